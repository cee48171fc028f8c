// Fused bf16 MLP stacks for the small-network regime (gfx950 / CDNA4, wave64).
//
// A CTR model's MLPs are a few hundred units wide, so at a batch of a few thousand samples
// every single layer is far too little work for the chip: layer-by-layer GEMM launches are
// latency bound.  Here one workgroup owns a tile of 32 samples and carries it through ALL
// layers of a stack (bottom or top network, Section 3.1): the tile's activations stay in
// LDS as the MFMA A operand, the weights are streamed from L2 straight into MFMA B fragments
// (each weight is used once per tile, so staging them in LDS would buy nothing).  A small
// prep kernel at the start of every step rounds the replica's fp32 master weights to
// bfloat16 (nearest even, as the layer-wise path does on load) and lays them out in fragment
// order -- for every (32-column tile, 16-deep reduction step) the 64 lanes' 8 values are
// contiguous -- once for X W^T and once for dY W, so each fragment load is one fully
// coalesced 1 KB wave access and several reduction steps can be kept in flight.  Kernels:
//   prep     : fp32 W -> the two bf16 fragment-ordered copies;
//   forward  : x -> a_1 -> ... -> a_L (+ for the top stack the one-unit output layer, the
//              mean log-loss and dL/dlogit);
//   backward : dL/da_L -> ... -> dL/da_0 (data gradients only), ReLU-gated;
//   wgrad    : all weight and bias gradients of all layers in one grouped launch,
//              dW_l = dY_l^T X_l as 64x64 tiles, one block of four waves per tile; each wave
//              keeps the whole tile in registers over its quarter of the batch, the four
//              partial tiles are folded through LDS and stored once (added atomically only
//              when the batch is also split over blocks, one slice per ~1024 samples).
// Activations and gradients that cross kernels are stored TRANSPOSED ([unit][sample], bf16):
// an MFMA accumulator holds 4 consecutive samples of one unit per lane, so this is the cheap
// direction to store, it is the layout the ReLU gate wants to read, and it makes the batch
// dimension contiguous for the weight-gradient fragments (no LDS transpose anywhere).
#include "ss_internal.h"

namespace ss {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int TB = 32;     // samples per workgroup
constexpr int APAD = 8;    // bf16 elements of LDS row padding
constexpr int NT = 1024;   // threads per workgroup: 16 waves, one 32-column tile each (widths <= 512)

__device__ __forceinline__ uint16_t f2b(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float b2f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint32_t pk(float lo, float hi) {
  return (uint32_t)f2b(lo) | ((uint32_t)f2b(hi) << 16);
}

union Frag {
  bf16x8 v;
  uint32_t u[4];
  uint4 q;
};

// Fragment-ordered bf16 weights: element (tile, step, lane, j), 8 values per lane.
//   forward copy : tile = n/32, step = k/16, lane = n%32 + 32*((k%16)/8), j = k%8
//   backward copy: tile = k/32, step = n/16, lane = k%32 + 32*((n%16)/8), j = n%8
__device__ __forceinline__ Frag load_frag(const uint16_t* __restrict__ Wsw, int tile, int steps,
                                          int step, int lane) {
  Frag f;
  f.q = *(const uint4*)(Wsw + (((size_t)tile * steps + step) * 64 + lane) * 8);
  return f;
}

// One layer's product for a 32-sample tile.  A workgroup has 16 waves; wave w owns the 32
// output columns of tile w (widths up to 512), so acc is one 32x32 accumulator.  A comes from
// LDS (row stride lda bf16), B fragments from the fragment-ordered copy.  DEPTH reduction
// steps (8 or 4) are kept in flight per wave (16 waves x 8 steps x 1 KB = 128 KB of weights
// requested at once); steps is a multiple of DEPTH (the reduction length is zero padded), the
// loop body has no branches, so the loads stay in flight behind the MFMAs, and the last group
// is peeled off so that no request is issued that nobody will use.  The first
// group is loaded separately (load_group) so that the caller can issue it early -- before the
// input tile is staged, or before the previous layer's epilogue -- and its latency is hidden.
template <int DEPTH>
__device__ __forceinline__ void load_group(Frag (&q)[8], const uint16_t* __restrict__ Wsw,
                                           int steps, int tile, int lane) {
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) q[d] = load_frag(Wsw, tile, steps, d, lane);
}

template <int DEPTH>
__device__ __forceinline__ void run_gemm(f32x16& acc, Frag (&q)[8],
                                         const uint16_t* __restrict__ A, int lda, int steps,
                                         int tile, int lane, const uint16_t* __restrict__ Wsw) {
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  int s0 = 0;
  for (; s0 + DEPTH < steps; s0 += DEPTH) {  // every group but the last refills its slots
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const bf16x8 a = *(const bf16x8*)(A + frow * lda + (s0 + d) * 16 + fk);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[d].v, acc, 0, 0, 0);
      q[d] = load_frag(Wsw, tile, steps, s0 + DEPTH + d, lane);
    }
  }
#pragma unroll
  for (int d = 0; d < DEPTH; ++d) {  // last group: nothing left to request
    const bf16x8 a = *(const bf16x8*)(A + frow * lda + (s0 + d) * 16 + fk);
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, q[d].v, acc, 0, 0, 0);
  }
}

__device__ __forceinline__ void load_group_n(int depth, Frag (&q)[8],
                                             const uint16_t* __restrict__ Wsw, int steps, int tile,
                                             int lane) {
  if (depth == 8) load_group<8>(q, Wsw, steps, tile, lane);
  else load_group<4>(q, Wsw, steps, tile, lane);
}
__device__ __forceinline__ void run_gemm_n(int depth, f32x16& acc, Frag (&q)[8],
                                           const uint16_t* __restrict__ A, int lda, int steps,
                                           int tile, int lane, const uint16_t* __restrict__ Wsw) {
  if (depth == 8) run_gemm<8>(acc, q, A, lda, steps, tile, lane, Wsw);
  else run_gemm<4>(acc, q, A, lda, steps, tile, lane, Wsw);
}

}  // namespace

// ------------------------------------------------------------------------------------------
// Prep: fp32 master weights -> bf16 in fragment order (both copies), one thread per 8 values.
__global__ __launch_bounds__(256) void mlp_prep_kernel(PrepArgs g) {
  const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;  // index of an 8-value fragment
  // the step's dense-gradient accumulator is cleared here (the later kernels add into it)
  if (g.zero) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = v; i < g.zero_n; i += stride) g.zero[i] = 0.f;
  }
  if (g.cast_dst) {
    const int64_t stride = (int64_t)gridDim.x * 256, n = (int64_t)g.cast_rows * g.cast_ld;
    for (int64_t i = v; i < n; i += stride) {
      const int r = (int)(i / g.cast_ld), c = (int)(i - (int64_t)r * g.cast_ld);
      g.cast_dst[i] = (c < g.cast_cols) ? f2b(g.cast_src[(size_t)r * g.cast_cols + c]) : (uint16_t)0;
    }
  }
  if (v >= g.total_frags) return;
  int l = 0;
  while (l + 1 < g.n_layers && v >= g.L[l + 1].frag_base) ++l;
  const PrepLayer L = g.L[l];
  int64_t r = v - L.frag_base;
  const bool bwd = r >= L.frags_fwd;
  if (bwd) r -= L.frags_fwd;
  const int lane = (int)(r & 63);
  const int64_t ts = r >> 6;
  Frag f;
  float e[8];
  if (!bwd) {
    const int steps = L.kp_f / 16;
    const int tile = (int)(ts / steps), step = (int)(ts - (int64_t)tile * steps);
    const int n = tile * 32 + (lane & 31), k = step * 16 + (lane >> 5) * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = (n < L.out && k + j < L.in) ? L.W[(size_t)n * L.in + k + j] : 0.f;
  } else {
    const int steps = L.kp_r / 16;
    const int tile = (int)(ts / steps), step = (int)(ts - (int64_t)tile * steps);
    const int k = tile * 32 + (lane & 31), n = step * 16 + (lane >> 5) * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) e[j] = (k < L.in && n + j < L.out) ? L.W[(size_t)(n + j) * L.in + k] : 0.f;
  }
  f.u[0] = pk(e[0], e[1]); f.u[1] = pk(e[2], e[3]); f.u[2] = pk(e[4], e[5]); f.u[3] = pk(e[6], e[7]);
  *(uint4*)((bwd ? L.Wr : L.Wf) + r * 8) = f.q;
}

// ------------------------------------------------------------------------------------------
// Forward.
__global__ __launch_bounds__(NT) void mlp_fused_fwd_kernel(FusedFwdArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* buf[2] = {smem, smem + g.lds_elems0};
  __shared__ float wl_s[512];
  __shared__ float wloss[16];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = blockIdx.x * TB;
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  // ---- first layer's weights and bias, and the tail's weights: requested before anything else
  Frag q[8];
  float bcur = 0.f, bnext = 0.f;
  {
    const FusedLayer L = g.L[0];
    if (wave * 32 < L.out) {
      load_group_n(L.depth_f, q, L.Wf, L.kp_f / 16, wave, lane);
      const int n = wave * 32 + col_in;
      if (n < L.out) bcur = L.b[n];
    }
  }
  float wl_r = 0.f;
  if (g.has_tail && tid < g.L[g.n_layers - 1].out) wl_r = g.w_last[tid];
  // ---- stage the input tile (bf16, zero padded columns and rows), then write its transposed
  //      copy for the weight-gradient kernel from LDS
  {
    const int Kp = g.L[0].kp_f, lda = Kp + APAD;
    const bool vec = !g.x_is_f32 && (g.ldx % 8 == 0) && ((((uintptr_t)g.x) & 15) == 0);
    if (vec) {
      const uint16_t* xs = (const uint16_t*)g.x;
      for (int i = tid; i < TB * (Kp / 8); i += NT) {
        const int r = i / (Kp / 8), k = (i - r * (Kp / 8)) * 8, b = b0 + r;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (b < g.B) {
          if (k + 8 <= g.in0) {
            v = *(const uint4*)(xs + (size_t)b * g.ldx + k);
          } else if (k < g.in0) {
            uint32_t e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = (k + j < g.in0) ? (uint32_t)xs[(size_t)b * g.ldx + k + j] : 0u;
            v = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                           e[6] | (e[7] << 16));
          }
        }
        *(uint4*)(buf[0] + r * lda + k) = v;
      }
    } else {
      for (int i = tid; i < TB * Kp; i += NT) {
        const int r = i / Kp, k = i - r * Kp, b = b0 + r;
        uint16_t v = 0;
        if (b < g.B && k < g.in0)
          v = g.x_is_f32 ? f2b(((const float*)g.x)[(size_t)b * g.ldx + k])
                         : ((const uint16_t*)g.x)[(size_t)b * g.ldx + k];
        buf[0][r * lda + k] = v;
      }
    }
    if (g.has_tail && tid < 512) wl_s[tid] = b2f(f2b(wl_r));
    __syncthreads();
    if (g.xT) {  // 8 consecutive samples of one input unit per thread: one 16-byte store
      for (int i = tid; i < g.in0 * (TB / 8); i += NT) {
        const int k = i / (TB / 8), r = (i - k * (TB / 8)) * 8, b = b0 + r;
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = buf[0][(r + j) * lda + k];
        uint16_t* p = g.xT + (size_t)k * g.ldT + b;
        if (b + 8 <= g.B) {
          *(uint4*)p = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                                  e[6] | (e[7] << 16));
        } else {
          for (int j = 0; j < 8 && b + j < g.B; ++j) p[j] = (uint16_t)e[j];
        }
      }
    }
  }
  for (int l = 0; l < g.n_layers; ++l) {
    const FusedLayer L = g.L[l];
    const uint16_t* A = buf[l & 1];
    uint16_t* O = buf[(l + 1) & 1];
    const int Kp = L.kp_f, lda = Kp + APAD;
    const bool last = (l == g.n_layers - 1);
    const int Np = last ? g.kp_tail : g.L[l + 1].kp_f, ldo = Np + APAD;
    const int ntiles = (L.out + 31) / 32;
    const bool active = wave < ntiles;
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    if (active) run_gemm_n(L.depth_f, acc, q, A, lda, Kp / 16, wave, lane, L.Wf);
    if (!last) {  // next layer's first fragments and bias fly during this layer's epilogue
      const FusedLayer N = g.L[l + 1];
      bnext = 0.f;
      if (wave * 32 < N.out) {
        load_group_n(N.depth_f, q, N.Wf, N.kp_f / 16, wave, lane);
        const int n = wave * 32 + col_in;
        if (n < N.out) bnext = N.b[n];
      }
    }
    const bool relu = !last || g.relu_last;
    if (active) {
      const int n = wave * 32 + col_in;
      const bool nok = n < L.out;
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int r = e4 * 8 + row_in;  // rows r .. r+3
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = acc[e4 * 4 + i] + bcur;
          if (relu) v[i] = fmaxf(v[i], 0.f);
        }
        if (n < Np) {
#pragma unroll
          for (int i = 0; i < 4; ++i) O[(r + i) * ldo + n] = nok ? f2b(v[i]) : (uint16_t)0;
        }
        if (nok) {
          const int b = b0 + r;
          if (g.actT[l] && b < g.B) {  // 4 consecutive samples of unit n: one 8-byte store
            uint16_t* p = g.actT[l] + (size_t)n * g.ldT + b;
            if (b + 3 < g.B) {
              *(uint2*)p = make_uint2(pk(v[0], v[1]), pk(v[2], v[3]));
            } else {
              for (int i = 0; i < 4 && b + i < g.B; ++i) p[i] = f2b(v[i]);
            }
          }
          if (last && g.out_f32) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (b + i < g.B) g.out_f32[(size_t)(b + i) * L.out + n] = v[i];
          }
        }
      }
    }
    // padded columns no tile covers must read as zero in the next product
    for (int i = tid; i < TB * (Np - ntiles * 32); i += NT) {
      const int w = Np - ntiles * 32, r = i / w, n = ntiles * 32 + (i - r * w);
      O[r * ldo + n] = 0;
    }
    bcur = bnext;
    __syncthreads();
  }
  // ---- top stack only: one-unit output layer, loss and dL/dlogit (32 threads per sample)
  if (g.has_tail) {
    const uint16_t* A = buf[g.n_layers & 1];
    const int in = g.L[g.n_layers - 1].out, lda = g.kp_tail + APAD;
    const int r = tid >> 5, sub = tid & 31, b = b0 + r;
    float s = 0.f;
    for (int k = sub; k < in; k += 32) s += b2f(A[r * lda + k]) * wl_s[k];
#pragma unroll
    for (int off = 1; off < 32; off <<= 1) s += __shfl_xor(s, off);
    float lossv = 0.f;
    const float invB = 1.0f / (float)g.B;
    if (sub == 0 && b < g.B) {
      const float lg = s + g.b_last[0], t = g.y[b];
      const float ex = expf(-fabsf(lg));
      lossv = fmaxf(lg, 0.f) - lg * t + log1pf(ex);
      const float p = (lg >= 0.f) ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
      g.logits[b] = lg;
      if (g.dlogit) g.dlogit[b] = (p - t) * invB;
    }
    // block sum of the 32 per-sample losses (two samples per wave)
    lossv += __shfl_xor(lossv, 32);
    if (lane == 0) wloss[wave] = lossv;
    __syncthreads();
    if (tid == 0) {
      float tot = 0.f;
#pragma unroll
      for (int i = 0; i < 16; ++i) tot += wloss[i];
      atomicAdd(g.loss, tot * invB);
    }
  }
}

// ------------------------------------------------------------------------------------------
// Backward (data gradients through the stack).
__global__ __launch_bounds__(NT) void mlp_fused_bwd_kernel(FusedBwdArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* buf[2] = {smem, smem + g.lds_elems0};
  __shared__ float dl[TB], dlq[TB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = blockIdx.x * TB;
  const int nl = g.n_layers;
  const int wlast = g.L[nl - 1].out;  // width of the stack's output
  const int Wp0 = g.L[nl - 1].kp_r, ld0 = Wp0 + APAD;
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  const bool full_tile = (b0 + TB <= g.B);
  // ---- the first product's weight fragments are requested before anything else
  Frag q[8];
  const bool any_product = !(nl == 1 && !g.d_out_f32);
  if (any_product) {
    const FusedLayer L = g.L[nl - 1];
    if (wave * 32 < L.in) load_group_n(L.depth_r, q, L.Wr, L.kp_r / 16, wave, lane);
  }
  // ---- incoming gradient tile -> LDS buffer 0 (+ transposed copy for the weight gradients)
  if (g.dlogit) {
    // top stack: dL/da = q(dlogit_b) q(w_k), gated by a > 0; plus the output layer's own
    // weight and bias gradients
    if (tid < TB) {
      const float v = (b0 + tid < g.B) ? g.dlogit[b0 + tid] : 0.f;
      dl[tid] = v;
      dlq[tid] = b2f(f2b(v));
    }
    __syncthreads();
    const uint16_t* aT = g.actT[nl - 1];
    if (full_tile) {
      // four threads per unit, eight samples each: the 32 samples of unit k are 64 contiguous
      // bytes in both transposed arrays, 16 of them per thread
      for (int i = tid; i < Wp0 * 4; i += NT) {
        const int k = i >> 2, c = i & 3;
        const bool kok = k < wlast;
        const float wq = kok ? b2f(f2b(g.w_last[k])) : 0.f;
        float acc = 0.f;
        uint4 av = make_uint4(0, 0, 0, 0);
        if (kok) av = *((const uint4*)(aT + (size_t)k * g.ldT + b0) + c);
        const uint32_t w4[4] = {av.x, av.y, av.z, av.w};
        uint32_t o4[4];
#pragma unroll
        for (int h2 = 0; h2 < 4; ++h2) {
          uint32_t ow = 0;
#pragma unroll
          for (int q2 = 0; q2 < 2; ++q2) {
            const int r = c * 8 + h2 * 2 + q2;
            const uint16_t a = (uint16_t)(w4[h2] >> (16 * q2));
            acc += dlq[r] * b2f(a);
            const uint16_t out = (kok && (int16_t)a > 0) ? f2b(dlq[r] * wq) : (uint16_t)0;
            buf[0][r * ld0 + k] = out;
            ow |= (uint32_t)out << (16 * q2);
          }
          o4[h2] = ow;
        }
        if (kok) *((uint4*)(g.dYT[nl - 1] + (size_t)k * g.ldT + b0) + c) = make_uint4(o4[0], o4[1], o4[2], o4[3]);
        // the four threads of a unit are neighbouring lanes
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        if (kok && c == 0) atomicAdd(g.g_w_last + k, acc);
      }
    } else {
      for (int k = tid; k < Wp0; k += NT) {
        const bool kok = k < wlast;
        const float wq = kok ? b2f(f2b(g.w_last[k])) : 0.f;
        float acc = 0.f;
        for (int r = 0; r < TB; ++r) {
          const int b = b0 + r;
          uint16_t out = 0;
          if (kok && b < g.B) {
            const uint16_t a = aT[(size_t)k * g.ldT + b];
            acc += dlq[r] * b2f(a);
            out = ((int16_t)a > 0) ? f2b(dlq[r] * wq) : (uint16_t)0;
            g.dYT[nl - 1][(size_t)k * g.ldT + b] = out;
          }
          buf[0][r * ld0 + k] = out;
        }
        if (kok) atomicAdd(g.g_w_last + k, acc);
      }
    }
    if (tid == 0) {
      float sb = 0.f;
      for (int r = 0; r < TB; ++r) sb += dl[r];
      atomicAdd(g.g_b_last, sb);
    }
  } else {
    // bottom stack: dz0 arrives in fp32, already gated
    const int Wp = Wp0;
    const bool vec = (wlast % 4 == 0) && (g.ld_d_in % 4 == 0);
    for (int i = tid; i < TB * (Wp / 4); i += NT) {
      const int r = i / (Wp / 4), k = (i - r * (Wp / 4)) * 4, b = b0 + r;
      float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
      if (b < g.B && k < wlast) {
        const float* p = g.d_in_f32 + (size_t)b * g.ld_d_in + k;
        if (vec) v = *(const float4*)p;
        else { v.x = p[0]; if (k + 1 < wlast) v.y = p[1]; if (k + 2 < wlast) v.z = p[2]; if (k + 3 < wlast) v.w = p[3]; }
      }
      *(uint2*)(buf[0] + r * ld0 + k) = make_uint2(pk(v.x, v.y), pk(v.z, v.w));
    }
    __syncthreads();
    for (int i = tid; i < wlast * (TB / 8); i += NT) {
      const int k = i / (TB / 8), r = (i - k * (TB / 8)) * 8, b = b0 + r;
      uint32_t e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = buf[0][(r + j) * ld0 + k];
      uint16_t* p = g.dYT[nl - 1] + (size_t)k * g.ldT + b;
      if (b + 8 <= g.B) {
        *(uint4*)p = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                                e[6] | (e[7] << 16));
      } else {
        for (int j = 0; j < 8 && b + j < g.B; ++j) p[j] = (uint16_t)e[j];
      }
    }
  }
  __syncthreads();
  int cur = 0;
  for (int l = nl - 1; l >= 0; --l) {
    if (l == 0 && !g.d_out_f32) break;  // the stack's input needs no gradient
    const FusedLayer L = g.L[l];
    const uint16_t* A = buf[cur];
    uint16_t* O = buf[cur ^ 1];
    const int Kred = L.kp_r, lda = Kred + APAD;  // reduction over this layer's outputs
    const int Np = (l > 0) ? g.L[l - 1].kp_r : 0, ldo = Np + APAD;  // result = next reduction
    const int ntiles = (L.in + 31) / 32;
    const bool active = wave < ntiles;
    const int k = wave * 32 + col_in;
    const bool kok = active && k < L.in;
    // ReLU gates of this lane's results (activations of the layer below), requested now so
    // that they arrive while the product runs
    uint2 gate[4];
#pragma unroll
    for (int e4 = 0; e4 < 4; ++e4) {
      gate[e4] = make_uint2(0, 0);
      if (l > 0 && full_tile && kok)
        gate[e4] = *(const uint2*)(g.actT[l - 1] + (size_t)k * g.ldT + b0 + e4 * 8 + row_in);
    }
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
    if (active) run_gemm_n(L.depth_r, acc, q, A, lda, Kred / 16, wave, lane, L.Wr);
    if (l > 1 || (l == 1 && g.d_out_f32)) {  // next product's first fragments
      const FusedLayer N = g.L[l - 1];
      if (wave * 32 < N.in) load_group_n(N.depth_r, q, N.Wr, N.kp_r / 16, wave, lane);
    }
    if (active) {
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int r = e4 * 8 + row_in, b = b0 + r;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = acc[e4 * 4 + i];
        if (l > 0) {
          // gate with the previous layer's activation, keep for the next product and for
          // the weight gradients
          uint16_t o[4] = {0, 0, 0, 0};
          if (kok && b < g.B) {
            uint16_t* dp = g.dYT[l - 1] + (size_t)k * g.ldT + b;
            if (full_tile) {
              const uint2 a = gate[e4];
              const uint16_t av[4] = {(uint16_t)a.x, (uint16_t)(a.x >> 16), (uint16_t)a.y,
                                      (uint16_t)(a.y >> 16)};
#pragma unroll
              for (int i = 0; i < 4; ++i) o[i] = ((int16_t)av[i] > 0) ? f2b(v[i]) : (uint16_t)0;
              *(uint2*)dp = make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16),
                                       (uint32_t)o[2] | ((uint32_t)o[3] << 16));
            } else {
              const uint16_t* ap = g.actT[l - 1] + (size_t)k * g.ldT + b;
              for (int i = 0; i < 4 && b + i < g.B; ++i) {
                o[i] = ((int16_t)ap[i] > 0) ? f2b(v[i]) : (uint16_t)0;
                dp[i] = o[i];
              }
            }
          }
          if (k < Np) {
#pragma unroll
            for (int i = 0; i < 4; ++i) O[(r + i) * ldo + k] = o[i];
          }
        } else if (kok) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (b + i < g.B) g.d_out_f32[(size_t)(b + i) * g.ld_d_out + k] = v[i];
        }
      }
    }
    if (l > 0) {
      for (int i = tid; i < TB * (Np - ntiles * 32); i += NT) {
        const int w = Np - ntiles * 32, r = i / w, kk = ntiles * 32 + (i - r * w);
        O[r * ldo + kk] = 0;
      }
    }
    cur ^= 1;
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Grouped weight gradients.  One block = one 64x64 tile of one layer's dW over one slice of
// the batch (blockIdx.x walks the tile table, blockIdx.y the slices); its four waves split the
// slice's samples, each keeping the whole 64x64 tile (2x2 MFMA tiles) in registers, and fold
// their sums through LDS.  Both fragments are 16-byte global loads (the batch is the
// contiguous dimension of the transposed operands).  Tiles with k0 == 0 also produce the bias
// gradient through one extra MFMA per row block against a fragment of ones.
constexpr int WG_T = 64;            // tile edge
constexpr int WG_LD = WG_T + 1;     // LDS row pitch (floats)
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void mlp_wgrad_grouped_kernel(WgradArgs g) {
  extern __shared__ float wg_red[];  // [4][64][65] tile sums + [4][64] bias sums
  float* const redb = wg_red + 4 * WG_T * WG_LD;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int4 t = g.tiles[blockIdx.x];
  const WgradLayer L = g.L[t.x];
  const int n0 = t.y, k0 = t.z;
  const int nsplit = gridDim.y * 4;
  const int per = (((g.B + nsplit - 1) / nsplit) + 15) & ~15;
  const int bbeg = (blockIdx.y * 4 + wave) * per;
  const int bend = min(g.B, bbeg + per);
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const uint16_t* ap[2];
  const uint16_t* bp[2];
  bool aok[2], bok[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int n = n0 + i * 32 + frow, k = k0 + i * 32 + frow;
    aok[i] = n < L.out; bok[i] = k < L.in;
    ap[i] = L.dYT + (size_t)(aok[i] ? n : 0) * g.ldT;
    bp[i] = L.XT + (size_t)(bok[i] ? k : 0) * g.ldT;
  }
  const bool do_bias = (k0 == 0);
  f32x16 acc[2][2], accb[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) { accb[i][e] = 0.f; acc[i][0][e] = 0.f; acc[i][1][e] = 0.f; }
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  auto ld = [&](const uint16_t* p, bool ok, int b) {
    Frag f;
    f.q = make_uint4(0, 0, 0, 0);
    if (ok && b < bend) {
      if (b + 8 <= bend) {
        f.q = *(const uint4*)(p + b);
      } else {
        uint32_t e[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) e[j] = (b + j < bend) ? (uint32_t)p[b + j] : 0u;
        f.q = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                         e[6] | (e[7] << 16));
      }
    }
    return f;
  };
  constexpr int WD = 4;  // batch steps of 16 samples in flight
  Frag a[WD][2], b[WD][2];
#pragma unroll
  for (int d = 0; d < WD; ++d)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[d][i] = ld(ap[i], aok[i], bbeg + d * 16 + fk);
      b[d][i] = ld(bp[i], bok[i], bbeg + d * 16 + fk);
    }
  for (int bb = bbeg; bb < bend; bb += 16 * WD) {
#pragma unroll
    for (int d = 0; d < WD; ++d) {
      if (bb + d * 16 < bend) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[d][i].v, b[d][j].v, acc[i][j], 0, 0, 0);
          if (do_bias) accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[d][i].v, ones, accb[i], 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          a[d][i] = ld(ap[i], aok[i], bb + (d + WD) * 16 + fk);
          b[d][i] = ld(bp[i], bok[i], bb + (d + WD) * 16 + fk);
        }
      }
    }
  }
  // every wave lays its tile down in LDS; then all 256 threads add the four copies, 16
  // outputs each, and store (or add atomically when the batch is split over blocks)
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  float* mine = wg_red + wave * WG_T * WG_LD;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int rr = i * 32 + (e >> 2) * 8 + row_in + (e & 3);
#pragma unroll
      for (int j = 0; j < 2; ++j) mine[rr * WG_LD + j * 32 + col_in] = acc[i][j][e];
      if (do_bias && col_in == 0) redb[wave * WG_T + rr] = accb[i][e];
    }
  }
  __syncthreads();
  const bool atomic = gridDim.y > 1;
#pragma unroll
  for (int u = 0; u < 16; ++u) {
    const int idx = threadIdx.x + 256 * u;   // consecutive threads: consecutive columns
    const int rr = idx >> 6, cc = idx & 63;
    const int nn = n0 + rr, kk = k0 + cc;
    const float v = (wg_red[rr * WG_LD + cc] + wg_red[WG_T * WG_LD + rr * WG_LD + cc]) +
                    (wg_red[2 * WG_T * WG_LD + rr * WG_LD + cc] + wg_red[3 * WG_T * WG_LD + rr * WG_LD + cc]);
    if (nn < L.out && kk < L.in) {
      if (atomic) atomicAdd(L.gW + (size_t)nn * L.in + kk, v);
      else L.gW[(size_t)nn * L.in + kk] = v;
    }
  }
  if (do_bias && threadIdx.x < WG_T) {
    const int nn = n0 + threadIdx.x;
    const float vb = (redb[threadIdx.x] + redb[WG_T + threadIdx.x]) +
                     (redb[2 * WG_T + threadIdx.x] + redb[3 * WG_T + threadIdx.x]);
    if (nn < L.out) {
      if (atomic) atomicAdd(L.gb + nn, vb);
      else L.gb[nn] = vb;
    }
  }
}

// ------------------------------------------------------------------------------------------
size_t fused_lds_bytes(const int* widths, int n_widths, size_t* elems0) {
  // widths[i] = padded row length of the i-th LDS tile of a launch; tile i lives in buffer i & 1
  size_t m[2] = {0, 0};
  for (int i = 0; i < n_widths; ++i) {
    const size_t e = (size_t)TB * (widths[i] + APAD);
    if (e > m[i & 1]) m[i & 1] = e;
  }
  if (elems0) *elems0 = m[0];
  return (m[0] + m[1]) * sizeof(uint16_t);
}

void launch_mlp_fused_fwd(const FusedFwdArgs& a, size_t lds_bytes, hipStream_t s) {
  hipLaunchKernelGGL(mlp_fused_fwd_kernel, dim3(ceil_div(a.B, TB)), dim3(NT), lds_bytes, s, a);
}

void launch_mlp_fused_bwd(const FusedBwdArgs& a, size_t lds_bytes, hipStream_t s) {
  hipLaunchKernelGGL(mlp_fused_bwd_kernel, dim3(ceil_div(a.B, TB)), dim3(NT), lds_bytes, s, a);
}

void launch_mlp_prep(const PrepArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(mlp_prep_kernel, dim3(ceil_div(a.total_frags, 256)), dim3(256), 0, s, a);
}

void launch_mlp_wgrad_grouped(const WgradArgs& a, int n_tiles, hipStream_t s) {
  // batch slices of about 256 samples per wave: fewer, longer slices cost less in atomics
  // and LDS folds than they lose in parallelism once several streams share the chip
  int gy = a.B / (4 * 256);
  if (gy < 1) gy = 1;
  if (gy > 8) gy = 8;
  const size_t lds = (size_t)(4 * WG_T * WG_LD + 4 * WG_T) * sizeof(float);
  hipLaunchKernelGGL(mlp_wgrad_grouped_kernel, dim3(n_tiles, gy), dim3(256), lds, s, a);
}

}  // namespace ss
