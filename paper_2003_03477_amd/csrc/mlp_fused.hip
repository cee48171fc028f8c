// Fused bf16 MLP stacks for the small-network regime (gfx950 / CDNA4, wave64).
//
// A CTR model's MLPs are a few hundred units wide, so at a batch of a few thousand samples
// every single layer is far too little work for the chip: layer-by-layer GEMM launches are
// latency bound.  Here one workgroup owns a tile of 32 samples and carries it through ALL
// layers of a stack (bottom or top network, Section 3.1): the tile's activations stay in
// LDS as the MFMA A operand, the weights are streamed from L2/HBM straight into MFMA B
// fragments (each weight is used once per tile, so staging them in LDS would buy nothing)
// and are rounded from the fp32 master copy to bfloat16 on the way, exactly as the
// layer-wise path does.  Three kernels:
//   forward  : x -> a_1 -> ... -> a_L (+ for the top stack the one-unit output layer, the
//              mean log-loss and dL/dlogit);
//   backward : dL/da_L -> ... -> dL/da_0 (data gradients only), ReLU-gated;
//   wgrad    : all weight and bias gradients of all layers in one grouped launch,
//              dW_l = dY_l^T X_l as wave-sized 32x32 tiles over batch slices, accumulated
//              with atomics.
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
constexpr int MAXT = 4;    // 32-column tiles per wave (4 waves -> widths up to 512)

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

// B fragment for the forward product X W^T: 8 consecutive k of weight row n (fp32 -> bf16).
struct RawK {
  float4 a, b;
};
__device__ __forceinline__ RawK load_w_rowk(const float* __restrict__ W, int ld, int n, int k,
                                            int N, int K) {
  RawK r;
  r.a = make_float4(0.f, 0.f, 0.f, 0.f);
  r.b = r.a;
  if (n < N) {
    const float* p = W + (size_t)n * ld + k;
    if (k + 8 <= K && ((((uintptr_t)p) & 15) == 0)) {
      r.a = *(const float4*)p;
      r.b = *(const float4*)(p + 4);
    } else {
      float e[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) e[j] = (k + j < K) ? p[j] : 0.f;
      r.a = make_float4(e[0], e[1], e[2], e[3]);
      r.b = make_float4(e[4], e[5], e[6], e[7]);
    }
  }
  return r;
}
__device__ __forceinline__ bf16x8 cvt(const RawK& r) {
  Frag f;
  f.u[0] = pk(r.a.x, r.a.y); f.u[1] = pk(r.a.z, r.a.w);
  f.u[2] = pk(r.b.x, r.b.y); f.u[3] = pk(r.b.z, r.b.w);
  return f.v;
}

// B fragment for the data gradient dY W: 8 consecutive rows n of weight column k.
struct RawN {
  float e[8];
};
__device__ __forceinline__ RawN load_w_coln(const float* __restrict__ W, int ld, int n, int k,
                                            int N, int K) {
  RawN r;
#pragma unroll
  for (int j = 0; j < 8; ++j) r.e[j] = (k < K && n + j < N) ? W[(size_t)(n + j) * ld + k] : 0.f;
  return r;
}
__device__ __forceinline__ bf16x8 cvt(const RawN& r) {
  Frag f;
  f.u[0] = pk(r.e[0], r.e[1]); f.u[1] = pk(r.e[2], r.e[3]);
  f.u[2] = pk(r.e[4], r.e[5]); f.u[3] = pk(r.e[6], r.e[7]);
  return f.v;
}

// acc[j] (+)= A_tile[32 x Kred] * B, for this wave's column tiles j (tile index w + 4j).
// A comes from LDS (row stride lda bf16), B fragments from global through `loadB(tile_col,
// kred)`; the fragments of reduction step s+1 are in flight during the MFMAs of step s.
template <typename Raw, typename LoadB>
__device__ __forceinline__ void tile_gemm(f32x16 (&acc)[MAXT], const uint16_t* __restrict__ A,
                                          int lda, int Kred_pad, int ntiles_mine, int lane,
                                          LoadB loadB) {
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  Raw cur[MAXT], nxt[MAXT];
#pragma unroll
  for (int j = 0; j < MAXT; ++j)
    if (j < ntiles_mine) cur[j] = loadB(j, fk);
  for (int k0 = 0; k0 < Kred_pad; k0 += 16) {
    if (k0 + 16 < Kred_pad) {
#pragma unroll
      for (int j = 0; j < MAXT; ++j)
        if (j < ntiles_mine) nxt[j] = loadB(j, k0 + 16 + fk);
    }
    const bf16x8 a = *(const bf16x8*)(A + frow * lda + k0 + fk);
#pragma unroll
    for (int j = 0; j < MAXT; ++j)
      if (j < ntiles_mine)
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, cvt(cur[j]), acc[j], 0, 0, 0);
#pragma unroll
    for (int j = 0; j < MAXT; ++j) cur[j] = nxt[j];
  }
}

__device__ __forceinline__ void zero_acc(f32x16 (&acc)[MAXT]) {
#pragma unroll
  for (int j = 0; j < MAXT; ++j)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
}

__device__ __forceinline__ int pad16(int k) { return (k + 15) & ~15; }

}  // namespace

// ------------------------------------------------------------------------------------------
// Forward.
__global__ __launch_bounds__(256) void mlp_fused_fwd_kernel(FusedFwdArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* buf[2] = {smem, smem + g.lds_elems0};
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = blockIdx.x * TB;
  // ---- stage the input tile (bf16, zero padded to a multiple of 16 columns and 32 rows),
  //      and its transposed copy for the weight-gradient kernel
  {
    const int Kp = pad16(g.in0), lda = Kp + APAD;
    for (int i = tid; i < TB * Kp; i += 256) {
      const int r = i / Kp, k = i - r * Kp, b = b0 + r;
      uint16_t v = 0;
      if (b < g.B && k < g.in0)
        v = g.x_is_f32 ? f2b(((const float*)g.x)[(size_t)b * g.ldx + k])
                       : ((const uint16_t*)g.x)[(size_t)b * g.ldx + k];
      buf[0][r * lda + k] = v;
    }
    if (g.xT) {
      for (int i = tid; i < g.in0 * TB; i += 256) {
        const int k = i / TB, r = i - k * TB, b = b0 + r;
        if (b < g.B) {
          const uint16_t v = g.x_is_f32 ? f2b(((const float*)g.x)[(size_t)b * g.ldx + k])
                                        : ((const uint16_t*)g.x)[(size_t)b * g.ldx + k];
          g.xT[(size_t)k * g.ldT + b] = v;
        }
      }
    }
  }
  __syncthreads();
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  for (int l = 0; l < g.n_layers; ++l) {
    const FusedLayer L = g.L[l];
    const uint16_t* A = buf[l & 1];
    uint16_t* O = buf[(l + 1) & 1];
    const int Kp = pad16(L.in), lda = Kp + APAD;
    const int Np = pad16(L.out), ldo = Np + APAD;
    const int ntiles = (L.out + 31) / 32;
    const int mine = (ntiles > wave) ? (ntiles - wave + 3) / 4 : 0;
    f32x16 acc[MAXT];
    zero_acc(acc);
    tile_gemm<RawK>(acc, A, lda, Kp, mine, lane, [&](int j, int k) {
      return load_w_rowk(L.W, L.in, (wave + 4 * j) * 32 + col_in, k, L.out, L.in);
    });
    const bool last = (l == g.n_layers - 1);
    const bool relu = !last || g.relu_last;
#pragma unroll
    for (int j = 0; j < MAXT; ++j) {
      if (j >= mine) continue;
      const int n = (wave + 4 * j) * 32 + col_in;
      const bool nok = n < L.out;
      const float bv = nok ? L.b[n] : 0.f;
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int r = e4 * 8 + row_in;  // rows r .. r+3
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          v[i] = acc[j][e4 * 4 + i] + bv;
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
    __syncthreads();
  }
  // ---- top stack only: one-unit output layer, loss and dL/dlogit (8 threads per sample)
  if (g.has_tail) {
    const uint16_t* A = buf[g.n_layers & 1];
    const int in = g.L[g.n_layers - 1].out, lda = pad16(in) + APAD;
    const int r = tid >> 3, sub = tid & 7, b = b0 + r;
    float s = 0.f;
    for (int k = sub; k < in; k += 8) s += b2f(A[r * lda + k]) * b2f(f2b(g.w_last[k]));
    s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4);
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
    // block sum of the 32 per-sample losses
    __shared__ float wl[4];
    float ws = lossv;
    for (int off = 32; off > 0; off >>= 1) ws += __shfl_xor(ws, off);
    if (lane == 0) wl[wave] = ws;
    __syncthreads();
    if (tid == 0) atomicAdd(g.loss, (wl[0] + wl[1] + wl[2] + wl[3]) * invB);
  }
}

// ------------------------------------------------------------------------------------------
// Backward (data gradients through the stack).
__global__ __launch_bounds__(256) void mlp_fused_bwd_kernel(FusedBwdArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* buf[2] = {smem, smem + g.lds_elems0};
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int b0 = blockIdx.x * TB;
  const int nl = g.n_layers;
  const int wlast = g.L[nl - 1].out;  // width of the stack's output
  const int ld0 = pad16(wlast) + APAD;
  // ---- incoming gradient tile -> LDS buffer 0 (+ transposed copy for the weight gradients)
  if (g.dlogit) {
    // top stack: dL/da = q(dlogit_b) q(w_k), gated by a > 0; plus the output layer's own
    // weight and bias gradients
    __shared__ float dl[TB], dlq[TB];
    if (tid < TB) {
      const float v = (b0 + tid < g.B) ? g.dlogit[b0 + tid] : 0.f;
      dl[tid] = v;
      dlq[tid] = b2f(f2b(v));
    }
    __syncthreads();
    const uint16_t* aT = g.actT[nl - 1];
    for (int k = tid; k < pad16(wlast); k += 256) {
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
    if (tid == 0) {
      float sb = 0.f;
      for (int r = 0; r < TB; ++r) sb += dl[r];
      atomicAdd(g.g_b_last, sb);
    }
  } else {
    // bottom stack: dz0 arrives in fp32, already gated
    for (int i = tid; i < TB * pad16(wlast); i += 256) {
      const int r = i / pad16(wlast), k = i - r * pad16(wlast), b = b0 + r;
      uint16_t v = 0;
      if (b < g.B && k < wlast) v = f2b(g.d_in_f32[(size_t)b * g.ld_d_in + k]);
      buf[0][r * ld0 + k] = v;
    }
    for (int i = tid; i < wlast * TB; i += 256) {
      const int k = i / TB, r = i - k * TB, b = b0 + r;
      if (b < g.B) g.dYT[nl - 1][(size_t)k * g.ldT + b] = f2b(g.d_in_f32[(size_t)b * g.ld_d_in + k]);
    }
  }
  __syncthreads();
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  int cur = 0;
  for (int l = nl - 1; l >= 0; --l) {
    if (l == 0 && !g.d_out_f32) break;  // the stack's input needs no gradient
    const FusedLayer L = g.L[l];
    const uint16_t* A = buf[cur];
    uint16_t* O = buf[cur ^ 1];
    const int Kred = pad16(L.out), lda = Kred + APAD;  // reduction over this layer's outputs
    const int Np = pad16(L.in), ldo = Np + APAD;       // result columns = this layer's inputs
    const int ntiles = (L.in + 31) / 32;
    const int mine = (ntiles > wave) ? (ntiles - wave + 3) / 4 : 0;
    f32x16 acc[MAXT];
    zero_acc(acc);
    tile_gemm<RawN>(acc, A, lda, Kred, mine, lane, [&](int j, int n) {
      return load_w_coln(L.W, L.in, n, (wave + 4 * j) * 32 + col_in, L.out, L.in);
    });
#pragma unroll
    for (int j = 0; j < MAXT; ++j) {
      if (j >= mine) continue;
      const int k = (wave + 4 * j) * 32 + col_in;
      const bool kok = k < L.in;
#pragma unroll
      for (int e4 = 0; e4 < 4; ++e4) {
        const int r = e4 * 8 + row_in, b = b0 + r;
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = acc[j][e4 * 4 + i];
        if (l > 0) {
          // gate with the previous layer's activation, keep for the next product and for
          // the weight gradients
          uint16_t o[4] = {0, 0, 0, 0};
          if (kok && b < g.B) {
            const uint16_t* ap = g.actT[l - 1] + (size_t)k * g.ldT + b;
            uint16_t* dp = g.dYT[l - 1] + (size_t)k * g.ldT + b;
            if (b + 3 < g.B) {
              const uint2 a = *(const uint2*)ap;
              const uint16_t av[4] = {(uint16_t)a.x, (uint16_t)(a.x >> 16), (uint16_t)a.y,
                                      (uint16_t)(a.y >> 16)};
#pragma unroll
              for (int i = 0; i < 4; ++i) o[i] = ((int16_t)av[i] > 0) ? f2b(v[i]) : (uint16_t)0;
              *(uint2*)dp = make_uint2((uint32_t)o[0] | ((uint32_t)o[1] << 16),
                                       (uint32_t)o[2] | ((uint32_t)o[3] << 16));
            } else {
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
    cur ^= 1;
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------
// Grouped weight gradients.  One wave = one 32x32 tile of one layer's dW over one slice of
// the batch; blockIdx.x walks the tile table, the 4 waves of a block and blockIdx.y split the
// batch.  Both fragments are 16-byte global loads (the batch is the contiguous dimension of
// the transposed operands).  Tiles with k0 == 0 also produce the bias gradient through one
// extra MFMA against a fragment of ones.
__global__ __launch_bounds__(256) void mlp_wgrad_grouped_kernel(WgradArgs g) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int4 t = g.tiles[blockIdx.x];
  const WgradLayer L = g.L[t.x];
  const int n0 = t.y, k0 = t.z;
  const int nsplit = gridDim.y * 4;
  const int per = (((g.B + nsplit - 1) / nsplit) + 15) & ~15;
  const int bbeg = (blockIdx.y * 4 + wave) * per;
  const int bend = min(g.B, bbeg + per);
  if (bbeg >= bend) return;
  const int frow = lane & 31, fk = (lane >> 5) * 8;
  const int n = n0 + frow, k = k0 + frow;
  const uint16_t* ap = L.dYT + (size_t)n * g.ldT;
  const uint16_t* bp = L.XT + (size_t)k * g.ldT;
  const bool aok = n < L.out, bok = k < L.in;
  const bool do_bias = (k0 == 0);
  f32x16 acc, accb;
#pragma unroll
  for (int e = 0; e < 16; ++e) { acc[e] = 0.f; accb[e] = 0.f; }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;
  auto ld = [&](const uint16_t* p, bool ok, int b) {
    Frag f;
    f.q = make_uint4(0, 0, 0, 0);
    if (ok) {
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
  Frag a = ld(ap, aok, bbeg + fk), b = ld(bp, bok, bbeg + fk);
  for (int bb = bbeg; bb < bend; bb += 16) {
    Frag an, bn;
    an.q = make_uint4(0, 0, 0, 0);
    bn.q = an.q;
    if (bb + 16 < bend) {
      an = ld(ap, aok, bb + 16 + fk);
      bn = ld(bp, bok, bb + 16 + fk);
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
    if (do_bias) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, ones, accb, 0, 0, 0);
    a = an;
    b = bn;
  }
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  const int kk = k0 + col_in;
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int nn = n0 + (e >> 2) * 8 + row_in + (e & 3);
    if (nn < L.out) {
      if (kk < L.in) atomicAdd(L.gW + (size_t)nn * L.in + kk, acc[e]);
      if (do_bias && col_in == 0) atomicAdd(L.gb + nn, accb[e]);
    }
  }
}

// ------------------------------------------------------------------------------------------
size_t fused_lds_bytes(const int* widths, int n_widths, size_t* elems0) {
  // widths[0] = stack input, widths[i] = output of layer i-1; buffer (i & 1) holds widths[i]
  size_t m[2] = {0, 0};
  for (int i = 0; i < n_widths; ++i) {
    const size_t e = (size_t)TB * (((widths[i] + 15) & ~15) + APAD);
    if (e > m[i & 1]) m[i & 1] = e;
  }
  if (elems0) *elems0 = m[0];
  return (m[0] + m[1]) * sizeof(uint16_t);
}

void launch_mlp_fused_fwd(const FusedFwdArgs& a, size_t lds_bytes, hipStream_t s) {
  hipLaunchKernelGGL(mlp_fused_fwd_kernel, dim3(ceil_div(a.B, TB)), dim3(256), lds_bytes, s, a);
}

void launch_mlp_fused_bwd(const FusedBwdArgs& a, size_t lds_bytes, hipStream_t s) {
  hipLaunchKernelGGL(mlp_fused_bwd_kernel, dim3(ceil_div(a.B, TB)), dim3(256), lds_bytes, s, a);
}

void launch_mlp_wgrad_grouped(const WgradArgs& a, int n_tiles, hipStream_t s) {
  // batch slices of at least 128 samples per wave
  int gy = a.B / (4 * 128);
  if (gy < 1) gy = 1;
  if (gy > 16) gy = 16;
  hipLaunchKernelGGL(mlp_wgrad_grouped_kernel, dim3(n_tiles, gy), dim3(256), 0, s, a);
}

}  // namespace ss
