// bf16 MFMA GEMM for the wide-layer regime (gfx950 / CDNA4, wave64):
//     C[M,N] = A[M,K] * B[N,K]^T,   both operands bfloat16 with the reduction dimension
// contiguous, fp32 accumulation on v_mfma_f32_32x32x16_bf16.
// All three GEMMs of a layer have this form once bf16 copies exist in both orientations:
//     forward           Y  = X  * W^T      A = X  [B][in],    B = W   [out][in]
//     data gradient     dX = dY * W        A = dY [B][out],   B = W^T [in][out]
//     weight gradient   dW = dY^T * X      A = dY^T [out][B], B = X^T [in][B]
// The epilogue of the forward / data-gradient GEMM therefore writes its bf16 result twice,
// row-major (operand A of the next layer) and transposed (operand of the weight gradient);
// both go through LDS so that every global store is a full 16-byte vector of a contiguous row.
//
// Block = 256 threads = 2x2 waves, block tile 128x128, wave tile 64x64 (2x2 MFMA tiles),
// reduction step 64.  Two register stages hold the global loads of the next two steps while the
// MFMAs run on the LDS copy of the current one (two LDS buffers, one barrier per step).
// Operand rows beyond M / N are clamped to the last valid row on load and discarded on store;
// the reduction length must be a multiple of 64 with zero padding in at least one operand
// (and finite values in the other), so the main loop has no edge handling at all.
#include <mutex>

#include "ss_internal.h"

namespace ss {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int TM = 128, TN = 128, TK = 64;
constexpr int LDK = TK + 8;     // LDS row pitch of an operand tile (bf16 elements)
constexpr int LDC = 128 + 8;    // LDS row pitch of an output tile
constexpr int OP_ELEMS = TM * LDK;
constexpr size_t NT_LDS_BYTES = (size_t)4 * OP_ELEMS * sizeof(uint16_t);
static_assert(2 * 128 * LDC <= 4 * OP_ELEMS, "output tiles must fit the operand buffers");

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

struct Dev {
  const uint16_t* A; int lda;
  const uint16_t* B; int ldb;
  int M, N, K;                      // K: multiple of 64
  uint16_t* C; int ldc;             // bf16 row-major [M][ldc] (columns N..ldc-1 are zeroed) or null
  uint16_t* CT; int ldct;           // bf16 transposed [N][ldct] (columns M.. zeroed up to the tile end) or null
  float* C32; int ldc32;            // fp32 output (store, or atomicAdd when split > 1) or null
  int epi; const float* bias;
  const uint16_t* mask; int ldmask;     // [M][ldmask]: keep C(m,n) where mask > 0
  const uint16_t* maskT; int ldmaskT;   // [N][ldmaskT]: the same gate for CT
  float* row_sum;                   // [M] (+)= sum_k A(m,k), or null
  int tiles_m, tiles_n, split, k_per_split;
  long long split_stride;           // > 0: slice z of a split reduction stores to C32 + z * stride
};

__device__ __forceinline__ uint4 gate8(uint4 x, uint4 m) {
  const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ms[4] = {m.x, m.y, m.z, m.w};
  uint32_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = ((int16_t)(ms[i] & 0xFFFFu) > 0) ? 0x0000FFFFu : 0u;
    const uint32_t hi = ((int16_t)(ms[i] >> 16) > 0) ? 0xFFFF0000u : 0u;
    o[i] = xs[i] & (lo | hi);
  }
  return make_uint4(o[0], o[1], o[2], o[3]);
}

// zero the elements j >= valid (0..8) of a vector of 8 bf16
__device__ __forceinline__ uint4 keep_first(uint4 x, int valid) {
  if (valid >= 8) return x;
  uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = (2 * i < valid) ? 0x0000FFFFu : 0u;
    const uint32_t hi = (2 * i + 1 < valid) ? 0xFFFF0000u : 0u;
    w[i] &= (lo | hi);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

// one register stage = this thread's four 16-byte pieces of each operand tile
__device__ __forceinline__ void fetch8(u32x4 (&pa)[4], u32x4 (&pb)[4], const uint16_t* __restrict__ A,
                                       const uint16_t* __restrict__ B, const int (&aoff)[4],
                                       const int (&boff)[4], int ko) {
#pragma unroll
  for (int i = 0; i < 4; ++i) pa[i] = *(const u32x4*)(A + aoff[i] + ko);
#pragma unroll
  for (int i = 0; i < 4; ++i) pb[i] = *(const u32x4*)(B + boff[i] + ko);
}
__device__ __forceinline__ void stash8(const u32x4 (&pa)[4], const u32x4 (&pb)[4], uint16_t* as,
                                       uint16_t* bs) {
#pragma unroll
  for (int i = 0; i < 4; ++i) *(u32x4*)(as + 32 * i * LDK) = pa[i];
#pragma unroll
  for (int i = 0; i < 4; ++i) *(u32x4*)(bs + 32 * i * LDK) = pb[i];
}

template <bool ROWSUM>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_nt_kernel(Dev g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* const As0 = smem;
  uint16_t* const As1 = smem + OP_ELEMS;
  uint16_t* const Bs0 = smem + 2 * OP_ELEMS;
  uint16_t* const Bs1 = smem + 3 * OP_ELEMS;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // consecutive tiles (same rows of A) go to the same XCD, whose L2 then serves the re-reads
  const int total = g.tiles_m * g.tiles_n;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int tm = id / g.tiles_n, tn = id - tm * g.tiles_n;
  const int m0 = tm * TM, n0 = tn * TN;
  const int kbeg = blockIdx.y * g.k_per_split;
  const int kend = min(g.K, kbeg + g.k_per_split);
  const int nk = (kend - kbeg) / TK;
  if (nk <= 0) return;
  const bool do_rs = ROWSUM && tn == 0 && wn == 0;

  // this thread's four 16-byte pieces of each operand tile: rows tid/8 + 32 i, k offset (tid%8)*8
  const int lrow = tid >> 3, lk = (tid & 7) * 8;
  int aoff[4], boff[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    aoff[i] = min(m0 + lrow + 32 * i, g.M - 1) * g.lda + lk + kbeg;
    boff[i] = min(n0 + lrow + 32 * i, g.N - 1) * g.ldb + lk + kbeg;
  }
  u32x4 ra0[4], rb0[4], ra1[4], rb1[4];  // the two register stages

  f32x16 acc[2][2], accr[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) accr[i][e] = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  auto compute = [&](const uint16_t* as, const uint16_t* bs) {
    // fragments of reduction sub-step kk+1 are requested from LDS before the MFMAs of kk
    bf16x8 a[2][2], b[2][2];
    const uint16_t* ar = as + (wm * 64 + frow) * LDK + fk;
    const uint16_t* br = bs + (wn * 64 + frow) * LDK + fk;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[0][i] = *(const bf16x8*)(ar + i * 32 * LDK);
      b[0][i] = *(const bf16x8*)(br + i * 32 * LDK);
    }
#pragma unroll
    for (int q = 0; q < TK / 16; ++q) {
      const int cur = q & 1, nxt = cur ^ 1;
      if (q + 1 < TK / 16) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          a[nxt][i] = *(const bf16x8*)(ar + i * 32 * LDK + (q + 1) * 16);
          b[nxt][i] = *(const bf16x8*)(br + i * 32 * LDK + (q + 1) * 16);
        }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], b[cur][j], acc[i][j], 0, 0, 0);
      if (ROWSUM) {
        if (do_rs) {
#pragma unroll
          for (int i = 0; i < 2; ++i)
            accr[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i], ones, accr[i], 0, 0, 0);
        }
      }
    }
  };

  const int soff = lrow * LDK + lk;  // this thread's first piece inside an LDS operand tile
  fetch8(ra0, rb0, g.A, g.B, aoff, boff, 0);
  fetch8(ra1, rb1, g.A, g.B, aoff, boff, min(1, nk - 1) * TK);
  stash8(ra0, rb0, As0 + soff, Bs0 + soff);
  fetch8(ra0, rb0, g.A, g.B, aoff, boff, min(2, nk - 1) * TK);
  __syncthreads();
  // steady state: every step is followed by an unconditional stash + fetch (fetches past the
  // end are clamped re-reads), so the wait before a stash only covers the older stage
  int it = 0;
  for (; it + 2 < nk; it += 2) {
    compute(As0, Bs0);
    stash8(ra1, rb1, As1 + soff, Bs1 + soff);
    fetch8(ra1, rb1, g.A, g.B, aoff, boff, min(it + 3, nk - 1) * TK);
    __syncthreads();
    compute(As1, Bs1);
    stash8(ra0, rb0, As0 + soff, Bs0 + soff);
    fetch8(ra0, rb0, g.A, g.B, aoff, boff, min(it + 4, nk - 1) * TK);
    __syncthreads();
  }
  compute(As0, Bs0);  // one or two steps are left
  if (it + 1 < nk) {
    stash8(ra1, rb1, As1 + soff, Bs1 + soff);
    __syncthreads();
    compute(As1, Bs1);
  }

  // accumulator element e of a 32x32 tile: row = (e/4)*8 + (lane/32)*4 + e%4, col = lane%32
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
  if (ROWSUM) {
    if (do_rs && col_in == 0) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int gm = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + row_in + (e & 3);
          if (gm < g.M) {
            if (g.split > 1) atomicAdd(g.row_sum + gm, accr[i][e]);
            else g.row_sum[gm] = accr[i][e];
          }
        }
    }
  }
  const bool first_split = (blockIdx.y == 0);
  if (g.C32) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int gn = n0 + wn * 64 + j * 32 + col_in;
        if (gn >= g.N) continue;
        const float bv = ((g.epi & EPI_BIAS) && first_split) ? g.bias[gn] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int gm = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + row_in + (e & 3);
          if (gm >= g.M) continue;
          float v = acc[i][j][e] + bv;
          if (g.epi & EPI_RELU) v = fmaxf(v, 0.f);
          if (g.split > 1 && g.split_stride == 0) atomicAdd(g.C32 + (size_t)gm * g.ldc32 + gn, v);
          else g.C32[(size_t)blockIdx.y * g.split_stride + (size_t)gm * g.ldc32 + gn] = v;
        }
      }
    return;
  }

  // bf16 outputs: round in registers, lay the tile out in LDS in both orientations, then store
  __syncthreads();  // every wave is done reading the operand buffers
  uint16_t* const Cs = smem;               // [128][LDC], row = m
  uint16_t* const CTs = smem + 128 * LDC;  // [128][LDC], row = n
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int c = wn * 64 + j * 32 + col_in;
      const int gn = n0 + c;
      const float bv = ((g.epi & EPI_BIAS) && gn < g.N) ? g.bias[gn] : 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int r = wm * 64 + i * 32 + q * 8 + row_in;
        uint16_t h[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          float v = acc[i][j][q * 4 + u] + bv;
          if (g.epi & EPI_RELU) v = fmaxf(v, 0.f);
          h[u] = f2bf(v);
          Cs[(r + u) * LDC + c] = h[u];
        }
        *(uint2*)(CTs + c * LDC + r) =
            make_uint2((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16));
      }
    }
  __syncthreads();
  const bool gated = (g.epi & EPI_MASK) != 0;
  if (g.C) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int v = tid + 256 * q;
      const int r = v >> 4, c = (v & 15) * 8;
      const int gm = m0 + r, gn = n0 + c;
      if (gm < g.M && gn < g.ldc) {
        uint4 x = *(const uint4*)(Cs + r * LDC + c);
        if (gated) x = gate8(x, *(const uint4*)(g.mask + (size_t)gm * g.ldmask + gn));
        x = keep_first(x, g.N - gn);
        *(uint4*)(g.C + (size_t)gm * g.ldc + gn) = x;
      }
    }
  }
  if (g.CT) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int v = tid + 256 * q;
      const int r = v >> 4, c = (v & 15) * 8;  // r: output unit within the tile, c: sample
      const int gn = n0 + r, gm = m0 + c;
      if (gn < g.N && gm < g.ldct) {
        uint4 x = *(const uint4*)(CTs + r * LDC + c);
        if (gated) x = gate8(x, *(const uint4*)(g.maskT + (size_t)gn * g.ldmaskT + gm));
        x = keep_first(x, g.M - gm);
        *(uint4*)(g.CT + (size_t)gn * g.ldct + gm) = x;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Cast + transpose of one activation matrix: in [M][ld_in] (fp32 or bf16, N valid columns) ->
// out [M][ld_out] bf16 (optional, columns N..ld_out-1 zeroed) and outT [N][ldt] bf16 (optional,
// columns M.. zeroed up to the end of the last 64-sample tile, capped at ldt).  64x64 tiles.
template <bool F32>
__global__ __launch_bounds__(256) void cast_transpose_kernel(const void* __restrict__ in, int ld_in,
                                                             int M, int N, uint16_t* __restrict__ out,
                                                             int ld_out, uint16_t* __restrict__ outT,
                                                             int ldt) {
  __shared__ uint16_t t[64][66];
  const int m0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    const int gm = m0 + r, gn = n0 + c;
    uint16_t h = 0;
    if (gm < M && gn < N) {
      if (F32) h = f2bf(((const float*)in)[(size_t)gm * ld_in + gn]);
      else h = ((const uint16_t*)in)[(size_t)gm * ld_in + gn];
    }
    t[r][c] = h;
    if (out && gm < M && gn < ld_out) out[(size_t)gm * ld_out + gn] = h;
  }
  __syncthreads();
  if (outT) {
    for (int i = threadIdx.x; i < 64 * 64; i += 256) {
      const int c = i >> 6, r = i & 63;  // consecutive threads walk the samples of one unit
      const int gm = m0 + r, gn = n0 + c;
      if (gn < N && gm < ldt) outT[(size_t)gn * ldt + gm] = t[r][c];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Per-step bf16 snapshot of a replica's weight matrices in both orientations, zero padded to
// the pitches the GEMM expects, plus the clearing of the step's gradient accumulator.
__global__ __launch_bounds__(256) void weights_bf16_kernel(WeightsBf16Args a) {
  __shared__ uint16_t t[64][66];
  // clear the gradient accumulator (grid-stride)
  if (a.zero) {
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < a.zero_n; i += stride) a.zero[i] = 0.f;
  }
  int l = 0;
  while (l + 1 < a.n_layers && (int)blockIdx.x >= a.L[l + 1].tile_base) ++l;
  const WeightsBf16Layer L = a.L[l];
  const int tile = blockIdx.x - L.tile_base;
  const int tk = (L.ldw + 63) / 64;           // tiles along `in` (covers the padding)
  const int n0 = (tile / tk) * 64, k0 = (tile % tk) * 64;
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int r = i >> 6, c = i & 63;
    const int n = n0 + r, k = k0 + c;
    uint16_t h = 0;
    if (n < L.out && k < L.in) h = f2bf(L.W[(size_t)n * L.in + k]);
    t[r][c] = h;
    if (n < L.out && k < L.ldw) L.Wb[(size_t)n * L.ldw + k] = h;
  }
  __syncthreads();
  for (int i = threadIdx.x; i < 64 * 64; i += 256) {
    const int c = i >> 6, r = i & 63;  // consecutive threads walk the output units of one input
    const int n = n0 + r, k = k0 + c;
    if (k < L.in && n < L.ldwt) L.WbT[(size_t)k * L.ldwt + n] = t[r][c];
  }
}

__global__ __launch_bounds__(256) void reduce_slices_kernel(ReduceArgs a) {
  int k = 0;
  while (k + 1 < a.n_seg && (int)blockIdx.x >= a.seg[k + 1].block_base) ++k;
  const ReduceSegment sg = a.seg[k];
  const int64_t base = (int64_t)(blockIdx.x - sg.block_base) * 1024;  // 1024 elements per block
  const bool vec = ((sg.n & 3) == 0) && ((((uintptr_t)sg.out) & 15) == 0);
  if (vec) {
    const int64_t i = base + threadIdx.x * 4;
    if (i >= sg.n) return;
    float4 acc = *(const float4*)(sg.part + i);
    for (int z = 1; z < sg.slices; ++z) {
      const float4 v = *(const float4*)(sg.part + (int64_t)z * sg.stride + i);
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
    *(float4*)(sg.out + i) = acc;
  } else {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = base + threadIdx.x + 256 * u;
      if (i < sg.n) {
        float acc = sg.part[i];
        for (int z = 1; z < sg.slices; ++z) acc += sg.part[(int64_t)z * sg.stride + i];
        sg.out[i] = acc;
      }
    }
  }
}

}  // namespace

void launch_reduce_slices(const ReduceArgs& a, int total_blocks, hipStream_t s) {
  if (total_blocks > 0)
    hipLaunchKernelGGL(reduce_slices_kernel, dim3(total_blocks), dim3(256), 0, s, a);
}

int launch_gemm_nt(const GemmNtArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return 0;
  // the kernels use more than 64 KB of dynamic LDS: raise their limit once per process
  static std::once_flag attr_once;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute((const void*)gemm_nt_kernel<true>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)NT_LDS_BYTES);
    (void)hipFuncSetAttribute((const void*)gemm_nt_kernel<false>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)NT_LDS_BYTES);
  });
  Dev g;
  g.A = a.A; g.lda = a.lda; g.B = a.B; g.ldb = a.ldb; g.M = a.M; g.N = a.N; g.K = a.K;
  g.C = a.C; g.ldc = a.ldc; g.CT = a.CT; g.ldct = a.ldct; g.C32 = a.C_f32; g.ldc32 = a.ldc32;
  g.epi = a.epi; g.bias = a.bias; g.mask = a.mask; g.ldmask = a.ldmask;
  g.maskT = a.maskT; g.ldmaskT = a.ldmaskT; g.row_sum = a.row_sum;
  g.tiles_m = ceil_div(a.M, TM); g.tiles_n = ceil_div(a.N, TN);
  int split = a.split_k < 1 ? 1 : a.split_k;
  int kps = ceil_div(ceil_div(a.K, split), TK) * TK;
  split = ceil_div(a.K, kps);
  g.split = split; g.k_per_split = kps;
  g.split_stride = split > 1 ? a.split_stride : 0;
  const dim3 grid(g.tiles_m * g.tiles_n, split);
  if (a.row_sum)
    hipLaunchKernelGGL(gemm_nt_kernel<true>, grid, dim3(256), NT_LDS_BYTES, s, g);
  else
    hipLaunchKernelGGL(gemm_nt_kernel<false>, grid, dim3(256), NT_LDS_BYTES, s, g);
  return split;
}

void launch_cast_transpose(const void* in, int in_is_f32, int ld_in, int M, int N, uint16_t* out,
                           int ld_out, uint16_t* outT, int ldt, hipStream_t s) {
  if (M <= 0 || N <= 0) return;
  // the row-major copy is padded to ld_out columns, so the grid covers max(N, ld_out) columns
  const int cols = (out && ld_out > N) ? ld_out : N;
  const dim3 grid(ceil_div(M, 64), ceil_div(cols, 64));
  if (in_is_f32)
    hipLaunchKernelGGL(cast_transpose_kernel<true>, grid, dim3(256), 0, s, in, ld_in, M, N, out,
                       ld_out, outT, ldt);
  else
    hipLaunchKernelGGL(cast_transpose_kernel<false>, grid, dim3(256), 0, s, in, ld_in, M, N, out,
                       ld_out, outT, ldt);
}

void launch_weights_bf16(const WeightsBf16Args& a, int total_tiles, hipStream_t s) {
  hipLaunchKernelGGL(weights_bf16_kernel, dim3(total_tiles), dim3(256), 0, s, a);
}

}  // namespace ss
