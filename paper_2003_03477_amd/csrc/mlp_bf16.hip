// bf16 MFMA GEMM for the MLP layers (gfx950 / CDNA4, wave64).
// Every MLP GEMM of a step -- forward X W^T, data gradient dY W, weight gradient dY^T X --
// rounds both operands to bfloat16 (nearest even) and accumulates in fp32 on the matrix
// cores with v_mfma_f32_32x32x16_bf16.  Operands are read in whatever layout they already
// have in HBM (fp32 master weights, fp32 or bf16 activations, reduction dimension contiguous
// or strided) and are converted / transposed on their way into LDS, so no bf16 weight copy
// has to be kept coherent with the SGD and shadow-sync writers of the fp32 replica.
//
// Block = 256 threads = 2x2 waves; each wave owns WM x WN MFMA tiles of 32x32.
// LDS tiles are [rows][BK] bf16 with the reduction dimension contiguous, so a lane's MFMA
// fragment (8 consecutive k of one row) is a single 16-byte LDS read.  Two LDS buffers: the
// global loads of tile i+1 are issued into registers before the MFMAs of tile i and stored
// to the other buffer after them, one barrier per K step.
// The bias gradient of a weight-gradient GEMM (row sums of dY^T) rides along as one extra
// MFMA against an all-ones fragment.
#include "ss_internal.h"

namespace ss {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int KPAD = 8;  // bf16 elements of row padding (16 bytes)

__device__ __forceinline__ uint16_t to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  return (uint32_t)to_bf16(lo) | ((uint32_t)to_bf16(hi) << 16);
}

// Register staging of one operand tile [ROWS][BK].  elem(r, k) lives at
//   KC:    base + r*ld + k        (reduction dimension contiguous)
//   else:  base + k*ld + r        (row dimension contiguous)
template <int ROWS, int BK, bool F32, bool KC>
struct Stage {
  static constexpr int NV = ROWS * BK / 8 / 256;  // 8-element vectors per thread
  static constexpr int LDSK = BK + KPAD;
  float4 f[F32 ? 2 * NV : 1];
  uint4 h[F32 ? 1 : NV];

  __device__ __forceinline__ static void coords(int v, int& r, int& k) {
    if (KC) { r = v / (BK / 8); k = (v % (BK / 8)) * 8; }
    else    { k = v / (ROWS / 8); r = (v % (ROWS / 8)) * 8; }
  }

  __device__ __forceinline__ void fetch(const void* __restrict__ base, int64_t ld, int r0, int k0,
                                        int R, int K, int tid) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int r, k;
      coords(tid + 256 * i, r, k);
      const int gr = r0 + r, gk = k0 + k;
      const int64_t off = KC ? ((int64_t)gr * ld + gk) : ((int64_t)gk * ld + gr);
      const bool full = KC ? ((gr < R) && (gk + 8 <= K)) : ((gk < K) && (gr + 8 <= R));
      if (F32) {
        const float* p = (const float*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          f[2 * i] = *(const float4*)p;
          f[2 * i + 1] = *(const float4*)(p + 4);
        } else {
          float e[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const bool in = KC ? (gr < R && gk + j < K) : (gk < K && gr + j < R);
            e[j] = in ? p[j] : 0.f;
          }
          f[2 * i] = make_float4(e[0], e[1], e[2], e[3]);
          f[2 * i + 1] = make_float4(e[4], e[5], e[6], e[7]);
        }
      } else {
        const uint16_t* p = (const uint16_t*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          h[i] = *(const uint4*)p;
        } else {
          uint32_t e[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            const bool in = KC ? (gr < R && gk + j < K) : (gk < K && gr + j < R);
            e[j] = in ? (uint32_t)p[j] : 0u;
          }
          h[i] = make_uint4(e[0] | (e[1] << 16), e[2] | (e[3] << 16), e[4] | (e[5] << 16),
                            e[6] | (e[7] << 16));
        }
      }
    }
  }

  __device__ __forceinline__ void stash(uint16_t* __restrict__ tile, int tid) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      int r, k;
      coords(tid + 256 * i, r, k);
      uint4 x;
      if (F32) {
        const float4 a = f[2 * i], b = f[2 * i + 1];
        x = make_uint4(pack2(a.x, a.y), pack2(a.z, a.w), pack2(b.x, b.y), pack2(b.z, b.w));
      } else {
        x = h[i];
      }
      if (KC) {
        *(uint4*)(tile + r * LDSK + k) = x;
      } else {
        const uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
        for (int j = 0; j < 8; ++j)
          tile[(r + j) * LDSK + k] = (uint16_t)(w[j >> 1] >> ((j & 1) * 16));
      }
    }
  }
};

struct GemmDev {
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  int M, N, K;
  float* C_f32; uint16_t* C_bf16; int ldc;
  int epi; const float* bias; const uint16_t* mask; int ldmask;
  float* row_sum;  // [M] += sum_k A(m,k)  (bias gradient of a weight-gradient GEMM) or null
  int split_k; int k_per_split;
};

template <int WM, int WN, int BK, bool A_F32, bool A_KC, bool B_F32, bool B_KC>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmDev g) {
  constexpr int BM = 64 * WM, BN = 64 * WN, LDSK = BK + KPAD;
  __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDSK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDSK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * g.k_per_split;
  const int kend = min(g.K, kbeg + g.k_per_split);
  const int nk = (kend - kbeg + BK - 1) / BK;
  const bool do_rs = (g.row_sum != nullptr) && blockIdx.x == 0 && wn == 0;

  f32x16 acc[WM][WN], accr[WM];
#pragma unroll
  for (int i = 0; i < WM; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) accr[i][e] = 0.f;
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  Stage<BM, BK, A_F32, A_KC> sa;
  Stage<BN, BK, B_F32, B_KC> sb;
  if (nk > 0) {
    sa.fetch(g.A, g.lda, m0, kbeg, g.M, kend, tid);
    sb.fetch(g.B, g.ldb, n0, kbeg, g.N, kend, tid);
    sa.stash(As[0], tid);
    sb.stash(Bs[0], tid);
  }
  __syncthreads();

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  for (int it = 0; it < nk; ++it) {
    const int cur = it & 1;
    const bool more = (it + 1 < nk);
    if (more) {
      sa.fetch(g.A, g.lda, m0, kbeg + (it + 1) * BK, g.M, kend, tid);
      sb.fetch(g.B, g.ldb, n0, kbeg + (it + 1) * BK, g.N, kend, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 a[WM], b[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        a[i] = *(const bf16x8*)(As[cur] + ((wm * WM + i) * 32 + frow) * LDSK + kk + fk);
#pragma unroll
      for (int j = 0; j < WN; ++j)
        b[j] = *(const bf16x8*)(Bs[cur] + ((wn * WN + j) * 32 + frow) * LDSK + kk + fk);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      if (do_rs) {
#pragma unroll
        for (int i = 0; i < WM; ++i)
          accr[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], ones, accr[i], 0, 0, 0);
      }
    }
    if (more) {
      sa.stash(As[cur ^ 1], tid);
      sb.stash(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // accumulator element e of a 32x32 tile: row = (e/4)*8 + (lane/32)*4 + e%4, col = lane%32
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < WM; ++i) {
#pragma unroll
    for (int j = 0; j < WN; ++j) {
      const int gn = n0 + (wn * WN + j) * 32 + col_in;
      if (gn >= g.N) continue;
      const float bv = ((g.epi & EPI_BIAS) && blockIdx.z == 0) ? g.bias[gn] : 0.f;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gm = m0 + (wm * WM + i) * 32 + (e >> 2) * 8 + row_in + (e & 3);
        if (gm >= g.M) continue;
        float v = acc[i][j][e] + bv;
        if (g.epi & EPI_RELU) v = fmaxf(v, 0.f);
        if (g.epi & EPI_MASK) {
          const int16_t mk = (int16_t)g.mask[(size_t)gm * g.ldmask + gn];
          v = (mk > 0) ? v : 0.f;
        }
        if (g.C_bf16) g.C_bf16[(size_t)gm * g.ldc + gn] = to_bf16(v);
        else if (g.split_k > 1) atomicAdd(g.C_f32 + (size_t)gm * g.ldc + gn, v);
        else g.C_f32[(size_t)gm * g.ldc + gn] = v;
      }
    }
    if (do_rs && col_in == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gm = m0 + (wm * WM + i) * 32 + (e >> 2) * 8 + row_in + (e & 3);
        if (gm < g.M) {
          if (g.split_k > 1) atomicAdd(g.row_sum + gm, accr[i][e]);
          else g.row_sum[gm] = accr[i][e];
        }
      }
    }
  }
}

template <int WM, int WN, int BK>
static void dispatch(const GemmBf16Args& a, const GemmDev& g, dim3 grid, hipStream_t s) {
  const int key = (a.a_is_f32 ? 8 : 0) | (a.a_kcontig ? 4 : 0) | (a.b_is_f32 ? 2 : 0) |
                  (a.b_kcontig ? 1 : 0);
#define CASE(k, AF, AK, BF, BKc)                                                                  \
  case k:                                                                                         \
    hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, BK, AF, AK, BF, BKc>), grid, dim3(256), 0, s, g); \
    break;
  switch (key) {
    CASE(0, false, false, false, false) CASE(1, false, false, false, true)
    CASE(2, false, false, true, false) CASE(3, false, false, true, true)
    CASE(4, false, true, false, false) CASE(5, false, true, false, true)
    CASE(6, false, true, true, false) CASE(7, false, true, true, true)
    CASE(8, true, false, false, false) CASE(9, true, false, false, true)
    CASE(10, true, false, true, false) CASE(11, true, false, true, true)
    CASE(12, true, true, false, false) CASE(13, true, true, false, true)
    CASE(14, true, true, true, false) CASE(15, true, true, true, true)
  }
#undef CASE
}

void launch_gemm_bf16(const GemmBf16Args& a, hipStream_t s) {
  if (a.M == 0 || a.N == 0) return;
  GemmDev g;
  g.A = a.A; g.lda = a.lda; g.B = a.B; g.ldb = a.ldb;
  g.M = a.M; g.N = a.N; g.K = a.K;
  g.C_f32 = a.C_f32; g.C_bf16 = a.C_bf16; g.ldc = a.ldc;
  g.epi = a.epi; g.bias = a.bias; g.mask = a.mask; g.ldmask = a.ldmask;
  g.row_sum = a.row_sum;
  const bool big = (int64_t)ceil_div(a.M, 64) * ceil_div(a.N, 64) >= 2048;
  const int bk = big ? 32 : 64;
  int split = a.split_k < 1 ? 1 : a.split_k;
  int kps = ceil_div(ceil_div(a.K, split), bk) * bk;
  if (kps < bk) kps = bk;
  split = ceil_div(a.K, kps);
  if (split < 1) split = 1;
  g.split_k = split; g.k_per_split = kps;
  if (big) {
    dim3 grid(ceil_div(a.N, 128), ceil_div(a.M, 128), split);
    dispatch<2, 2, 32>(a, g, grid, s);
  } else {
    dim3 grid(ceil_div(a.N, 64), ceil_div(a.M, 64), split);
    dispatch<1, 1, 64>(a, g, grid, s);
  }
}

// ------------------------------------------------------------------------------------------
// Last top layer (one output unit) fused with the loss: logit_b = <q(x_b), q(w)> + bias,
// mean log-loss max(l,0) - l*y + log1p(exp(-|l|)) accumulated into *loss (zeroed earlier in
// the step), dlogit_b = (sigmoid(l) - y)/B.  16 lanes per sample.
__global__ __launch_bounds__(256) void last_layer_fwd_loss_kernel(
    const uint16_t* __restrict__ X, int ldx, const float* __restrict__ w,
    const float* __restrict__ bias, const float* __restrict__ y, int B, int in,
    float* __restrict__ logits, float* __restrict__ dlogit, float* __restrict__ loss) {
  __shared__ float part[16];
  const int sub = threadIdx.x & 15, sl = threadIdx.x >> 4;
  const int b = blockIdx.x * 16 + sl;
  float s = 0.f;
  if (b < B) {
    const uint16_t* xr = X + (size_t)b * ldx;
    for (int k = sub * 8; k < in; k += 128) {
      if (k + 8 <= in && ((((uintptr_t)(xr + k)) & 15) == 0)) {
        const uint4 xv = *(const uint4*)(xr + k);
        const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float xf = bf16_to_f32((uint16_t)(xw[j >> 1] >> ((j & 1) * 16)));
          s += xf * bf16_to_f32(to_bf16(w[k + j]));
        }
      } else {
        for (int j = 0; j < 8 && k + j < in; ++j)
          s += bf16_to_f32(xr[k + j]) * bf16_to_f32(to_bf16(w[k + j]));
      }
    }
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) s += __shfl_xor(s, off);
  float lossv = 0.f;
  const float invB = 1.0f / (float)B;
  if (b < B && sub == 0) {
    const float l = s + bias[0], t = y[b];
    const float ex = expf(-fabsf(l));
    lossv = fmaxf(l, 0.f) - l * t + log1pf(ex);
    const float p = (l >= 0.f) ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    logits[b] = l;
    if (dlogit) dlogit[b] = (p - t) * invB;
  }
  if (sub == 0) part[sl] = lossv;
  __syncthreads();
  if (threadIdx.x == 0) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += part[i];
    atomicAdd(loss, tot * invB);
  }
}

void launch_last_layer_fwd_loss(const uint16_t* X, int ldx, const float* w, const float* bias,
                                const float* y, int B, int in, float* logits, float* dlogit,
                                float* loss, hipStream_t s) {
  hipLaunchKernelGGL(last_layer_fwd_loss_kernel, dim3(ceil_div(B, 16)), dim3(256), 0, s, X, ldx, w,
                     bias, y, B, in, logits, dlogit, loss);
}

// Backward of that layer in one pass over X: dX[b,k] = q(dlogit_b) q(w_k) gated by X[b,k] > 0,
// gW[k] += sum_b q(dlogit_b) X[b,k], gb += sum_b dlogit_b.  A block owns LAST_ROWS_PB samples.
constexpr int LAST_ROWS_PB = 32;
__global__ __launch_bounds__(256) void last_layer_bwd_kernel(
    const uint16_t* __restrict__ X, int ldx, const float* __restrict__ w,
    const float* __restrict__ dlogit, int B, int in, uint16_t* __restrict__ dX, int lddx,
    float* __restrict__ gW, float* __restrict__ gb) {
  __shared__ float dl[LAST_ROWS_PB], dlq[LAST_ROWS_PB];
  const int b0 = blockIdx.x * LAST_ROWS_PB;
  const int nb = min(LAST_ROWS_PB, B - b0);
  if (threadIdx.x < LAST_ROWS_PB) {
    const float v = ((int)threadIdx.x < nb) ? dlogit[b0 + threadIdx.x] : 0.f;
    dl[threadIdx.x] = v;
    dlq[threadIdx.x] = bf16_to_f32(to_bf16(v));
  }
  __syncthreads();
  for (int k = threadIdx.x; k < in; k += 256) {
    const float wq = bf16_to_f32(to_bf16(w[k]));
    float acc = 0.f;
    for (int r = 0; r < nb; ++r) {
      const uint16_t xb = X[(size_t)(b0 + r) * ldx + k];
      const float d = dlq[r];
      acc += d * bf16_to_f32(xb);
      dX[(size_t)(b0 + r) * lddx + k] = ((int16_t)xb > 0) ? to_bf16(d * wq) : (uint16_t)0;
    }
    atomicAdd(gW + k, acc);
  }
  if (threadIdx.x == 0) {
    float sb = 0.f;
    for (int r = 0; r < nb; ++r) sb += dl[r];
    atomicAdd(gb, sb);
  }
}

void launch_last_layer_bwd(const uint16_t* X, int ldx, const float* w, const float* dlogit, int B,
                           int in, uint16_t* dX, int lddx, float* gW, float* gb, hipStream_t s) {
  hipLaunchKernelGGL(last_layer_bwd_kernel, dim3(ceil_div(B, LAST_ROWS_PB)), dim3(256), 0, s, X,
                     ldx, w, dlogit, B, in, dX, lddx, gW, gb);
}

}  // namespace ss
