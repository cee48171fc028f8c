// bf16 MFMA GEMM for the MLP layers (gfx950 / CDNA4, wave64).
// Every MLP GEMM of a step -- forward X W^T, data gradient dY W, weight gradient dY^T X --
// rounds both operands to bfloat16 (nearest even) and accumulates in fp32 on the matrix
// cores with v_mfma_f32_32x32x16_bf16.  Operands are read in whatever layout they already
// have in HBM (fp32 master weights, fp32 or bf16 activations, reduction dimension contiguous
// or strided) and are converted / transposed on their way into LDS, so no bf16 weight copy
// has to be kept coherent with the SGD and shadow-sync writers of the fp32 replica.
//
// Block = 256 threads = 2x2 waves; each wave owns WM x WN MFMA tiles of 32x32.
// LDS tiles are [rows][BK] bf16 with the reduction dimension contiguous; a lane's MFMA
// fragment (8 consecutive k of one row) is a single 16-byte LDS read.
#include "ss_internal.h"

namespace ss {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 32;
constexpr int KPAD = 8;  // bf16 elements of row padding (16 bytes)
constexpr int LDSK = BK + KPAD;

__device__ __forceinline__ uint16_t to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t h) {
  return __uint_as_float((uint32_t)h << 16);
}

// Load one operand tile [ROWS][BK] into LDS as bf16.  elem(r, k) lives at
//   kcontig:  base + r*ld + k        (reduction dimension contiguous)
//   else:     base + k*ld + r        (row dimension contiguous)
template <int ROWS, bool F32, bool KCONTIG>
__device__ __forceinline__ void load_tile(uint16_t* __restrict__ tile, const void* __restrict__ base,
                                          int64_t ld, int r0, int k0, int R, int K, int tid) {
  constexpr int VEC = 8;
  constexpr int NVEC = ROWS * BK / VEC;
  for (int v = tid; v < NVEC; v += 256) {
    int r, k;
    if (KCONTIG) { r = v / (BK / VEC); k = (v % (BK / VEC)) * VEC; }
    else         { k = v / (ROWS / VEC); r = (v % (ROWS / VEC)) * VEC; }
    __attribute__((aligned(16))) uint16_t x[VEC];
    const int gr = r0 + r, gk = k0 + k;
    if (KCONTIG) {
      const int64_t off = (int64_t)gr * ld + gk;
      const bool full = (gr < R) && (gk + VEC <= K);
      if (F32) {
        const float* p = (const float*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
          x[0] = to_bf16(a.x); x[1] = to_bf16(a.y); x[2] = to_bf16(a.z); x[3] = to_bf16(a.w);
          x[4] = to_bf16(b.x); x[5] = to_bf16(b.y); x[6] = to_bf16(b.z); x[7] = to_bf16(b.w);
        } else {
#pragma unroll
          for (int i = 0; i < VEC; ++i)
            x[i] = (gr < R && gk + i < K) ? to_bf16(p[i]) : (uint16_t)0;
        }
      } else {
        const uint16_t* p = (const uint16_t*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          *(uint4*)x = *(const uint4*)p;
        } else {
#pragma unroll
          for (int i = 0; i < VEC; ++i) x[i] = (gr < R && gk + i < K) ? p[i] : (uint16_t)0;
        }
      }
      *(uint4*)(tile + r * LDSK + k) = *(uint4*)x;
    } else {
      const int64_t off = (int64_t)gk * ld + gr;
      const bool full = (gk < K) && (gr + VEC <= R);
      if (F32) {
        const float* p = (const float*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          const float4 a = *(const float4*)p, b = *(const float4*)(p + 4);
          x[0] = to_bf16(a.x); x[1] = to_bf16(a.y); x[2] = to_bf16(a.z); x[3] = to_bf16(a.w);
          x[4] = to_bf16(b.x); x[5] = to_bf16(b.y); x[6] = to_bf16(b.z); x[7] = to_bf16(b.w);
        } else {
#pragma unroll
          for (int i = 0; i < VEC; ++i)
            x[i] = (gk < K && gr + i < R) ? to_bf16(p[i]) : (uint16_t)0;
        }
      } else {
        const uint16_t* p = (const uint16_t*)base + off;
        if (full && ((((uintptr_t)p) & 15) == 0)) {
          *(uint4*)x = *(const uint4*)p;
        } else {
#pragma unroll
          for (int i = 0; i < VEC; ++i) x[i] = (gk < K && gr + i < R) ? p[i] : (uint16_t)0;
        }
      }
#pragma unroll
      for (int i = 0; i < VEC; ++i) tile[(r + i) * LDSK + k] = x[i];
    }
  }
}

struct GemmDev {
  const void* A; int64_t lda;
  const void* B; int64_t ldb;
  int M, N, K;
  float* C_f32; uint16_t* C_bf16; int ldc;
  int epi; const float* bias; const uint16_t* mask; int ldmask;
  int split_k; int k_per_split;
};

template <int WM, int WN, bool A_F32, bool A_KC, bool B_F32, bool B_KC>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmDev g) {
  constexpr int BM = 64 * WM, BN = 64 * WN;
  __shared__ __attribute__((aligned(16))) uint16_t As[BM * LDSK];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[BN * LDSK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int kbeg = blockIdx.z * g.k_per_split;
  const int kend = min(g.K, kbeg + g.k_per_split);
  f32x16 acc[WM][WN];
#pragma unroll
  for (int i = 0; i < WM; ++i)
#pragma unroll
    for (int j = 0; j < WN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int frow = lane & 31, fk = (lane >> 5) * 8;
  for (int k0 = kbeg; k0 < kend; k0 += BK) {
    load_tile<BM, A_F32, A_KC>(As, g.A, g.lda, m0, k0, g.M, kend, tid);
    load_tile<BN, B_F32, B_KC>(Bs, g.B, g.ldb, n0, k0, g.N, kend, tid);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 a[WM], b[WN];
#pragma unroll
      for (int i = 0; i < WM; ++i)
        a[i] = *(const bf16x8*)(As + ((wm * WM + i) * 32 + frow) * LDSK + kk + fk);
#pragma unroll
      for (int j = 0; j < WN; ++j)
        b[j] = *(const bf16x8*)(Bs + ((wn * WN + j) * 32 + frow) * LDSK + kk + fk);
#pragma unroll
      for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }

  // accumulator element e of a 32x32 tile: row = (e/4)*8 + (lane/32)*4 + e%4, col = lane%32
  const int col_in = lane & 31, row_in = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < WM; ++i)
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
}

template <int WM, int WN>
static void dispatch(const GemmBf16Args& a, const GemmDev& g, dim3 grid, hipStream_t s) {
  const int key = (a.a_is_f32 ? 8 : 0) | (a.a_kcontig ? 4 : 0) | (a.b_is_f32 ? 2 : 0) |
                  (a.b_kcontig ? 1 : 0);
#define CASE(k, AF, AK, BF, BKc)                                                              \
  case k:                                                                                     \
    hipLaunchKernelGGL((gemm_bf16_kernel<WM, WN, AF, AK, BF, BKc>), grid, dim3(256), 0, s, g); \
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
  int split = a.split_k < 1 ? 1 : a.split_k;
  int kps = ceil_div(ceil_div(a.K, split), BK) * BK;
  if (kps < BK) kps = BK;
  split = ceil_div(a.K, kps);
  if (split < 1) split = 1;
  g.split_k = split; g.k_per_split = kps;
  const bool big = (a.M >= 1024 && a.N >= 512);
  if (big) {
    dim3 grid(ceil_div(a.N, 128), ceil_div(a.M, 128), split);
    dispatch<2, 2>(a, g, grid, s);
  } else {
    dim3 grid(ceil_div(a.N, 64), ceil_div(a.M, 64), split);
    dispatch<1, 1>(a, g, grid, s);
  }
}

__global__ __launch_bounds__(256) void col_sum_bf16_kernel(const uint16_t* __restrict__ dY, int ld,
                                                           int M, int N, float* __restrict__ db) {
  __shared__ float part[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), strip = threadIdx.x >> 6;
  float s = 0.f;
  if (c < N)
    for (int m = strip; m < M; m += 4) s += bf16_to_f32(dY[(size_t)m * ld + c]);
  part[strip][threadIdx.x & 63] = s;
  __syncthreads();
  if (strip == 0 && c < N)
    db[c] = (part[0][threadIdx.x] + part[1][threadIdx.x]) +
            (part[2][threadIdx.x] + part[3][threadIdx.x]);
}

void launch_col_sum_bf16(const uint16_t* dY, int ld, int M, int N, float* db, hipStream_t s) {
  if (N == 0) return;
  hipLaunchKernelGGL(col_sum_bf16_kernel, dim3(ceil_div(N, 64)), dim3(256), 0, s, dY, ld, M, N,
                     db);
}

}  // namespace ss
