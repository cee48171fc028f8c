// fp32 MLP pieces (gfx950): a general strided LDS-tiled GEMM with fused bias / ReLU /
// ReLU-gate epilogues, bias gradients, the log-loss, and the lock-free SGD step.  This path
// serves models configured for fp32 arithmetic end to end; the bf16 MFMA paths live in
// mlp_fused.hip and gemm_mfma.hip.  Bottom / top networks and their place in the step:
// Section 3.1 "Trainer".
#include "ss_internal.h"

namespace ss {

constexpr int TM = 64, TN = 64, TK = 16;

// C[M,N] = A[M,K] * B[K,N], any strides; 256 threads, each a 4x4 micro-tile.
__global__ __launch_bounds__(256) void gemm_f32_kernel(
    const float* __restrict__ A, int64_t sam, int64_t sak, const float* __restrict__ Bm,
    int64_t sbk, int64_t sbn, float* __restrict__ C, int ldc, int M, int N, int K, int epi,
    const float* __restrict__ bias, const float* __restrict__ mask, int ldmask) {
  __shared__ float As[TK][TM + 4];
  __shared__ float Bs[TK][TN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * TM, n0 = blockIdx.x * TN;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += TK) {
    for (int i = tid; i < TM * TK; i += 256) {
      // walk the contiguous dimension of each operand with consecutive threads
      int mm, kk;
      if (sak == 1) { kk = i % TK; mm = i / TK; } else { mm = i % TM; kk = i / TM; }
      const int gm = m0 + mm, gk = k0 + kk;
      As[kk][mm] = (gm < M && gk < K) ? A[gm * sam + gk * sak] : 0.f;
    }
    for (int i = tid; i < TN * TK; i += 256) {
      int nn, kk;
      if (sbk == 1) { kk = i % TK; nn = i / TK; } else { nn = i % TN; kk = i / TN; }
      const int gn = n0 + nn, gk = k0 + kk;
      Bs[kk][nn] = (gn < N && gk < K) ? Bm[gk * sbk + gn * sbn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int gm = m0 + ty * 4 + i;
    if (gm >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gn = n0 + tx * 4 + j;
      if (gn >= N) continue;
      float v = acc[i][j];
      if (epi & EPI_BIAS) v += bias[gn];
      if (epi & EPI_RELU) v = fmaxf(v, 0.f);
      if (epi & EPI_MASK) v = (mask[(size_t)gm * ldmask + gn] > 0.f) ? v : 0.f;
      C[(size_t)gm * ldc + gn] = v;
    }
  }
}

void launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* Bm, int64_t sbk,
                     int64_t sbn, float* C, int ldc, int M, int N, int K, int epi,
                     const float* bias, const float* mask, int ldmask, hipStream_t s) {
  if (M == 0 || N == 0) return;
  dim3 grid(ceil_div(N, TN), ceil_div(M, TM)), block(256);
  hipLaunchKernelGGL(gemm_f32_kernel, grid, block, 0, s, A, sam, sak, Bm, sbk, sbn, C, ldc, M, N,
                     K, epi, bias, mask, ldmask);
}

// db[n] = sum_m dY[m, n]; one block per 64 columns, 16 row strips folded through LDS.
__global__ __launch_bounds__(1024) void col_sum_f32_kernel(const float* __restrict__ dY, int ld,
                                                           int M, int N, float* __restrict__ db) {
  __shared__ float part[16][64];
  const int cl = threadIdx.x & 63, c = blockIdx.x * 64 + cl, strip = threadIdx.x >> 6;
  float s = 0.f;
  if (c < N)
    for (int m = strip; m < M; m += 16) s += dY[(size_t)m * ld + c];
  part[strip][cl] = s;
  __syncthreads();
  if (strip == 0 && c < N) {
    float tot = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) tot += part[i][cl];
    db[c] = tot;
  }
}

void launch_col_sum_f32(const float* dY, int ld, int M, int N, float* db, hipStream_t s) {
  if (N == 0) return;
  hipLaunchKernelGGL(col_sum_f32_kernel, dim3(ceil_div(N, 64)), dim3(1024), 0, s, dY, ld, M, N, db);
}

// Mean binary cross-entropy on the logit, max(l,0) - l*y + log1p(exp(-|l|)), and its
// gradient (sigmoid(l) - y)/B.  One block; B is at most a few thousand.
__global__ __launch_bounds__(1024) void bce_loss_kernel(const float* __restrict__ logit,
                                                        const float* __restrict__ y, int B,
                                                        float* __restrict__ loss,
                                                        float* __restrict__ dlogit) {
  __shared__ float part[16];
  float s = 0.f;
  const float invB = 1.0f / (float)B;
  for (int b = threadIdx.x; b < B; b += 1024) {
    const float l = logit[b], t = y[b];
    const float ex = expf(-fabsf(l));
    s += fmaxf(l, 0.f) - l * t + log1pf(ex);
    const float p = (l >= 0.f) ? 1.0f / (1.0f + ex) : ex / (1.0f + ex);
    if (dlogit) dlogit[b] = (p - t) * invB;
  }
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0 && loss) {
    float tot = 0.f;
    for (int i = 0; i < 16; ++i) tot += part[i];
    *loss = tot * invB;
  }
}

void launch_bce_loss(const float* logit, const float* y, int B, float* loss, float* dlogit,
                     hipStream_t s) {
  hipLaunchKernelGGL(bce_loss_kernel, dim3(1), dim3(1024), 0, s, logit, y, B, loss, dlogit);
}

__global__ __launch_bounds__(256) void metrics_kernel(const float* __restrict__ mean_loss,
                                                      const float* __restrict__ y, int B,
                                                      double* __restrict__ acc) {
  metrics_block(mean_loss, y, B, acc);
}

void launch_metrics(const float* mean_loss, const float* y, int B, double* acc, hipStream_t s) {
  hipLaunchKernelGGL(metrics_kernel, dim3(1), dim3(256), 0, s, mean_loss, y, B, acc);
}

// w -= lr * g.  Plain loads and stores: concurrent steps on one replica overwrite each other
// the way the paper's lock-free worker threads do (Section 3.2).  With acc != nullptr the
// launch carries one extra block that adds the step's loss and labels to the running metrics
// (the loss is final by the time the update runs).
__global__ __launch_bounds__(256) void sgd_kernel(float* __restrict__ w,
                                                  const float* __restrict__ g, int64_t n,
                                                  float lr, const float* __restrict__ mean_loss,
                                                  const float* __restrict__ y, int B,
                                                  double* __restrict__ acc) {
  const unsigned nb = acc ? gridDim.x - 1 : gridDim.x;
  if (blockIdx.x == nb) {
    metrics_block(mean_loss, y, B, acc);
    return;
  }
  // four floats per thread and trip (replicas and gradient buffers are 16-byte aligned)
  const int64_t n4 = n >> 2;
  const int64_t stride = (int64_t)nb * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    float4 wv = ((float4*)w)[i];
    const float4 gv = ((const float4*)g)[i];
    wv.x -= lr * gv.x; wv.y -= lr * gv.y; wv.z -= lr * gv.z; wv.w -= lr * gv.w;
    ((float4*)w)[i] = wv;
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const int64_t i = (n4 << 2) + threadIdx.x;
    w[i] -= lr * g[i];
  }
}

void launch_sgd(float* w, const float* g, int64_t n, float lr, const float* mean_loss,
                const float* y, int B, double* acc, hipStream_t s) {
  if (n == 0) return;
  int64_t blocks = ((n >> 2) + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  if (blocks < 1) blocks = 1;
  hipLaunchKernelGGL(sgd_kernel, dim3((unsigned)blocks + (acc ? 1u : 0u)), dim3(256), 0, s, w, g, n,
                     lr, mean_loss, y, B, acc);
}

}  // namespace ss
