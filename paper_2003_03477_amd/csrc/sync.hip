// Shadow synchronisation rounds (Algorithms 2, 3 and 4) as single fused, memory-bound
// kernels over K dense replicas resident in HBM.  Each element is read once and written
// once per vector it belongs to: 8(K+1) bytes/parameter for S-EASGD, 8K (+4 for w_global)
// for S-MA, 8K+16 for S-BMUF.  The K exchanges of one S-EASGD round are chained in
// registers, which equals K pairwise exchanges taken in ascending replica order.
#include "ss_internal.h"
#include "../../include/shadowsync.h"

namespace ss {

typedef float f32x4 __attribute__((ext_vector_type(4)));
template <bool NT>
__device__ __forceinline__ float4 ld4(const float* p) {
  if (NT) {
    f32x4 v = __builtin_nontemporal_load((const f32x4*)p);
    return make_float4(v.x, v.y, v.z, v.w);
  }
  return *(const float4*)p;
}
template <bool NT>
__device__ __forceinline__ void st4(float* p, float4 v) {
  if (NT) {
    f32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, (f32x4*)p);
  } else {
    *(float4*)p = v;
  }
}

#define SS_F4_OP(dst, expr)   \
  {                           \
    dst.x = expr(x);          \
    dst.y = expr(y);          \
    dst.z = expr(z);          \
    dst.w = expr(w);          \
  }

template <int K, int ALGO, bool NT>
__global__ __launch_bounds__(256) void sync_round_kernel(float* __restrict__ W, int64_t stride,
                                                         float* __restrict__ w_ps,
                                                         float* __restrict__ w_global,
                                                         float* __restrict__ v, int64_t n_vec,
                                                         float alpha, float eta, float mu) {
  const int64_t step = (int64_t)gridDim.x * blockDim.x;
  const float inv_k = 1.0f / (float)K;
  const float beta = 1.0f - alpha;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += step) {
    const int64_t o = 4 * i;
    float4 w[K];
#pragma unroll
    for (int k = 0; k < K; ++k) w[k] = ld4<NT>(W + k * stride + o);
    if constexpr (ALGO == SS_EASGD) {
      float4 c = ld4<NT>(w_ps + o);
#pragma unroll
      for (int k = 0; k < K; ++k) {
        float4 dl;
#define E(f) alpha * (w[k].f - c.f)
        SS_F4_OP(dl, E)
#undef E
        c.x += dl.x; c.y += dl.y; c.z += dl.z; c.w += dl.w;
        w[k].x -= dl.x; w[k].y -= dl.y; w[k].z -= dl.z; w[k].w -= dl.w;
      }
      st4<NT>(w_ps + o, c);
    } else if constexpr (ALGO == SS_EASGD_LITERAL) {
      float4 c = ld4<NT>(w_ps + o);
#pragma unroll
      for (int k = 0; k < K; ++k) {
#define E(f) beta * c.f + alpha * w[k].f
        SS_F4_OP(c, E)
#undef E
#define E(f) beta * w[k].f + alpha * c.f
        SS_F4_OP(w[k], E)
#undef E
      }
      st4<NT>(w_ps + o, c);
    } else {
      float4 m = w[0];
#pragma unroll
      for (int k = 1; k < K; ++k) {
        m.x += w[k].x; m.y += w[k].y; m.z += w[k].z; m.w += w[k].w;
      }
      m.x *= inv_k; m.y *= inv_k; m.z *= inv_k; m.w *= inv_k;
      float4 g;
      if constexpr (ALGO == SS_MA) {
        g = m;
      } else {  // SS_BMUF, SS_BMUF_NESTEROV
        float4 g0 = ld4<NT>(w_global + o), vv = ld4<NT>(v + o);
#define E(f) mu * vv.f + eta * (m.f - g0.f)
        SS_F4_OP(vv, E)
#undef E
        g.x = g0.x + vv.x; g.y = g0.y + vv.y; g.z = g0.z + vv.z; g.w = g0.w + vv.w;
        st4<NT>(v + o, vv);
        st4<NT>(w_global + o, g);
        if constexpr (ALGO == SS_BMUF_NESTEROV) {  // the replicas aim at the look-ahead point
          g.x += mu * vv.x; g.y += mu * vv.y; g.z += mu * vv.z; g.w += mu * vv.w;
        }
      }
      if constexpr (ALGO == SS_MA) st4<NT>(w_global + o, g);
#pragma unroll
      for (int k = 0; k < K; ++k) {
#define E(f) beta * w[k].f + alpha * g.f
        SS_F4_OP(w[k], E)
#undef E
      }
    }
#pragma unroll
    for (int k = 0; k < K; ++k) st4<NT>(W + k * stride + o, w[k]);
  }
}

template <int K>
static void launch_k(int algo, int64_t n_vec, float* W, int64_t stride, float* w_ps,
                     float* w_global, float* v, float alpha, float eta, float mu,
                     hipStream_t s) {
  // One float4 column of the K+1 vectors per thread, no grid-stride looping: measured faster
  // than a capped persistent grid on 50M-parameter replicas (5.2-5.4 TB/s against 4.9 TB/s,
  // and 5.0 TB/s for a plain device copy).  Streams that exceed the 256 MB memory-side cache
  // use non-temporal loads and stores; small replicas stay cacheable for the trainer kernels.
  int64_t blocks = (n_vec + 255) / 256;
  const int64_t cap = 1 << 30;
  if (blocks > cap) blocks = cap;
  const bool nt = (int64_t)(K + 1) * n_vec * 16 > (256ll << 20);
  dim3 g((unsigned)blocks), b(256);
#define SS_LAUNCH(A)                                                                              \
  if (nt)                                                                                         \
    hipLaunchKernelGGL((sync_round_kernel<K, A, true>), g, b, 0, s, W, stride, w_ps, w_global, v, \
                       n_vec, alpha, eta, mu);                                                    \
  else                                                                                            \
    hipLaunchKernelGGL((sync_round_kernel<K, A, false>), g, b, 0, s, W, stride, w_ps, w_global,   \
                       v, n_vec, alpha, eta, mu)
  switch (algo) {
    case SS_EASGD: SS_LAUNCH(SS_EASGD); break;
    case SS_EASGD_LITERAL: SS_LAUNCH(SS_EASGD_LITERAL); break;
    case SS_MA: SS_LAUNCH(SS_MA); break;
    case SS_BMUF_NESTEROV: SS_LAUNCH(SS_BMUF_NESTEROV); break;
    default: SS_LAUNCH(SS_BMUF); break;
  }
#undef SS_LAUNCH
}

// P is padded up to a multiple of 4 by the caller's layout (stride >= P rounded up).
int launch_sync_round(int algo, int K, int64_t P, int64_t stride, float* W, float* w_ps,
                      float* w_global, float* v, float alpha, float eta, float mu,
                      hipStream_t s) {
  if (K < 1 || K > 16 || P <= 0) return -1;
  int64_t n_vec = (P + 3) / 4;
  switch (K) {
#define C(k) case k: launch_k<k>(algo, n_vec, W, stride, w_ps, w_global, v, alpha, eta, mu, s); break;
    C(1) C(2) C(3) C(4) C(5) C(6) C(7) C(8) C(9) C(10) C(11) C(12) C(13) C(14) C(15) C(16)
#undef C
  }
  return 0;
}

// Mean of the K replicas (the alternative output model of Section 4, "Experimental Setup":
// the paper returns the first trainer's copy; the replica average is the other candidate),
// summed in replica order like the averaging rounds.
__global__ __launch_bounds__(256) void replica_mean_kernel(const float* __restrict__ W, int K,
                                                           int64_t stride, int64_t n_vec,
                                                           float* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_vec) return;
  float4 acc = ((const float4*)W)[i];
  for (int k = 1; k < K; ++k) {
    const float4 v = ((const float4*)(W + (size_t)k * stride))[i];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  const float inv = 1.0f / (float)K;
  ((float4*)out)[i] = make_float4(acc.x * inv, acc.y * inv, acc.z * inv, acc.w * inv);
}

void launch_replica_mean(const float* W, int K, int64_t stride, int64_t P, float* out,
                         hipStream_t s) {
  const int64_t n_vec = (P + 3) / 4;
  hipLaunchKernelGGL(replica_mean_kernel, dim3(ceil_div(n_vec, 256)), dim3(256), 0, s, W, K, stride,
                     n_vec, out);
}

}  // namespace ss
