// Table initialisation from a counter-based hash, and small fill kernels (gfx950).
// Algorithm 1 takes h0 as an input; the hash lets a multi-GB table be filled in place on
// the device while a host-side checker regenerates any single row from the same definition.
#include "ss_internal.h"

namespace ss {

__device__ __forceinline__ uint64_t mix64(uint64_t z) {  // splitmix64 output function
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

static inline uint64_t host_mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__device__ __forceinline__ float hash_value(uint64_t key, uint64_t idx) {
  uint64_t z = mix64(key + idx * 0x9E3779B97F4A7C15ull);
  int k = (int)(z >> 40) - (1 << 23);
  // 0.05f * 2^-23: the product k * scale is rounded once
  return (float)k * (0.05f * 1.1920928955078125e-07f);
}

// n_elems is a multiple of 4 (d is); each thread writes one float4.
__global__ __launch_bounds__(256) void table_hash_init_kernel(float4* __restrict__ h,
                                                              uint64_t n_vec, uint64_t key) {
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n_vec; i += stride) {
    float4 v;
    v.x = hash_value(key, 4 * i + 0);
    v.y = hash_value(key, 4 * i + 1);
    v.z = hash_value(key, 4 * i + 2);
    v.w = hash_value(key, 4 * i + 3);
    h[i] = v;
  }
}

void launch_table_hash_init(float* h, uint64_t n_elems, uint64_t seed, int table,
                            hipStream_t s) {
  if (n_elems == 0) return;
  uint64_t key = host_mix64(seed ^ ((uint64_t)(1000 + table) * 0xD1B54A32D192ED03ull));
  uint64_t n_vec = n_elems / 4;
  uint64_t blocks = (n_vec + 255) / 256;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(table_hash_init_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                     (float4*)h, n_vec, key);
}

template <typename T>
__global__ __launch_bounds__(256) void fill_kernel(T* __restrict__ p, uint64_t n, T v) {
  uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
  for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    p[i] = v;
}

void launch_fill_f32(float* p, uint64_t n, float v, hipStream_t s) {
  if (n == 0) return;
  uint64_t blocks = (n + 255) / 256;
  if (blocks > 32768) blocks = 32768;
  hipLaunchKernelGGL(fill_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
}

void launch_fill_u32(uint32_t* p, uint64_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return;
  uint64_t blocks = (n + 255) / 256;
  if (blocks > 32768) blocks = 32768;
  hipLaunchKernelGGL(fill_kernel<uint32_t>, dim3((unsigned)blocks), dim3(256), 0, s, p, n, v);
}

}  // namespace ss
