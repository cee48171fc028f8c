// Embedding kernels (gfx950): sum-pooled gather (forward) and, for the backward pass,
// segment detection over the row-sorted (row, position) pairs followed by one fused
// "sum the occurrences' gradients, then row-wise Adagrad" pass per distinct row
// (Section 3.1: pooling happens where the table lives; Section 3.2: lock-free optimiser
// updates with the Adagrad accumulator co-located with each row).
#include "ss_internal.h"

namespace ss {

// ------------------------------------------------------------------------------------------
// Forward.  One wavefront per bag.  A row of d floats is covered by LPR = d/4 lanes loading
// one float4 each, so a wave keeps 64/LPR rows in flight per load instruction.  The bag's
// index list is read once, coalesced, 64 ids at a time, and handed between lanes with
// cross-lane permutes; every lane owns fixed columns, partial sums of the 64/LPR row slots
// are folded with xor-shuffles at the end.
template <int LPR>
__global__ __launch_bounds__(256) void embedding_bag_fwd_kernel(
    const float* __restrict__ h, const int32_t* __restrict__ indices,
    const int32_t* __restrict__ offsets, TableMeta meta, int B, int T, float* __restrict__ e,
    uint32_t* __restrict__ keys, int32_t* __restrict__ bag_of_pos,
    float* __restrict__ zero_scalar) {
  constexpr int D = LPR * 4;
  constexpr int RPW = SS_WAVE / LPR;  // rows per wave-wide load
  // the step's loss accumulator is cleared here, ahead of the kernel that adds into it
  if (zero_scalar && blockIdx.x == 0 && threadIdx.x == 0) *zero_scalar = 0.f;
  const int lane = threadIdx.x & 63;
  const int bag = (int)((blockIdx.x * (uint64_t)blockDim.x + threadIdx.x) >> 6);  // t*B + b
  if (bag >= T * B) return;
  const int t = bag / B, b = bag - t * B;
  const int lo = offsets[bag], hi = offsets[bag + 1];
  const uint32_t base = meta.row_base[t];
  const int sub = lane / LPR, c4 = lane % LPR;
  const int ebag = b * T + t;
  float4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = lo; j0 < hi; j0 += SS_WAVE) {
    const int j = j0 + lane;
    uint32_t grow = 0;
    if (j < hi) {
      grow = base + (uint32_t)indices[j];
      keys[j] = grow;
      bag_of_pos[j] = ebag;
    }
    const int cnt = min(SS_WAVE, hi - j0);
    // trip count is wave-uniform so every lane takes part in every permute
    for (int it = 0; it < cnt; it += 2 * RPW) {
      const int ja = it + sub, jb = it + RPW + sub;
      const uint32_t ra = (uint32_t)__shfl((int)grow, ja & 63);
      const uint32_t rb = (uint32_t)__shfl((int)grow, jb & 63);
      float4 va = {0.f, 0.f, 0.f, 0.f}, vb = {0.f, 0.f, 0.f, 0.f};
      if (ja < cnt) va = *(const float4*)(h + (size_t)ra * D + c4 * 4);
      if (jb < cnt) vb = *(const float4*)(h + (size_t)rb * D + c4 * 4);
      acc0.x += va.x; acc0.y += va.y; acc0.z += va.z; acc0.w += va.w;
      acc1.x += vb.x; acc1.y += vb.y; acc1.z += vb.z; acc1.w += vb.w;
    }
  }
  float4 acc = {acc0.x + acc1.x, acc0.y + acc1.y, acc0.z + acc1.z, acc0.w + acc1.w};
#pragma unroll
  for (int off = LPR; off < SS_WAVE; off <<= 1) {
    acc.x += __shfl_xor(acc.x, off);
    acc.y += __shfl_xor(acc.y, off);
    acc.z += __shfl_xor(acc.z, off);
    acc.w += __shfl_xor(acc.w, off);
  }
  if (sub == 0) *(float4*)(e + (size_t)ebag * D + c4 * 4) = acc;
}

void launch_embedding_bag_fwd(const float* h, const int32_t* indices, const int32_t* offsets,
                              const TableMeta& meta, int B, int T, int d, float* e,
                              uint32_t* keys, int32_t* bag_of_pos, float* zero_scalar,
                              hipStream_t s) {
  const int64_t bags = (int64_t)B * T;
  if (bags == 0) return;
  dim3 grid((unsigned)ceil_div(bags, 4)), block(256);
#define L(LPR)                                                                               \
  hipLaunchKernelGGL((embedding_bag_fwd_kernel<LPR>), grid, block, 0, s, h, indices, offsets, \
                     meta, B, T, e, keys, bag_of_pos, zero_scalar)
  switch (d) {
    case 16: L(4); break;
    case 32: L(8); break;
    case 64: L(16); break;
    default: L(32); break;  // 128
  }
#undef L
}

// ------------------------------------------------------------------------------------------
// Segment starts: flag j where sorted_keys[j] != sorted_keys[j-1], count per block, scan the
// block counts, compact.  SEG_TILE elements per block.
constexpr int SEG_TILE = 2048;   // 256 threads x 8
constexpr uint32_t LONG_SEG = 256;  // segments longer than this go to the block-wide kernel

__device__ __forceinline__ bool is_head(const uint32_t* __restrict__ k, uint32_t j) {
  return j == 0 || k[j] != k[j - 1];
}

__global__ __launch_bounds__(256) void seg_count_kernel(const uint32_t* __restrict__ keys,
                                                        uint32_t n,
                                                        uint32_t* __restrict__ block_counts) {
  __shared__ uint32_t wsum[4];
  const uint32_t base = blockIdx.x * SEG_TILE;
  uint32_t c = 0;
  for (int r = 0; r < SEG_TILE / 256; ++r) {
    uint32_t j = base + r * 256 + threadIdx.x;
    if (j < n && is_head(keys, j)) ++c;
  }
  for (int off = 32; off > 0; off >>= 1) c += __shfl_xor((int)c, off);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) block_counts[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// Single block: exclusive scan of block_counts in place, total -> num_unique, sentinel
// seg_starts[U] = n, long-segment counter reset.
__global__ __launch_bounds__(1024) void seg_scan_kernel(uint32_t* __restrict__ block_counts,
                                                        int nblocks, uint32_t n,
                                                        uint32_t* __restrict__ num_unique,
                                                        uint32_t* __restrict__ seg_starts,
                                                        uint32_t* __restrict__ long_count) {
  __shared__ uint32_t part[1024];
  const int tid = threadIdx.x;
  const int per = (nblocks + 1023) / 1024;
  const int lo = tid * per, hi = min(nblocks, lo + per);
  uint32_t s = 0;
  for (int i = lo; i < hi; ++i) s += block_counts[i];
  part[tid] = s;
  __syncthreads();
  for (int off = 1; off < 1024; off <<= 1) {  // Hillis-Steele inclusive scan
    uint32_t v = (tid >= off) ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  uint32_t run = part[tid] - s;
  for (int i = lo; i < hi; ++i) {
    uint32_t c = block_counts[i];
    block_counts[i] = run;
    run += c;
  }
  if (tid == 1023) {
    uint32_t U = part[1023];
    *num_unique = U;
    seg_starts[U] = n;
    *long_count = 0;
  }
}

__global__ __launch_bounds__(256) void seg_compact_kernel(const uint32_t* __restrict__ keys,
                                                          uint32_t n,
                                                          const uint32_t* __restrict__ block_off,
                                                          uint32_t* __restrict__ seg_starts) {
  __shared__ uint32_t wcnt[4];
  __shared__ uint32_t running;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (threadIdx.x == 0) running = block_off[blockIdx.x];
  __syncthreads();
  const uint32_t base = blockIdx.x * SEG_TILE;
  for (int r = 0; r < SEG_TILE / 256; ++r) {
    const uint32_t j = base + r * 256 + threadIdx.x;
    const bool hd = (j < n) && is_head(keys, j);
    const uint64_t m = __ballot(hd);
    if (lane == 0) wcnt[wave] = (uint32_t)__popcll(m);
    __syncthreads();
    uint32_t before = running;
    for (int w = 0; w < wave; ++w) before += wcnt[w];
    if (hd) seg_starts[before + (uint32_t)__popcll(m & ((1ull << lane) - 1ull))] = j;
    __syncthreads();
    if (threadIdx.x == 0) running += wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
    __syncthreads();
  }
}

void launch_segment_starts(const uint32_t* sorted_keys, uint32_t n, const SegScratch& sc,
                           hipStream_t s) {
  const int nb = ceil_div(n, SEG_TILE);
  if (nb > 0)
    hipLaunchKernelGGL(seg_count_kernel, dim3(nb), dim3(256), 0, s, sorted_keys, n,
                       sc.block_counts);
  hipLaunchKernelGGL(seg_scan_kernel, dim3(1), dim3(1024), 0, s, sc.block_counts, nb, n,
                     sc.num_unique, sc.seg_starts, sc.long_count);
  if (nb > 0)
    hipLaunchKernelGGL(seg_compact_kernel, dim3(nb), dim3(256), 0, s, sorted_keys, n,
                       sc.block_counts, sc.seg_starts);
}

// ------------------------------------------------------------------------------------------
// Row update.  One LPR-lane group per distinct row; the group walks the row's occurrences
// in sorted order (ascending flat position), LPR occurrences per batch of index loads, adds
// the pooled-vector gradients they point at, then applies row-wise Adagrad:
//   G_r += mean_c g_r[c]^2 ;  h[r,:] -= lr * g_r / (sqrt(G_r) + eps).
// Segments longer than LONG_SEG are queued for the block-wide kernel below.
template <int LPR>
__device__ __forceinline__ void adagrad_apply(float4 g, uint32_t row, int c4, float* __restrict__ h,
                                              float* __restrict__ G, float lr, float eps) {
  constexpr int D = LPR * 4;
  float ss = g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w;
#pragma unroll
  for (int off = 1; off < LPR; off <<= 1) ss += __shfl_xor(ss, off);
  const float Gn = G[row] + ss * (1.0f / (float)D);
  const float scale = lr / (sqrtf(Gn) + eps);
  float4* hp = (float4*)(h + (size_t)row * D + c4 * 4);
  float4 hv = *hp;
  hv.x -= scale * g.x; hv.y -= scale * g.y; hv.z -= scale * g.z; hv.w -= scale * g.w;
  *hp = hv;
  if (c4 == 0) G[row] = Gn;
}

template <int LPR>
__global__ __launch_bounds__(256) void row_update_kernel(
    const uint32_t* __restrict__ sorted_keys, const int32_t* __restrict__ sorted_bag,
    const float* __restrict__ de, const uint32_t* __restrict__ seg_starts,
    const uint32_t* __restrict__ num_unique, uint32_t* __restrict__ long_list,
    uint32_t* __restrict__ long_count, float* __restrict__ h, float* __restrict__ G, float lr,
    float eps) {
  constexpr int D = LPR * 4;
  const uint32_t U = *num_unique;
  const int lane = threadIdx.x & 63;
  const int c4 = lane % LPR;
  const uint32_t groups = (uint32_t)(gridDim.x * (blockDim.x / LPR));
  for (uint32_t u = blockIdx.x * (blockDim.x / LPR) + threadIdx.x / LPR; u < U; u += groups) {
    const uint32_t start = seg_starts[u], end = seg_starts[u + 1];
    if (end - start > LONG_SEG) {
      if (c4 == 0) long_list[atomicAdd(long_count, 1u)] = u;
      continue;
    }
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    for (uint32_t k0 = start; k0 < end; k0 += LPR) {
      const uint32_t k = k0 + c4;
      int bag = 0;
      if (k < end) bag = sorted_bag[k];
      const int cnt = (int)min((uint32_t)LPR, end - k0);
      // group-uniform trip count: the source lane of every permute is an active lane
      for (int i = 0; i < cnt; ++i) {
        const int bg = __shfl(bag, i, LPR);
        const float4 v = *(const float4*)(de + (size_t)bg * D + c4 * 4);
        acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
      }
    }
    adagrad_apply<LPR>(acc, sorted_keys[start], c4, h, G, lr, eps);
  }
}

// One block per long segment: the 256/LPR groups take interleaved occurrences, four at a
// time so that several gradient rows are in flight per group; partial sums are folded
// through LDS and group 0 applies the update.
template <int LPR>
__global__ __launch_bounds__(256) void row_update_long_kernel(
    const uint32_t* __restrict__ sorted_keys, const int32_t* __restrict__ sorted_bag,
    const float* __restrict__ de, const uint32_t* __restrict__ seg_starts,
    const uint32_t* __restrict__ long_list, const uint32_t* __restrict__ long_count,
    float* __restrict__ h, float* __restrict__ G, float lr, float eps) {
  constexpr int D = LPR * 4;
  constexpr int NG = 256 / LPR;
  __shared__ float4 part[256];
  const uint32_t nlong = *long_count;
  const int c4 = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  for (uint32_t li = blockIdx.x; li < nlong; li += gridDim.x) {
    const uint32_t u = long_list[li];
    const uint32_t start = seg_starts[u], end = seg_starts[u + 1];
    float4 a0 = {0.f, 0.f, 0.f, 0.f}, a1 = a0, a2 = a0, a3 = a0;
    uint32_t k = start + grp;
    for (; k + 3 * NG < end; k += 4 * NG) {
      const int b0 = sorted_bag[k], b1 = sorted_bag[k + NG], b2 = sorted_bag[k + 2 * NG],
                b3 = sorted_bag[k + 3 * NG];
      const float4 v0 = *(const float4*)(de + (size_t)b0 * D + c4 * 4);
      const float4 v1 = *(const float4*)(de + (size_t)b1 * D + c4 * 4);
      const float4 v2 = *(const float4*)(de + (size_t)b2 * D + c4 * 4);
      const float4 v3 = *(const float4*)(de + (size_t)b3 * D + c4 * 4);
      a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
      a1.x += v1.x; a1.y += v1.y; a1.z += v1.z; a1.w += v1.w;
      a2.x += v2.x; a2.y += v2.y; a2.z += v2.z; a2.w += v2.w;
      a3.x += v3.x; a3.y += v3.y; a3.z += v3.z; a3.w += v3.w;
    }
    for (; k < end; k += NG) {
      const int b0 = sorted_bag[k];
      const float4 v0 = *(const float4*)(de + (size_t)b0 * D + c4 * 4);
      a0.x += v0.x; a0.y += v0.y; a0.z += v0.z; a0.w += v0.w;
    }
    float4 acc = {(a0.x + a1.x) + (a2.x + a3.x), (a0.y + a1.y) + (a2.y + a3.y),
                  (a0.z + a1.z) + (a2.z + a3.z), (a0.w + a1.w) + (a2.w + a3.w)};
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int half = NG / 2; half >= 1; half >>= 1) {
      if (grp < half) {
        float4 o = part[threadIdx.x + half * LPR];
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
        part[threadIdx.x] = acc;
      }
      __syncthreads();
    }
    if (grp == 0) adagrad_apply<LPR>(acc, sorted_keys[start], c4, h, G, lr, eps);
    __syncthreads();
  }
}

void launch_row_update(const uint32_t* sorted_keys, const int32_t* sorted_bag, const float* de,
                       uint32_t n, const SegScratch& sc, int d, float* h, float* G, float lr,
                       float eps, hipStream_t s) {
  if (n == 0) return;
  const int lpr = d / 4;
  const int groups_per_block = 256 / lpr;
  int blocks = ceil_div(n, groups_per_block);
  if (blocks > 256 * 16) blocks = 256 * 16;
#define L(LPR)                                                                                 \
  hipLaunchKernelGGL((row_update_kernel<LPR>), dim3(blocks), dim3(256), 0, s, sorted_keys,     \
                     sorted_bag, de, sc.seg_starts, sc.num_unique, sc.long_list, sc.long_count, \
                     h, G, lr, eps);                                                           \
  hipLaunchKernelGGL((row_update_long_kernel<LPR>), dim3(256), dim3(256), 0, s, sorted_keys,   \
                     sorted_bag, de, sc.seg_starts, sc.long_list, sc.long_count, h, G, lr, eps)
  switch (d) {
    case 16: L(4); break;
    case 32: L(8); break;
    case 64: L(16); break;
    default: L(32); break;
  }
#undef L
}

}  // namespace ss
