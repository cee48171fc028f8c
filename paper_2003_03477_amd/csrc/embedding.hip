// Embedding kernels (gfx950): sum-pooled gather (forward, Section 3.1: pooling happens where
// the table lives) and the compaction of segment starts over the row-sorted (row, position)
// pairs of the backward pass.  The row update itself lives in row_update.hip.
#include "ss_internal.h"

namespace ss {

// ------------------------------------------------------------------------------------------
// Forward.  One wavefront per bag.  A row of d floats is covered by LPR = d/4 lanes loading
// one float4 each, so a wave keeps 64/LPR rows in flight per load instruction.  The bag's
// index list is read once, coalesced, 64 ids at a time, and handed between lanes with
// cross-lane permutes; every lane owns fixed columns, partial sums of the 64/LPR row slots
// are folded with xor-shuffles at the end.
// With row shards (Section 3.1, "Embedding PS": a table too large for one parameter server is
// split by rows, every shard pools the rows it owns and the trainer adds the partial results)
// blockIdx.y is the shard: the wave walks the whole bag but only fetches and adds the rows
// inside its shard's range, and writes the bag's PARTIAL sum to its shard's slice of `e`
// ([shard][B*T][d]); embedding_combine_kernel adds the slices in shard order.
template <int LPR, bool SHARDED>
__global__ __launch_bounds__(256) void embedding_bag_fwd_kernel(
    const float* __restrict__ h, const int32_t* __restrict__ indices,
    const int32_t* __restrict__ offsets, TableMeta meta, int B, int T, float* __restrict__ e,
    uint32_t* __restrict__ keys, int32_t* __restrict__ bag_of_pos,
    float* __restrict__ zero_scalar, float* __restrict__ inv_len, int n_shards, SortPlanOut plan) {
  constexpr int D = LPR * 4;
  constexpr int RPW = SS_WAVE / LPR;  // rows per wave-wide load
  constexpr int NIF = 8;              // row loads in flight per lane
  const int shard = SHARDED ? blockIdx.y : 0;
  // the step's loss accumulator is cleared here, ahead of the kernel that adds into it
  if (zero_scalar && blockIdx.x == 0 && shard == 0 && threadIdx.x == 0) *zero_scalar = 0.f;
  const int lane = threadIdx.x & 63;
  // The last workgroup of the grid (a spare one: the launcher rounds up past the bags) leaves
  // the plan of the backward pass's sort behind: where every table's positions begin and how
  // many tiles of the sort precede them.
  if (plan.seg_lo && blockIdx.x == gridDim.x - 1 && shard == 0 && threadIdx.x < 64) {
    const uint32_t n_all = (uint32_t)offsets[(size_t)T * B];
    const uint32_t lo = lane < T ? (uint32_t)offsets[(size_t)lane * B] : n_all;
    uint32_t nxt = (uint32_t)__shfl_down((int)lo, 1);
    if (lane >= T - 1) nxt = n_all;
    const uint32_t tiles = lane < T ? (nxt - lo + plan.tile - 1) / plan.tile : 0u;
    uint32_t incl = tiles;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const uint32_t v = (uint32_t)__shfl_up((int)incl, off);
      if (lane >= off) incl += v;
    }
    if (lane < T) {
      plan.seg_lo[lane] = lo;
      plan.tile_base[lane] = incl - tiles;
    }
    if (lane == T - 1) {
      plan.seg_lo[T] = n_all;
      plan.tile_base[T] = incl;
    }
  }
  // Workgroups go to the chip's eight dies (each with its own L2) in turn; the grid is a
  // multiple of 8 and die x takes the x-th eighth of the bags (table-major), so that every L2
  // holds the hot rows of the one or two tables its die is working on instead of all eight
  // holding the same table's.
  const uint32_t per_die = gridDim.x >> 3;
  const uint32_t lb = (blockIdx.x & 7u) * per_die + (blockIdx.x >> 3);
  const int64_t bag64 = (int64_t)lb * (blockDim.x >> 6) + (threadIdx.x >> 6);  // t*B + b
  if (bag64 >= (int64_t)T * B) return;
  const int bag = (int)bag64;
  const int t = bag / B, b = bag - t * B;
  const int lo = offsets[bag], hi = offsets[bag + 1];
  const uint32_t base = meta.row_base[t];
  // this shard's rows of table t: [s_lo, s_hi) (everything when the tables are not split)
  uint32_t s_lo = 0, s_hi = 0xFFFFFFFFu;
  if (SHARDED) {
    const uint32_t rows_t = meta.row_base[t + 1] - base;
    const uint32_t per = (rows_t + n_shards - 1) / n_shards;
    s_lo = (uint32_t)shard * per;
    s_hi = s_lo + per;
    e += (size_t)shard * B * T * D;
  }
  const int sub = lane / LPR, c4 = lane % LPR;
  const int ebag = b * T + t;
  float4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
  for (int j0 = lo; j0 < hi; j0 += SS_WAVE) {
    const int j = j0 + lane;
    uint32_t grow = 0, lrow = 0xFFFFFFFFu;
    if (j < hi) {
      lrow = (uint32_t)indices[j];
      grow = base + lrow;
      if (keys && shard == 0) {   // (forward-only evaluation records nothing for a backward pass)
        keys[j] = grow;
        bag_of_pos[j] = ebag;
      }
    }
    const bool mine = !SHARDED || (lrow >= s_lo && lrow < s_hi);
    const int cnt = min(SS_WAVE, hi - j0);
    // trip count is wave-uniform so every lane takes part in every permute; NIF row loads per
    // lane are issued before the first is consumed (a bag of up to NIF * RPW ids is one round
    // trip to memory instead of one per pair of loads)
    for (int it = 0; it < cnt; it += NIF * RPW) {
      float4 v[NIF];
#pragma unroll
      for (int u = 0; u < NIF; ++u) {
        const int ju = it + u * RPW + sub;
        const uint32_t ru = (uint32_t)__shfl((int)grow, ju & 63);
        bool mu = true;
        if (SHARDED) mu = __shfl((int)mine, ju & 63) != 0;
        v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ju < cnt && mu) v[u] = *(const float4*)(h + (size_t)ru * D + c4 * 4);
      }
#pragma unroll
      for (int u = 0; u < NIF; u += 2) {
        acc0.x += v[u].x; acc0.y += v[u].y; acc0.z += v[u].z; acc0.w += v[u].w;
        acc1.x += v[u + 1].x; acc1.y += v[u + 1].y; acc1.z += v[u + 1].z; acc1.w += v[u + 1].w;
      }
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
  if (inv_len) {
    // mean pooling: the sum over the bag divided by its length; 1/length is kept per pooled
    // vector because every member's gradient carries the same factor.  With row shards the
    // partial sums stay sums; the combining kernel applies the factor.
    const float sc = (hi > lo) ? 1.0f / (float)(hi - lo) : 0.f;
    if (!SHARDED) { acc.x *= sc; acc.y *= sc; acc.z *= sc; acc.w *= sc; }
    if (lane == 0 && shard == 0) inv_len[ebag] = sc;
  }
  if (sub == 0) *(float4*)(e + (size_t)ebag * D + c4 * 4) = acc;
}

// Trainer side of partial pooling: e[v] = (sum over the shards, ascending, of part[s][v]) (times
// 1 / bag length under mean pooling).  One thread per float4.
__global__ __launch_bounds__(256) void embedding_combine_kernel(const float* __restrict__ part,
                                                                int n_shards, int64_t n_vec4,
                                                                int d4, const float* __restrict__ inv_len,
                                                                float* __restrict__ e) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_vec4) return;
  float4 acc = ((const float4*)part)[i];
  for (int s = 1; s < n_shards; ++s) {
    const float4 v = ((const float4*)part)[(int64_t)s * n_vec4 + i];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if (inv_len) {
    const float sc = inv_len[i / d4];
    acc.x *= sc; acc.y *= sc; acc.z *= sc; acc.w *= sc;
  }
  ((float4*)e)[i] = acc;
}

void launch_embedding_bag_fwd(const float* h, const int32_t* indices, const int32_t* offsets,
                              const TableMeta& meta, int B, int T, int d, float* e,
                              uint32_t* keys, int32_t* bag_of_pos, float* zero_scalar,
                              float* inv_len, int n_shards, float* e_part, const SortPlanOut& plan,
                              hipStream_t s) {
  const int64_t bags = (int64_t)B * T;
  if (bags == 0) return;
  const bool split = n_shards > 1;
  // (one workgroup more than the bags need: see the kernel)
  dim3 grid((unsigned)(ceil_div(ceil_div(bags, 4) + 1, 8) * 8), split ? n_shards : 1), block(256);
  float* out = split ? e_part : e;
#define L(LPR)                                                                                  \
  do {                                                                                          \
    if (split)                                                                                  \
      hipLaunchKernelGGL((embedding_bag_fwd_kernel<LPR, true>), grid, block, 0, s, h, indices,  \
                         offsets, meta, B, T, out, keys, bag_of_pos, zero_scalar, inv_len,      \
                         n_shards, plan);                                                       \
    else                                                                                        \
      hipLaunchKernelGGL((embedding_bag_fwd_kernel<LPR, false>), grid, block, 0, s, h, indices, \
                         offsets, meta, B, T, out, keys, bag_of_pos, zero_scalar, inv_len, 1,   \
                         plan);                                                                 \
  } while (0)
  switch (d) {
    case 16: L(4); break;
    case 32: L(8); break;
    case 64: L(16); break;
    default: L(32); break;  // 128
  }
#undef L
  if (split) {
    const int64_t n_vec4 = bags * (d / 4);
    hipLaunchKernelGGL(embedding_combine_kernel, dim3((unsigned)ceil_div(n_vec4, 256)), dim3(256), 0,
                       s, e_part, n_shards, n_vec4, d / 4, inv_len, e);
  }
}

// ------------------------------------------------------------------------------------------
// Segment starts: flag j where sorted_keys[j] != sorted_keys[j-1], count per block, scan the
// block counts, compact.  SEG_TILE elements per block.
constexpr int SEG_TILE = 2048;   // 256 threads x 8

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
// seg_starts[U] = n.
__global__ __launch_bounds__(1024) void seg_scan_kernel(uint32_t* __restrict__ block_counts,
                                                        int nblocks, uint32_t n,
                                                        uint32_t* __restrict__ num_unique,
                                                        uint32_t* __restrict__ seg_starts) {
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
                     sc.num_unique, sc.seg_starts);
  if (nb > 0)
    hipLaunchKernelGGL(seg_compact_kernel, dim3(nb), dim3(256), 0, s, sorted_keys, n,
                       sc.block_counts, sc.seg_starts);
}

}  // namespace ss
