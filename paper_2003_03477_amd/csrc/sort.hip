// Stable LSD radix sort of (global row, flat position) pairs, 8 bits per pass (gfx950).
// The embedding backward needs every distinct row's occurrences side by side and in
// ascending flat position, so equal keys must keep their input order: each pass is
// histogram -> per-digit scan over blocks -> stable scatter.
//
// A block owns a contiguous tile of 256*rounds elements; wave w of the block owns the w-th
// quarter of the tile and walks it 64 elements at a time, so "earlier in the tile" is
// (wave, round, lane) order.  Ranks among equal digits inside a wave come from 8 ballots
// (one per digit bit); running per-wave digit counts live in LDS.  The scatter first reorders
// its tile by digit inside LDS, so that elements with equal digits leave as contiguous runs.
#include "ss_internal.h"

namespace ss {

constexpr int RADIX_BITS = 8;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_THREADS = 256;
constexpr int SORT_WAVES = SORT_THREADS / SS_WAVE;
constexpr int MAX_ROUNDS = 16;

int sort_num_blocks(uint32_t n, int* rounds_out) {
  // one block per CU once there is enough work, tiles of at most 4096 elements: long tiles
  // give the scatter longer runs of equal digits, i.e. wider contiguous stores
  int rounds = (int)((n + 256u * SORT_THREADS - 1) / (256u * SORT_THREADS));
  if (rounds < 1) rounds = 1;
  if (rounds > MAX_ROUNDS) rounds = MAX_ROUNDS;
  if (rounds_out) *rounds_out = rounds;
  return ceil_div(n, (int64_t)SORT_THREADS * rounds);
}

int sort_max_blocks(uint32_t max_n) {
  // below the round cap a sort never uses more than 256 blocks; above it, tiles of 4096
  int b = ceil_div(max_n, (int64_t)SORT_THREADS * MAX_ROUNDS);
  return (b > 256 ? b : 256) + 1;
}

__global__ __launch_bounds__(SORT_THREADS) void radix_hist_kernel(
    const uint32_t* __restrict__ keys, uint32_t n, int shift, int rounds, int nblocks,
    uint32_t* __restrict__ block_hist) {
  __shared__ uint32_t hist[RADIX];
  hist[threadIdx.x] = 0;
  __syncthreads();
  const uint32_t base = blockIdx.x * (uint32_t)(SORT_THREADS * rounds);
  // the order inside the tile does not matter here: 16-byte loads, all issued up front
  const uint32_t end = min(n, base + (uint32_t)(SORT_THREADS * rounds));
  const uint32_t cnt = end > base ? end - base : 0u;
  const uint32_t nv = cnt / 4;
  const uint4* kv = (const uint4*)(keys + base);
  uint4 q[MAX_ROUNDS / 4];
#pragma unroll
  for (int i = 0; i < MAX_ROUNDS / 4; ++i) {
    const uint32_t v = threadIdx.x + i * SORT_THREADS;
    if (v < nv) q[i] = kv[v];
  }
#pragma unroll
  for (int i = 0; i < MAX_ROUNDS / 4; ++i) {
    const uint32_t v = threadIdx.x + i * SORT_THREADS;
    const bool valid = v < nv;
    const uint32_t d0 = valid ? (q[i].x >> shift) & (RADIX - 1) : 0u;
    const uint32_t d1 = valid ? (q[i].y >> shift) & (RADIX - 1) : 0u;
    const uint32_t d2 = valid ? (q[i].z >> shift) & (RADIX - 1) : 0u;
    const uint32_t d3 = valid ? (q[i].w >> shift) & (RADIX - 1) : 0u;
    // in the later passes the input is sorted by the lower digits and whole waves share one
    // digit: count those with a single LDS atomic instead of 256 colliding ones
    const bool same4 = (d0 == d1) && (d1 == d2) && (d2 == d3);
    const uint64_t vm = __ballot(valid);
    if (vm == 0) continue;
    const uint32_t lead = __builtin_amdgcn_readlane(d0, __builtin_ctzll(vm));
    const bool uniform = __ballot(valid && !(same4 && d0 == lead)) == 0;
    if (uniform) {
      if ((threadIdx.x & 63) == (uint32_t)__builtin_ctzll(vm)) atomicAdd(&hist[lead], 4u * (uint32_t)__popcll(vm));
    } else if (valid) {
      if (same4) {
        atomicAdd(&hist[d0], 4u);
      } else {
        atomicAdd(&hist[d0], 1u);
        atomicAdd(&hist[d1], 1u);
        atomicAdd(&hist[d2], 1u);
        atomicAdd(&hist[d3], 1u);
      }
    }
  }
  for (uint32_t j = base + nv * 4 + threadIdx.x; j < end; j += SORT_THREADS)
    atomicAdd(&hist[(keys[j] >> shift) & (RADIX - 1)], 1u);
  __syncthreads();
  block_hist[(size_t)threadIdx.x * nblocks + blockIdx.x] = hist[threadIdx.x];  // digit-major
}

// One block per digit: exclusive scan of that digit's counts over the blocks (in place) and
// the digit's total.
__global__ __launch_bounds__(256) void radix_scan_kernel(uint32_t* __restrict__ block_hist,
                                                         int nblocks,
                                                         uint32_t* __restrict__ digit_tot) {
  __shared__ uint32_t part[256];
  uint32_t* row = block_hist + (size_t)blockIdx.x * nblocks;
  const int tid = threadIdx.x;
  const int per = (nblocks + 255) / 256;
  const int lo = min(nblocks, tid * per), hi = min(nblocks, lo + per);
  uint32_t s = 0;
  for (int i = lo; i < hi; ++i) s += row[i];
  part[tid] = s;
  __syncthreads();
  for (int off = 1; off < 256; off <<= 1) {
    uint32_t v = (tid >= off) ? part[tid - off] : 0;
    __syncthreads();
    part[tid] += v;
    __syncthreads();
  }
  uint32_t run = part[tid] - s;
  for (int i = lo; i < hi; ++i) {
    uint32_t c = row[i];
    row[i] = run;
    run += c;
  }
  if (tid == 255) digit_tot[blockIdx.x] = part[255];
}

__global__ __launch_bounds__(SORT_THREADS) void radix_scatter_kernel(
    const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in, uint32_t n,
    int shift, int rounds, int nblocks, const uint32_t* __restrict__ block_hist,
    const uint32_t* __restrict__ digit_tot, uint32_t* __restrict__ keys_out,
    uint32_t* __restrict__ vals_out) {
  // per-wave running digit counts; volatile: lanes of one wave hand values to each other
  // through it between rounds without a barrier
  __shared__ volatile uint32_t wrun[SORT_WAVES][RADIX];
  __shared__ uint32_t gbase[RADIX];             // global start of this block's run of a digit
  __shared__ uint32_t lbase[RADIX];             // start of the digit inside the block's tile
  __shared__ uint32_t skey[SORT_THREADS * MAX_ROUNDS], sval[SORT_THREADS * MAX_ROUNDS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t tile = (uint32_t)(SORT_THREADS * rounds);
  const uint32_t wbase = blockIdx.x * tile + wave * (uint32_t)(SS_WAVE * rounds);
  // issue the loads first: this tile's keys and values, the digit totals, this block's offsets
  uint32_t key[MAX_ROUNDS], val[MAX_ROUNDS], rank[MAX_ROUNDS];
#pragma unroll
  for (int r = 0; r < MAX_ROUNDS; ++r) {
    if (r < rounds) {
      const uint32_t j = wbase + r * SS_WAVE + lane;
      key[r] = (j < n) ? keys_in[j] : 0xFFFFFFFFu;
      val[r] = (j < n && vals_in) ? vals_in[j] : j;
    }
  }
  const uint32_t dtot = digit_tot[tid];
  const uint32_t boff = block_hist[(size_t)tid * nblocks + blockIdx.x];
  for (int w = 0; w < SORT_WAVES; ++w) wrun[w][tid] = 0;
  __syncthreads();

#pragma unroll
  for (int r = 0; r < MAX_ROUNDS; ++r) {
    if (r < rounds) {
      const uint32_t j = wbase + r * SS_WAVE + lane;
      const bool valid = j < n;
      const uint32_t dg = (key[r] >> shift) & (RADIX - 1);
      uint64_t m = __ballot(valid);
      // a wave inside a long run of one hot row (passes after the first: equal keys are
      // neighbours) holds a single digit: every valid lane matches every other
      const uint32_t lead = __builtin_amdgcn_readfirstlane(dg);
      if (__ballot(valid && dg != lead) != 0) {
#pragma unroll
        for (int b = 0; b < RADIX_BITS; ++b) {
          const uint64_t bal = __ballot((dg >> b) & 1u);
          m &= ((dg >> b) & 1u) ? bal : ~bal;
        }
      }
      // m = valid lanes of this wave holding the same digit (includes this lane if valid)
      const uint32_t before = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
      uint32_t prev = 0;
      if (valid) prev = wrun[wave][dg];
      // every lane has read the running count before the group's last lane bumps it: LDS
      // operations of one wave complete in program order
      if (valid && (m >> lane) == 1ull) wrun[wave][dg] = prev + (uint32_t)__popcll(m);
      rank[r] = prev + before;
    }
  }
  __syncthreads();
  // per digit: exclusive prefix of the per-wave counts over the waves; the digit's count in
  // this tile feeds the scan over digits below
  uint32_t cnt = 0;
  for (int w = 0; w < SORT_WAVES; ++w) {
    const uint32_t c = wrun[w][tid];
    wrun[w][tid] = cnt;
    cnt += c;
  }
  // two exclusive scans over the 256 digits at once: digit totals of the whole array (global
  // digit starts) and digit counts of this tile (starts inside the tile)
  gbase[tid] = dtot;
  lbase[tid] = cnt;
  __syncthreads();
  for (int off = 1; off < RADIX; off <<= 1) {
    const uint32_t a = (tid >= off) ? gbase[tid - off] : 0;
    const uint32_t b = (tid >= off) ? lbase[tid - off] : 0;
    __syncthreads();
    gbase[tid] += a;
    lbase[tid] += b;
    __syncthreads();
  }
  const uint32_t gex = gbase[tid] - dtot, lex = lbase[tid] - cnt;
  __syncthreads();
  gbase[tid] = gex + boff;
  lbase[tid] = lex;
  __syncthreads();
  // reorder the tile by digit inside LDS (stable: wave, round, lane order within a digit)
#pragma unroll
  for (int r = 0; r < MAX_ROUNDS; ++r) {
    if (r < rounds) {
      const uint32_t j = wbase + r * SS_WAVE + lane;
      if (j < n) {
        const uint32_t dg = (key[r] >> shift) & (RADIX - 1);
        const uint32_t lp = lbase[dg] + wrun[wave][dg] + rank[r];
        skey[lp] = key[r];
        sval[lp] = val[r];
      }
    }
  }
  __syncthreads();
  // element i of the reordered tile goes to the i-th slot of its digit's run: neighbours in
  // the tile with the same digit are neighbours in the output
  const uint32_t count = min(tile, n - min(n, blockIdx.x * tile));
  for (uint32_t i = tid; i < count; i += SORT_THREADS) {
    const uint32_t k = skey[i], v = sval[i];
    const uint32_t dg = (k >> shift) & (RADIX - 1);
    const uint32_t dst = gbase[dg] + (i - lbase[dg]);
    keys_out[dst] = k;
    vals_out[dst] = v;
  }
}

void launch_sort_pairs(const uint32_t* keys, const uint32_t* vals, uint32_t n, int key_bits,
                       const SortScratch& sc, uint32_t** sorted_keys, uint32_t** sorted_vals,
                       hipStream_t s) {
  const uint32_t* kin = keys;
  const uint32_t* vin = vals;     // null: the value is the element's own position
  uint32_t* kout = sc.keys_a;
  uint32_t* kother = sc.keys_b;
  uint32_t* vout = sc.vals;
  uint32_t* vother = sc.vals_alt;
  int passes = (key_bits + RADIX_BITS - 1) / RADIX_BITS;
  if (passes < 1) passes = 1;
  int rounds = 1;
  const int nblocks = sort_num_blocks(n, &rounds);
  *sorted_keys = sc.keys_a;
  *sorted_vals = sc.vals;
  if (n == 0) return;
  for (int p = 0; p < passes; ++p) {
    const int shift = p * RADIX_BITS;
    hipLaunchKernelGGL(radix_hist_kernel, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin, n, shift,
                       rounds, nblocks, sc.block_hist);
    hipLaunchKernelGGL(radix_scan_kernel, dim3(RADIX), dim3(256), 0, s, sc.block_hist, nblocks,
                       sc.digit_tot);
    hipLaunchKernelGGL(radix_scatter_kernel, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin, vin, n,
                       shift, rounds, nblocks, sc.block_hist, sc.digit_tot, kout, vout);
    *sorted_keys = kout;
    *sorted_vals = vout;
    kin = kout; vin = vout;
    uint32_t* t = kout; kout = kother; kother = t;
    t = vout; vout = vother; vother = t;
  }
}

}  // namespace ss
