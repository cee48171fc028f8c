// Stable LSD radix sort of (global row, value) pairs, up to 10 bits per pass (gfx950).
// The embedding backward needs every distinct row's occurrences side by side and in
// ascending flat position, so equal keys must keep their input order: each pass is
// histogram -> per-digit scan over blocks -> stable scatter.
//
// The input is table-major (all positions of table 0, then table 1, ...) and the key is
// row_base[t] + row, so the tables' position ranges are already in key order: every table's
// range is sorted on its own, on the digits of the LOCAL row, with as many passes as that
// table's row count needs and digits of that table's own width: b bits of local row take
// ceil(b / max_digit_bits) passes of ceil(b / passes) bits each (with the default of 8 a table
// of 60 000 rows takes two passes of 8 bits, one of 40 million rows four of 7; with 10 a table
// of a million rows takes two passes of 10 bits), and a table's last pass writes into the
// common result buffers.  The ranges come from a
// plan the step's gather kernel leaves in the scratch (first position and first tile of every
// table); blocks map to (table, tile) through it.
//
// A block owns a contiguous tile of 256*rounds elements of one table; wave w of the block owns
// the w-th quarter of the tile and walks it 64 elements at a time, so "earlier in the tile" is
// (wave, round, lane) order.  Ranks among equal digits inside a wave come from one ballot per
// digit bit; running per-wave digit counts live in LDS.  The scatter first reorders
// its tile by digit inside LDS, so that elements with equal digits leave as contiguous runs.
#include "ss_internal.h"

namespace ss {

constexpr int RADIX_BITS_MAX = 10;             // widest digit any pass may use
constexpr int RADIX_MAX = 1 << RADIX_BITS_MAX;
constexpr int SORT_THREADS = 256;
constexpr int SORT_WAVES = SORT_THREADS / SS_WAVE;
constexpr int MAX_ROUNDS = 16;

// Tile length for n elements in all: one block per CU once there is enough work, tiles of at
// most 4096 elements (long tiles give the scatter longer runs of equal digits, i.e. wider
// contiguous stores).  Returns the number of tiles of an unsegmented array.
int sort_num_blocks(uint32_t n, int* rounds_out) {
  int rounds = (int)((n + 256u * SORT_THREADS - 1) / (256u * SORT_THREADS));
  if (rounds < 1) rounds = 1;
  if (rounds > MAX_ROUNDS) rounds = MAX_ROUNDS;
  if (rounds_out) *rounds_out = rounds;
  return ceil_div(n, (int64_t)SORT_THREADS * rounds);
}

uint32_t sort_tile(uint32_t n) {
  int rounds = 1;
  sort_num_blocks(n, &rounds);
  return (uint32_t)(SORT_THREADS * rounds);
}

int sort_max_blocks(uint32_t max_n) {
  // below the round cap a sort never uses more than 256 tiles; above it, tiles of 4096; every
  // table's range may end in one partial tile
  int b = ceil_div(max_n, (int64_t)SORT_THREADS * MAX_ROUNDS);
  return (b > 256 ? b : 256) + SS_MAX_TABLES + 1;
}

struct SegDev {
  const uint32_t* seg_lo;     // [T + 1]
  const uint32_t* tile_base;  // [T + 1]
  int T;
  // 32-bit entries on purpose: with a byte array here the compiler derived the address of
  // meta.row_base[t] from the byte address of passes[t] (base + t, plus 3 t), and a scalar load
  // ignores the two low bits of each of its address components
  int32_t passes[SS_MAX_TABLES];
  int32_t width[SS_MAX_TABLES];   // digit bits of the table's passes (1..RADIX_BITS_MAX)
  TableMeta meta;
};

// (table, tile inside the table) of this block, or false when the block is beyond the last tile
// or its table is done after `pass` passes.  Wave-uniform.
__device__ __forceinline__ bool seg_of_block(const SegDev& g, int pass, uint32_t tile, int& t,
                                             uint32_t& base, uint32_t& end) {
  const int lane = threadIdx.x & 63;
  const bool ge = lane < g.T && blockIdx.x >= g.tile_base[lane + 1];
  t = (int)__popcll(__ballot(ge));
  if (t >= g.T || (int)g.passes[t] <= pass) return false;
  base = g.seg_lo[t] + (blockIdx.x - g.tile_base[t]) * tile;
  end = min(g.seg_lo[t + 1], base + tile);
  return true;
}

__global__ __launch_bounds__(SORT_THREADS) void radix_hist_kernel(
    const uint32_t* __restrict__ keys, SegDev g, int pass, int rounds, int pitch,
    uint32_t* __restrict__ block_hist) {
  __shared__ uint32_t hist[RADIX_MAX];
  const uint32_t tile = (uint32_t)(SORT_THREADS * rounds);
  int t;
  uint32_t base, end;
  if (!seg_of_block(g, pass, tile, t, base, end)) return;
  const uint32_t rb = g.meta.row_base[t];
  const int width = g.width[t];
  const int shift = pass * width;
  const uint32_t dmask = (1u << width) - 1u;
  for (int d = threadIdx.x; d < RADIX_MAX; d += SORT_THREADS) hist[d] = 0;
  __syncthreads();
  // the order inside the tile does not matter here: 16-byte loads from the aligned start
  // below the tile, all issued up front; elements outside [base, end) are masked
  const uint32_t a0 = base & ~3u;
  const uint32_t nv = (end - a0 + 3) / 4;          // <= tile / 4 + 1 vectors
  const uint4* kv = (const uint4*)(keys + a0);
  constexpr int NV = MAX_ROUNDS / 4 + 1;
  uint4 q[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const uint32_t v = threadIdx.x + i * SORT_THREADS;
    // (the last vector of the array may reach past n by up to 3 elements: the buffers are
    // allocated in multiples of 4)
    if (v < nv) q[i] = kv[v];
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const uint32_t v = threadIdx.x + i * SORT_THREADS;
    const uint32_t j0 = a0 + 4 * v;
    const bool any = v < nv;
    const bool full = any && j0 >= base && j0 + 4 <= end;
    const uint32_t d0 = ((q[i].x - rb) >> shift) & dmask;
    const uint32_t d1 = ((q[i].y - rb) >> shift) & dmask;
    const uint32_t d2 = ((q[i].z - rb) >> shift) & dmask;
    const uint32_t d3 = ((q[i].w - rb) >> shift) & dmask;
    // inside a long run of one hot row whole waves share one digit: count those with a single
    // LDS atomic instead of 256 colliding ones
    const bool same4 = full && (d0 == d1) && (d1 == d2) && (d2 == d3);
    const uint64_t vm = __ballot(any);
    if (vm == 0) continue;
    const uint32_t lead = __builtin_amdgcn_readlane(d0, __builtin_ctzll(vm));
    const bool uniform = __ballot(any && !(same4 && d0 == lead)) == 0;
    if (uniform) {
      if ((threadIdx.x & 63) == (uint32_t)__builtin_ctzll(vm)) atomicAdd(&hist[lead], 4u * (uint32_t)__popcll(vm));
    } else if (any) {
      if (same4) {
        atomicAdd(&hist[d0], 4u);
      } else {
        if (j0 >= base && j0 < end) atomicAdd(&hist[d0], 1u);
        if (j0 + 1 >= base && j0 + 1 < end) atomicAdd(&hist[d1], 1u);
        if (j0 + 2 >= base && j0 + 2 < end) atomicAdd(&hist[d2], 1u);
        if (j0 + 3 >= base && j0 + 3 < end) atomicAdd(&hist[d3], 1u);
      }
    }
  }
  __syncthreads();
  for (uint32_t d = threadIdx.x; d <= dmask; d += SORT_THREADS)
    block_hist[(size_t)d * pitch + blockIdx.x] = hist[d];  // digit-major
}

// One wave per (digit, table): exclusive scan of that digit's counts over the table's tiles
// (in place) and the digit's total inside the table.
__global__ __launch_bounds__(64) void radix_scan_kernel(uint32_t* __restrict__ block_hist,
                                                        int pitch, SegDev g, int pass,
                                                        uint32_t* __restrict__ seg_tot) {
  const int t = blockIdx.y, lane = threadIdx.x;
  if ((int)g.passes[t] <= pass || (int)blockIdx.x >= (1 << g.width[t])) return;
  const uint32_t b0 = g.tile_base[t], nb = g.tile_base[t + 1] - b0;
  uint32_t* row = block_hist + (size_t)blockIdx.x * pitch + b0;
  const uint32_t per = (nb + 63) / 64;
  const uint32_t lo = min(nb, lane * per), hi = min(nb, lo + per);
  uint32_t s = 0;
  for (uint32_t i = lo; i < hi; ++i) s += row[i];
  uint32_t incl = s;
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t v = __shfl_up(incl, off);
    if (lane >= off) incl += v;
  }
  uint32_t run = incl - s;
  for (uint32_t i = lo; i < hi; ++i) {
    const uint32_t c = row[i];
    row[i] = run;
    run += c;
  }
  if (lane == 63) seg_tot[t * RADIX_MAX + blockIdx.x] = incl;
}

// RB: digit bits the kernel's LDS tables are sized for (the widest digit of any table of this
// sort); a table with narrower digits uses the first 2^width entries.
template <int RB>
__global__ __launch_bounds__(SORT_THREADS) void radix_scatter_kernel(
    const uint32_t* __restrict__ keys_in, const uint32_t* __restrict__ vals_in, SegDev g, int pass,
    int rounds, int pitch, const uint32_t* __restrict__ block_hist,
    const uint32_t* __restrict__ seg_tot, uint32_t* __restrict__ keys_mid,
    uint32_t* __restrict__ vals_mid, uint32_t* __restrict__ keys_fin,
    uint32_t* __restrict__ vals_fin) {
  constexpr int ND = 1 << RB;                   // digits the tables hold
  constexpr int DPT = ND / SORT_THREADS;        // consecutive digits per thread (1, 2 or 4)
  static_assert(DPT >= 1 && RB <= RADIX_BITS_MAX && RADIX_MAX == SORT_MAX_DIGITS, "digit tables are split over the block's threads");
  // per-wave running digit counts; volatile: lanes of one wave hand values to each other
  // through it between rounds without a barrier
  __shared__ volatile uint32_t wrun[SORT_WAVES][ND];
  __shared__ uint32_t gbase[ND];                // global start of this block's run of a digit
  __shared__ uint32_t lbase[ND];                // start of the digit inside the block's tile
  __shared__ uint32_t gsum[SORT_THREADS], lsum[SORT_THREADS];
  __shared__ uint32_t skey[SORT_THREADS * MAX_ROUNDS], sval[SORT_THREADS * MAX_ROUNDS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t tile = (uint32_t)(SORT_THREADS * rounds);
  int t;
  uint32_t base, n;   // n: end of this tile's elements
  if (!seg_of_block(g, pass, tile, t, base, n)) return;
  const uint32_t rb = g.meta.row_base[t];
  const int width = g.width[t];                 // <= RB
  const int shift = pass * width;
  const uint32_t dmask = (1u << width) - 1u;
  // a table's last pass writes the common result buffers
  const bool last = pass == (int)g.passes[t] - 1;
  uint32_t* __restrict__ keys_out = last ? keys_fin : keys_mid;
  uint32_t* __restrict__ vals_out = last ? vals_fin : vals_mid;
  const uint32_t wbase = base + wave * (uint32_t)(SS_WAVE * rounds);
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
  // this thread's digits: tid * DPT + i
  uint32_t dtot[DPT], boff[DPT];
  const uint32_t lo_t = g.seg_lo[t];
#pragma unroll
  for (int i = 0; i < DPT; ++i) {
    const uint32_t d = (uint32_t)(tid * DPT + i);
    const bool used = d <= dmask;
    dtot[i] = used ? seg_tot[t * RADIX_MAX + d] : 0u;
    boff[i] = used ? block_hist[(size_t)d * pitch + blockIdx.x] + lo_t : 0u;
  }
#pragma unroll
  for (int w = 0; w < SORT_WAVES; ++w)
#pragma unroll
    for (int i = 0; i < DPT; ++i) wrun[w][tid + i * SORT_THREADS] = 0;
  __syncthreads();

#pragma unroll
  for (int r = 0; r < MAX_ROUNDS; ++r) {
    if (r < rounds) {
      const uint32_t j = wbase + r * SS_WAVE + lane;
      const bool valid = j < n;
      const uint32_t dg = ((key[r] - rb) >> shift) & dmask;
      uint64_t m = __ballot(valid);
      // a wave inside a long run of one hot row (passes after the first: equal keys are
      // neighbours) holds a single digit: every valid lane matches every other
      const uint32_t lead = __builtin_amdgcn_readfirstlane(dg);
      if (__ballot(valid && dg != lead) != 0) {
#pragma unroll
        for (int b = 0; b < RB; ++b) {
          if (b < width) {   // wave-uniform
            const uint64_t bal = __ballot((dg >> b) & 1u);
            m &= ((dg >> b) & 1u) ? bal : ~bal;
          }
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
  uint32_t cnt[DPT];
  uint32_t gs = 0, ls = 0;
#pragma unroll
  for (int i = 0; i < DPT; ++i) {
    const int d = tid * DPT + i;
    uint32_t c0 = 0;
#pragma unroll
    for (int w = 0; w < SORT_WAVES; ++w) {
      const uint32_t c = wrun[w][d];
      wrun[w][d] = c0;
      c0 += c;
    }
    cnt[i] = c0;
    gs += dtot[i];
    ls += c0;
  }
  // two exclusive scans over the digits at once: digit totals of the table's whole range
  // (global digit starts) and digit counts of this tile (starts inside the tile); a thread's
  // consecutive digits are scanned in registers, the threads' sums in LDS
  gsum[tid] = gs;
  lsum[tid] = ls;
  __syncthreads();
  for (int off = 1; off < SORT_THREADS; off <<= 1) {
    const uint32_t a = (tid >= off) ? gsum[tid - off] : 0;
    const uint32_t b = (tid >= off) ? lsum[tid - off] : 0;
    __syncthreads();
    gsum[tid] += a;
    lsum[tid] += b;
    __syncthreads();
  }
  uint32_t gex = gsum[tid] - gs, lex = lsum[tid] - ls;
#pragma unroll
  for (int i = 0; i < DPT; ++i) {
    const int d = tid * DPT + i;
    gbase[d] = gex + boff[i];
    lbase[d] = lex;
    gex += dtot[i];
    lex += cnt[i];
  }
  __syncthreads();
  // reorder the tile by digit inside LDS (stable: wave, round, lane order within a digit)
#pragma unroll
  for (int r = 0; r < MAX_ROUNDS; ++r) {
    if (r < rounds) {
      const uint32_t j = wbase + r * SS_WAVE + lane;
      if (j < n) {
        const uint32_t dg = ((key[r] - rb) >> shift) & dmask;
        const uint32_t lp = lbase[dg] + wrun[wave][dg] + rank[r];
        skey[lp] = key[r];
        sval[lp] = val[r];
      }
    }
  }
  __syncthreads();
  // element i of the reordered tile goes to the i-th slot of its digit's run: neighbours in
  // the tile with the same digit are neighbours in the output
  const uint32_t count = n - base;
  for (uint32_t i = tid; i < count; i += SORT_THREADS) {
    const uint32_t k = skey[i], v = sval[i];
    const uint32_t dg = ((k - rb) >> shift) & dmask;
    const uint32_t dst = gbase[dg] + (i - lbase[dg]);
    keys_out[dst] = k;
    vals_out[dst] = v;
  }
}

void launch_sort_pairs(const uint32_t* keys, const uint32_t* vals, uint32_t n,
                       const SortSegments& seg, const SortScratch& sc, uint32_t** sorted_keys,
                       uint32_t** sorted_vals, hipStream_t s) {
  *sorted_keys = sc.keys_f;
  *sorted_vals = sc.vals_f;
  if (n == 0) return;
  int rounds = 1;
  sort_num_blocks(n, &rounds);
  const uint32_t tile = (uint32_t)(SORT_THREADS * rounds);
  // upper bound of the tiles: every table's range may end in a partial one
  const int nblocks = ceil_div(n, tile) + seg.T;
  const int pitch = nblocks;
  int dmax = seg.max_digit_bits;
  if (dmax < 8) dmax = 8;
  if (dmax > RADIX_BITS_MAX) dmax = RADIX_BITS_MAX;
  SegDev g;
  g.seg_lo = sc.seg_lo; g.tile_base = sc.tile_base; g.T = seg.T; g.meta = *seg.meta;
  int max_passes = 1, max_width = 1;
  for (int t = 0; t < seg.T; ++t) {
    // bits of the largest local row of the table, split evenly over the fewest passes
    const uint32_t rows = seg.meta->row_base[t + 1] - seg.meta->row_base[t];
    int bits = 1;
    while (bits < 32 && (1ull << bits) < rows) ++bits;
    const int p = (bits + dmax - 1) / dmax;
    const int w = (bits + p - 1) / p;
    g.passes[t] = p;
    g.width[t] = w;
    if (p > max_passes) max_passes = p;
    if (w > max_width) max_width = w;
  }
  for (int t = seg.T; t < SS_MAX_TABLES; ++t) { g.passes[t] = 0; g.width[t] = 1; }
  const uint32_t* kin = keys;
  const uint32_t* vin = vals;     // null: the value is the element's own position
  uint32_t* kmid = sc.keys_a; uint32_t* kother = sc.keys_b;
  uint32_t* vmid = sc.vals; uint32_t* vother = sc.vals_alt;
  for (int p = 0; p < max_passes; ++p) {
    hipLaunchKernelGGL(radix_hist_kernel, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin, g, p,
                       rounds, pitch, sc.block_hist);
    hipLaunchKernelGGL(radix_scan_kernel, dim3(1 << max_width, seg.T), dim3(64), 0, s,
                       sc.block_hist, pitch, g, p, sc.seg_tot);
    if (max_width <= 8)
      hipLaunchKernelGGL(radix_scatter_kernel<8>, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin, vin,
                         g, p, rounds, pitch, sc.block_hist, sc.seg_tot, kmid, vmid, sc.keys_f,
                         sc.vals_f);
    else if (max_width == 9)
      hipLaunchKernelGGL(radix_scatter_kernel<9>, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin, vin,
                         g, p, rounds, pitch, sc.block_hist, sc.seg_tot, kmid, vmid, sc.keys_f,
                         sc.vals_f);
    else
      hipLaunchKernelGGL(radix_scatter_kernel<10>, dim3(nblocks), dim3(SORT_THREADS), 0, s, kin,
                         vin, g, p, rounds, pitch, sc.block_hist, sc.seg_tot, kmid, vmid,
                         sc.keys_f, sc.vals_f);
    kin = kmid; vin = vmid;
    uint32_t* x = kmid; kmid = kother; kother = x;
    x = vmid; vmid = vother; vother = x;
  }
}

}  // namespace ss
