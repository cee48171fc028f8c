// Embedding backward, second half (gfx950): per distinct row, the sum of the pooled-vector
// gradients of all its occurrences, then ONE optimiser update of that row (Section 3.2:
// lock-free optimiser updates on the single shared copy of the tables, the optimiser's state
// kept beside each row; the section names Adagrad and Adam):
//   row-wise Adagrad   G_r += mean_c g_r[c]^2 ;  h[r,:] -= lr * g_r / (sqrt(G_r) + eps)
//   Adam (lazy)        t_r += 1 ; m = b1 m + (1-b1) g ; v = b2 v + (1-b2) g^2 ;
//                      h[r,:] -= lr * (m / (1-b1^t_r)) / (sqrt(v / (1-b2^t_r)) + eps)
//                      with m, v per element and the step count t_r per row (kept in G[r]):
//                      a row's state only moves in the steps that touch the row.
//
// Input: the (row, position) pairs sorted by row, as `sorted_keys` and the pooled-vector id
// `sorted_bag` of every sorted entry.  With Zipf-distributed ids the run lengths range from 1
// to thousands, so work is split by POSITION, not by row: a group of LPR = d/4 lanes owns a
// chunk of C = S * LPR consecutive sorted entries (S = 1, 2 or 4 slices of LPR, one entry per
// lane and slice, by problem size), whatever runs they belong to.
//   pass 1 (chunk kernel): walk the chunk; a run that begins and ends inside the chunk is
//     finished on the spot (gradient rows and table rows of a sub-block of 8 entries are all
//     in flight together).  A run cut by the chunk's edges leaves a partial sum: slot 0 for
//     the piece that continues a run from the previous chunk (flag 1 = the run ends here,
//     flag 4 = the whole chunk lies inside the run), slot 1 for the piece that opens a run
//     continuing into the next chunk (flag 2).
//   pass 2 (stitch kernel): the chunk that opened a run adds the slot-0 partials of the
//     following chunks up to the one that ends the run and applies the update; a run that
//     spans more than 30 further chunks is queued instead.
//   pass 3 (long-run kernel): one 1024-thread block per queued run finds the run's last chunk
//     by scanning the flags and sums the partials in parallel.
#include "ss_internal.h"

namespace ss {

// Table rows are read once and written once per step: they pass through the caches with the
// non-temporal hint, so that the gradient rows (each re-read once per member of its bag, from
// all over the sorted order) stay resident.
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
__device__ __forceinline__ float4 load_row_nt(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load((const f32x4_t*)p);
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_row_nt(float* p, float4 v) {
  f32x4_t t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, (f32x4_t*)p);
}

// A chunk is CHUNK_SLICES wave-slices of LPR entries: short enough for tens of thousands of
// chunks per step, long enough that few runs are cut by a chunk's edges (with Zipf-distributed
// ids almost every second pair of neighbours in the sorted order shares its row).
// Slices per chunk by problem size: long chunks pay off once there are enough of them to keep
// every CU busy (sized for the shortest chunk, which needs the most scratch).
static int chunk_slices(uint32_t n) { return n >= (1u << 21) ? 4 : (n >= (1u << 18) ? 2 : 1); }

int64_t row_update_chunks(int64_t max_ids, int d) {
  const int C = d / 4;
  return (max_ids + C - 1) / C + 1;
}

template <int CTRL>
__device__ __forceinline__ float lane_perm(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}

template <int LPR, bool ADAM>
__device__ __forceinline__ void apply_update(float4 g, float4 hv, float Gv, uint32_t row, int c4,
                                             const EmbOpt& o) {
  constexpr int D = LPR * 4;
  float* __restrict__ h = o.h;
  if (ADAM) {
    const size_t at = (size_t)row * D + c4 * 4;
    float4 m = *(const float4*)(o.M + at), v = *(const float4*)(o.V + at);
    const float t = Gv + 1.0f;
    const float b1 = o.beta1, b2 = o.beta2;
    m.x = b1 * m.x + (1.f - b1) * g.x; m.y = b1 * m.y + (1.f - b1) * g.y;
    m.z = b1 * m.z + (1.f - b1) * g.z; m.w = b1 * m.w + (1.f - b1) * g.w;
    v.x = b2 * v.x + (1.f - b2) * g.x * g.x; v.y = b2 * v.y + (1.f - b2) * g.y * g.y;
    v.z = b2 * v.z + (1.f - b2) * g.z * g.z; v.w = b2 * v.w + (1.f - b2) * g.w * g.w;
    const float c1 = 1.f - powf(b1, t), c2 = 1.f - powf(b2, t);
    const float s1 = o.lr / c1, s2 = 1.f / sqrtf(c2);
    hv.x -= s1 * m.x / (sqrtf(v.x) * s2 + o.eps); hv.y -= s1 * m.y / (sqrtf(v.y) * s2 + o.eps);
    hv.z -= s1 * m.z / (sqrtf(v.z) * s2 + o.eps); hv.w -= s1 * m.w / (sqrtf(v.w) * s2 + o.eps);
    *(float4*)(o.M + at) = m;
    *(float4*)(o.V + at) = v;
    *(float4*)(h + at) = hv;
    if (c4 == 0) o.G[row] = t;
    return;
  }
  // sum of squares over the row's LPR lanes, every lane ending with the total: lane-permute
  // modifiers of the adds instead of LDS round trips (pairs, quads, then the mirrored half of
  // 8 and of 16 lanes -- each half already holds one value)
  float ss = g.x * g.x + g.y * g.y + g.z * g.z + g.w * g.w;
  ss += lane_perm<0xB1>(ss);                  // quad_perm [1,0,3,2]
  ss += lane_perm<0x4E>(ss);                  // quad_perm [2,3,0,1]
  if (LPR >= 8) ss += lane_perm<0x141>(ss);   // row_half_mirror
  if (LPR >= 16) ss += lane_perm<0x140>(ss);  // row_mirror
  if (LPR >= 32) ss += __shfl_xor(ss, 16);
  const float Gn = Gv + ss * (1.0f / (float)D);
  // hardware square root and reciprocal (one ulp each)
  const float scale = o.lr * __builtin_amdgcn_rcpf(__builtin_amdgcn_sqrtf(Gn) + o.eps);
  hv.x -= scale * g.x; hv.y -= scale * g.y; hv.z -= scale * g.z; hv.w -= scale * g.w;
  store_row_nt(h + (size_t)row * D + c4 * 4, hv);
  if (c4 == 0) o.G[row] = Gn;
}

template <int LPR, bool ADAM, int CHUNK_SLICES>
__global__ __launch_bounds__(256) void row_update_chunk_kernel(
    const uint32_t* __restrict__ keys, const int32_t* __restrict__ bags,
    const float* __restrict__ de, uint32_t n, EmbOpt o, float* __restrict__ parts,
    uint32_t* __restrict__ flags, uint32_t* __restrict__ long_count,
    const float* __restrict__ inv_len, int by_die) {
  const float* __restrict__ h = o.h;
  const float* __restrict__ G = o.G;
  constexpr int D = LPR * 4, C = CHUNK_SLICES * LPR, SUB = (LPR < 8 ? LPR : 8);
  if (blockIdx.x == 0 && threadIdx.x == 0) *long_count = 0;  // consumed by the later passes
  const int lane = threadIdx.x & 63, c = lane % LPR, gw = lane / LPR;
  const uint32_t nchunks = (n + C - 1) / C;
  // Workgroups go to the chip's eight dies (each with its own L2) in turn.  When the whole
  // grid is resident at once (by_die; the grid is then a multiple of 8) die x takes the x-th
  // eighth of the sorted order, so that a die works inside one or two tables (keys are
  // table-major) and its L2 holds their gradient rows de[:, t, :] and accumulators.  Larger
  // grids run in plain order: measured faster there although the die-wise order halves the
  // L2 misses (Large workload: 289 against 309 us).
  const uint32_t per_die = gridDim.x >> 3;
  const uint32_t lb = by_die ? (blockIdx.x & 7u) * per_die + (blockIdx.x >> 3) : blockIdx.x;
  const uint32_t g = lb * (256 / LPR) + threadIdx.x / LPR;
  const bool live = g < nchunks;
  const uint32_t gmask = (LPR == 32) ? 0xFFFFFFFFu : ((1u << LPR) - 1u);
  float4 acc = {0.f, 0.f, 0.f, 0.f};
  bool started = false;  // the current run began at a head inside this chunk
  bool open = false;     // the last entry seen so far did not end its run
  uint32_t fl = 0;
  float4* part0 = (float4*)(parts + ((size_t)g * 2 + 0) * D) + c;
  float4* part1 = (float4*)(parts + ((size_t)g * 2 + 1) * D) + c;
  // every slice's index work first (one entry per lane and slice; every lane of the wave
  // takes part in all ballots), so that all index loads are in flight together
  uint32_t key_s[CHUNK_SLICES], hm_s[CHUNK_SLICES], tm_s[CHUNK_SLICES];
  int bag_s[CHUNK_SLICES], nv_s[CHUNK_SLICES];
#pragma unroll
  for (int sl = 0; sl < CHUNK_SLICES; ++sl) {
    const uint32_t j = g * C + sl * LPR + c;
    const bool valid = live && j < n;
    key_s[sl] = valid ? keys[j] : 0u;
    bag_s[sl] = valid ? bags[j] : 0;
    const bool head = valid && (j == 0 || keys[j - 1] != key_s[sl]);
    const bool tail = valid && (j + 1 == n || keys[j + 1] != key_s[sl]);
    const uint64_t hb = __ballot(head), tb = __ballot(tail), vb = __ballot(valid);
    hm_s[sl] = (uint32_t)(hb >> (gw * LPR)) & gmask;
    tm_s[sl] = (uint32_t)(tb >> (gw * LPR)) & gmask;
    nv_s[sl] = __popc((uint32_t)(vb >> (gw * LPR)) & gmask);  // valid entries form a prefix
  }
  // staging registers of a sub-block: gradient rows, and the table row, accumulator and row
  // id of the entries that end a run.  Declared (and given a value) once: an entry's registers
  // are only read under the condition they were loaded under, so nothing is cleared per
  // sub-block.
  float4 v[SUB], hv[SUB];
  float Gv[SUB];
  uint32_t rw[SUB];
#pragma unroll
  for (int i = 0; i < SUB; ++i) {
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    hv[i] = v[i];
    Gv[i] = 0.f;
    rw[i] = 0;
  }
#pragma unroll
  for (int sl = 0; sl < CHUNK_SLICES; ++sl) {
    const uint32_t key = key_s[sl], hm = hm_s[sl], tm = tm_s[sl];
    const int bag = bag_s[sl], nv = nv_s[sl];
    for (int s0 = 0; s0 < nv; s0 += SUB) {
#pragma unroll
      for (int i = 0; i < SUB; ++i) {
        const int p = s0 + i;
        const int bg = __shfl(bag, p, LPR);
        if (p < nv) {
          v[i] = *(const float4*)(de + (size_t)bg * D + c * 4);
          if (inv_len) {  // mean pooling: d(mean)/d(member) = 1 / bag length
            const float sc = inv_len[bg];
            v[i].x *= sc; v[i].y *= sc; v[i].z *= sc; v[i].w *= sc;
          }
          if ((tm >> p) & 1u) {
            // (the row is only needed where a run ends; the condition is uniform over the
            // group's lanes, which is all the permute reads from)
            rw[i] = (uint32_t)__shfl((int)key, p, LPR);
            hv[i] = load_row_nt(h + (size_t)rw[i] * D + c * 4);
            Gv[i] = G[rw[i]];
          }
        }
      }
#pragma unroll
      for (int i = 0; i < SUB; ++i) {
        const int p = s0 + i;
        if (p < nv) {
          if ((hm >> p) & 1u) {
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
            started = true;
          }
          acc.x += v[i].x; acc.y += v[i].y; acc.z += v[i].z; acc.w += v[i].w;
          open = true;
          if ((tm >> p) & 1u) {
            if (started) {
              apply_update<LPR, ADAM>(acc, hv[i], Gv[i], rw[i], c, o);
            } else {
              *part0 = acc;  // end of a run that came in from the previous chunk
              fl |= 1u;
            }
            acc = make_float4(0.f, 0.f, 0.f, 0.f);
            started = false;
            open = false;
          }
        }
      }
    }
  }
  if (!live) return;
  if (open) {  // the last run goes on into the next chunk
    if (started) { *part1 = acc; fl |= 2u; }
    else { *part0 = acc; fl |= 4u; }
  }
  if (c == 0) flags[g] = fl;
}

template <int LPR, bool ADAM, int CHUNK_SLICES>
__global__ __launch_bounds__(256) void row_update_stitch_kernel(
    const uint32_t* __restrict__ keys, uint32_t n, float* __restrict__ parts,
    const uint32_t* __restrict__ flags, EmbOpt o, uint32_t* __restrict__ long_list,
    uint32_t* __restrict__ long_count) {
  const float* __restrict__ h = o.h;
  const float* __restrict__ G = o.G;
  constexpr int D = LPR * 4, C = CHUNK_SLICES * LPR, MAXB = 16;
  const int c = threadIdx.x % LPR;
  const uint32_t nchunks = (n + C - 1) / C;
  const uint32_t g = blockIdx.x * (256 / LPR) + threadIdx.x / LPR;
  if (g >= nchunks) return;
  if (!(flags[g] & 2u)) return;
  // an open run at the end of chunk g means the chunk is full: its last entry is (g+1)*C-1
  const uint32_t row = keys[(g + 1) * C - 1];
  const float4 hv = *(const float4*)(h + (size_t)row * D + c * 4);
  const float Gv = G[row];
  float4* mine = (float4*)(parts + ((size_t)g * 2 + 1) * D) + c;
  float4 acc = *mine;
  uint32_t g2 = g + 1;
  int batch = 2;
  bool done = false;
  for (int round = 0; round < 4 && !done; ++round) {  // 2 + 4 + 8 + 16 chunks
    float4 p[MAXB];
    uint32_t f[MAXB];
#pragma unroll
    for (int i = 0; i < MAXB; ++i) {
      const uint32_t gi = g2 + i;
      p[i] = make_float4(0.f, 0.f, 0.f, 0.f);
      f[i] = 1u;  // past the last chunk: treat as the end of the run
      if (i < batch && gi < nchunks) {
        f[i] = flags[gi];
        p[i] = *((const float4*)(parts + ((size_t)gi * 2 + 0) * D) + c);
      }
    }
#pragma unroll
    for (int i = 0; i < MAXB; ++i) {
      if (!done && i < batch) {
        acc.x += p[i].x; acc.y += p[i].y; acc.z += p[i].z; acc.w += p[i].w;
        if (!(f[i] & 4u)) done = true;
      }
    }
    g2 += batch;
    batch = min(MAXB, batch * 2);
  }
  if (done) {
    apply_update<LPR, ADAM>(acc, hv, Gv, row, c, o);
  } else {
    *mine = acc;  // sum so far; the long-run kernel continues from chunk g2
    if (c == 0) {
      const uint32_t slot = atomicAdd(long_count, 1u);
      long_list[2 * slot] = g;
      long_list[2 * slot + 1] = g2;
    }
  }
}

template <int LPR, bool ADAM, int CHUNK_SLICES>
__global__ __launch_bounds__(1024) void row_update_long_kernel(
    const uint32_t* __restrict__ keys, uint32_t n, const float* __restrict__ parts,
    const uint32_t* __restrict__ flags, EmbOpt o, const uint32_t* __restrict__ long_list,
    const uint32_t* __restrict__ long_count) {
  const float* __restrict__ h = o.h;
  const float* __restrict__ G = o.G;
  constexpr int D = LPR * 4, C = CHUNK_SLICES * LPR, NG = 1024 / LPR;
  __shared__ float4 red[1024];
  __shared__ uint32_t last_chunk;
  const uint32_t nchunks = (n + C - 1) / C;
  const uint32_t nlong = *long_count;
  const int c = threadIdx.x % LPR, grp = threadIdx.x / LPR;
  for (uint32_t li = blockIdx.x; li < nlong; li += gridDim.x) {
    const uint32_t g = long_list[2 * li], g2 = long_list[2 * li + 1];
    // the run's last chunk: the first one at or after g2 whose flags lack "whole chunk inside"
    if (threadIdx.x == 0) last_chunk = nchunks - 1;
    __syncthreads();
    for (uint32_t base = g2; base < nchunks; base += 1024) {
      const uint32_t gi = base + threadIdx.x;
      if (gi < nchunks && !(flags[gi] & 4u)) atomicMin(&last_chunk, gi);
      __syncthreads();
      if (last_chunk < base + 1024) break;  // block-uniform: read after the barrier
      __syncthreads();
    }
    __syncthreads();
    const uint32_t ge = last_chunk;
    float4 acc = {0.f, 0.f, 0.f, 0.f};
    {
      // four partial sums in flight per lane: the loop is bound by load latency otherwise
      float4 a4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) a4[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      for (uint32_t gi = g2 + grp; gi <= ge; gi += 4 * NG) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const uint32_t gu = gi + u * NG;
          if (gu <= ge) {
            const float4 v = *((const float4*)(parts + ((size_t)gu * 2 + 0) * D) + c);
            a4[u].x += v.x; a4[u].y += v.y; a4[u].z += v.z; a4[u].w += v.w;
          }
        }
      }
      acc.x = (a4[0].x + a4[1].x) + (a4[2].x + a4[3].x);
      acc.y = (a4[0].y + a4[1].y) + (a4[2].y + a4[3].y);
      acc.z = (a4[0].z + a4[1].z) + (a4[2].z + a4[3].z);
      acc.w = (a4[0].w + a4[1].w) + (a4[2].w + a4[3].w);
    }
    red[threadIdx.x] = acc;
    __syncthreads();
    for (int half = NG / 2; half >= 1; half >>= 1) {
      if (grp < half) {
        const float4 o = red[threadIdx.x + half * LPR];
        acc.x += o.x; acc.y += o.y; acc.z += o.z; acc.w += o.w;
        red[threadIdx.x] = acc;
      }
      __syncthreads();
    }
    if (grp == 0) {
      const float4 first = *((const float4*)(parts + ((size_t)g * 2 + 1) * D) + c);
      acc.x += first.x; acc.y += first.y; acc.z += first.z; acc.w += first.w;
      const uint32_t row = keys[(g + 1) * C - 1];
      const float4 hv = *(const float4*)(h + (size_t)row * D + c * 4);
      apply_update<LPR, ADAM>(acc, hv, G[row], row, c, o);
    }
    __syncthreads();
  }
}

void launch_row_update_chunk(const uint32_t* sorted_keys, const int32_t* sorted_bag,
                             const float* de, uint32_t n, const RowUpdateScratch& sc, int d,
                             const EmbOpt& o, const float* inv_len, hipStream_t s) {
  if (n == 0) return;
  const int lpr = d / 4, ch = chunk_slices(n), C = ch * lpr;
  const int64_t nchunks = ((int64_t)n + C - 1) / C;
  int blocks = ceil_div(nchunks, 256 / lpr);
  const int by_die = blocks <= 2048;
  if (by_die) blocks = ceil_div(blocks, 8) * 8;
#define L(LPR, A, CH)                                                                          \
  hipLaunchKernelGGL((row_update_chunk_kernel<LPR, A, CH>), dim3(blocks), dim3(256), 0, s,    \
                     sorted_keys, sorted_bag, de, n, o, sc.parts, sc.flags, sc.long_count, inv_len, by_die)
#define LC(LPR, A) do { if (ch == 4) { L(LPR, A, 4); } else if (ch == 2) { L(LPR, A, 2); } else { L(LPR, A, 1); } } while (0)
#define LA(LPR) do { if (o.adam) LC(LPR, true); else LC(LPR, false); } while (0)
  switch (d) {
    case 16: LA(4); break;
    case 32: LA(8); break;
    case 64: LA(16); break;
    default: LA(32); break;
  }
#undef LA
#undef LC
#undef L
}

void launch_row_update_finish(const uint32_t* sorted_keys, uint32_t n, const RowUpdateScratch& sc,
                              int d, const EmbOpt& o, hipStream_t s) {
  if (n == 0) return;
  const int lpr = d / 4, ch = chunk_slices(n), C = ch * lpr;
  const int64_t nchunks = ((int64_t)n + C - 1) / C;
  const int blocks = ceil_div(nchunks, 256 / lpr);
  // one block per long run; their number is only known on the device, so the grid is sized
  // for the worst case that matters (a run is long from about 30 chunks on) and capped
  const int64_t lb = nchunks / 512 + 16;
  const int long_blocks = (int)(lb > 512 ? 512 : lb);
#define L(LPR, A, CH)                                                                             \
  hipLaunchKernelGGL((row_update_stitch_kernel<LPR, A, CH>), dim3(blocks), dim3(256), 0, s,      \
                     sorted_keys, n, sc.parts, sc.flags, o, sc.long_list, sc.long_count);         \
  hipLaunchKernelGGL((row_update_long_kernel<LPR, A, CH>), dim3(long_blocks), dim3(1024), 0, s,  \
                     sorted_keys, n, sc.parts, sc.flags, o, sc.long_list, sc.long_count)
#define LC(LPR, A) do { if (ch == 4) { L(LPR, A, 4); } else if (ch == 2) { L(LPR, A, 2); } else { L(LPR, A, 1); } } while (0)
#define LA(LPR) do { if (o.adam) LC(LPR, true); else LC(LPR, false); } while (0)
  switch (d) {
    case 16: LA(4); break;
    case 32: LA(8); break;
    case 64: LA(16); break;
    default: LA(32); break;
  }
#undef LA
#undef LC
#undef L
}

}  // namespace ss
