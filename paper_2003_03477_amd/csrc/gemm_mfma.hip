// bf16 MFMA GEMMs of the layer-wise MLP path (gfx950 / CDNA4, wave64, v_mfma_f32_32x32x16_bf16,
// fp32 accumulation).  Activations and activation gradients live in HBM as plain row-major
// bf16 matrices [sample][unit]; the step's weights are a bf16 snapshot laid out in MFMA
// fragment order (see mlp_fused.hip: for every (32-unit tile, 16-deep reduction step) the 64
// lanes' 8 values are contiguous), once for X W^T and once for dY W.
//
//   gemm_xw_kernel      forward  Y = act(X W^T + b)  and data gradient  dX = gate(dY W):
//                       the activation operand is staged through LDS, the weight operand comes
//                       straight from the fragment-ordered copy as coalesced 1 KB wave loads
//                       (L2-resident, 8 reduction steps in flight), so LDS carries one operand
//                       only.  Block = 2x2 waves, tile 128x128 (wave tile 64x64), two blocks per
//                       CU (256x128 tiles with one block per CU measured 12 % slower on
//                       8192x1024x1024).  The MFMA operands are swapped (the accumulator then
//                       holds four consecutive output units of one sample per lane); results
//                       are laid out in LDS and stored as 16-byte vectors of contiguous rows.
//   gemm_wgrad_kernel   weight gradients  dW = dY^T X  (+ bias gradients as an MFMA against
//                       ones) of ALL layers in one grouped launch over (layer, tile, batch
//                       slice).  Both operands are read row-major and transposed on their way
//                       into LDS (4 samples x 8 units per thread, byte permutes, 8-byte LDS
//                       stores), so no transposed copy of any activation exists in HBM.  Every
//                       slice stores its partial sums; reduce_slices_kernel adds them up.
//
// LDS operand tiles are [rows][64] bf16 with 128-byte rows and no padding; the 16-byte chunk c
// of row r sits at chunk c ^ ((r ^ (r >> 3)) & 7), which spreads both the 16-byte fragment
// reads (32 consecutive rows, one chunk) and the 8-byte transposing stores (rows 8 apart) over
// the banks.
#include <mutex>

#include "ss_internal.h"

namespace ss {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

namespace {

constexpr int TK = 64;        // reduction step
constexpr int CP = 128 + 8;   // LDS row pitch of a bf16 output tile (elements)
constexpr int CPF = 128 + 4;  // LDS row pitch of an fp32 output tile (floats)

union Frag {
  bf16x8 v;
  u32x4 q;
};

__device__ __forceinline__ uint16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
__device__ __forceinline__ uint32_t pk2(float lo, float hi) {
  return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}
__device__ __forceinline__ int swz(int r) { return (r ^ (r >> 3)) & 7; }
// element offset of 16-byte chunk c of row r inside an operand tile
__device__ __forceinline__ int tile_off(int r, int c) { return r * TK + ((c ^ swz(r)) << 3); }

__device__ __forceinline__ uint4 gate8(uint4 x, uint4 m) {
  const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ms[4] = {m.x, m.y, m.z, m.w};
  uint32_t o[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = ((int16_t)(ms[i] & 0xFFFFu) > 0) ? 0x0000FFFFu : 0u;
    const uint32_t hi = ((int16_t)(ms[i] >> 16) > 0) ? 0xFFFF0000u : 0u;
    o[i] = xs[i] & (lo | hi);
  }
  return make_uint4(o[0], o[1], o[2], o[3]);
}
// zero the elements j >= valid (0..8) of a vector of 8 bf16
__device__ __forceinline__ uint4 keep_first(uint4 x, int valid) {
  if (valid >= 8) return x;
  uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t lo = (2 * i < valid) ? 0x0000FFFFu : 0u;
    const uint32_t hi = (2 * i + 1 < valid) ? 0xFFFF0000u : 0u;
    w[i] &= (lo | hi);
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// ------------------------------------------------------------------------------------------
struct XwDev {
  const uint16_t* A; int lda;       // [M][lda] bf16, K (multiple of 64) finite columns
  const uint16_t* Bf;               // fragment-ordered weights: tile = n / 32, step = k / 16
  int M, N, K;
  int n_tiles32;                    // 32-unit tiles in Bf (N rounded up to 32, / 32)
  uint16_t* C; int ldc;             // bf16 [M][ldc], columns N..ldc-1 zeroed
  float* C32; int ldc32;            // or fp32 [M][ldc32]
  int epi; const float* bias;
  const uint16_t* mask; int ldmask; // [M][ldmask]: keep C(m,n) where mask > 0 (EPI_MASK)
  int tiles_m, tiles_n;
  int stream_out;                   // bf16 output stored non-temporally
};

// (ROLE: 0 = a layer's forward product, 1 = a data gradient.  Same code; the two get their
// own names in a profiler's kernel list, as they have their own classes in the event timing.)
template <int ROLE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_xw_kernel(XwDev g) {
  constexpr int BM = 128;
  constexpr int MT = BM / 64;   // 32-row tiles per wave along M
  constexpr int NA = BM / 32;   // 16-byte pieces of the A tile per thread and step
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  uint16_t* const As0 = smem;
  uint16_t* const As1 = smem + BM * TK;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  // consecutive tiles (same rows of A) go to the same XCD, whose L2 then serves the re-reads
  const int total = g.tiles_m * g.tiles_n;
  int id = blockIdx.x;
  if ((total & 7) == 0) id = (id & 7) * (total >> 3) + (id >> 3);
  const int tm = id / g.tiles_n, tn = id - tm * g.tiles_n;
  const int m0 = tm * BM, n0 = tn * 128;
  const int nk = g.K / TK;          // >= 1
  const int steps16 = nk * 4;

  // activation operand: piece i of this thread = row (tid/8 + 32 i), chunk tid%8
  const int lrow = tid >> 3, lch = tid & 7;
  const uint16_t* aptr[NA];
  int lds_a[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int r = lrow + 32 * i;
    aptr[i] = g.A + (size_t)min(m0 + r, g.M - 1) * g.lda + lch * 8;
    lds_a[i] = tile_off(r, lch);
  }
  // weight operand: this wave's two 32-unit tiles (clamped; results of tiles beyond N are
  // dropped at the store)
  const uint16_t* bptr[2];
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int t = min((n0 >> 5) + wn * 2 + j, g.n_tiles32 - 1);
    bptr[j] = g.Bf + ((size_t)t * steps16 * 64 + lane) * 8;
  }
  auto load_b = [&](Frag (&dst)[2], int step16) {
    const int s = min(step16, steps16 - 1);   // past the end: a harmless re-read
#pragma unroll
    for (int j = 0; j < 2; ++j) dst[j].q = *(const u32x4*)(bptr[j] + (size_t)s * 512);
  };

  // Accumulators with the MFMA operands swapped: rows = output units, columns = samples, so a
  // lane holds four consecutive units of one sample per group of four elements.
  f32x16 acc[MT][2];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  u32x4 ra0[NA], ra1[NA];   // two register stages of the activation tile
  auto fetch = [&](u32x4 (&r)[NA], int step) {
    const int ko = min(step, nk - 1) * TK;
#pragma unroll
    for (int i = 0; i < NA; ++i) r[i] = *(const u32x4*)(aptr[i] + ko);
  };
  auto stash = [&](const u32x4 (&r)[NA], uint16_t* as) {
#pragma unroll
    for (int i = 0; i < NA; ++i) *(u32x4*)(as + lds_a[i]) = r[i];
  };

  Frag bq[8][2];            // weight fragments of the next 8 reduction steps of 16
#pragma unroll
  for (int d = 0; d < 8; ++d) load_b(bq[d], d);

  const int frow = lane & 31, fh = lane >> 5;
  int arow[MT];
#pragma unroll
  for (int i = 0; i < MT; ++i) arow[i] = wm * (BM / 2) + i * 32 + frow;

  // one reduction step of 64 on LDS buffer `as`; H = which half of the weight ring it uses;
  // base16 = index of its first step of 16 (the ring slot is refilled with step + 8)
  auto compute = [&](const uint16_t* as, auto H, int base16) {
    constexpr int h = decltype(H)::value;
    Frag a[2][MT];
#pragma unroll
    for (int i = 0; i < MT; ++i) a[0][i].q = *(const u32x4*)(as + tile_off(arow[i], fh));
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int cur = q & 1, nxt = cur ^ 1;
      if (q + 1 < 4) {
#pragma unroll
        for (int i = 0; i < MT; ++i)
          a[nxt][i].q = *(const u32x4*)(as + tile_off(arow[i], 2 * (q + 1) + fh));
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bq[4 * h + q][j].v, a[cur][i].v, acc[i][j], 0, 0, 0);
      load_b(bq[4 * h + q], base16 + q + 8);
    }
  };
  using H0 = std::integral_constant<int, 0>;
  using H1 = std::integral_constant<int, 1>;

  fetch(ra0, 0);
  fetch(ra1, 1);
  stash(ra0, As0);
  fetch(ra0, 2);
  __syncthreads();
  int it = 0;
  for (; it + 2 < nk; it += 2) {
    compute(As0, H0{}, it * 4);
    stash(ra1, As1);
    fetch(ra1, it + 3);
    __syncthreads();
    compute(As1, H1{}, it * 4 + 4);
    stash(ra0, As0);
    fetch(ra0, it + 4);
    __syncthreads();
  }
  // the bias of this lane's 2 x 16 output units is requested ahead of the last step(s), whose
  // MFMAs cover the latency
  const int l31 = lane & 31, l4 = (lane >> 5) * 4;
  float bv[2][4][4];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int eg = 0; eg < 4; ++eg)
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int gn = n0 + wn * 64 + j * 32 + eg * 8 + l4 + u;
        bv[j][eg][u] = ((g.epi & EPI_BIAS) && gn < g.N) ? g.bias[gn] : 0.f;
      }
  compute(As0, H0{}, it * 4);   // one or two steps are left
  if (it + 1 < nk) {
    stash(ra1, As1);
    __syncthreads();
    compute(As1, H1{}, it * 4 + 4);
  }

  // Epilogue.  Element e of an accumulator = unit (e/4)*8 + (lane/32)*4 + e%4 of its 32-unit
  // tile, sample = lane%32.  The tile is laid out in LDS ([sample][unit], bf16 or fp32), then
  // every thread stores 16-byte vectors of contiguous rows.
  __syncthreads();   // every wave is done reading the operand buffers
  const bool gated = (g.epi & EPI_MASK) != 0;
  const int oc = (tid & 15) * 8;          // bf16 output: this thread's 8 units of rows tid/16 + 16 q
  uint4 mk[BM / 16];
  if (gated) {                            // the gate's activations, requested before the LDS pass
#pragma unroll
    for (int q = 0; q < BM / 16; ++q) {
      const int gm = m0 + (tid >> 4) + 16 * q, gn = n0 + oc;
      mk[q] = (gm < g.M && gn < g.ldc) ? *(const uint4*)(g.mask + (size_t)gm * g.ldmask + gn)
                                        : make_uint4(0, 0, 0, 0);
    }
  }
  if (g.C32 == nullptr) {
    uint16_t* const Cs = smem;   // [BM][CP]
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int eg = 0; eg < 4; ++eg) {
        const int nl = wn * 64 + j * 32 + eg * 8 + l4;   // first of four units (tile-local)
#pragma unroll
        for (int i = 0; i < MT; ++i) {
          const int ml = wm * (BM / 2) + i * 32 + l31;
          float v[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            v[u] = acc[i][j][eg * 4 + u] + bv[j][eg][u];
            if (g.epi & EPI_RELU) v[u] = fmaxf(v[u], 0.f);
          }
          *(uint2*)(Cs + ml * CP + nl) = make_uint2(pk2(v[0], v[1]), pk2(v[2], v[3]));
        }
      }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < BM / 16; ++q) {
      const int r = (tid >> 4) + 16 * q;
      const int gm = m0 + r, gn = n0 + oc;
      if (gm < g.M && gn < g.ldc) {
        uint4 x = *(const uint4*)(Cs + r * CP + oc);
        if (gated) x = gate8(x, mk[q]);
        x = keep_first(x, g.N - gn);
        uint16_t* dst = g.C + (size_t)gm * g.ldc + gn;
        if (g.stream_out) {   // large outputs bypass the L2 (the reader is a later kernel)
          __builtin_nontemporal_store(x.x, (uint32_t*)dst);
          __builtin_nontemporal_store(x.y, (uint32_t*)dst + 1);
          __builtin_nontemporal_store(x.z, (uint32_t*)dst + 2);
          __builtin_nontemporal_store(x.w, (uint32_t*)dst + 3);
        } else {
          *(uint4*)dst = x;
        }
      }
    }
    return;
  }
  // fp32 output (bottom output z0, gradient w.r.t. the interaction output)
  float* const Cf = (float*)smem;   // [BM][CPF]
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int eg = 0; eg < 4; ++eg) {
      const int nl = wn * 64 + j * 32 + eg * 8 + l4;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int ml = wm * (BM / 2) + i * 32 + l31;
        float4 v;
        v.x = acc[i][j][eg * 4 + 0] + bv[j][eg][0]; v.y = acc[i][j][eg * 4 + 1] + bv[j][eg][1];
        v.z = acc[i][j][eg * 4 + 2] + bv[j][eg][2]; v.w = acc[i][j][eg * 4 + 3] + bv[j][eg][3];
        if (g.epi & EPI_RELU) { v.x = fmaxf(v.x, 0.f); v.y = fmaxf(v.y, 0.f); v.z = fmaxf(v.z, 0.f); v.w = fmaxf(v.w, 0.f); }
        *(float4*)(Cf + ml * CPF + nl) = v;
      }
    }
  __syncthreads();
  const bool vec = ((g.ldc32 & 3) == 0) && ((((uintptr_t)g.C32) & 15) == 0);
#pragma unroll
  for (int q = 0; q < BM / 8; ++q) {
    const int r = (tid >> 5) + 8 * q, c = (tid & 31) * 4;   // 32 threads x 4 floats per row
    const int gm = m0 + r, gn = n0 + c;
    if (gm >= g.M || gn >= g.N) continue;
    const float4 v = *(const float4*)(Cf + r * CPF + c);
    float* dst = g.C32 + (size_t)gm * g.ldc32 + gn;
    if (vec && gn + 4 <= g.N) {
      *(float4*)dst = v;
    } else {
      const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (gn + u < g.N) dst[u] = e[u];
    }
  }
}

// ------------------------------------------------------------------------------------------
// Weight gradients, grouped.
__device__ __forceinline__ uint32_t perm_lo(uint32_t a, uint32_t b) {  // (a.lo16, b.lo16)
  return __builtin_amdgcn_perm(b, a, 0x05040100u);
}
__device__ __forceinline__ uint32_t perm_hi(uint32_t a, uint32_t b) {  // (a.hi16, b.hi16)
  return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

// one register stage: four 16-byte rows (4 consecutive samples, 8 units) of each operand
struct WgStage {
  u32x4 a[4], b[4];
};

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void gemm_wgrad_kernel(WgradGroupArgs g) {
  extern __shared__ __attribute__((aligned(16))) uint16_t smem[];
  constexpr int OP = 128 * TK;
  uint16_t* const As0 = smem;
  uint16_t* const As1 = smem + OP;
  uint16_t* const Bs0 = smem + 2 * OP;
  uint16_t* const Bs1 = smem + 3 * OP;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int id = blockIdx.x;
  if ((g.n_tiles & 7) == 0) id = (id & 7) * (g.n_tiles >> 3) + (id >> 3);
  const int4 t = g.tiles[id];               // (layer, first unit of dY, first unit of X, slice)
  if (t.x < 0) return;                      // padding entry
  const WgradGroupLayer L = g.L[t.x];
  const int m0 = t.y, n0 = t.z;
  const int bbeg = t.w * L.slice_len;
  const int bend = min(g.B, bbeg + L.slice_len);
  const int nk = (bend - bbeg + TK - 1) / TK;
  if (nk <= 0) return;                      // (an empty slice still owns a zeroed partial: see host)

  // staging: thread = (unit chunk of 8: tid%16, sample group of 4: tid/16)
  const int cidx = tid & 15, qq = tid >> 4;
  const int ca = m0 + cidx * 8, cb = n0 + cidx * 8;
  const bool a_ok = ca < L.ldy, b_ok = cb < L.ldx;      // inside the row pitch (padding is zero)
  const uint16_t* const ap = L.dY + ca;
  const uint16_t* const bp = L.X + cb;
  auto fetch = [&](WgStage& s, int step) {
    const int b0 = bbeg + min(step, nk - 1) * TK + qq * 4;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int b = b0 + i;
      const bool ok = b < bend;
      const u32x4 z = {0u, 0u, 0u, 0u};
      s.a[i] = (ok && a_ok) ? *(const u32x4*)(ap + (size_t)b * L.ldy) : z;
      s.b[i] = (ok && b_ok) ? *(const u32x4*)(bp + (size_t)b * L.ldx) : z;
    }
  };
  // transposed store of a 4 (samples) x 8 (units) micro-tile: unit row 8*cidx + j receives the
  // four samples 4*qq .. 4*qq+3 as one 8-byte store
  int st_off[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) st_off[j] = tile_off(cidx * 8 + j, qq >> 1) + (qq & 1) * 4;
  auto stash_one = [&](const u32x4 (&r)[4], uint16_t* dst) {
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t x0 = r[0][w], x1 = r[1][w], x2 = r[2][w], x3 = r[3][w];
      *(uint2*)(dst + st_off[2 * w]) = make_uint2(perm_lo(x0, x1), perm_lo(x2, x3));
      *(uint2*)(dst + st_off[2 * w + 1]) = make_uint2(perm_hi(x0, x1), perm_hi(x2, x3));
    }
  };
  auto stash = [&](const WgStage& s, uint16_t* as, uint16_t* bs) {
    stash_one(s.a, as);
    stash_one(s.b, bs);
  };

  const bool do_bias = (n0 == 0 && wn == 0);
  f32x16 acc[2][2], accb[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) accb[i][e] = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }
  bf16x8 ones;
#pragma unroll
  for (int e = 0; e < 8; ++e) ones[e] = (__bf16)1.0f;

  const int frow = lane & 31, fh = lane >> 5;
  int arow[2], brow[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    arow[i] = wm * 64 + i * 32 + frow;
    brow[i] = wn * 64 + i * 32 + frow;
  }
  auto compute = [&](const uint16_t* as, const uint16_t* bs) {
    Frag a[2][2], b[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a[0][i].q = *(const u32x4*)(as + tile_off(arow[i], fh));
      b[0][i].q = *(const u32x4*)(bs + tile_off(brow[i], fh));
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int cur = q & 1, nxt = cur ^ 1;
      if (q + 1 < 4) {
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          a[nxt][i].q = *(const u32x4*)(as + tile_off(arow[i], 2 * (q + 1) + fh));
          b[nxt][i].q = *(const u32x4*)(bs + tile_off(brow[i], 2 * (q + 1) + fh));
        }
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i].v, b[cur][j].v, acc[i][j], 0, 0, 0);
      if (do_bias) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
          accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][i].v, ones, accb[i], 0, 0, 0);
      }
    }
  };

  WgStage s0, s1;
  fetch(s0, 0);
  fetch(s1, 1);
  stash(s0, As0, Bs0);
  fetch(s0, 2);
  __syncthreads();
  int it = 0;
  for (; it + 2 < nk; it += 2) {
    compute(As0, Bs0);
    stash(s1, As1, Bs1);
    fetch(s1, it + 3);
    __syncthreads();
    compute(As1, Bs1);
    stash(s0, As0, Bs0);
    fetch(s0, it + 4);
    __syncthreads();
  }
  compute(As0, Bs0);
  if (it + 1 < nk) {
    stash(s1, As1, Bs1);
    __syncthreads();
    compute(As1, Bs1);
  }
  // NOTE: steps past the end re-stage the last tile but are never computed on.

  // this slice's partial sums: [out][in] followed by [out] bias sums
  float* const out = L.part + (size_t)t.w * L.part_stride;
  const int l31 = lane & 31, l4 = (lane >> 5) * 4;
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int gn = n0 + wn * 64 + j * 32 + l31;
      if (gn >= L.in) continue;
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gm = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + l4 + (e & 3);
        if (gm < L.out) out[(size_t)gm * L.in + gn] = acc[i][j][e];
      }
    }
    if (do_bias && l31 == 0) {
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int gm = m0 + wm * 64 + i * 32 + (e >> 2) * 8 + l4 + (e & 3);
        if (gm < L.out) out[(size_t)L.out * L.in + gm] = accb[i][e];
      }
    }
  }
}

// out[i] = sum over the slices of part[z * stride + i] (and the SGD step on w); 1024 elements
// per block; the block after the last segment's feeds the metrics accumulators
__global__ __launch_bounds__(256) void reduce_slices_kernel(ReduceArgs a, int total_blocks) {
  if ((int)blockIdx.x == total_blocks) {
    metrics_block(a.mean_loss, a.y, a.B, a.acc);
    return;
  }
  int k = 0;
  while (k + 1 < a.n_seg && (int)blockIdx.x >= a.seg[k + 1].block_base) ++k;
  const ReduceSegment sg = a.seg[k];
  const int64_t base = (int64_t)(blockIdx.x - sg.block_base) * 1024;
  const bool vec = ((sg.n & 3) == 0) && ((sg.stride & 3) == 0) && ((((uintptr_t)sg.out) & 15) == 0) &&
                   ((((uintptr_t)sg.part) & 15) == 0) && ((((uintptr_t)sg.w) & 15) == 0);
  if (vec) {
    const int64_t i = base + threadIdx.x * 4;
    if (i >= sg.n) return;
    // the replica's element and up to eight slices' partial sums are requested together; the
    // slices are added in ascending order all the same
    float4 wv = make_float4(0.f, 0.f, 0.f, 0.f);
    if (sg.w) wv = *(const float4*)(sg.w + i);
    float4 acc = *(const float4*)(sg.part + i);
    for (int z0 = 1; z0 < sg.slices; z0 += 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (z0 + u < sg.slices) v[u] = *(const float4*)(sg.part + (int64_t)(z0 + u) * sg.stride + i);
#pragma unroll
      for (int u = 0; u < 8; ++u)
        if (z0 + u < sg.slices) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    *(float4*)(sg.out + i) = acc;
    if (sg.w) {
      wv.x -= a.lr * acc.x; wv.y -= a.lr * acc.y; wv.z -= a.lr * acc.z; wv.w -= a.lr * acc.w;
      *(float4*)(sg.w + i) = wv;
    }
  } else {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int64_t i = base + threadIdx.x + 256 * u;
      if (i < sg.n) {
        float acc = sg.part[i];
        for (int z0 = 1; z0 < sg.slices; z0 += 8) {
          float v[8];
#pragma unroll
          for (int q = 0; q < 8; ++q)
            if (z0 + q < sg.slices) v[q] = sg.part[(int64_t)(z0 + q) * sg.stride + i];
#pragma unroll
          for (int q = 0; q < 8; ++q)
            if (z0 + q < sg.slices) acc += v[q];
        }
        sg.out[i] = acc;
        if (sg.w) sg.w[i] -= a.lr * acc;
      }
    }
  }
}

}  // namespace

void launch_reduce_slices(const ReduceArgs& a, int total_blocks, hipStream_t s) {
  if (total_blocks > 0)
    hipLaunchKernelGGL(reduce_slices_kernel, dim3(total_blocks + (a.acc ? 1 : 0)), dim3(256), 0, s,
                       a, total_blocks);
}

void launch_gemm_xw(const GemmXwArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0 || a.K <= 0) return;
  // operand double buffer (2 x 16 KB), reused by the output tile: bf16 [128][136] or fp32 [128][132]
  constexpr size_t LDS = (size_t)128 * CPF * 4;
  static_assert(LDS >= (size_t)2 * 128 * TK * 2 && LDS >= (size_t)128 * CP * 2, "output tile must cover the buffers");
  static std::once_flag attr_once;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute((const void*)gemm_xw_kernel<0>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)LDS);
    (void)hipFuncSetAttribute((const void*)gemm_xw_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                              (int)LDS);
  });
  XwDev g;
  g.A = a.A; g.lda = a.lda; g.Bf = a.Bf; g.M = a.M; g.N = a.N; g.K = a.K;
  g.n_tiles32 = (a.N + 31) / 32;
  g.C = a.C; g.ldc = a.ldc; g.C32 = a.C_f32; g.ldc32 = a.ldc32;
  g.epi = a.epi; g.bias = a.bias; g.mask = a.mask; g.ldmask = a.ldmask;
  g.tiles_n = ceil_div(a.N, 128);
  g.tiles_m = ceil_div(a.M, 128);
  g.stream_out = ((int64_t)a.M * a.N * 2 >= (8ll << 20)) ? 1 : 0;
  // a launch with the bf16 output asks for half the LDS of an fp32 one: four of its
  // workgroups fit a CU beside other streams' kernels instead of two
  constexpr size_t LDS_BF16 = (size_t)128 * CP * 2;
  static_assert(LDS_BF16 >= (size_t)2 * 128 * TK * 2, "bf16 output tile must cover the buffers");
  if (a.role == 0)
    hipLaunchKernelGGL(gemm_xw_kernel<0>, dim3(g.tiles_m * g.tiles_n), dim3(256),
                       a.C_f32 ? LDS : LDS_BF16, s, g);
  else
    hipLaunchKernelGGL(gemm_xw_kernel<1>, dim3(g.tiles_m * g.tiles_n), dim3(256),
                       a.C_f32 ? LDS : LDS_BF16, s, g);
}

void launch_gemm_wgrad(const WgradGroupArgs& a, hipStream_t s) {
  if (a.n_tiles <= 0) return;
  constexpr size_t LDS = (size_t)4 * 128 * TK * 2;
  static std::once_flag attr_once;
  std::call_once(attr_once, [] {
    (void)hipFuncSetAttribute((const void*)gemm_wgrad_kernel,
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
  });
  hipLaunchKernelGGL(gemm_wgrad_kernel, dim3(a.n_tiles), dim3(256), LDS, s, a);
}

}  // namespace ss
