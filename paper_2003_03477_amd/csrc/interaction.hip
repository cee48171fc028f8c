// Pairwise-dot feature interaction, forward and backward (gfx950).
// Per sample the T+1 vectors V = [z0; e_0; ...; e_{T-1}] (d floats each) are staged in LDS
// by one wavefront; the forward emits z0 followed by <V_r, V_c> for the strictly lower
// triangle in row-major order, the backward applies the product rule
// dV_r = sum_{c != r} S[r][c] V_c with S the symmetric matrix of incoming pair gradients.
// This is the "feature interaction" component between the bottom and top networks of the
// model reviewed in Section 3.1; it is bandwidth-bound work (Section 4.3 notes these ops are
// what saturates a trainer's memory bandwidth), so it stays on the vector ALUs in fp32.
#include "ss_internal.h"

namespace ss {

__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// r(r-1)/2 <= p < r(r+1)/2  ->  pair p is (r, c = p - r(r-1)/2), r >= 1
__device__ __forceinline__ void pair_of(int p, int& r, int& c) {
  int rr = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)p)) * 0.5f);
  while (rr * (rr - 1) / 2 > p) --rr;
  while (rr * (rr + 1) / 2 <= p) ++rr;
  r = rr;
  c = p - rr * (rr - 1) / 2;
}

// The sample's tile [T+1][d] (no row padding), loaded straight into LDS: every load
// instruction moves 64 x 16 bytes from per-lane global addresses to 1 KB of consecutive LDS
// (lane l's 16 bytes at byte 16 l of the chunk), no registers in between, so all of a sample's
// loads are in flight together.  The caller waits for them (vector-memory counter) before the
// tile is read.  SWZ: the 16-byte piece k of row r sits in slot k ^ (r mod d/4) of its row, for
// readers whose lanes read the same piece of different rows at once (rows are a multiple of
// the bank width apart); without it piece k is slot k (readers whose lanes share the row).
template <bool SWZ>
__device__ __forceinline__ void stage_V_direct(float* Vs, const float* __restrict__ z0,
                                               const float* __restrict__ e, int b, int T, int d,
                                               int lane) {
  const int vec_per_row = d / 4;   // a power of two
  const int total = (T + 1) * vec_per_row;
  for (int i0 = 0; i0 < total; i0 += SS_WAVE) {
    const int i = i0 + lane;
    if (i < total) {
      const int r = i / vec_per_row, slot = i - r * vec_per_row;
      const int k4 = SWZ ? (slot ^ (r & (vec_per_row - 1))) : slot;
      const float* src = (r == 0) ? (z0 + (size_t)b * d) : (e + ((size_t)b * T + (r - 1)) * d);
      __builtin_amdgcn_global_load_lds(
          (const __attribute__((address_space(1))) void*)(src + 4 * k4),
          (__attribute__((address_space(3))) void*)(Vs + 4 * i0), 16, 0, 0);
    }
  }
}

// Forward.  The Gram matrix V V^T of a sample is computed in 4x4 register blocks of its lower
// triangle: a task (rb, cb <= rb) reads rows 4 rb .. 4 rb + 3 and 4 cb .. 4 cb + 3 piece by
// piece (8 LDS reads of 16 bytes feed 64 FMAs) and is shared by KS neighbouring lanes, each
// summing a 1/KS share of the d columns; the lanes' sums are added with lane exchanges.  The
// entries below the diagonal go to an LDS copy of the output row, which the wave then writes
// out in consecutive order.  With at most 64 pairs (KS == 0) a lane computes one pair instead.
__global__ __launch_bounds__(256) void interaction_fwd_kernel(
    const float* __restrict__ z0, const float* __restrict__ e, int B, int T, int d, int KS,
    float* __restrict__ f, int ldf, uint16_t* __restrict__ f_bf16, int ldf_bf16) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int vec_per_row = d / 4, vmask = vec_per_row - 1;
  const int n1 = T + 1, n1p = (n1 + 3) & ~3;
  const int npairs = T * (T + 1) / 2;
  const int F = d + npairs;
  const int row_blocks = n1p / 4, ntasks = row_blocks * (row_blocks + 1) / 2;
  // per wave: the tile (rows n1 .. n1p-1 are never written: they only feed entries that are
  // dropped), then the pair values
  float* Vs = smem + (size_t)wave * (n1p * d + ((npairs + 3) & ~3));   // swizzled rows
  float* Fs = Vs + n1p * d;
  const int kshare = KS ? vec_per_row / KS : 0;
  for (int b0 = blockIdx.x * 4; b0 < B; b0 += gridDim.x * 4) {
    const int b = b0 + wave;
    if (b < B) stage_V_direct<true>(Vs, z0, e, b, T, d, lane);
    __builtin_amdgcn_s_waitcnt(0);   // the direct loads have landed
    __syncthreads();
    if (b < B) {
      for (int k = lane; k < d; k += SS_WAVE) {
        const float v = Vs[k];       // row 0 is not permuted
        if (f) f[(size_t)b * ldf + k] = v;
        if (f_bf16) f_bf16[(size_t)b * ldf_bf16 + k] = f32_to_bf16(v);
      }
      if (KS == 0) {
        // few pairs (at most one per lane): a lane takes a whole pair and writes it itself
        const int p = lane;
        if (p < npairs) {
          int r, c;
          pair_of(p, r, c);
          const float* vr = Vs + r * d;
          const float* vc = Vs + c * d;
          const int xr = r & vmask, xc = c & vmask;
          float4 acc = {0.f, 0.f, 0.f, 0.f};
          for (int k4 = 0; k4 < vec_per_row; ++k4) {
            const float4 x = *(const float4*)(vr + ((k4 ^ xr) << 2));
            const float4 y = *(const float4*)(vc + ((k4 ^ xc) << 2));
            acc.x += x.x * y.x; acc.y += x.y * y.y; acc.z += x.z * y.z; acc.w += x.w * y.w;
          }
          Fs[p] = (acc.x + acc.y) + (acc.z + acc.w);
        }
      }
      // (ntasks * KS <= 64, or KS == 1: the KS lanes of a task are neighbours in one round)
      for (int u0 = 0; u0 < ntasks * KS; u0 += SS_WAVE) {
        const int u = u0 + lane;
        const bool on = u < ntasks * KS;
        const int t = on ? u / KS : 0, ks = u % KS;
        int rb1, cb;
        pair_of(t, rb1, cb);         // t = rb (rb + 1) / 2 + cb with rb = rb1 - 1 >= cb
        const int r0 = (rb1 - 1) * 4, c0 = cb * 4;
        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
        if (on) {
          for (int k4 = ks * kshare; k4 < (ks + 1) * kshare; ++k4) {
            float4 x[4], y[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              x[i] = *(const float4*)(Vs + (r0 + i) * d + ((k4 ^ ((r0 + i) & vmask)) << 2));
              y[i] = *(const float4*)(Vs + (c0 + i) * d + ((k4 ^ ((c0 + i) & vmask)) << 2));
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
              for (int j = 0; j < 4; ++j)
                acc[i][j] += (x[i].x * y[j].x + x[i].y * y[j].y) + (x[i].z * y[j].z + x[i].w * y[j].w);
          }
        }
        for (int m = 1; m < KS; m <<= 1) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[i][j] += __shfl_xor(acc[i][j], m);
        }
        if (on && ks == 0) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
              const int r = r0 + i, c = c0 + j;
              if (r < n1 && c < r) Fs[r * (r - 1) / 2 + c] = acc[i][j];
            }
        }
      }
    }
    __syncthreads();   // (a wave reads what its own lanes wrote; the barrier is for the compiler)
    if (b < B) {
      for (int p = lane; p < npairs; p += SS_WAVE) {
        const float dot = Fs[p];
        if (f) f[(size_t)b * ldf + d + p] = dot;
        if (f_bf16) f_bf16[(size_t)b * ldf_bf16 + d + p] = f32_to_bf16(dot);
      }
      if (f_bf16)
        for (int k = F + lane; k < ldf_bf16; k += SS_WAVE) f_bf16[(size_t)b * ldf_bf16 + k] = 0;
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(256) void interaction_bwd_kernel(
    const float* __restrict__ z0, const float* __restrict__ e, const float* __restrict__ df,
    int lddf, int B, int T, int d, float* __restrict__ dz0, float* __restrict__ de,
    uint16_t* __restrict__ dz0_bf16, int ld16) {
  extern __shared__ float smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int ld = d;                // no row padding: all lanes of a wave read the same row of V
  const int n1 = T + 1;
  const int n1p = (n1 + 3) & ~3;   // pitch of S: a lane reads four neighbouring entries at once
  float* Vs = smem + (size_t)wave * (n1 * ld + n1 * n1p);  // float4-aligned regions
  float* Ss = Vs + n1 * ld;
  const int npairs = T * (T + 1) / 2;
  const int vec_per_row = d / 4;
  const int row_blocks = n1p / 4;
  for (int b0 = blockIdx.x * 4; b0 < B; b0 += gridDim.x * 4) {
    const int b = b0 + wave;
    if (b < B) {
      stage_V_direct<false>(Vs, z0, e, b, T, d, lane);
      // S is symmetric with a zero diagonal; the pitch padding (rows n1 .. n1p-1 of a column)
      // only feeds output rows that do not exist
      for (int i = lane; i < n1; i += SS_WAVE) Ss[i * n1p + i] = 0.f;
      for (int p = lane; p < npairs; p += SS_WAVE) {
        int r, c;
        pair_of(p, r, c);
        const float s = df[(size_t)b * lddf + d + p];
        Ss[r * n1p + c] = s;
        Ss[c * n1p + r] = s;
      }
    }
    __builtin_amdgcn_s_waitcnt(0);   // the direct loads into Vs have landed
    __syncthreads();
    if (b < B) {
      // a lane owns four output rows r0..r0+3 and four columns 4 k4..4 k4+3: per source row c
      // one 16-byte read of S[c][r0..r0+3] (= S[r0..r0+3][c]) and one of V[c] feed 16 FMAs
      for (int i = lane; i < row_blocks * vec_per_row; i += SS_WAVE) {
        const int rb = i / vec_per_row, k4 = i - rb * vec_per_row;
        const int r0 = rb * 4;
        float4 acc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int c = 0; c < n1; ++c) {
          const float4 s4 = *(const float4*)(Ss + c * n1p + r0);
          const float4 v = *(const float4*)(Vs + c * ld + 4 * k4);
          const float sj[4] = {s4.x, s4.y, s4.z, s4.w};
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            acc[j].x += sj[j] * v.x; acc[j].y += sj[j] * v.y;
            acc[j].z += sj[j] * v.z; acc[j].w += sj[j] * v.w;
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int r = r0 + j;
          if (r >= n1) continue;
          if (r == 0) {
            const float4 pass = *(const float4*)(df + (size_t)b * lddf + 4 * k4);
            const float4 z = *(const float4*)(Vs + 4 * k4);
            float4 o;  // gradient w.r.t. the bottom MLP's last pre-activation: ReLU gate
            o.x = z.x > 0.f ? acc[j].x + pass.x : 0.f;
            o.y = z.y > 0.f ? acc[j].y + pass.y : 0.f;
            o.z = z.z > 0.f ? acc[j].z + pass.z : 0.f;
            o.w = z.w > 0.f ? acc[j].w + pass.w : 0.f;
            *(float4*)(dz0 + (size_t)b * d + 4 * k4) = o;
            if (dz0_bf16) {  // the same values as the bottom stack's bf16 GEMM operand
              uint16_t* q = dz0_bf16 + (size_t)b * ld16 + 4 * k4;
              *(uint2*)q = make_uint2((uint32_t)f32_to_bf16(o.x) | ((uint32_t)f32_to_bf16(o.y) << 16),
                                      (uint32_t)f32_to_bf16(o.z) | ((uint32_t)f32_to_bf16(o.w) << 16));
            }
          } else {
            *(float4*)(de + ((size_t)b * T + (r - 1)) * d + 4 * k4) = acc[j];
          }
        }
      }
      if (dz0_bf16)   // zero padding of the operand row
        for (int k = d + lane; k < ld16; k += SS_WAVE) dz0_bf16[(size_t)b * ld16 + k] = 0;
    }
    __syncthreads();
  }
}

void launch_interaction_fwd(const float* z0, const float* e, int B, int T, int d, float* f,
                            int ldf, uint16_t* f_bf16, int ldf_bf16, hipStream_t s) {
  if (B == 0) return;
  const int n1p = (T + 1 + 3) & ~3, npairs = T * (T + 1) / 2;
  const size_t shm = (size_t)4 * (n1p * d + ((npairs + 3) & ~3)) * sizeof(float);
  // lanes that share a block of the Gram matrix: as many as keep all tasks in one round
  const int rbk = n1p / 4, ntasks = rbk * (rbk + 1) / 2;
  int KS = 1;
  while (ntasks * KS * 2 <= SS_WAVE && KS * 2 <= d / 4) KS *= 2;
  if (npairs <= SS_WAVE) KS = 0;   // one pair per lane is cheaper than sharing blocks
  int blocks = ceil_div(B, 4);
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(interaction_fwd_kernel, dim3(blocks), dim3(256), shm, s, z0, e, B, T, d, KS,
                     f, ldf, f_bf16, ldf_bf16);
}

void launch_interaction_bwd(const float* z0, const float* e, const float* df, int lddf, int B,
                            int T, int d, float* dz0, float* de, uint16_t* dz0_bf16, int ld16,
                            hipStream_t s) {
  if (B == 0) return;
  const int n1 = T + 1;
  const int n1p = (n1 + 3) & ~3;
  const size_t shm = (size_t)4 * (n1 * d + n1 * n1p) * sizeof(float);
  int blocks = ceil_div(B, 4);
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(interaction_bwd_kernel, dim3(blocks), dim3(256), shm, s, z0, e, df, lddf, B,
                     T, d, dz0, de, dz0_bf16, ld16);
}

}  // namespace ss
