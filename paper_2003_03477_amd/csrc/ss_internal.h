// Internal declarations shared by the HIP translation units of libshadowsync (gfx950).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define SS_MAX_TABLES 64
#define SS_WAVE 64

namespace ss {

// First global row of every table; passed to kernels by value (kernarg memory).
struct TableMeta {
  uint32_t row_base[SS_MAX_TABLES + 1];
};

static inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---------------------------------------------------------------------------- init.hip
void launch_table_hash_init(float* h, uint64_t n_elems, uint64_t seed, int table,
                            hipStream_t s);
void launch_fill_f32(float* p, uint64_t n, float v, hipStream_t s);
void launch_fill_u32(uint32_t* p, uint64_t n, uint32_t v, hipStream_t s);

// ---------------------------------------------------------------------------- embedding.hip
// Sum-pooled gather: e[b,t,:] = sum_j h[row_base[t] + indices[j], :].  Also records, for the
// backward pass, the sort key (global row) and the pooled-vector index b*T+t of every flat
// position.
// n_shards > 1: every table is split into n_shards equal row ranges, each range pools the rows
// it owns into e_part[shard][b*T+t][d] and a second launch adds the partial results in shard
// order into e (partial pooling).
// Where the gather leaves the plan of the backward pass's sort (all null / zero: no plan):
// seg_lo[t] = first position of table t (seg_lo[T] = number of ids), tile_base[t] = tiles of
// `tile` elements before table t.
struct SortPlanOut {
  uint32_t* seg_lo;
  uint32_t* tile_base;
  uint32_t tile;
};
void launch_embedding_bag_fwd(const float* h, const int32_t* indices, const int32_t* offsets,
                              const TableMeta& meta, int B, int T, int d, float* e,
                              uint32_t* keys, int32_t* bag_of_pos, float* zero_scalar,
                              float* inv_len, int n_shards, float* e_part, const SortPlanOut& plan, hipStream_t s);

struct SegScratch {
  uint32_t* block_counts;  // [seg_blocks]
  uint32_t* seg_starts;    // [max_ids + 1]
  uint32_t* num_unique;    // [1]
};
// Heads of runs of equal keys in a sorted key array -> compacted start offsets.
void launch_segment_starts(const uint32_t* sorted_keys, uint32_t n, const SegScratch& sc,
                           hipStream_t s);
// ---------------------------------------------------------------------------- row_update.hip
struct RowUpdateScratch {
  float* parts;     // [row_update_chunks(max_ids, d) * 2 * d] partial sums of runs cut by chunks
  uint32_t* flags;  // [row_update_chunks(max_ids, d)]
  uint32_t* long_list;   // [2 * (row_update_chunks(max_ids, d) / 30 + 2)] (first, next) chunk pairs
  uint32_t* long_count;  // [1]
};
int64_t row_update_chunks(int64_t max_ids, int d);
// Table optimiser of the row update: h and its state beside the rows.  adam = 0: row-wise
// Adagrad, G = one accumulator per row.  adam = 1: Adam, M / V = first / second moments per
// element, G = the row's own step count.
struct EmbOpt {
  float* h; float* G; float* M; float* V;
  float lr, eps, beta1, beta2;
  int adam;
};
// Per distinct row: g = sum of de over its occurrences (all of them first), then one optimiser
// update of that row.  Input: keys sorted ascending with the pooled-vector id of each entry.
void launch_row_update_chunk(const uint32_t* sorted_keys, const int32_t* sorted_bag,
                             const float* de, uint32_t n, const RowUpdateScratch& sc, int d,
                             const EmbOpt& o, const float* inv_len, hipStream_t s);
void launch_row_update_finish(const uint32_t* sorted_keys, uint32_t n, const RowUpdateScratch& sc,
                              int d, const EmbOpt& o, hipStream_t s);

// ---------------------------------------------------------------------------- sort.hip
struct SortScratch {
  uint32_t* keys_a;     // [max_ids + 4] ping-pong buffers of the passes
  uint32_t* keys_b;     // [max_ids + 4]
  uint32_t* keys_f;     // [max_ids + 4] result
  uint32_t* vals;       // [max_ids + 4]
  uint32_t* vals_alt;   // [max_ids + 4]
  uint32_t* vals_f;     // [max_ids + 4] result
  uint32_t* block_hist; // [SORT_MAX_DIGITS * max_sort_blocks]
  uint32_t* seg_tot;    // [SS_MAX_TABLES * SORT_MAX_DIGITS] digit totals per table
  uint32_t* seg_lo;     // [SS_MAX_TABLES + 1] first position of every table (the plan, kept
  uint32_t* tile_base;  // [SS_MAX_TABLES + 1]  between calls)
};
constexpr int SORT_MAX_DIGITS = 1024;   // values of the widest digit (10 bits) a pass may use
int sort_num_blocks(uint32_t n, int* rounds_out);
int sort_max_blocks(uint32_t max_n);
uint32_t sort_tile(uint32_t n);   // tile length the sort of n elements uses
// The tables of the batch being sorted; their position ranges are read from the plan in the
// scratch (seg_lo, tile_base: written by the gather of the same step, see SortPlanOut, for the
// tile length sort_tile(n)).
struct SortSegments {
  int T;
  const TableMeta* meta;
  int max_digit_bits;   // 8..10: widest digit of a pass
};
// Stable LSD radix sort of (key, value) pairs, every table's range on its own local rows;
// vals == nullptr sorts (key, position).  The inputs (at least max_ids + 4 elements long) are
// left as they are; the sorted arrays are returned through the out pointers.
void launch_sort_pairs(const uint32_t* keys, const uint32_t* vals, uint32_t n,
                       const SortSegments& seg, const SortScratch& sc, uint32_t** sorted_keys,
                       uint32_t** sorted_vals, hipStream_t s);

// ---------------------------------------------------------------------------- interaction.hip
// f[b] = [z0[b], <V_r, V_c> for r>c], V = [z0[b]; e[b,0..T-1]].  Writes fp32 f (ldf floats per
// row) and, if f_bf16 != nullptr, a bf16 copy with row stride ldf_bf16 (zero padded).
void launch_interaction_fwd(const float* z0, const float* e, int B, int T, int d, float* f,
                            int ldf, uint16_t* f_bf16, int ldf_bf16, hipStream_t s);
// dz0 (masked by z0 > 0) and de from df; dz0_bf16 (optional): dz0 once more as bf16 rows of
// pitch ld16 (a multiple of 4, zero padded).
void launch_interaction_bwd(const float* z0, const float* e, const float* df, int lddf, int B,
                            int T, int d, float* dz0, float* de, uint16_t* dz0_bf16, int ld16,
                            hipStream_t s);

// ---------------------------------------------------------------------------- mlp_fp32.hip
enum : int { EPI_NONE = 0, EPI_BIAS = 1, EPI_RELU = 2, EPI_MASK = 4 };
// C[M,N] (ldc) = A*B with A(m,k) = A[m*sam + k*sak], B(k,n) = B[k*sbk + n*sbn];
// + bias[n] (EPI_BIAS), ReLU (EPI_RELU), zero where mask[m*ldmask+n] <= 0 (EPI_MASK).
void launch_gemm_f32(const float* A, int64_t sam, int64_t sak, const float* Bm, int64_t sbk,
                     int64_t sbn, float* C, int ldc, int M, int N, int K, int epi,
                     const float* bias, const float* mask, int ldmask, hipStream_t s);
// db[n] = sum_m dY[m*ld + n]
void launch_col_sum_f32(const float* dY, int ld, int M, int N, float* db, hipStream_t s);
// loss = mean_b bce(logit_b, y_b) ; dlogit_b = (sigmoid(logit_b) - y_b) / B
void launch_bce_loss(const float* logit, const float* y, int B, float* loss, float* dlogit,
                     hipStream_t s);
// w -= lr * g   (lock-free, plain loads and stores); with acc != nullptr one extra block adds
// (mean_loss * B, sum of labels, B) to the three doubles at acc
void launch_sgd(float* w, const float* g, int64_t n, float lr, const float* mean_loss,
                const float* y, int B, double* acc, hipStream_t s);
// the same accumulation as a launch of its own (evaluation steps)
void launch_metrics(const float* mean_loss, const float* y, int B, double* acc, hipStream_t s);

// Running sums behind the normalised entropy (Section 4, "Evaluation Metrics"): one block adds
// the batch's summed log-loss (mean * B), its number of positive labels and B to three doubles.
__device__ __forceinline__ void metrics_block(const float* __restrict__ mean_loss,
                                              const float* __restrict__ y, int B,
                                              double* __restrict__ acc) {
  __shared__ float part[4];
  float s = 0.f;
  for (int b = threadIdx.x; b < B; b += 256) s += y[b];
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    atomicAdd(acc + 0, (double)mean_loss[0] * (double)B);
    atomicAdd(acc + 1, (double)((part[0] + part[1]) + (part[2] + part[3])));
    atomicAdd(acc + 2, (double)B);
  }
}

// ---------------------------------------------------------------------------- mlp_last.hip
// Last top layer (one output unit) fused with the mean log-loss (accumulated into *loss,
// which must be zero) and its gradient.
void launch_last_layer_fwd_loss(const uint16_t* X, int ldx, const float* w, const float* bias,
                                const float* y, int B, int in, float* logits, float* dlogit,
                                float* loss, hipStream_t s);
// forward, loss and the layer's whole backward in one launch (training steps); the data
// gradient goes either as bf16, gated by X > 0, to dX, or as fp32 without a gate to dX32.
// The weight and bias gradients are added into LAST_GRAD_COPIES partial copies (copy c at
// gpart + c * gstride: `in` weight sums, then the bias sum; zeroed by the caller), block b into
// copy b % LAST_GRAD_COPIES: thousands of atomic adds onto the few cache lines of one copy
// serialise in the L2.  The reduction that ends the backward adds the copies up.
constexpr int LAST_GRAD_COPIES = 16;
void launch_last_layer_train(const uint16_t* X, int ldx, const float* w, const float* bias,
                             const float* y, int B, int in, float* logits, float* dlogit,
                             float* loss, uint16_t* dX, int lddx, float* dX32, int lddx32,
                             float* gpart, int gstride, hipStream_t s);
// ---------------------------------------------------------------------------- gemm_mfma.hip
#define SS_NT_MAX_LAYERS 16
// C[M,N] = A[M,K] W^T (+ bias, ReLU, gate): A bf16 row-major with K (a multiple of 64) finite
// columns per row, the weight operand a fragment-ordered bf16 copy (tile = n / 32, step =
// k / 16, zero padded to 32 units and 64 reduction elements).  Output: bf16 C [M][ldc] (columns
// N..ldc-1 zeroed; under EPI_MASK kept where mask > 0) or fp32 C_f32 [M][ldc32].
struct GemmXwArgs {
  const uint16_t* A; int lda;
  const uint16_t* Bf;
  int M, N, K;
  uint16_t* C; int ldc;
  float* C_f32; int ldc32;
  int epi; const float* bias;
  const uint16_t* mask; int ldmask;
  int role;   // 0: forward product, 1: data gradient (separate kernel names for profilers)
};
void launch_gemm_xw(const GemmXwArgs& a, hipStream_t s);
// Weight gradients of all layers in one launch.  Layer l: part[z] (z = batch slice) receives
// dY[slice]^T X[slice] as [out][in] fp32 followed by the [out] column sums of dY[slice]; dY
// [B][ldy] and X [B][ldx] are row-major bf16 whose pitch padding is zero.  tiles: device table
// of (layer, first unit of dY, first unit of X, slice), 128x128 tiles, padded to a multiple of
// 8 entries with layer = -1.
struct WgradGroupLayer {
  const uint16_t* dY; int ldy;
  const uint16_t* X; int ldx;
  float* part; int64_t part_stride;
  int out, in;
  int slice_len;      // samples per slice, a multiple of 64
};
struct WgradGroupArgs {
  WgradGroupLayer L[SS_NT_MAX_LAYERS];
  const int4* tiles;
  int n_tiles;
  int B;
};
void launch_gemm_wgrad(const WgradGroupArgs& a, hipStream_t s);
// out[i] = sum over the slices of part[z * stride + i], for up to 16 segments in one launch
// out[i] = sum over the slices of part[z * stride + i]; with w != nullptr also the SGD step
// w[i] -= lr * out[i] (plain loads and stores: lock-free, Section 3.2).  With acc != nullptr the
// launch carries one more block that adds the step's loss and labels to the running metrics.
struct ReduceSegment { const float* part; float* out; float* w; int64_t n, stride; int slices; int block_base; };
struct ReduceArgs {
  ReduceSegment seg[16]; int n_seg;
  float lr;
  const float* mean_loss; const float* y; int B; double* acc;
};
void launch_reduce_slices(const ReduceArgs& a, int total_blocks, hipStream_t s);

// ---------------------------------------------------------------------------- mlp_fused.hip
#define SS_FUSED_MAX_LAYERS 8
struct FusedLayer {
  const uint16_t* Wf;  // bf16 weights in fragment order for X W^T
  const uint16_t* Wr;  // bf16 weights in fragment order for dY W
  const float* b;      // [out] fp32
  int in, out;
  int kp_f, depth_f;   // X W^T: zero-padded reduction length (multiple of 16*depth_f)
  int kp_r, depth_r;   // dY W:  zero-padded reduction length (multiple of 16*depth_r)
};
struct PrepLayer {
  const float* W;      // [out][in] fp32 master weights
  uint16_t* Wf;
  uint16_t* Wr;
  int in, out;
  int kp_f, kp_r;
  int64_t frag_base;   // first 8-value fragment of this layer in the launch
  int64_t frags_fwd;   // fragments of the forward copy (the backward copy follows)
};
struct PrepArgs {
  int n_layers;
  PrepLayer L[2 * SS_FUSED_MAX_LAYERS];
  int64_t total_frags;
  float* zero;      // optional: zero_n floats cleared by the same launch
  int64_t zero_n;
  // optional: fp32 rows [cast_rows][cast_cols] -> bf16 rows of pitch cast_ld, zero padded (the
  // dense input as the first GEMM's operand)
  const float* cast_src;
  uint16_t* cast_dst;
  int cast_rows, cast_cols, cast_ld;
};
void launch_mlp_prep(const PrepArgs& a, hipStream_t s);
struct FusedFwdArgs {
  int n_layers;
  FusedLayer L[SS_FUSED_MAX_LAYERS];
  int B, ldT;
  const void* x; int x_is_f32; int ldx; int in0;  // stack input [B, in0]
  uint16_t* xT;                                   // [in0][ldT] transposed bf16 copy, or null
  uint16_t* actT[SS_FUSED_MAX_LAYERS];            // [out_l][ldT] transposed bf16 output, or null
  float* out_f32;                                 // last layer's output [B, out] fp32, or null
  int relu_last;
  int kp_tail;                                    // padded row length of the last output tile
  int has_tail;                                   // top stack: one-unit layer + loss
  const float* w_last; const float* b_last; const float* y;
  float* logits; float* dlogit; float* loss;
  unsigned lds_elems0;                            // bf16 elements of LDS buffer 0
};
struct FusedBwdArgs {
  int n_layers;
  FusedLayer L[SS_FUSED_MAX_LAYERS];
  int B, ldT;
  const float* d_in_f32; int ld_d_in;             // bottom stack: gated dL/dz0 [B, d]
  const float* dlogit; const float* w_last;       // top stack: tail
  float* g_w_last; float* g_b_last;
  const uint16_t* actT[SS_FUSED_MAX_LAYERS];      // outputs of layer l (for the ReLU gates)
  uint16_t* dYT[SS_FUSED_MAX_LAYERS];             // [out_l][ldT] gradient w.r.t. layer l's output
  float* d_out_f32; int ld_d_out;                 // gradient w.r.t. the stack input, or null
  unsigned lds_elems0;
};
struct WgradLayer {
  const uint16_t* dYT;  // [out][ldT]
  const uint16_t* XT;   // [in][ldT]
  float* gW;            // [out][in]
  float* gb;            // [out]
  int in, out;
};
struct WgradArgs {
  WgradLayer L[2 * SS_FUSED_MAX_LAYERS];
  const int4* tiles;    // device: (layer, n0, k0, 0) per 64x64 tile
  int B, ldT;
};
size_t fused_lds_bytes(const int* widths, int n_widths, size_t* elems0);
void launch_mlp_fused_fwd(const FusedFwdArgs& a, size_t lds_bytes, hipStream_t s);
void launch_mlp_fused_bwd(const FusedBwdArgs& a, size_t lds_bytes, hipStream_t s);
void launch_mlp_wgrad_grouped(const WgradArgs& a, int n_tiles, hipStream_t s);

// ---------------------------------------------------------------------------- sync.hip
int launch_sync_round(int algo, int K, int64_t P, int64_t stride, float* W, float* w_ps,
                      float* w_global, float* v, float alpha, float eta, float mu,
                      hipStream_t s);
// out[0..P) = mean over the K replicas (P rounded up to 4 floats is read and written)
void launch_replica_mean(const float* W, int K, int64_t stride, int64_t P, float* out,
                         hipStream_t s);

}  // namespace ss
