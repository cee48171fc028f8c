// C ABI of libshadowsync: context, workspace layout, and the host-side sequencing of one
// worker iteration and one shadow round (Algorithm 1).  No device memory is allocated here:
// everything is carved out of the caller's workspace.
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>
#include <thread>
#include <vector>

#include "../../include/shadowsync.h"
#include "ss_internal.h"

using namespace ss;

// Scratch of ss_eval_step_static: activations of one forward pass, for callers that may not
// allocate and hold no worker slot.  One copy per GPU the library runs on, kept until the
// process ends; the kernels reach it through the address ss_init looks up, never by this name.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

namespace {

constexpr int MAX_LAYERS = 16;
constexpr size_t ALIGN = 256;

struct Layer {
  int in, out;
  int64_t w_off, b_off;  // offsets inside the dense vector
};

struct Slot {
  // forward
  float* act_f32[MAX_LAYERS];      // fp32 path: output of layer l
  uint16_t* act_bf16[MAX_LAYERS];  // bf16 path: output of hidden layers
  float* z0;                       // output of the last bottom layer (fp32 in both paths)
  float* e;                        // [B,T,d]
  float* e_part = nullptr;         // [shards][B,T,d] partial pooling results (row-sharded tables)
  float* inv_len;                  // [B,T] 1 / bag length (mean pooling)
  float* f;                        // [B,ldf]
  uint16_t* f_bf16;                // [B,ldf16]
  float* logits;                   // [B]
  float* loss;                     // [1]
  // backward
  float* dlogit;                   // [B]
  float* grads;                    // [P]
  float* dbuf[2];                  // fp32 path ping-pong [B, maxw]
  float* df;                       // [B,ldf]
  float* dz0;                      // [B,d]
  float* de;                       // [B,T,d]
  // fused-MLP path: transposed bf16 copies [unit][ldT]
  uint16_t* xT;                    // dense input
  uint16_t* fT;                    // interaction output
  uint16_t* actT[MAX_LAYERS];      // output of hidden layer l
  uint16_t* dYT[MAX_LAYERS];       // gradient w.r.t. the output of layer l
  uint16_t* wsw;                   // bf16 fragment-ordered weights of the step's replica
  // layer-wise path: bf16 dense input, row-major gradient w.r.t. every layer's output, partial
  // weight gradients of the batch slices
  uint16_t* xb;                    // [B][pin[0]]
  uint16_t* dYr[MAX_LAYERS];       // [B][pout[l]]
  float* wg_part;
  // embedding backward
  uint32_t* keys;                  // [max_ids] global row of every position (the sort's input, kept)
  int32_t* bag_of_pos;             // [max_ids] pooled-vector id of every position (the sort's values)
  SortScratch sort;
  SegScratch seg;
  RowUpdateScratch upd;
  // results of the last step (for ss_read_debug)
  uint32_t* sorted_keys = nullptr;
  uint32_t* sorted_bag = nullptr;  // pooled-vector id of every sorted entry
  uint32_t last_n = 0;             // ids of the last forward pass (training or evaluation)
  uint32_t sort_n = 0;             // ids of the last TRAINING step: length of the sorted arrays
  int last_B = 0;
  bool seg_valid = false;
  bool trained = false;
};

struct Carver {
  char* base;
  size_t off = 0;
  explicit Carver(void* b) : base((char*)b) {}
  template <typename T>
  T* take(size_t count) {
    off = (off + ALIGN - 1) / ALIGN * ALIGN;
    T* p = base ? (T*)(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

}  // namespace

struct ss_ctx {
  // configuration
  int T, d, num_dense, K, max_batch, num_slots, prec;
  bool pool_mean = false;          // mean instead of sum pooling
  int row_shards = 1;              // row shards per table (partial pooling); 1 = not split
  int sort_digit_bits = 8;         // widest digit of a pass of the backward's radix sort
  int64_t max_ids;
  std::vector<int64_t> rows;
  std::vector<Layer> layers;
  int n_bot_layers, n_top_layers;
  int64_t P, Pstride;
  int F, ldf, ldf16, maxw;
  bool fused = false;              // small-network regime: fused per-sample-tile MLP kernels
  int ldT = 0;
  size_t lds_fwd_bot = 0, lds_fwd_top = 0, lds_bwd_bot = 0, lds_bwd_top = 0;
  size_t e0_fwd_bot = 0, e0_fwd_top = 0, e0_bwd_bot = 0, e0_bwd_top = 0;
  std::vector<int64_t> wsw_f, wsw_r;  // per layer: offsets of the two fragment-ordered copies
  std::vector<int> kp_f, kp_r, depth_f, depth_r;  // per layer: padded reduction lengths, prefetch depths
  int64_t wsw_elems = 0;
  bool wide = false;               // wide-layer regime: one 128x128-tile GEMM per layer and pass
  std::vector<int> pin, pout;      // per layer: row pitches of bf16 matrices with in / out columns
  std::vector<int64_t> wg_off, wg_stride;  // per layer: its batch slices inside Slot::wg_part
  int64_t wg_elems = 0;
  int wg_slices = 1, wg_slice_len = 0;     // batch slices of the grouped weight-gradient launch
  int last_stride = 4;                     // floats per partial copy of the output unit's gradients
  std::vector<int4> wgrad_tiles;   // host copy of the tile table
  int4* wgrad_tiles_dev = nullptr;
  float lr_dense, lr_emb, eps;
  bool adam = false;               // table optimiser: Adam instead of row-wise Adagrad
  float beta1 = 0.9f, beta2 = 0.999f;
  uint64_t seed;
  int device;
  TableMeta meta;
  uint64_t total_rows;
  // device memory
  float* h;
  float* G;
  float* M = nullptr;  // Adam: first / second moments, [total_rows, d] each
  float* V = nullptr;
  float* W;  // K replicas, stride Pstride
  float* w_ps;
  float* w_global;
  float* v;
  float* w_mean;  // replica average, filled on request (ss_read_dense with which = -4)
  double* metrics;  // [2][4]: (sum of log-loss, positive labels, examples, unused) train / eval
  unsigned char* static_scratch = nullptr;  // this device's copy of the file-scope array
  std::vector<Slot> slots;
  // state
  std::mutex err_mu;               // guards err: concurrent callers may fail at the same time
  std::string err;
  std::atomic<int> sticky{0};
  std::vector<std::atomic<uint64_t>> steps;
  std::atomic<uint64_t> rounds{0}, examples{0}, exchanges{0};
  // shadow loop
  std::thread shadow;
  std::atomic<bool> shadow_run{false};
  std::atomic<int64_t> shadow_period_us{0};
  // profiling
  std::mutex prof_mu;
  std::atomic<uint32_t> prof_mask{0};
  std::atomic<uint32_t> prof_every[SS_K_COUNT];   // per class: bracket one launch in so many
  std::atomic<uint32_t> prof_seen[SS_K_COUNT];
  struct ProfPool {
    std::vector<std::pair<hipEvent_t, hipEvent_t>> ev;
    size_t used = 0;
  } prof[SS_K_COUNT];

  explicit ss_ctx(int k) : steps(k) {
    for (auto& a : steps) a.store(0);
    for (auto& a : prof_seen) a.store(0);
    for (auto& a : prof_every) a.store(1);
  }
};

static std::mutex g_init_err_mu;
static std::string g_init_err;

static int fail(ss_ctx* ctx, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) {
    std::lock_guard<std::mutex> lk(ctx->err_mu);
    ctx->err = buf;
  } else {
    std::lock_guard<std::mutex> lk(g_init_err_mu);
    g_init_err = buf;
  }
  return code;
}

static int check_hip(ss_ctx* ctx, hipError_t e, const char* what) {
  if (e == hipSuccess) return SS_OK;
  if (ctx) ctx->sticky = 1;
  return fail(ctx, SS_EDEVICE, "%s: %s", what, hipGetErrorString(e));
}

#define HIP_TRY(ctx, call)                                     \
  do {                                                         \
    int _rc = check_hip(ctx, (call), #call);                   \
    if (_rc != SS_OK) return _rc;                              \
  } while (0)

// ------------------------------------------------------------------------------------------
// Layout.  Returns total bytes; fills ctx pointers when base != nullptr.
static int validate(const ss_config* c, std::string& why) {
  char b[256];
#define BAD(...) do { snprintf(b, sizeof b, __VA_ARGS__); why = b; return SS_EINVAL; } while (0)
  if (!c) BAD("null config");
  if (c->num_tables < 1 || c->num_tables > SS_MAX_TABLES) BAD("num_tables must be 1..%d", SS_MAX_TABLES);
  if (!c->rows || !c->bot_dims || !c->top_dims) BAD("null rows/bot_dims/top_dims");
  if (c->emb_dim != 16 && c->emb_dim != 32 && c->emb_dim != 64 && c->emb_dim != 128)
    BAD("emb_dim must be 16, 32, 64 or 128");
  if (c->n_bot < 2 || c->n_top < 2 || (c->n_bot - 1) + (c->n_top - 1) > MAX_LAYERS)
    BAD("need 1..%d MLP layers in total", MAX_LAYERS);
  if (c->num_dense < 1 || c->bot_dims[0] != c->num_dense) BAD("bot_dims[0] must equal num_dense");
  if (c->bot_dims[c->n_bot - 1] != c->emb_dim) BAD("last bottom width must equal emb_dim");
  const int T = c->num_tables;
  if (c->top_dims[0] != c->emb_dim + T * (T + 1) / 2)
    BAD("top_dims[0] must be emb_dim + T(T+1)/2 = %d", c->emb_dim + T * (T + 1) / 2);
  if (c->top_dims[c->n_top - 1] != 1) BAD("last top width must be 1");
  for (int i = 0; i < c->n_bot; ++i) if (c->bot_dims[i] < 1) BAD("bad bottom width");
  for (int i = 0; i < c->n_top; ++i) if (c->top_dims[i] < 1) BAD("bad top width");
  if (c->mlp_prec == SS_BF16) {
    // the bf16 kernels index padded [batch][width] operands with 32 bits
    int maxw = 0;
    for (int i = 0; i < c->n_bot; ++i) maxw = c->bot_dims[i] > maxw ? c->bot_dims[i] : maxw;
    for (int i = 0; i < c->n_top; ++i) maxw = c->top_dims[i] > maxw ? c->top_dims[i] : maxw;
    if (((int64_t)maxw + 128) * ((int64_t)c->max_batch + 128) >= (1ll << 31))
      BAD("max_batch x widest layer too large for the bf16 MLP kernels");
  }
  uint64_t tot = 0;
  for (int t = 0; t < T; ++t) {
    if (c->rows[t] < 1) BAD("table %d has no rows", t);
    tot += (uint64_t)c->rows[t];
  }
  if (tot >= (1ull << 32)) BAD("total rows must be < 2^32");
  if (c->num_replicas < 1 || c->num_replicas > 16) BAD("num_replicas must be 1..16");
  if (c->max_batch < 1 || c->max_batch > (1 << 20)) BAD("bad max_batch");
  if (c->max_ids < 1 || c->max_ids >= (1ll << 31)) BAD("max_ids must be 1..2^31-1");
  if ((int64_t)c->max_batch * T >= (1ll << 31)) BAD("max_batch * num_tables too large");
  if (c->num_worker_slots < 1 || c->num_worker_slots > 64) BAD("num_worker_slots must be 1..64");
  if (c->mlp_prec != SS_FP32 && c->mlp_prec != SS_BF16) BAD("bad mlp_prec");
  if (c->pooling != SS_POOL_SUM && c->pooling != SS_POOL_MEAN) BAD("bad pooling mode");
  if (c->mlp_path != SS_MLP_AUTO && c->mlp_path != SS_MLP_LAYERWISE) BAD("bad mlp_path");
  if (c->emb_row_shards < 0 || c->emb_row_shards > 64) BAD("emb_row_shards must be 0..64");
  if (c->sort_digit_bits != 0 && (c->sort_digit_bits < 8 || c->sort_digit_bits > 10))
    BAD("sort_digit_bits must be 0 (default), 8, 9 or 10");
  if (c->emb_optimizer != SS_OPT_ROWWISE_ADAGRAD && c->emb_optimizer != SS_OPT_ADAM)
    BAD("bad emb_optimizer");
  if (c->emb_optimizer == SS_OPT_ADAM &&
      !(c->adam_beta1 >= 0.f && c->adam_beta1 < 1.f && c->adam_beta2 >= 0.f && c->adam_beta2 < 1.f))
    BAD("Adam betas must lie in [0, 1)");
  {  // LDS of the interaction kernels, four samples per workgroup (see interaction.hip)
    const int n1 = T + 1, n1p = (n1 + 3) & ~3, np4 = (T * (T + 1) / 2 + 3) & ~3;
    const size_t fwd = (size_t)4 * (n1p * c->emb_dim + np4) * 4;
    const size_t bwd = (size_t)4 * (n1 * c->emb_dim + n1 * n1p) * 4;
    if (fwd > 64 * 1024 || bwd > 64 * 1024)
      BAD("interaction tile (T+1) x d does not fit the LDS budget");
  }
#undef BAD
  return SS_OK;
}

// Per-caller scratch of one step for a batch of up to B samples and n ids: activations,
// gradients, sort and row-update buffers.  fwd_only leaves out everything only a training step
// touches (the forward kernels skip outputs whose pointer is null).
static void carve_slot(const ss_ctx* x, Carver& cv, Slot& s, int B, int64_t n, bool fwd_only) {
  const int L = (int)x->layers.size();
  for (int l = 0; l < L; ++l) {
    s.act_f32[l] = nullptr;
    s.act_bf16[l] = nullptr;
    s.actT[l] = s.dYT[l] = nullptr;
    s.dYr[l] = nullptr;
    const bool is_z0 = (l == x->n_bot_layers - 1), is_logit = (l == L - 1);
    if (is_z0 || is_logit) continue;
    if (x->prec == SS_FP32) s.act_f32[l] = cv.take<float>((size_t)B * x->layers[l].out);
    else if (!x->fused) s.act_bf16[l] = cv.take<uint16_t>((size_t)B * (x->wide ? x->pout[l] : x->layers[l].out));
  }
  s.z0 = cv.take<float>((size_t)B * x->d);
  s.e = cv.take<float>((size_t)B * x->T * x->d);
  s.e_part = x->row_shards > 1 ? cv.take<float>((size_t)x->row_shards * B * x->T * x->d) : nullptr;
  s.inv_len = cv.take<float>((size_t)B * x->T);
  s.f = cv.take<float>((size_t)B * x->ldf);
  s.f_bf16 = (x->prec == SS_BF16) ? cv.take<uint16_t>((size_t)B * x->ldf16) : nullptr;
  s.logits = cv.take<float>(B);
  s.loss = cv.take<float>(64);
  s.xT = s.fT = nullptr;
  s.wsw = nullptr;
  s.xb = nullptr;
  s.wg_part = nullptr;
  s.dlogit = s.grads = s.df = s.dz0 = s.de = nullptr;
  s.dbuf[0] = s.dbuf[1] = nullptr;
  if (x->fused || x->wide) s.wsw = cv.take<uint16_t>((size_t)x->wsw_elems);
  if (x->wide) s.xb = cv.take<uint16_t>((size_t)B * x->pin[0]);
  if (fwd_only) return;
  s.dlogit = cv.take<float>(B);
  // (followed by the partial copies of the output unit's gradients, cleared with it)
  s.grads = cv.take<float>(x->Pstride + (size_t)LAST_GRAD_COPIES * x->last_stride);
  for (int i = 0; i < 2; ++i) {
    if (x->prec == SS_FP32) s.dbuf[i] = cv.take<float>((size_t)B * x->maxw);
  }
  s.df = cv.take<float>((size_t)B * x->ldf);
  s.dz0 = cv.take<float>((size_t)B * x->d);
  s.de = cv.take<float>((size_t)B * x->T * x->d);
  if (x->wide) {
    s.wg_part = cv.take<float>((size_t)x->wg_elems);
    for (int l = 0; l < L - 1; ++l) s.dYr[l] = cv.take<uint16_t>((size_t)B * x->pout[l]);
  }
  if (x->fused) {
    s.xT = cv.take<uint16_t>((size_t)x->num_dense * x->ldT);
    s.fT = cv.take<uint16_t>((size_t)x->F * x->ldT);
    for (int l = 0; l < L - 1; ++l) {
      if (l != x->n_bot_layers - 1) s.actT[l] = cv.take<uint16_t>((size_t)x->layers[l].out * x->ldT);
      s.dYT[l] = cv.take<uint16_t>((size_t)x->layers[l].out * x->ldT);
    }
  }
  const int sort_blocks = sort_max_blocks((uint32_t)n);
  const int seg_blocks = ceil_div(n, 2048) + 1;
  // (+4: the sort's histogram reads whole 16-byte vectors up to the end of the array)
  s.keys = cv.take<uint32_t>(n + 4);
  s.bag_of_pos = cv.take<int32_t>(n + 4);
  s.sort.keys_a = cv.take<uint32_t>(n + 4);
  s.sort.keys_b = cv.take<uint32_t>(n + 4);
  s.sort.keys_f = cv.take<uint32_t>(n + 4);
  s.sort.vals = cv.take<uint32_t>(n + 4);
  s.sort.vals_alt = cv.take<uint32_t>(n + 4);
  s.sort.vals_f = cv.take<uint32_t>(n + 4);
  s.sort.block_hist = cv.take<uint32_t>((size_t)SORT_MAX_DIGITS * sort_blocks);
  s.sort.seg_tot = cv.take<uint32_t>((size_t)SS_MAX_TABLES * SORT_MAX_DIGITS);
  s.sort.seg_lo = cv.take<uint32_t>(SS_MAX_TABLES + 1);
  s.sort.tile_base = cv.take<uint32_t>(SS_MAX_TABLES + 1);
  s.seg.block_counts = cv.take<uint32_t>(seg_blocks);
  s.seg.seg_starts = cv.take<uint32_t>(n + 1);
  s.seg.num_unique = cv.take<uint32_t>(64);
  s.upd.parts = cv.take<float>((size_t)row_update_chunks(n, x->d) * 2 * x->d);
  s.upd.flags = cv.take<uint32_t>((size_t)row_update_chunks(n, x->d));
  s.upd.long_list = cv.take<uint32_t>(2 * ((size_t)row_update_chunks(n, x->d) / 30 + 2));
  s.upd.long_count = cv.take<uint32_t>(64);
}

static size_t layout(ss_ctx* x, void* base) {
  Carver cv(base);
  const int B = x->max_batch;
  const int64_t n = x->max_ids;
  x->h = cv.take<float>(x->total_rows * (uint64_t)x->d);
  x->G = cv.take<float>(x->total_rows);
  if (x->adam) {
    x->M = cv.take<float>(x->total_rows * (uint64_t)x->d);
    x->V = cv.take<float>(x->total_rows * (uint64_t)x->d);
  }
  x->W = cv.take<float>((size_t)x->K * x->Pstride);
  x->w_ps = cv.take<float>(x->Pstride);
  x->w_global = cv.take<float>(x->Pstride);
  x->v = cv.take<float>(x->Pstride);
  x->w_mean = cv.take<float>(x->Pstride);
  x->metrics = cv.take<double>(8);
  x->wgrad_tiles_dev = x->wgrad_tiles.empty() ? nullptr : cv.take<int4>(x->wgrad_tiles.size());
  for (Slot& s : x->slots) carve_slot(x, cv, s, B, n, false);
  return (cv.off + ALIGN - 1) / ALIGN * ALIGN;
}

static ss_ctx* make_ctx(const ss_config* c) {
  ss_ctx* x = new ss_ctx(c->num_replicas);
  x->T = c->num_tables; x->d = c->emb_dim; x->num_dense = c->num_dense;
  x->K = c->num_replicas; x->max_batch = c->max_batch; x->max_ids = c->max_ids;
  x->num_slots = c->num_worker_slots; x->prec = c->mlp_prec;
  x->pool_mean = (c->pooling == SS_POOL_MEAN);
  x->row_shards = c->emb_row_shards < 1 ? 1 : c->emb_row_shards;
  x->sort_digit_bits = c->sort_digit_bits == 0 ? 8 : c->sort_digit_bits;
  x->lr_dense = c->lr_dense; x->lr_emb = c->lr_emb; x->eps = c->adagrad_eps; x->seed = c->seed;
  x->adam = (c->emb_optimizer == SS_OPT_ADAM);
  x->beta1 = c->adam_beta1; x->beta2 = c->adam_beta2;
  x->rows.assign(c->rows, c->rows + c->num_tables);
  uint64_t base = 0;
  memset(&x->meta, 0, sizeof x->meta);
  for (int t = 0; t < x->T; ++t) { x->meta.row_base[t] = (uint32_t)base; base += (uint64_t)x->rows[t]; }
  x->meta.row_base[x->T] = (uint32_t)base;
  x->total_rows = base;
  int64_t off = 0;
  int maxw = 1;
  auto add = [&](const int32_t* dims, int n) {
    for (int i = 0; i + 1 < n; ++i) {
      Layer l; l.in = dims[i]; l.out = dims[i + 1];
      l.w_off = off; off += (int64_t)l.in * l.out;
      l.b_off = off; off += l.out;
      x->layers.push_back(l);
      if (l.in > maxw) maxw = l.in;
      if (l.out > maxw) maxw = l.out;
    }
  };
  add(c->bot_dims, c->n_bot);
  add(c->top_dims, c->n_top);
  x->n_bot_layers = c->n_bot - 1; x->n_top_layers = c->n_top - 1;
  x->P = off;
  x->Pstride = (off + 255) / 256 * 256;
  x->last_stride = (x->layers.back().in + 1 + 3) / 4 * 4;
  x->F = c->top_dims[0];
  x->ldf = (x->F + 7) / 8 * 8;
  x->ldf16 = (x->F + 7) / 8 * 8;
  x->maxw = maxw;
  x->slots.resize(x->num_slots);
  // Fused MLP kernels: bf16, at least one hidden top layer, every width <= 512, stacks of at
  // most SS_FUSED_MAX_LAYERS layers, and the two LDS activation buffers within 64 KB.
  {
    const int nb = x->n_bot_layers, nt = x->n_top_layers, nh = nt - 1;
    bool ok = x->prec == SS_BF16 && nh >= 1 && nb <= SS_FUSED_MAX_LAYERS &&
              nh <= SS_FUSED_MAX_LAYERS && maxw <= 512 && c->mlp_path == SS_MLP_AUTO;
    auto round_up = [](int v, int m) { return (v + m - 1) / m * m; };
    // Both MFMA paths read the step's weights from fragment-ordered bf16 copies whose reduction
    // lengths are zero padded to a multiple of 64; the fused kernels' prefetch depth of a layer
    // is the larger of 8 / 4 reduction steps that divides its step count.
    if (x->prec == SS_BF16) {
      auto depth_for = [](int kp) {
        const int steps = kp / 16;
        return steps % 8 == 0 ? 8 : 4;
      };
      for (int l = 0; l < nb + nh; ++l) {
        const Layer& ly = x->layers[l];
        x->kp_f.push_back(round_up(ly.in, 64));
        x->depth_f.push_back(depth_for(x->kp_f.back()));
        x->kp_r.push_back(round_up(ly.out, 64));
        x->depth_r.push_back(depth_for(x->kp_r.back()));
        x->wsw_f.push_back(x->wsw_elems);
        x->wsw_elems += (int64_t)((ly.out + 31) / 32 * 32) * x->kp_f[l];
        x->wsw_r.push_back(x->wsw_elems);
        x->wsw_elems += (int64_t)((ly.in + 31) / 32 * 32) * x->kp_r[l];
      }
    }
    if (ok) {
      // LDS tiles of each launch, in the order they are produced (tile i -> buffer i & 1)
      std::vector<int> fb, ft, rb, rt;
      for (int l = 0; l < nb; ++l) fb.push_back(x->kp_f[l]);
      fb.push_back(round_up(x->layers[nb - 1].out, 64));
      for (int l = nb; l < nb + nh; ++l) ft.push_back(x->kp_f[l]);
      ft.push_back(round_up(x->layers[nb + nh - 1].out, 64));
      for (int l = nb - 1; l >= 0; --l) rb.push_back(x->kp_r[l]);
      for (int l = nb + nh - 1; l >= nb; --l) rt.push_back(x->kp_r[l]);
      x->lds_fwd_bot = fused_lds_bytes(fb.data(), (int)fb.size(), &x->e0_fwd_bot);
      x->lds_fwd_top = fused_lds_bytes(ft.data(), (int)ft.size(), &x->e0_fwd_top);
      x->lds_bwd_bot = fused_lds_bytes(rb.data(), (int)rb.size(), &x->e0_bwd_bot);
      x->lds_bwd_top = fused_lds_bytes(rt.data(), (int)rt.size(), &x->e0_bwd_top);
      const size_t lim = 150 * 1024;
      ok = x->lds_fwd_bot <= lim && x->lds_fwd_top <= lim && x->lds_bwd_bot <= lim &&
           x->lds_bwd_top <= lim;
    }
    x->fused = ok;
    x->ldT = (x->max_batch + 7) / 8 * 8;
    // Layer-wise regime: every other bf16 model.  Activations and their gradients are
    // row-major bf16 whose pitch is a multiple of 64 elements (zero padded, so no GEMM handles
    // an edge along its reduction).
    x->wide = !ok && x->prec == SS_BF16;
    if (x->wide) {
      // row pitches: multiples of 64 elements, never a multiple of 256 (rows that are a power
      // of two apart would all fall on the same memory channel)
      auto pitch = [](int v) { const int p = (v + 63) / 64 * 64; return (p % 256 == 0) ? p + 64 : p; };
      x->ldf16 = pitch(x->F);
      int total_tiles = 0;
      for (size_t l = 0; l + 1 < x->layers.size(); ++l) {
        const Layer& ly = x->layers[l];
        x->pin.push_back(pitch(ly.in)); x->pout.push_back(pitch(ly.out));
        total_tiles += ceil_div(ly.out, 128) * ceil_div(ly.in, 128);
      }
      // Weight gradients: ONE launch over (layer, 128x128 tile, batch slice).  The batch is cut
      // into as many slices as keep about two blocks per CU busy (each at least 256 samples
      // long); a slice stores its partial [out][in] + [out] sums, one reduction launch adds them.
      const int Bp = round_up(x->max_batch, 64);
      int slices = 512 / total_tiles;
      if (slices > Bp / 256) slices = Bp / 256;
      if (slices > 32) slices = 32;
      if (slices < 1) slices = 1;
      x->wg_slice_len = round_up(ceil_div(Bp, slices), 64);
      x->wg_slices = ceil_div(Bp, x->wg_slice_len);
      for (size_t l = 0; l + 1 < x->layers.size(); ++l) {
        const Layer& ly = x->layers[l];
        const int64_t stride = ((int64_t)ly.out * ly.in + ly.out + 3) / 4 * 4;
        x->wg_off.push_back(x->wg_elems);
        x->wg_stride.push_back(stride);
        x->wg_elems += stride * x->wg_slices;
        for (int z = 0; z < x->wg_slices; ++z)
          for (int m0 = 0; m0 < ly.out; m0 += 128)
            for (int n0 = 0; n0 < ly.in; n0 += 128)
              x->wgrad_tiles.push_back(make_int4((int)l, m0, n0, z));
      }
      while (x->wgrad_tiles.size() % 8) x->wgrad_tiles.push_back(make_int4(-1, 0, 0, 0));
    }
    if (ok) {
      // weight-gradient tiles of every layer except the one-unit output layer
      for (int l = 0; l < nb + nh; ++l)
        for (int n0 = 0; n0 < x->layers[l].out; n0 += 64)
          for (int k0 = 0; k0 < x->layers[l].in; k0 += 64)
            x->wgrad_tiles.push_back(make_int4(l, n0, k0, 0));
    }
  }
  return x;
}

// ------------------------------------------------------------------------------------------
extern "C" {

size_t ss_workspace_bytes(const ss_config* cfg) {
  std::string why;
  if (validate(cfg, why) != SS_OK) { fail(nullptr, SS_EINVAL, "%s", why.c_str()); return 0; }
  ss_ctx* x = make_ctx(cfg);
  size_t bytes = layout(x, nullptr);
  delete x;
  return bytes;
}

int ss_init(const ss_config* cfg, void* dev_workspace, size_t bytes, ss_ctx** out) {
  if (!out) return fail(nullptr, SS_EINVAL, "null out pointer");
  *out = nullptr;
  std::string why;
  if (validate(cfg, why) != SS_OK) return fail(nullptr, SS_EINVAL, "%s", why.c_str());
  if (!dev_workspace || ((uintptr_t)dev_workspace % ALIGN) != 0)
    return fail(nullptr, SS_EINVAL, "workspace must be non-null and %zu-byte aligned", ALIGN);
  ss_ctx* x = make_ctx(cfg);
  const size_t need = layout(x, dev_workspace);
  if (bytes < need) {
    delete x;
    return fail(nullptr, SS_ENOMEM, "workspace too small: %zu bytes given, %zu needed", bytes, need);
  }
  hipError_t e = hipGetDevice(&x->device);
  if (e != hipSuccess) {
    delete x;
    return fail(nullptr, SS_EDEVICE, "hipGetDevice: %s", hipGetErrorString(e));
  }
  // this device's address of the static scratch array (every GPU holds its own copy)
  e = hipGetSymbolAddress((void**)&x->static_scratch, HIP_SYMBOL(scratch));
  if (e != hipSuccess || !x->static_scratch) {
    delete x;
    return fail(nullptr, SS_EDEVICE, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
  }
  // optimiser state and momentum start at zero (Algorithm 1 initialisation)
  launch_fill_f32(x->G, x->total_rows, 0.f, nullptr);
  if (x->adam) {
    launch_fill_f32(x->M, x->total_rows * (uint64_t)x->d, 0.f, nullptr);
    launch_fill_f32(x->V, x->total_rows * (uint64_t)x->d, 0.f, nullptr);
  }
  launch_fill_f32(x->v, (uint64_t)x->Pstride, 0.f, nullptr);
  launch_fill_f32(x->W, (uint64_t)x->K * x->Pstride, 0.f, nullptr);
  launch_fill_f32(x->w_ps, (uint64_t)x->Pstride, 0.f, nullptr);
  launch_fill_f32(x->w_global, (uint64_t)x->Pstride, 0.f, nullptr);
  launch_fill_f32((float*)x->metrics, 16, 0.f, nullptr);
  for (Slot& s : x->slots) launch_fill_f32(s.grads, (uint64_t)x->Pstride, 0.f, nullptr);
  if (x->wide) {
    // the pitch padding of these row-major bf16 buffers is read as an operand (against zero
    // weights, or as zero contributions to a weight gradient) and only partly rewritten by the
    // kernels, so it holds zeros from the start
    const int L = (int)x->layers.size();
    for (Slot& s : x->slots) {
      launch_fill_f32((float*)s.xb, (uint64_t)x->max_batch * x->pin[0] / 2, 0.f, nullptr);
      if (s.f_bf16) launch_fill_f32((float*)s.f_bf16, (uint64_t)x->max_batch * x->ldf16 / 2, 0.f, nullptr);
      for (int l = 0; l < L - 1; ++l) {
        launch_fill_f32((float*)s.dYr[l], (uint64_t)x->max_batch * x->pout[l] / 2, 0.f, nullptr);
        if (s.act_bf16[l])
          launch_fill_f32((float*)s.act_bf16[l], (uint64_t)x->max_batch * x->pout[l] / 2, 0.f, nullptr);
      }
    }
  }
  if (!x->wgrad_tiles.empty())
    (void)hipMemcpy(x->wgrad_tiles_dev, x->wgrad_tiles.data(), x->wgrad_tiles.size() * sizeof(int4),
                    hipMemcpyHostToDevice);
  e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    delete x;
    return fail(nullptr, SS_EDEVICE, "init kernels: %s", hipGetErrorString(e));
  }
  *out = x;
  return SS_OK;
}

void ss_destroy(ss_ctx* ctx) {
  if (!ctx) return;
  ss_shadow_stop(ctx);
  (void)hipDeviceSynchronize();
  for (auto& pool : ctx->prof)
    for (auto& p : pool.ev) { (void)hipEventDestroy(p.first); (void)hipEventDestroy(p.second); }
  delete ctx;
}

const char* ss_last_error(const ss_ctx* ctx) {
  // the text is copied under the lock into storage owned by the calling thread, so the pointer
  // stays valid while other threads fail
  static thread_local std::string copy;
  if (ctx) {
    std::lock_guard<std::mutex> lk(const_cast<ss_ctx*>(ctx)->err_mu);
    copy = ctx->err;
  } else {
    std::lock_guard<std::mutex> lk(g_init_err_mu);
    copy = g_init_err;
  }
  return copy.c_str();
}

int64_t ss_num_params(const ss_ctx* ctx) { return ctx ? ctx->P : -1; }

int ss_init_tables_hash(ss_ctx* ctx, void* stream) {
  if (!ctx) return SS_EINVAL;
  hipStream_t s = (hipStream_t)stream;
  for (int t = 0; t < ctx->T; ++t)
    launch_table_hash_init(ctx->h + (size_t)ctx->meta.row_base[t] * ctx->d,
                           (uint64_t)ctx->rows[t] * ctx->d, ctx->seed, t, s);
  launch_fill_f32(ctx->G, ctx->total_rows, 0.f, s);
  if (ctx->adam) {
    launch_fill_f32(ctx->M, ctx->total_rows * (uint64_t)ctx->d, 0.f, s);
    launch_fill_f32(ctx->V, ctx->total_rows * (uint64_t)ctx->d, 0.f, s);
  }
  return check_hip(ctx, hipGetLastError(), "table init");
}

int ss_write_rows(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                  const float* host_rows) {
  if (!ctx) return SS_EINVAL;
  if (table < 0 || table >= ctx->T || first_row < 0 || n_rows < 0 ||
      first_row + n_rows > ctx->rows[table] || (!host_rows && n_rows))
    return fail(ctx, SS_EINVAL, "ss_write_rows: bad table/row range");
  if (n_rows == 0) return SS_OK;
  const size_t r0 = (size_t)ctx->meta.row_base[table] + first_row;
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(ctx->h + r0 * ctx->d, host_rows, (size_t)n_rows * ctx->d * sizeof(float),
                         hipMemcpyHostToDevice));
  launch_fill_f32(ctx->G + r0, (uint64_t)n_rows, 0.f, nullptr);
  if (ctx->adam) {
    launch_fill_f32(ctx->M + r0 * ctx->d, (uint64_t)n_rows * ctx->d, 0.f, nullptr);
    launch_fill_f32(ctx->V + r0 * ctx->d, (uint64_t)n_rows * ctx->d, 0.f, nullptr);
  }
  HIP_TRY(ctx, hipDeviceSynchronize());
  return SS_OK;
}

int ss_write_adam_state(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                        const float* host_m, const float* host_v) {
  if (!ctx) return SS_EINVAL;
  if (!ctx->adam) return fail(ctx, SS_ESTATE, "the table optimiser is not Adam");
  if (table < 0 || table >= ctx->T || first_row < 0 || n_rows < 0 ||
      first_row + n_rows > ctx->rows[table])
    return fail(ctx, SS_EINVAL, "ss_write_adam_state: bad table/row range");
  if (n_rows == 0) return SS_OK;
  const size_t r0 = (size_t)ctx->meta.row_base[table] + first_row;
  const size_t bytes = (size_t)n_rows * ctx->d * sizeof(float);
  HIP_TRY(ctx, hipDeviceSynchronize());
  if (host_m) HIP_TRY(ctx, hipMemcpy(ctx->M + r0 * ctx->d, host_m, bytes, hipMemcpyHostToDevice));
  if (host_v) HIP_TRY(ctx, hipMemcpy(ctx->V + r0 * ctx->d, host_v, bytes, hipMemcpyHostToDevice));
  return SS_OK;
}

int ss_write_adagrad(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                     const float* host_acc) {
  if (!ctx) return SS_EINVAL;
  if (table < 0 || table >= ctx->T || first_row < 0 || n_rows < 0 ||
      first_row + n_rows > ctx->rows[table] || (!host_acc && n_rows))
    return fail(ctx, SS_EINVAL, "ss_write_adagrad: bad table/row range");
  if (n_rows == 0) return SS_OK;
  const size_t r0 = (size_t)ctx->meta.row_base[table] + first_row;
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(ctx->G + r0, host_acc, (size_t)n_rows * sizeof(float),
                         hipMemcpyHostToDevice));
  return SS_OK;
}

static float* dense_ptr(ss_ctx* ctx, int which) {
  if (which >= 0 && which < ctx->K) return ctx->W + (size_t)which * ctx->Pstride;
  if (which == -1) return ctx->w_ps;
  if (which == -2) return ctx->w_global;
  if (which == -3) return ctx->v;
  return nullptr;
}

int ss_init_dense(ss_ctx* ctx, const float* host_w0) {
  if (!ctx || !host_w0) return SS_EINVAL;
  HIP_TRY(ctx, hipDeviceSynchronize());
  for (int which = -2; which < ctx->K; ++which)
    HIP_TRY(ctx, hipMemcpy(dense_ptr(ctx, which), host_w0, (size_t)ctx->P * sizeof(float),
                           hipMemcpyHostToDevice));
  launch_fill_f32(ctx->v, (uint64_t)ctx->Pstride, 0.f, nullptr);
  HIP_TRY(ctx, hipDeviceSynchronize());
  return SS_OK;
}

int ss_read_dense(ss_ctx* ctx, int32_t which, float* host_out, int64_t n) {
  if (!ctx || !host_out) return SS_EINVAL;
  float* p = (which == -4) ? ctx->w_mean : dense_ptr(ctx, which);
  if (!p || n != ctx->P) return fail(ctx, SS_EINVAL, "ss_read_dense: bad selector or length");
  HIP_TRY(ctx, hipDeviceSynchronize());
  if (which == -4) {
    launch_replica_mean(ctx->W, ctx->K, ctx->Pstride, ctx->P, ctx->w_mean, nullptr);
    HIP_TRY(ctx, hipDeviceSynchronize());
  }
  HIP_TRY(ctx, hipMemcpy(host_out, p, (size_t)n * sizeof(float), hipMemcpyDeviceToHost));
  return SS_OK;
}

int ss_write_dense(ss_ctx* ctx, int32_t which, const float* host_in, int64_t n) {
  if (!ctx || !host_in) return SS_EINVAL;
  float* p = dense_ptr(ctx, which);
  if (!p || n != ctx->P) return fail(ctx, SS_EINVAL, "ss_write_dense: bad selector or length");
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemcpy(p, host_in, (size_t)n * sizeof(float), hipMemcpyHostToDevice));
  return SS_OK;
}

int ss_read_rows(ss_ctx* ctx, int32_t table, const int64_t* rows, int64_t n, float* host_rows_out,
                 float* host_adagrad_out) {
  if (!ctx || (!rows && n)) return SS_EINVAL;
  if (table < 0 || table >= ctx->T || n < 0) return fail(ctx, SS_EINVAL, "ss_read_rows: bad table");
  for (int64_t i = 0; i < n; ++i)
    if (rows[i] < 0 || rows[i] >= ctx->rows[table])
      return fail(ctx, SS_EINVAL, "ss_read_rows: row %lld out of range", (long long)rows[i]);
  HIP_TRY(ctx, hipDeviceSynchronize());
  const size_t base = ctx->meta.row_base[table];
  // contiguous runs are copied in one piece
  int64_t i = 0;
  while (i < n) {
    int64_t j = i + 1;
    while (j < n && rows[j] == rows[j - 1] + 1) ++j;
    const size_t r = base + (size_t)rows[i];
    if (host_rows_out)
      HIP_TRY(ctx, hipMemcpy(host_rows_out + (size_t)i * ctx->d, ctx->h + r * ctx->d,
                             (size_t)(j - i) * ctx->d * sizeof(float), hipMemcpyDeviceToHost));
    if (host_adagrad_out)
      HIP_TRY(ctx, hipMemcpy(host_adagrad_out + i, ctx->G + r, (size_t)(j - i) * sizeof(float),
                             hipMemcpyDeviceToHost));
    i = j;
  }
  return SS_OK;
}

int ss_read_adam_state(ss_ctx* ctx, int32_t table, const int64_t* rows, int64_t n,
                       float* host_m_out, float* host_v_out) {
  if (!ctx || (!rows && n)) return SS_EINVAL;
  if (!ctx->adam) return fail(ctx, SS_ESTATE, "the table optimiser is not Adam");
  if (table < 0 || table >= ctx->T || n < 0) return fail(ctx, SS_EINVAL, "ss_read_adam_state: bad table");
  for (int64_t i = 0; i < n; ++i)
    if (rows[i] < 0 || rows[i] >= ctx->rows[table])
      return fail(ctx, SS_EINVAL, "ss_read_adam_state: row %lld out of range", (long long)rows[i]);
  HIP_TRY(ctx, hipDeviceSynchronize());
  const size_t base = ctx->meta.row_base[table];
  int64_t i = 0;
  while (i < n) {   // contiguous runs are copied in one piece
    int64_t j = i + 1;
    while (j < n && rows[j] == rows[j - 1] + 1) ++j;
    const size_t r = base + (size_t)rows[i];
    const size_t bytes = (size_t)(j - i) * ctx->d * sizeof(float);
    if (host_m_out)
      HIP_TRY(ctx, hipMemcpy(host_m_out + (size_t)i * ctx->d, ctx->M + r * ctx->d, bytes, hipMemcpyDeviceToHost));
    if (host_v_out)
      HIP_TRY(ctx, hipMemcpy(host_v_out + (size_t)i * ctx->d, ctx->V + r * ctx->d, bytes, hipMemcpyDeviceToHost));
    i = j;
  }
  return SS_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------
// Event brackets around one kernel class.
namespace {
struct ProfScope {
  ss_ctx* x; hipStream_t s; hipEvent_t stop = nullptr;
  ProfScope(ss_ctx* ctx, int id, hipStream_t st) : x(ctx), s(st) {
    if (!(x->prof_mask.load(std::memory_order_relaxed) & (1u << id))) return;
    const uint32_t every = x->prof_every[id].load(std::memory_order_relaxed);
    // launches are picked by a hash of their running number, not by its remainder: a step's
    // launches of one class cycle through the layers, and a fixed stride would always land on
    // the same ones
    if (every > 1 &&
        ((x->prof_seen[id].fetch_add(1, std::memory_order_relaxed) * 0x9E3779B1u) >> 12) % every != 0)
      return;
    std::lock_guard<std::mutex> lk(x->prof_mu);
    auto& pool = x->prof[id];
    if (!(x->prof_mask.load() & (1u << id)) || pool.used >= pool.ev.size()) return;
    auto& p = pool.ev[pool.used++];
    (void)hipEventRecord(p.first, s);
    stop = p.second;
  }
  ~ProfScope() { if (stop) (void)hipEventRecord(stop, s); }
};
}  // namespace

// ------------------------------------------------------------------------------------------
// One worker iteration.
static int check_batch(ss_ctx* x, int replica, int slot, const ss_batch* b) {
  if (!b) return fail(x, SS_EINVAL, "null batch");
  if (x->sticky) return SS_EDEVICE;
  if (replica < 0 || replica >= x->K) return fail(x, SS_EINVAL, "replica %d out of range", replica);
  if (slot < 0 || slot >= x->num_slots) return fail(x, SS_EINVAL, "worker slot %d out of range", slot);
  if (b->batch < 1 || b->batch > x->max_batch)
    return fail(x, SS_EINVAL, "batch %d outside 1..%d", b->batch, x->max_batch);
  if (b->num_ids < 0 || b->num_ids > x->max_ids)
    return fail(x, SS_EINVAL, "num_ids %lld outside 0..%lld", (long long)b->num_ids, (long long)x->max_ids);
  if (!b->dense || !b->labels || !b->offsets || (!b->indices && b->num_ids))
    return fail(x, SS_EINVAL, "null batch buffer");
  return SS_OK;
}

// bf16 models with at least one hidden top layer run the one-unit output layer and the loss
// (and that layer's backward) as fused kernels instead of GEMMs with a single column.
// bf16 models run the one-unit output layer, the loss and dL/dlogit in one kernel
static bool fused_last(const ss_ctx* x) { return x->prec == SS_BF16; }

// ---- fused-MLP path -------------------------------------------------------------------------
static void fill_stack(const ss_ctx* x, const Slot& s, const float* w, int l0, int n,
                       FusedLayer* out) {
  for (int i = 0; i < n; ++i) {
    const Layer& ly = x->layers[l0 + i];
    out[i].Wf = s.wsw + x->wsw_f[l0 + i]; out[i].Wr = s.wsw + x->wsw_r[l0 + i];
    out[i].b = w + ly.b_off; out[i].in = ly.in; out[i].out = ly.out;
    out[i].kp_f = x->kp_f[l0 + i]; out[i].depth_f = x->depth_f[l0 + i];
    out[i].kp_r = x->kp_r[l0 + i]; out[i].depth_r = x->depth_r[l0 + i];
  }
}

// Training steps: the gather also writes the plan of the step's sort into the slot.
static SortPlanOut sort_plan_of(const Slot& s, const ss_batch* bt, bool train) {
  if (!train || bt->num_ids <= 0) return SortPlanOut{nullptr, nullptr, 0};
  return SortPlanOut{s.sort.seg_lo, s.sort.tile_base, sort_tile((uint32_t)bt->num_ids)};
}

static void launch_weight_snapshot(ss_ctx* x, Slot& s, const float* w, bool train,
                                   const ss_batch* cast_dense, hipStream_t st);

static void forward_fused(ss_ctx* x, Slot& s, const float* w, const ss_batch* bt, float* loss,
                          bool train, hipStream_t st) {
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers, nh = x->n_top_layers - 1;
  {
    ProfScope ps(x, SS_K_MLP, st);
    launch_weight_snapshot(x, s, w, train, nullptr, st);
    FusedFwdArgs a{};
    a.n_layers = nb; fill_stack(x, s, w, 0, nb, a.L);
    a.B = B; a.ldT = x->ldT;
    a.x = bt->dense; a.x_is_f32 = 1; a.ldx = x->num_dense; a.in0 = x->num_dense;
    a.xT = train ? s.xT : nullptr;
    for (int l = 0; l < nb; ++l) a.actT[l] = s.actT[l];
    a.out_f32 = s.z0; a.relu_last = 1; a.has_tail = 0;
    a.kp_tail = (x->layers[nb - 1].out + 63) / 64 * 64;
    a.lds_elems0 = (unsigned)x->e0_fwd_bot;
    { ProfScope pk(x, SS_K_MLP_FWD, st); launch_mlp_fused_fwd(a, x->lds_fwd_bot, st); }
  }
  {
    ProfScope ps(x, SS_K_GATHER, st);
    launch_embedding_bag_fwd(x->h, bt->indices, bt->offsets, x->meta, B, x->T, x->d, s.e,
                             train ? s.keys : nullptr, s.bag_of_pos, loss, x->pool_mean ? s.inv_len : nullptr, x->row_shards,
                             s.e_part, sort_plan_of(s, bt, train), st);
  }
  {
    ProfScope ps(x, SS_K_INTERACT_FWD, st);
    launch_interaction_fwd(s.z0, s.e, B, x->T, x->d, s.f, x->ldf, s.f_bf16, x->ldf16, st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    FusedFwdArgs a{};
    a.n_layers = nh; fill_stack(x, s, w, nb, nh, a.L);
    a.B = B; a.ldT = x->ldT;
    a.x = s.f_bf16; a.x_is_f32 = 0; a.ldx = x->ldf16; a.in0 = x->F;
    a.xT = train ? s.fT : nullptr;
    for (int l = 0; l < nh; ++l) a.actT[l] = s.actT[nb + l];
    a.out_f32 = nullptr; a.relu_last = 1; a.has_tail = 1;
    a.kp_tail = (x->layers[nb + nh - 1].out + 63) / 64 * 64;
    const Layer& last = x->layers[L - 1];
    a.w_last = w + last.w_off; a.b_last = w + last.b_off; a.y = bt->labels;
    a.logits = s.logits; a.dlogit = train ? s.dlogit : nullptr; a.loss = loss;
    a.lds_elems0 = (unsigned)x->e0_fwd_top;
    { ProfScope pk(x, SS_K_MLP_FWD, st); launch_mlp_fused_fwd(a, x->lds_fwd_top, st); }
  }
}

static void backward_fused(ss_ctx* x, Slot& s, const float* w, const ss_batch* bt, hipStream_t st) {
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers, nh = x->n_top_layers - 1;
  {
    ProfScope ps(x, SS_K_MLP, st);
    FusedBwdArgs a{};  // (the gradient accumulator was cleared by the step's prep launch)
    a.n_layers = nh; fill_stack(x, s, w, nb, nh, a.L);
    a.B = B; a.ldT = x->ldT;
    const Layer& last = x->layers[L - 1];
    a.dlogit = s.dlogit; a.w_last = w + last.w_off;
    a.g_w_last = s.grads + last.w_off; a.g_b_last = s.grads + last.b_off;
    for (int l = 0; l < nh; ++l) { a.actT[l] = s.actT[nb + l]; a.dYT[l] = s.dYT[nb + l]; }
    a.d_out_f32 = s.df; a.ld_d_out = x->ldf;
    a.lds_elems0 = (unsigned)x->e0_bwd_top;
    { ProfScope pk(x, SS_K_MLP_DGRAD, st); launch_mlp_fused_bwd(a, x->lds_bwd_top, st); }
  }
  {
    ProfScope ps(x, SS_K_INTERACT_BWD, st);
    launch_interaction_bwd(s.z0, s.e, s.df, x->ldf, B, x->T, x->d, s.dz0, s.de, nullptr, 0, st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    FusedBwdArgs a{};
    a.n_layers = nb; fill_stack(x, s, w, 0, nb, a.L);
    a.B = B; a.ldT = x->ldT;
    a.d_in_f32 = s.dz0; a.ld_d_in = x->d;
    for (int l = 0; l < nb; ++l) { a.actT[l] = s.actT[l]; a.dYT[l] = s.dYT[l]; }
    a.d_out_f32 = nullptr;
    a.lds_elems0 = (unsigned)x->e0_bwd_bot;
    { ProfScope pk(x, SS_K_MLP_DGRAD, st); launch_mlp_fused_bwd(a, x->lds_bwd_bot, st); }
    WgradArgs g{};
    for (int l = 0; l < nb + nh; ++l) {
      const Layer& ly = x->layers[l];
      g.L[l].dYT = s.dYT[l];
      g.L[l].XT = (l == 0) ? s.xT : (l == nb) ? s.fT : s.actT[l - 1];
      g.L[l].gW = s.grads + ly.w_off; g.L[l].gb = s.grads + ly.b_off;
      g.L[l].in = ly.in; g.L[l].out = ly.out;
    }
    g.tiles = x->wgrad_tiles_dev; g.B = B; g.ldT = x->ldT;
    { ProfScope pk(x, SS_K_MLP_WGRAD, st); launch_mlp_wgrad_grouped(g, (int)x->wgrad_tiles.size(), st); }
  }
}

// ---- layer-wise path ------------------------------------------------------------------------
// this step's snapshot of the replica: bf16, MFMA fragment order, both products (also clears
// the step's gradient accumulator when training)
static void launch_weight_snapshot(ss_ctx* x, Slot& s, const float* w, bool train,
                                   const ss_batch* cast_dense, hipStream_t st) {
  const int nl = (int)x->layers.size() - 1;
  PrepArgs pa{};
  pa.n_layers = nl;
  int64_t base = 0;
  for (int l = 0; l < nl; ++l) {
    const Layer& ly = x->layers[l];
    PrepLayer& pl = pa.L[l];
    pl.W = w + ly.w_off; pl.Wf = s.wsw + x->wsw_f[l]; pl.Wr = s.wsw + x->wsw_r[l];
    pl.in = ly.in; pl.out = ly.out; pl.frag_base = base;
    pl.kp_f = x->kp_f[l]; pl.kp_r = x->kp_r[l];
    pl.frags_fwd = (x->wsw_r[l] - x->wsw_f[l]) / 8;
    const int64_t end = (l + 1 < nl) ? x->wsw_f[l + 1] : x->wsw_elems;
    base += (end - x->wsw_f[l]) / 8;
  }
  pa.total_frags = base;
  pa.zero = train ? s.grads : nullptr;
  pa.zero_n = x->wide ? x->Pstride + (int64_t)LAST_GRAD_COPIES * x->last_stride : x->P;
  if (cast_dense) {   // layer-wise path: the dense input as bf16 rows of the first GEMM's pitch
    pa.cast_src = cast_dense->dense; pa.cast_dst = s.xb;
    pa.cast_rows = cast_dense->batch; pa.cast_cols = x->num_dense; pa.cast_ld = x->pin[0];
  }
  launch_mlp_prep(pa, st);
}

static void forward_wide(ss_ctx* x, Slot& s, const float* w, const ss_batch* bt, float* loss,
                         bool train, hipStream_t st) {
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers;
  auto layer_fwd = [&](int l, const uint16_t* in, int ld_in) {
    const Layer& ly = x->layers[l];
    GemmXwArgs a{};
    a.A = in; a.lda = ld_in; a.Bf = s.wsw + x->wsw_f[l];
    a.M = B; a.N = ly.out; a.K = x->kp_f[l];
    a.epi = EPI_BIAS | EPI_RELU; a.bias = w + ly.b_off;
    if (l == nb - 1) { a.C_f32 = s.z0; a.ldc32 = x->d; }
    else { a.C = s.act_bf16[l]; a.ldc = x->pout[l]; }
    { ProfScope pk(x, SS_K_MLP_FWD, st); launch_gemm_xw(a, st); }
  };
  {
    ProfScope ps(x, SS_K_MLP, st);
    launch_weight_snapshot(x, s, w, train, bt, st);
    const uint16_t* in = s.xb; int ld_in = x->pin[0];
    for (int l = 0; l < nb; ++l) {
      layer_fwd(l, in, ld_in);
      in = s.act_bf16[l]; ld_in = x->pout[l];
    }
  }
  {
    ProfScope ps(x, SS_K_GATHER, st);
    launch_embedding_bag_fwd(x->h, bt->indices, bt->offsets, x->meta, B, x->T, x->d, s.e,
                             train ? s.keys : nullptr, s.bag_of_pos, loss, x->pool_mean ? s.inv_len : nullptr, x->row_shards,
                             s.e_part, sort_plan_of(s, bt, train), st);
  }
  {
    ProfScope ps(x, SS_K_INTERACT_FWD, st);
    launch_interaction_fwd(s.z0, s.e, B, x->T, x->d, s.f, x->ldf, s.f_bf16, x->ldf16, st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    const uint16_t* in = s.f_bf16; int ld_in = x->ldf16;
    for (int l = nb; l < L - 1; ++l) {
      layer_fwd(l, in, ld_in);
      in = s.act_bf16[l]; ld_in = x->pout[l];
    }
    const Layer& last = x->layers[L - 1];
    if (!train) {
      launch_last_layer_fwd_loss(in, ld_in, w + last.w_off, w + last.b_off, bt->labels, B, last.in,
                                 s.logits, nullptr, loss, st);
    } else if (L - 1 == nb) {
      // training: the output unit's forward, loss and backward are one launch.  Without a
      // hidden top layer it reads the interaction output and its data gradient is the fp32
      // gradient w.r.t. that output (no gate: f is no ReLU output)
      launch_last_layer_train(in, ld_in, w + last.w_off, w + last.b_off, bt->labels, B, last.in,
                              s.logits, s.dlogit, loss, nullptr, 0, s.df, x->ldf,
                              s.grads + x->Pstride, x->last_stride, st);
    } else {
      launch_last_layer_train(in, ld_in, w + last.w_off, w + last.b_off, bt->labels, B, last.in,
                              s.logits, s.dlogit, loss, s.dYr[L - 2], x->pout[L - 2], nullptr, 0,
                              s.grads + x->Pstride, x->last_stride, st);
    }
  }
}

static void backward_wide(ss_ctx* x, Slot& s, float* w_rw, const float* loss, const ss_batch* bt,
                          hipStream_t st) {
  const float* w = w_rw;
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers;
  // gradient w.r.t. the input of layer l from the gradient w.r.t. its output (dYr[l])
  auto layer_dgrad = [&](int l) {
    const Layer& ly = x->layers[l];
    GemmXwArgs a{};
    a.A = s.dYr[l]; a.lda = x->pout[l]; a.Bf = s.wsw + x->wsw_r[l];
    a.M = B; a.N = ly.in; a.K = x->kp_r[l]; a.role = 1;
    if (l == nb) {
      a.C_f32 = s.df; a.ldc32 = x->ldf; a.epi = EPI_NONE;
    } else {
      a.C = s.dYr[l - 1]; a.ldc = x->pout[l - 1];
      a.epi = EPI_MASK; a.mask = s.act_bf16[l - 1]; a.ldmask = x->pout[l - 1];
    }
    { ProfScope pk(x, SS_K_MLP_DGRAD, st); launch_gemm_xw(a, st); }
  };
  {
    ProfScope ps(x, SS_K_MLP, st);  // (the gradient accumulator was cleared by the weight snapshot)
    // (the output unit's backward ran with its forward: launch_last_layer_train)
    for (int l = L - 2; l >= nb; --l) layer_dgrad(l);
  }
  {
    ProfScope ps(x, SS_K_INTERACT_BWD, st);
    launch_interaction_bwd(s.z0, s.e, s.df, x->ldf, B, x->T, x->d, s.dz0, s.de,
                           s.dYr[nb - 1], x->pout[nb - 1], st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    for (int l = nb - 1; l >= 1; --l) layer_dgrad(l);
    // weight and bias gradients of every layer but the one-unit output layer: one grouped
    // launch over (layer, tile, batch slice), then one launch that adds the slices up
    WgradGroupArgs g{};
    ReduceArgs red{};
    int red_blocks = 0;
    const int slices = ceil_div(B, x->wg_slice_len);   // slices that hold samples of this batch
    for (int l = 0; l < L - 1; ++l) {
      const Layer& ly = x->layers[l];
      WgradGroupLayer& q = g.L[l];
      q.dY = s.dYr[l]; q.ldy = x->pout[l];
      if (l == 0) { q.X = s.xb; q.ldx = x->pin[0]; }
      else if (l == nb) { q.X = s.f_bf16; q.ldx = x->ldf16; }
      else { q.X = s.act_bf16[l - 1]; q.ldx = x->pout[l - 1]; }
      q.part = s.wg_part + x->wg_off[l]; q.part_stride = x->wg_stride[l];
      q.out = ly.out; q.in = ly.in; q.slice_len = x->wg_slice_len;
      ReduceSegment& sg = red.seg[red.n_seg++];
      sg.part = q.part; sg.out = s.grads + ly.w_off; sg.n = (int64_t)ly.out * ly.in + ly.out;
      sg.stride = q.part_stride; sg.slices = slices; sg.block_base = red_blocks;
      red_blocks += ceil_div(sg.n, 1024);
    }
    g.tiles = x->wgrad_tiles_dev; g.n_tiles = (int)x->wgrad_tiles.size(); g.B = B;
    { ProfScope pk(x, SS_K_MLP_WGRAD, st); launch_gemm_wgrad(g, st); }
    // the reduction is also the step's SGD update of the replica ("update local param w^(i)":
    // lock-free) and feeds the Train-NE accumulators; the output unit's gradients, left in
    // partial copies by its own launch, ride along as one more segment
    const Layer& last = x->layers[L - 1];
    ReduceSegment& lg = red.seg[red.n_seg++];
    lg.part = s.grads + x->Pstride; lg.out = s.grads + last.w_off; lg.n = (int64_t)last.in + 1;
    lg.stride = x->last_stride; lg.slices = LAST_GRAD_COPIES; lg.block_base = red_blocks;
    red_blocks += ceil_div(lg.n, 1024);
    for (int k = 0; k < red.n_seg; ++k) red.seg[k].w = w_rw + (red.seg[k].out - s.grads);
    red.lr = x->lr_dense; red.mean_loss = loss; red.y = bt->labels; red.B = B; red.acc = x->metrics;
    launch_reduce_slices(red, red_blocks, st);
  }
}

// ---- fp32 path: every layer one GEMM on the vector units -------------------------------------
static void forward_f32(ss_ctx* x, Slot& s, const float* w, const ss_batch* bt, float* loss,
                        bool train, hipStream_t st) {
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers;
  (void)loss;
  {
    ProfScope ps(x, SS_K_MLP, st);
    const float* in = bt->dense; int ld_in = x->num_dense;
    for (int l = 0; l < nb; ++l) {
      const Layer& ly = x->layers[l];
      float* out = (l == nb - 1) ? s.z0 : s.act_f32[l];
      launch_gemm_f32(in, ld_in, 1, w + ly.w_off, 1, ly.in, out, ly.out, B, ly.out, ly.in,
                      EPI_BIAS | EPI_RELU, w + ly.b_off, nullptr, 0, st);
      in = out; ld_in = ly.out;
    }
  }
  // look-ups (pooled where the table lives) and interaction
  {
    ProfScope ps(x, SS_K_GATHER, st);
    launch_embedding_bag_fwd(x->h, bt->indices, bt->offsets, x->meta, B, x->T, x->d, s.e,
                             train ? s.keys : nullptr, s.bag_of_pos, nullptr,
                             x->pool_mean ? s.inv_len : nullptr, x->row_shards, s.e_part, sort_plan_of(s, bt, train), st);
  }
  {
    ProfScope ps(x, SS_K_INTERACT_FWD, st);
    launch_interaction_fwd(s.z0, s.e, B, x->T, x->d, s.f, x->ldf, nullptr, 0, st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    const float* in = s.f; int ld_in = x->ldf;
    for (int l = nb; l < L; ++l) {
      const Layer& ly = x->layers[l];
      const bool last = (l == L - 1);
      float* out = last ? s.logits : s.act_f32[l];
      launch_gemm_f32(in, ld_in, 1, w + ly.w_off, 1, ly.in, out, ly.out, B, ly.out, ly.in,
                      last ? EPI_BIAS : (EPI_BIAS | EPI_RELU), w + ly.b_off, nullptr, 0, st);
      in = out; ld_in = ly.out;
    }
  }
}

static void backward_f32(ss_ctx* x, Slot& s, const float* w, const ss_batch* bt, hipStream_t st) {
  const int B = bt->batch, L = (int)x->layers.size(), nb = x->n_bot_layers;
  // layers l_hi .. l_lo from the gradient d0 w.r.t. the output of layer l_hi
  auto run_layers = [&](int l_hi, int l_lo, const float* d0, int ldd0) {
    const float* dcur = d0; int ldd = ldd0; int pp = 0;
    for (int l = l_hi; l >= l_lo; --l) {
      const Layer& ly = x->layers[l];
      const float* xin; int ldx;
      if (l == 0) { xin = bt->dense; ldx = x->num_dense; }
      else if (l == nb) { xin = s.f; ldx = x->ldf; }
      else { xin = s.act_f32[l - 1]; ldx = x->layers[l - 1].out; }
      launch_gemm_f32(dcur, 1, ldd, xin, ldx, 1, s.grads + ly.w_off, ly.in, ly.out, ly.in, B,
                      EPI_NONE, nullptr, nullptr, 0, st);
      launch_col_sum_f32(dcur, ldd, B, ly.out, s.grads + ly.b_off, st);
      if (l != 0) {
        const bool to_df = (l == nb);            // gradient w.r.t. the interaction output
        float* out = to_df ? s.df : s.dbuf[pp];
        const int ldo = to_df ? x->ldf : ly.in;
        launch_gemm_f32(dcur, ldd, 1, w + ly.w_off, ly.in, 1, out, ldo, B, ly.in, ly.out,
                        to_df ? EPI_NONE : EPI_MASK, nullptr, to_df ? nullptr : xin, ldx, st);
        dcur = out; ldd = ldo; pp ^= 1;
      }
    }
  };
  {
    ProfScope ps(x, SS_K_MLP, st);
    run_layers(L - 1, nb, s.dlogit, 1);
  }
  {
    ProfScope ps(x, SS_K_INTERACT_BWD, st);
    launch_interaction_bwd(s.z0, s.e, s.df, x->ldf, B, x->T, x->d, s.dz0, s.de, nullptr, 0, st);
  }
  {
    ProfScope ps(x, SS_K_MLP, st);
    run_layers(nb - 1, 0, s.dz0, x->d);
  }
}

static int train_or_eval(ss_ctx* x, int replica, int slot, const ss_batch* bt, void* stream,
                         float* dev_loss_out, bool train) {
  if (!x) return SS_EINVAL;
  int rc = check_batch(x, replica, slot, bt);
  if (rc != SS_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  Slot& s = x->slots[slot];
  float* w = x->W + (size_t)replica * x->Pstride;
  const int B = bt->batch;
  const uint32_t n = (uint32_t)bt->num_ids;
  float* loss = dev_loss_out ? dev_loss_out : s.loss;
  if (x->fused) forward_fused(x, s, w, bt, loss, train, st);
  else if (x->wide) forward_wide(x, s, w, bt, loss, train, st);
  else forward_f32(x, s, w, bt, loss, train, st);
  if (!fused_last(x)) launch_bce_loss(s.logits, bt->labels, B, loss, train ? s.dlogit : nullptr, st);
  s.last_B = B;
  s.last_n = n;
  if (!train) launch_metrics(loss, bt->labels, B, x->metrics + 4, st);
  if (train) {
    s.sort_n = n;
    if (x->fused) backward_fused(x, s, w, bt, st);
    else if (x->wide) backward_wide(x, s, w, loss, bt, st);
    else backward_f32(x, s, w, bt, st);
    // "update local param w^(i)": lock-free SGD on the replica (the layer-wise path's last
    // kernel has already applied it)
    if (!x->wide) launch_sgd(w, s.grads, x->P, x->lr_dense, loss, bt->labels, B, x->metrics, st);
    // "update h": stable sort by row, one Adagrad update per distinct row
    {
      ProfScope ps(x, SS_K_SORT, st);
      // the value carried through the passes is the pooled-vector id of the position: equal
      // rows keep the order of their positions (stable), and the update needs nothing else
      const SortSegments seg{x->T, &x->meta, x->sort_digit_bits};   // (the tables' ranges: planned by the gather)
      launch_sort_pairs(s.keys, (const uint32_t*)s.bag_of_pos, n, seg, s.sort, &s.sorted_keys,
                        &s.sorted_bag, st);
      s.seg_valid = false;  // compacted segment starts are produced on demand (ss_read_debug)
    }
    const EmbOpt opt{x->h, x->G, x->M, x->V, x->lr_emb, x->eps, x->beta1, x->beta2, x->adam ? 1 : 0};
    {
      ProfScope all(x, SS_K_ROW_UPDATE, st);
      {
        ProfScope ps(x, SS_K_ROW_UPDATE_CHUNK, st);
        launch_row_update_chunk(s.sorted_keys, (const int32_t*)s.sorted_bag, s.de, n, s.upd, x->d, opt,
                                x->pool_mean ? s.inv_len : nullptr, st);
      }
      launch_row_update_finish(s.sorted_keys, n, s.upd, x->d, opt, st);
    }
    s.trained = true;
    x->steps[replica].fetch_add(1);
    x->examples.fetch_add((uint64_t)B);
  }
  return check_hip(x, hipGetLastError(), train ? "ss_train_step" : "ss_eval_step");
}

extern "C" {

int ss_train_step(ss_ctx* ctx, int32_t replica, int32_t worker_slot, const ss_batch* batch,
                  void* stream, float* dev_loss_out) {
  return train_or_eval(ctx, replica, worker_slot, batch, stream, dev_loss_out, true);
}

int ss_eval_step(ss_ctx* ctx, int32_t replica, int32_t worker_slot, const ss_batch* batch,
                 void* stream, float* dev_loss_out) {
  return train_or_eval(ctx, replica, worker_slot, batch, stream, dev_loss_out, false);
}

int ss_eval_step_static(ss_ctx* ctx, int32_t replica, const ss_batch* batch, void* stream,
                        float* dev_loss_out, float* dev_logits_out) {
  if (!ctx) return SS_EINVAL;
  int rc = check_batch(ctx, replica, 0, batch);
  if (rc != SS_OK) return rc;
  if (!dev_loss_out) return fail(ctx, SS_EINVAL, "ss_eval_step_static: dev_loss_out must not be NULL");
  // forward-only scratch for exactly this batch, laid out in the static array
  Slot s;
  Carver sizing(nullptr);
  carve_slot(ctx, sizing, s, batch->batch, batch->num_ids, true);
  const size_t need = (sizing.off + ALIGN - 1) / ALIGN * ALIGN;
  if (need > STATIC_SCRATCH_BYTES)
    return fail(ctx, SS_ENOMEM,
                "ss_eval_step_static: a batch of %d needs %zu bytes of scratch, the static array "
                "holds %zu (use ss_eval_step with a worker slot)",
                batch->batch, need, STATIC_SCRATCH_BYTES);
  hipStream_t st = (hipStream_t)stream;
  Carver cv(ctx->static_scratch);
  carve_slot(ctx, cv, s, batch->batch, batch->num_ids, true);
  // the array keeps the last call's contents, and the layer-wise kernels read the pitch padding
  // of their operands: the part this call uses starts from zero (a fill kernel, so that the
  // call may be captured into a graph)
  launch_fill_f32((float*)ctx->static_scratch, (uint64_t)(need / 4), 0.f, st);
  if (dev_logits_out) s.logits = dev_logits_out;
  const float* w = ctx->W + (size_t)replica * ctx->Pstride;
  if (ctx->fused) forward_fused(ctx, s, w, batch, dev_loss_out, false, st);
  else if (ctx->wide) forward_wide(ctx, s, w, batch, dev_loss_out, false, st);
  else forward_f32(ctx, s, w, batch, dev_loss_out, false, st);
  if (!fused_last(ctx)) launch_bce_loss(s.logits, batch->labels, batch->batch, dev_loss_out, nullptr, st);
  launch_metrics(dev_loss_out, batch->labels, batch->batch, ctx->metrics + 4, st);
  return check_hip(ctx, hipGetLastError(), "ss_eval_step_static");
}

// ------------------------------------------------------------------------------------------
int ss_sync_round(int32_t algo, int32_t K, int64_t P, int64_t stride, float* dev_replicas,
                  float* dev_w_ps, float* dev_w_global, float* dev_v, float alpha, float eta,
                  float momentum, void* stream) {
  if (algo < SS_EASGD || algo > SS_BMUF_NESTEROV || K < 1 || K > 16 || P < 1 || (P & 3) ||
      stride < P || (stride & 3) || !dev_replicas)
    return SS_EINVAL;
  const bool easgd = (algo == SS_EASGD || algo == SS_EASGD_LITERAL);
  if (easgd && !dev_w_ps) return SS_EINVAL;
  if (!easgd && !dev_w_global) return SS_EINVAL;
  if ((algo == SS_BMUF || algo == SS_BMUF_NESTEROV) && !dev_v) return SS_EINVAL;
  uintptr_t al = (uintptr_t)dev_replicas | (uintptr_t)dev_w_ps | (uintptr_t)dev_w_global |
                 (uintptr_t)dev_v;
  if (al & 15) return SS_EINVAL;
  launch_sync_round(algo, K, P, stride, dev_replicas, dev_w_ps, dev_w_global, dev_v, alpha, eta,
                    momentum, (hipStream_t)stream);
  return hipGetLastError() == hipSuccess ? SS_OK : SS_EDEVICE;
}

static int sync_once(ss_ctx* x, int algo, float alpha, float eta, float mu, hipStream_t st) {
  {
    ProfScope ps(x, SS_K_SYNC, st);
    // vectors are padded to Pstride (multiple of 256 floats); the pad is carried along
    launch_sync_round(algo, x->K, x->Pstride, x->Pstride, x->W, x->w_ps, x->w_global, x->v, alpha,
                      eta, mu, st);
  }
  x->rounds.fetch_add(1);
  return check_hip(x, hipGetLastError(), "ss_shadow_sync");
}

int ss_shadow_sync(ss_ctx* ctx, int32_t algo, float alpha, float eta, float momentum, void* stream) {
  if (!ctx) return SS_EINVAL;
  if (ctx->sticky) return SS_EDEVICE;
  if (algo < SS_EASGD || algo > SS_BMUF_NESTEROV) return fail(ctx, SS_EINVAL, "unknown sync rule %d", algo);
  if (ctx->shadow_run) return fail(ctx, SS_ESTATE, "shadow loop is running");
  return sync_once(ctx, algo, alpha, eta, momentum, (hipStream_t)stream);
}

int ss_easgd_exchange(ss_ctx* ctx, int32_t algo, int32_t replica, float alpha, void* stream) {
  if (!ctx) return SS_EINVAL;
  if (ctx->sticky) return SS_EDEVICE;
  if (algo != SS_EASGD && algo != SS_EASGD_LITERAL)
    return fail(ctx, SS_EINVAL, "ss_easgd_exchange: rule %d is not an EASGD rule", algo);
  if (replica < 0 || replica >= ctx->K) return fail(ctx, SS_EINVAL, "replica %d out of range", replica);
  hipStream_t st = (hipStream_t)stream;
  {
    ProfScope ps(ctx, SS_K_SYNC, st);
    launch_sync_round(algo, 1, ctx->Pstride, ctx->Pstride, ctx->W + (size_t)replica * ctx->Pstride,
                      ctx->w_ps, nullptr, nullptr, alpha, 1.f, 0.f, st);
  }
  ctx->exchanges.fetch_add(1);
  return check_hip(ctx, hipGetLastError(), "ss_easgd_exchange");
}

int ss_shadow_start(ss_ctx* ctx, int32_t algo, float alpha, float eta, float momentum, void* stream) {
  if (!ctx) return SS_EINVAL;
  if (algo < SS_EASGD || algo > SS_BMUF_NESTEROV) return fail(ctx, SS_EINVAL, "unknown sync rule %d", algo);
  if (ctx->shadow_run.exchange(true)) return fail(ctx, SS_ESTATE, "shadow loop already running");
  hipStream_t st = (hipStream_t)stream;
  ctx->shadow = std::thread([ctx, algo, alpha, eta, momentum, st]() {
    if (hipSetDevice(ctx->device) != hipSuccess) { ctx->sticky = 1; return; }
    // Algorithm 1, shadow loop (Section 3.2): rounds follow one another, uncoupled from the workers
    auto next = std::chrono::steady_clock::now();
    while (ctx->shadow_run.load()) {
      if (sync_once(ctx, algo, alpha, eta, momentum, st) != SS_OK) break;
      if (hipStreamSynchronize(st) != hipSuccess) { ctx->sticky = 1; break; }
      const int64_t period = ctx->shadow_period_us.load(std::memory_order_relaxed);
      if (period > 0) {
        // rounds START at least `period` apart; sleep in short slices so that a stop request
        // is seen promptly
        next += std::chrono::microseconds(period);
        const auto now = std::chrono::steady_clock::now();
        if (next < now) next = now;
        while (ctx->shadow_run.load() && std::chrono::steady_clock::now() < next) {
          const auto left = next - std::chrono::steady_clock::now();
          std::this_thread::sleep_for(left > std::chrono::microseconds(200)
                                          ? std::chrono::microseconds(200)
                                          : std::chrono::duration_cast<std::chrono::microseconds>(left));
        }
      }
    }
  });
  return SS_OK;
}

int ss_shadow_pace(ss_ctx* ctx, int64_t min_period_us) {
  if (!ctx) return SS_EINVAL;
  if (min_period_us < 0) return fail(ctx, SS_EINVAL, "shadow period must be >= 0");
  ctx->shadow_period_us = min_period_us;
  return SS_OK;
}

int ss_shadow_stop(ss_ctx* ctx) {
  if (!ctx) return SS_EINVAL;
  if (!ctx->shadow_run.exchange(false)) {
    if (ctx->shadow.joinable()) ctx->shadow.join();
    return SS_OK;
  }
  if (ctx->shadow.joinable()) ctx->shadow.join();
  return ctx->sticky ? SS_EDEVICE : SS_OK;
}

// ------------------------------------------------------------------------------------------
int ss_read_debug(ss_ctx* ctx, int32_t worker_slot, int32_t item, void* host_out, size_t bytes,
                  size_t* size_out) {
  if (!ctx) return SS_EINVAL;
  if (worker_slot < 0 || worker_slot >= ctx->num_slots) return fail(ctx, SS_EINVAL, "bad slot");
  Slot& s = ctx->slots[worker_slot];
  HIP_TRY(ctx, hipDeviceSynchronize());
  const size_t B = (size_t)s.last_B, n = s.last_n, ns = s.sort_n;
  const void* src = nullptr; size_t size = 0; size_t pitch_src = 0, width = 0, rows = 0;
  uint32_t U = 0;
  if (item == SS_DBG_SEG_STARTS || item == SS_DBG_NUM_UNIQUE) {
    if (!s.trained) return fail(ctx, SS_ESTATE, "no training step has run on this slot yet");
    if (!s.seg_valid) {
      // the row update works on the runs of equal keys directly; the compacted list of run
      // starts is derived from the same sorted keys when somebody asks for it
      launch_segment_starts(s.sorted_keys, s.sort_n, s.seg, nullptr);
      HIP_TRY(ctx, hipDeviceSynchronize());
      s.seg_valid = true;
    }
    HIP_TRY(ctx, hipMemcpy(&U, s.seg.num_unique, 4, hipMemcpyDeviceToHost));
  }
  if (item == SS_DBG_SORTED_POS) {
    // The step's sort carries pooled-vector ids, not positions.  The positions come from
    // sorting the step's keys (kept) once more with each element's own position as its value:
    // the same stable passes, so the same permutation.  The step's sorted arrays are rebuilt
    // afterwards (the passes share their buffers).
    if (!s.trained) return fail(ctx, SS_ESTATE, "no training step has run on this slot yet");
    if (size_out) *size_out = ns * 4;
    if (!host_out || bytes == 0 || ns == 0) return SS_OK;
    uint32_t *k = nullptr, *v = nullptr;
    // (the tables' position ranges are those the step's own sort left in its plan)
    const SortSegments seg{ctx->T, &ctx->meta, ctx->sort_digit_bits};
    launch_sort_pairs(s.keys, nullptr, s.sort_n, seg, s.sort, &k, &v, nullptr);
    HIP_TRY(ctx, hipDeviceSynchronize());
    HIP_TRY(ctx, hipMemcpy(host_out, v, bytes < ns * 4 ? bytes : ns * 4, hipMemcpyDeviceToHost));
    launch_sort_pairs(s.keys, (const uint32_t*)s.bag_of_pos, s.sort_n, seg, s.sort,
                      &s.sorted_keys, &s.sorted_bag, nullptr);
    HIP_TRY(ctx, hipDeviceSynchronize());
    return SS_OK;
  }
  const int L = (int)ctx->layers.size();
  if (item >= SS_DBG_HIDDEN_ACT && item < SS_DBG_HIDDEN_ACT + L) {
    // hidden activations live in a path-specific layout (fp32 or bf16, row-major with a padded
    // pitch, or transposed [unit][sample]); they are brought to float [B, out] on the host
    const int l = item - SS_DBG_HIDDEN_ACT;
    if (l == ctx->n_bot_layers - 1 || l == L - 1)
      return fail(ctx, SS_EINVAL, "layer %d has no hidden activation buffer", l);
    const size_t out = (size_t)ctx->layers[l].out;
    const size_t sz = B * out * 4;
    if (size_out) *size_out = sz;
    if (!host_out || bytes == 0 || sz == 0) return SS_OK;
    if (bytes < sz) return fail(ctx, SS_EINVAL, "buffer too small for a hidden activation");
    float* dst = (float*)host_out;
    if (ctx->prec == SS_FP32) {
      HIP_TRY(ctx, hipMemcpy(dst, s.act_f32[l], sz, hipMemcpyDeviceToHost));
      return SS_OK;
    }
    const bool transposed = ctx->fused;
    const size_t pitch = transposed ? (size_t)ctx->ldT : (ctx->wide ? (size_t)ctx->pout[l] : out);
    const size_t n_rows = transposed ? out : B;
    std::vector<uint16_t> raw(n_rows * pitch);
    HIP_TRY(ctx, hipMemcpy(raw.data(), transposed ? s.actT[l] : s.act_bf16[l], raw.size() * 2,
                           hipMemcpyDeviceToHost));
    for (size_t b = 0; b < B; ++b)
      for (size_t u = 0; u < out; ++u) {
        const uint32_t bits = (uint32_t)(transposed ? raw[u * pitch + b] : raw[b * pitch + u]) << 16;
        memcpy(&dst[b * out + u], &bits, 4);
      }
    return SS_OK;
  }
  switch (item) {
    case SS_DBG_Z0: src = s.z0; size = B * ctx->d * 4; break;
    case SS_DBG_POOLED_PARTIALS:
      if (ctx->row_shards <= 1) return fail(ctx, SS_ESTATE, "the tables are not row-sharded");
      src = s.e_part; size = (size_t)ctx->row_shards * B * ctx->T * ctx->d * 4; break;
    case SS_DBG_POOLED: src = s.e; size = B * ctx->T * ctx->d * 4; break;
    case SS_DBG_INTERACT: src = s.f; rows = B; width = (size_t)ctx->F * 4; pitch_src = (size_t)ctx->ldf * 4; size = rows * width; break;
    case SS_DBG_LOGITS: src = s.logits; size = B * 4; break;
    case SS_DBG_DENSE_GRAD: src = s.grads; size = (size_t)ctx->P * 4; break;
    case SS_DBG_POOLED_GRAD: src = s.de; size = B * ctx->T * ctx->d * 4; break;
    case SS_DBG_SORTED_ROWS: src = s.sorted_keys; size = ns * 4; break;
    case SS_DBG_SORTED_BAG: src = s.sorted_bag; size = ns * 4; break;
    case SS_DBG_SEG_STARTS: src = s.seg.seg_starts; size = (size_t)U * 4; break;
    case SS_DBG_NUM_UNIQUE: src = s.seg.num_unique; size = 4; break;
    case SS_DBG_BAG_OF_POS: src = s.bag_of_pos; size = ns * 4; break;
    default: return fail(ctx, SS_EINVAL, "unknown debug item %d", item);
  }
  if (size_out) *size_out = size;
  if (!host_out || bytes == 0 || size == 0) return SS_OK;
  if (!src) return fail(ctx, SS_ESTATE, "no step has run on this slot yet");
  if (rows) {
    if (bytes < size) return fail(ctx, SS_EINVAL, "buffer too small for a strided item");
    HIP_TRY(ctx, hipMemcpy2D(host_out, width, src, pitch_src, width, rows, hipMemcpyDeviceToHost));
  } else {
    HIP_TRY(ctx, hipMemcpy(host_out, src, bytes < size ? bytes : size, hipMemcpyDeviceToHost));
  }
  return SS_OK;
}

int ss_metrics_read(ss_ctx* ctx, int32_t which, double* host_out4) {
  if (!ctx || !host_out4) return SS_EINVAL;
  if (which != 0 && which != 1) return fail(ctx, SS_EINVAL, "metrics selector must be 0 (train) or 1 (eval)");
  HIP_TRY(ctx, hipDeviceSynchronize());
  double acc[4];
  HIP_TRY(ctx, hipMemcpy(acc, ctx->metrics + 4 * which, sizeof acc, hipMemcpyDeviceToHost));
  const double n = acc[2];
  const double nan = std::nan("");
  host_out4[0] = n;
  host_out4[1] = n > 0 ? acc[0] / n : nan;
  host_out4[2] = n > 0 ? acc[1] / n : nan;
  const double p = host_out4[2];
  host_out4[3] = (n > 0 && p > 0.0 && p < 1.0)
                     ? host_out4[1] / -(p * std::log(p) + (1.0 - p) * std::log(1.0 - p))
                     : nan;
  return SS_OK;
}

int ss_metrics_reset(ss_ctx* ctx, int32_t which) {
  if (!ctx) return SS_EINVAL;
  if (which != 0 && which != 1) return fail(ctx, SS_EINVAL, "metrics selector must be 0 (train) or 1 (eval)");
  HIP_TRY(ctx, hipDeviceSynchronize());
  HIP_TRY(ctx, hipMemset(ctx->metrics + 4 * which, 0, 4 * sizeof(double)));
  HIP_TRY(ctx, hipDeviceSynchronize());
  return SS_OK;
}

int ss_get_counters(ss_ctx* ctx, uint64_t* steps_per_replica, uint64_t* rounds, uint64_t* examples) {
  if (!ctx) return SS_EINVAL;
  if (steps_per_replica)
    for (int i = 0; i < ctx->K; ++i) steps_per_replica[i] = ctx->steps[i].load();
  if (rounds) *rounds = ctx->rounds.load();
  if (examples) *examples = ctx->examples.load();
  return SS_OK;
}

int ss_profile_arm(ss_ctx* ctx, uint32_t kernel_mask) {
  if (!ctx) return SS_EINVAL;
  if (kernel_mask >> SS_K_COUNT) return fail(ctx, SS_EINVAL, "bad kernel mask");
  std::lock_guard<std::mutex> lk(ctx->prof_mu);
  for (int id = 1; id < SS_K_COUNT; ++id) {
    if (!(kernel_mask & (1u << id))) continue;
    auto& pool = ctx->prof[id];
    if (pool.ev.empty()) {
      pool.ev.resize(4096);
      for (auto& p : pool.ev) {
        HIP_TRY(ctx, hipEventCreate(&p.first));
        HIP_TRY(ctx, hipEventCreate(&p.second));
      }
    }
    pool.used = 0;
    ctx->prof_seen[id] = 0;
  }
  ctx->prof_mask = kernel_mask & ~1u;
  return SS_OK;
}

int ss_profile_sample(ss_ctx* ctx, int32_t every) {
  if (!ctx) return SS_EINVAL;
  if (every < 1) return fail(ctx, SS_EINVAL, "sampling interval must be >= 1");
  for (int id = 0; id < SS_K_COUNT; ++id) ctx->prof_every[id] = (uint32_t)every;
  return SS_OK;
}

int ss_profile_sample_class(ss_ctx* ctx, int32_t kernel_id, int32_t every) {
  if (!ctx) return SS_EINVAL;
  if (kernel_id < 1 || kernel_id >= SS_K_COUNT) return fail(ctx, SS_EINVAL, "bad kernel id");
  if (every < 1) return fail(ctx, SS_EINVAL, "sampling interval must be >= 1");
  ctx->prof_every[kernel_id] = (uint32_t)every;
  return SS_OK;
}

int ss_profile_read(ss_ctx* ctx, int32_t kernel_id, int64_t* launches, double* total_ms) {
  if (!ctx) return SS_EINVAL;
  if (kernel_id < 1 || kernel_id >= SS_K_COUNT) return fail(ctx, SS_EINVAL, "bad kernel id");
  HIP_TRY(ctx, hipDeviceSynchronize());
  std::lock_guard<std::mutex> lk(ctx->prof_mu);
  ctx->prof_mask = ctx->prof_mask.load() & ~(1u << kernel_id);
  auto& pool = ctx->prof[kernel_id];
  double tot = 0;
  for (size_t i = 0; i < pool.used; ++i) {
    float ms = 0;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, pool.ev[i].first, pool.ev[i].second));
    tot += ms;
  }
  if (launches) *launches = (int64_t)pool.used;
  if (total_ms) *total_ms = tot;
  pool.used = 0;
  return SS_OK;
}

}  // extern "C"
