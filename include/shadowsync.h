/*
 * shadowsync.h — C ABI of the MI355X (gfx950) ShadowSync hot-path library.
 *
 * One trainer's click-through-rate training step (ShadowSync, arXiv 2003.03477,
 * Section 3.1 "Trainer" and Section 3.2 "Optimization Strategies") and the background
 * ("shadow") synchronisation of Algorithms 1-4 over K dense-parameter replicas that all
 * live in the HBM of one GPU.  The calls follow Algorithm 1: initialise the tables h and
 * the replicas w^(i) (and w^PS / w^global); a worker iteration = ss_train_step(replica,
 * batch) = "update h; update w^(i)"; a shadow iteration = ss_shadow_sync(algo, ...) =
 * "sync w^(i)"; after training read back h and w^(1) (Section 4, "Experimental Setup").
 *
 * Conventions
 *  - Every function returns SS_OK (0) or a negative ss_status; text via ss_last_error().
 *    No exception or C++ type crosses this boundary.
 *  - "dev" pointers are device (HBM) addresses, "host" pointers are host addresses.
 *  - The library allocates NO device memory: the caller passes one workspace of
 *    ss_workspace_bytes() bytes (256-byte aligned) that must outlive the context, and
 *    owns every batch buffer.  The library owns only the host-side ss_ctx.
 *  - All device work is enqueued asynchronously on the hipStream_t passed as `stream`
 *    (cast to void*; NULL = the default stream).  ss_read_* synchronise the device.
 *  - Thread safety: ss_train_step may be called concurrently from different host threads
 *    with different worker slots; two calls on one slot must be ordered by the caller
 *    (same stream, or an event).  Concurrent steps race on h and on w^(replica) exactly as
 *    the paper's lock-free worker threads do.  Shape errors are reported; the CONTENT of
 *    indices/offsets is not validated on the hot path (rows must be < rows[t], offsets
 *    non-decreasing with offsets[0] = 0 and offsets[T*B] = num_ids).
 *
 * Dense parameter vector (exposed by ss_read_dense / ss_init_dense): bottom-MLP layers then
 * top-MLP layers, each W[out][in] row-major followed by b[out]; P floats, no padding.
 */
#ifndef SHADOWSYNC_H
#define SHADOWSYNC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ss_ctx ss_ctx;

typedef enum {
  SS_OK = 0,
  SS_EINVAL = -1,  /* bad shape, index or argument                                   */
  SS_ENOMEM = -2,  /* workspace too small                                            */
  SS_EDEVICE = -3, /* a HIP call failed; sticky for the context                      */
  SS_ESTATE = -4   /* call not valid in the current state (e.g. shadow loop running) */
} ss_status;

/* Synchronisation rule of one shadow round. */
typedef enum {
  SS_EASGD = 0,         /* Algorithm 2, symmetric elastic exchange (conserves mass)   */
  SS_MA = 1,            /* Algorithm 3                                               */
  SS_BMUF = 2,          /* Algorithm 4 with optional block momentum                  */
  SS_EASGD_LITERAL = 3, /* Algorithm 2 with its two lines executed one after another */
  SS_BMUF_NESTEROV = 4  /* Algorithm 4 with Nesterov block momentum: v and w^global as in
                           SS_BMUF, replicas pulled towards w^global + momentum * v        */
} ss_algo;

typedef enum { SS_FP32 = 0, SS_BF16 = 1 } ss_mlp_prec;

/* Pooling of a bag's rows (Section 3.1): SS_POOL_SUM adds them, SS_POOL_MEAN (the pooling of
 * the paper's example) divides the sum by the bag's length; the gradient of every member then
 * carries 1 / length. */
typedef enum { SS_POOL_SUM = 0, SS_POOL_MEAN = 1 } ss_pooling;

/* Which bf16 MLP kernels run the model.  SS_MLP_AUTO picks by layer width: the per-sample-tile
 * fused kernels when every width is <= 512, the layer-wise 128x128-tile MFMA GEMMs otherwise.
 * SS_MLP_LAYERWISE forces the layer-wise GEMMs for any width.  Ignored under SS_FP32. */
typedef enum { SS_MLP_AUTO = 0, SS_MLP_LAYERWISE = 1 } ss_mlp_path;

/* Optimiser of the embedding tables (Section 3.2, "Embedding Tables: Hogwild Updates": lock-free
 * updates with the optimiser's auxiliary state co-located with the rows; the section names
 * Adagrad and Adam).  SS_OPT_ROWWISE_ADAGRAD: one accumulator per row, G += mean_c g^2,
 * h -= lr g / (sqrt(G) + eps).  SS_OPT_ADAM: first and second moments per element, one step
 * count per row; a row's state advances only in the steps that touch it (t_r += 1;
 * m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; h -= lr (m / (1-b1^t_r)) / (sqrt(v / (1-b2^t_r)) + eps)).
 * Either way the gradients of all occurrences of a row in the batch are summed first and the
 * row gets one update per step. */
typedef enum { SS_OPT_ROWWISE_ADAGRAD = 0, SS_OPT_ADAM = 1 } ss_emb_optimizer;

typedef struct {
  int32_t num_tables;        /* T, 1..64                                                  */
  const int64_t* rows;       /* host [T] rows per table; sum < 2^32                      */
  int32_t emb_dim;           /* d: 16, 32, 64 or 128                                     */
  int32_t num_dense;         /* width of the dense-feature input                        */
  int32_t n_bot;             /* entries in bot_dims (layers + 1)                        */
  const int32_t* bot_dims;   /* host, e.g. {13,256,128,64}; last must equal emb_dim     */
  int32_t n_top;             /* entries in top_dims                                     */
  const int32_t* top_dims;   /* host, e.g. {100,512,256,1}; first must equal
                                emb_dim + T(T+1)/2 and last must be 1                    */
  int32_t num_replicas;      /* K >= 1 dense replicas w^(i)                              */
  int32_t max_batch;         /* largest batch any step will pass                        */
  int64_t max_ids;           /* largest num_ids any step will pass (< 2^31)             */
  int32_t num_worker_slots;  /* concurrent ss_train_step callers (private scratch each) */
  int32_t mlp_prec;          /* ss_mlp_prec: SS_BF16 rounds the inputs of every MLP GEMM
                                to bfloat16 (fp32 accumulate, fp32 master weights)       */
  float lr_dense;            /* SGD step on w^(i)                                        */
  float lr_emb;              /* row-wise Adagrad step on h                               */
  float adagrad_eps;
  uint64_t seed;             /* seed of the counter-based table initialiser             */
  int32_t pooling;           /* ss_pooling                                               */
  int32_t mlp_path;          /* ss_mlp_path                                              */
  int32_t emb_optimizer;     /* ss_emb_optimizer; lr_emb and adagrad_eps serve both      */
  float adam_beta1;          /* SS_OPT_ADAM only (0 <= beta < 1)                         */
  float adam_beta2;
  int32_t emb_row_shards;    /* 0 or 1: tables are not split.  S > 1 (Section 3.1, "Embedding
                                PS": a table too large for one server is split by rows, each
                                part pools what it owns, the trainer adds the partial results):
                                every table is cut into S equal row ranges, the look-up pools
                                per range and a second kernel adds the S partial vectors in
                                range order                                              */
  int32_t sort_digit_bits;   /* widest digit of a pass of the stable radix sort that orders the
                                batch's (row, position) pairs for the table update: 8, 9 or 10;
                                0 picks the default (8: wider digits take fewer passes, but
                                each pass scatters into shorter runs and measured slower on
                                both configured workloads).  A table whose local rows take b
                                bits is sorted in ceil(b / this) passes of equal width; the
                                sorted order does not depend on it                         */
} ss_config;

/* One mini-batch.  All pointers are DEVICE pointers owned by the caller and must stay
 * valid until the step's stream work has completed.  Table-major CSR: bag (t, b) is
 * indices[offsets[t*batch + b] .. offsets[t*batch + b + 1]).  An empty bag pools to 0. */
typedef struct {
  int32_t batch;           /* B <= max_batch                                            */
  int64_t num_ids;         /* n = offsets[T*B] <= max_ids (host copy of that value)     */
  const float* dense;      /* dev [B, num_dense] row-major                              */
  const float* labels;     /* dev [B], 0 or 1                                           */
  const int32_t* indices;  /* dev [n], row within its table                             */
  const int32_t* offsets;  /* dev [T*B + 1]                                             */
} ss_batch;

/* Placement of the tables on embedding parameter servers (host only, no device work; Section
 * 3.1, "Embedding PS": every table's look-up cost is profiled and the tables are bin-packed so
 * that the servers carry similar costs; tables too large for one server are partitioned).
 * Tables with more than max_rows_per_shard rows (> 0) are cut into ceil(rows / limit) equal row
 * ranges whose cost is their share of the table's; the parts are packed by the
 * longest-processing-time rule (decreasing cost, each to the least loaded server, ties to the
 * lower index).  out_shards (host, capacity entries) receives the parts in (table, first row)
 * order, *out_num_shards their number (also when capacity is too small: SS_ENOMEM),
 * out_ps_cost (host [num_ps], may be NULL) the cost per server. */
typedef struct {
  int32_t table;
  int64_t first_row;
  int64_t rows;
  double cost;
  int32_t ps;
} ss_shard;
int ss_plan_placement(int32_t num_tables, const int64_t* rows, const double* cost, int32_t num_ps,
                      int64_t max_rows_per_shard, ss_shard* out_shards, int32_t capacity,
                      int32_t* out_num_shards, double* out_ps_cost);

/* Device bytes ss_init needs for this configuration (0 on an invalid configuration). */
size_t ss_workspace_bytes(const ss_config* cfg);

/* Algorithm 1, initialisation: lay out h (+ Adagrad state), the K replicas, w^PS,
 * w^global, the momentum buffer and the per-slot scratch inside `dev_workspace`; zero the
 * optimiser state.  Runs on the current HIP device; synchronous.  */
int ss_init(const ss_config* cfg, void* dev_workspace, size_t bytes, ss_ctx** out);
void ss_destroy(ss_ctx* ctx);
const char* ss_last_error(const ss_ctx* ctx); /* NULL ctx: error of the last failed ss_init */

/* h <- h0 for every table from the counter-based hash of (seed, table, row, column):
 * value = (u24 - 2^23) * (0.05 * 2^-23), u24 = top 24 bits of
 * mix64(mix64(seed ^ (1000+table)*0xD1B54A32D192ED03) + (row*d+col)*0x9E3779B97F4A7C15),
 * mix64 = the splitmix64 output function.  Also zeroes the Adagrad accumulators. */
int ss_init_tables_hash(ss_ctx* ctx, void* stream);

/* h[table, first_row .. first_row+n_rows) <- host values [n_rows, d]; accumulators of
 * those rows <- 0.  Synchronous. */
int ss_write_rows(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                  const float* host_rows);
/* Adagrad accumulators G of the same row range <- host values [n_rows] (restoring a saved
 * optimiser state; Section 3.2 keeps this state beside the rows).  Synchronous. */
int ss_write_adagrad(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                     const float* host_acc);

/* SS_OPT_ADAM: moments of the same row range <- host values [n_rows, d] each (either may be
 * NULL); the rows' step counts are written with ss_write_adagrad.  Synchronous. */
int ss_write_adam_state(ss_ctx* ctx, int32_t table, int64_t first_row, int64_t n_rows,
                        const float* host_m, const float* host_v);

/* Algorithm 1: w^(i) <- w0 for all i, w^PS <- w0, w^global <- w0 (Algorithms 3, 4), v <- 0.
 * host_w0 holds P floats.  Synchronous. */
int ss_init_dense(ss_ctx* ctx, const float* host_w0);

/* Number of dense parameters P of the configured model. */
int64_t ss_num_params(const ss_ctx* ctx);

/* One worker iteration for one batch on replica `replica` (Algorithm 1 worker loop;
 * Section 3.1 "Trainer"): bottom MLP, sum-pooled look-ups, pairwise-dot interaction, top
 * MLP, mean log-loss, backward, then w^(replica) -= lr_dense * grad (lock-free) and one
 * row-wise Adagrad update per distinct touched row of h with the gradients of all its
 * occurrences summed first (stable sort by row, segmented reduction).
 * dev_loss_out (device, 1 float, may be NULL) receives the mean log-loss BEFORE the update. */
int ss_train_step(ss_ctx* ctx, int32_t replica, int32_t worker_slot, const ss_batch* batch,
                  void* stream, float* dev_loss_out);

/* Forward pass only: mean log-loss of replica `replica` on the batch, nothing is updated
 * (the quantity whose ratio to the label entropy is the paper's NE, Section 4). */
int ss_eval_step(ss_ctx* ctx, int32_t replica, int32_t worker_slot, const ss_batch* batch,
                 void* stream, float* dev_loss_out);

/* ss_eval_step for callers that cannot allocate and hold no worker slot (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the forward pass keeps its
 * activations in a static device array of the library (8 MiB per GPU, held until the process
 * ends) instead of a worker slot's part of the workspace.  The call allocates nothing and uses
 * no memset node.  dev_loss_out (device, 1 float, required) receives the batch's mean log-loss,
 * dev_logits_out (device, [batch] floats, may be NULL) the logits; the eval NE accumulator is
 * advanced as by ss_eval_step.  Returns SS_ENOMEM, with the sizes in ss_last_error, when the
 * batch's activations (and the model's bf16 weight snapshot) exceed the array.  All calls on
 * one GPU share the array: calls that overlap in time -- on different streams, contexts or
 * host threads -- race; order them on one stream. */
int ss_eval_step_static(ss_ctx* ctx, int32_t replica, const ss_batch* batch, void* stream,
                        float* dev_loss_out, float* dev_logits_out);

/* One shadow round over all K replicas, i ascending, element-wise (Algorithms 2-4):
 *  SS_EASGD: for each i: delta = alpha (w^(i) - w^PS); w^PS += delta; w^(i) -= delta
 *  SS_MA:    w^global = mean_i w^(i); w^(i) = (1-alpha) w^(i) + alpha w^global
 *  SS_BMUF:  m = mean_i w^(i); v = momentum v + eta (m - w^global); w^global += v;
 *            w^(i) = (1-alpha) w^(i) + alpha w^global
 *  SS_BMUF_NESTEROV: v and w^global as in SS_BMUF;
 *            w^(i) = (1-alpha) w^(i) + alpha (w^global + momentum v)
 * eta and momentum are used by SS_BMUF and SS_BMUF_NESTEROV only.  One fused, memory-bound
 * kernel. */
int ss_shadow_sync(ss_ctx* ctx, int32_t algo, float alpha, float eta, float momentum,
                   void* stream);

/* Algorithm 2 for ONE trainer: the elastic exchange of w^(replica) with w^PS only (what a
 * single trainer's shadow thread does per iteration; a round of ss_shadow_sync(SS_EASGD) is
 * this for replica 0..K-1 in order).  algo is SS_EASGD or SS_EASGD_LITERAL.  Enqueued on
 * `stream`: the shadow stream for background sync, or a worker's own stream for the
 * foreground variant (FR-EASGD, Section 4) in which the worker syncs every k iterations. */
int ss_easgd_exchange(ss_ctx* ctx, int32_t algo, int32_t replica, float alpha, void* stream);

/* The same round on caller-owned device vectors (no context needed): `dev_replicas` holds
 * K vectors of P floats, vector i starting at dev_replicas + i*stride (stride >= P,
 * multiple of 4; all pointers 16-byte aligned).  dev_w_ps is used by the EASGD rules,
 * dev_w_global by MA/BMUF, dev_v by BMUF; unused ones may be NULL.  K <= 16. */
int ss_sync_round(int32_t algo, int32_t K, int64_t P, int64_t stride, float* dev_replicas,
                  float* dev_w_ps, float* dev_w_global, float* dev_v, float alpha, float eta,
                  float momentum, void* stream);

/* Algorithm 1's shadow thread (shadow loop; Section 3.2): a host thread owned by the context
 * that enqueues rounds on `stream` one after another, with no coupling to the worker
 * iterations, until ss_shadow_stop.  The stream must not be used by the caller while the loop
 * runs. */
int ss_shadow_start(ss_ctx* ctx, int32_t algo, float alpha, float eta, float momentum,
                    void* stream);
int ss_shadow_stop(ss_ctx* ctx);
/* Pace of the shadow loop: the thread starts rounds at least min_period_us apart (0, the
 * default: back to back).  The paper's loop is paced by its network (Section 4.2 reports one
 * round per 5-12 trainer iterations); inside one HBM a round is a single short kernel, and
 * this is the knob that sets the average sync gap.  May be changed while the loop runs. */
int ss_shadow_pace(ss_ctx* ctx, int64_t min_period_us);

/* Read-back (synchronises the device first).  which: 0..K-1 = w^(which), -1 = w^PS,
 * -2 = w^global, -3 = v, -4 = the mean of the K replicas, computed on the device at the time
 * of the call (Section 4, "Experimental Setup": the model returned is the first trainer's
 * copy, which = 0; the replica average is the alternative).  n must equal P.
 * ss_write_dense accepts 0..K-1, -1, -2, -3. */
int ss_read_dense(ss_ctx* ctx, int32_t which, float* host_out, int64_t n);
int ss_write_dense(ss_ctx* ctx, int32_t which, const float* host_in, int64_t n);
/* rows: host [n] row ids of `table`; host_rows_out [n, d] and host_adagrad_out [n] may
 * each be NULL.  Under SS_OPT_ADAM host_adagrad_out receives the rows' step counts and
 * ss_read_adam_state the moments ([n, d] each, either may be NULL). */
int ss_read_rows(ss_ctx* ctx, int32_t table, const int64_t* rows, int64_t n,
                 float* host_rows_out, float* host_adagrad_out);
int ss_read_adam_state(ss_ctx* ctx, int32_t table, const int64_t* rows, int64_t n,
                       float* host_m_out, float* host_v_out);

/* Intermediates of the LAST step run on a worker slot, for element-wise checks
 * (synchronises first).  Forward results (pooled vectors, interaction, logits, activations)
 * are those of the last ss_train_step OR ss_eval_step; the index work (sorted rows and
 * positions, segment starts, bag ids) and the gradients are those of the last ss_train_step.  Copies min(bytes, size) bytes; returns the full size in bytes
 * through *size_out (may be NULL). */
typedef enum {
  SS_DBG_POOLED = 0,       /* float  [B, T, d]   pooled embeddings e                       */
  SS_DBG_INTERACT = 1,     /* float  [B, F]      interaction output f                      */
  SS_DBG_LOGITS = 2,       /* float  [B]                                                    */
  SS_DBG_DENSE_GRAD = 3,   /* float  [P]         gradient of the mean loss w.r.t. w         */
  SS_DBG_POOLED_GRAD = 4,  /* float  [B, T, d]   de                                         */
  SS_DBG_SORTED_ROWS = 5,  /* uint32 [n]         global row (row_base[t]+row), ascending    */
  SS_DBG_SORTED_POS = 6,   /* uint32 [n]         flat position of each sorted entry (made on
                              demand: the step's keys sorted once more with positions as
                              the values; the step itself carries SS_DBG_SORTED_BAG)      */
  SS_DBG_SEG_STARTS = 7,   /* uint32 [U]         sorted index where each distinct row starts */
  SS_DBG_NUM_UNIQUE = 8,   /* uint32 [1]         U                                          */
  SS_DBG_BAG_OF_POS = 9,   /* int32  [n]         b*T + t of each flat position              */
  SS_DBG_Z0 = 10,          /* float  [B, d]      output of the bottom MLP (after its ReLU)  */
  SS_DBG_POOLED_PARTIALS = 11, /* float [S, B, T, d] partial pooling results per row shard
                                  (sums, before any 1/length factor); emb_row_shards > 1   */
  SS_DBG_SORTED_BAG = 12,  /* int32  [n]         b*T + t of each sorted entry: the values the
                              step's sort carries (the update sums de[b, t, :] of a row's
                              entries in this order)                                       */
  SS_DBG_HIDDEN_ACT = 32   /* SS_DBG_HIDDEN_ACT + l: float [B, out_l], output of hidden layer l
                              (layers counted over the whole model, bottom first; not the
                              bottom output, not the logit) as the device stores it, i.e.
                              after ReLU and, under SS_BF16, after rounding to bfloat16      */
} ss_debug_item;
int ss_read_debug(ss_ctx* ctx, int32_t worker_slot, int32_t item, void* host_out, size_t bytes,
                  size_t* size_out);

/* Counters (Section 4: EPS; Section 4.1: average sync gap = trainer iterations per sync).
 * steps_per_replica: host [K]; any pointer may be NULL. */
int ss_get_counters(ss_ctx* ctx, uint64_t* steps_per_replica, uint64_t* rounds,
                    uint64_t* examples);

/* Normalised entropy (Section 4, "Evaluation Metrics"): NE = mean log-loss / entropy of the
 * empirical click rate of the same examples.  The library keeps two running accumulators on
 * the device: which = 0, TRAIN -- every ss_train_step adds its batch's log-loss BEFORE the update
 * (each example is predicted by a model that has not yet trained on it: the paper's
 * progressive Train NE); which = 1, EVAL -- every ss_eval_step adds its batch.
 * ss_metrics_read synchronises the device and fills out[0..3] = number of examples, mean
 * log-loss, click rate, NE (NaN while the click rate is 0 or 1, or no example was seen).
 * ss_metrics_reset zeroes one accumulator (synchronous). */
int ss_metrics_read(ss_ctx* ctx, int32_t which, double* host_out4);
int ss_metrics_reset(ss_ctx* ctx, int32_t which);

/* Kernel timing with HIP events recorded on the launching stream.  ss_profile_arm takes a bit
 * mask (bit i = ss_kernel_id i); from then on every launch of an armed class is bracketed by
 * an event pair (at most 4096 brackets per class); ss_profile_sample(every) thins that to every
 * `every`-th launch of each armed class (default 1), which keeps the cost of the brackets out
 * of a timed run.  ss_profile_read synchronises the device,
 * returns the number of brackets of one class and their summed duration in ms, and disarms
 * that class.  Classes marked "one kernel" bracket exactly one kernel launch, so their average
 * is comparable with a profiler's per-kernel average; the others bracket a group of launches. */
typedef enum {
  SS_K_NONE = 0,
  SS_K_GATHER = 1,            /* one kernel: embedding gather + sum pooling                  */
  SS_K_SORT = 2,              /* group: all radix-sort passes of a step                      */
  SS_K_ROW_UPDATE_CHUNK = 3,  /* one kernel: chunk pass of the segmented reduction + Adagrad */
  SS_K_SYNC = 4,              /* one kernel: one shadow round                                */
  SS_K_MLP = 5,               /* group: MLP kernels (bottom fwd / top fwd / top bwd / bottom bwd) */
  SS_K_INTERACT_FWD = 6,      /* one kernel                                                  */
  SS_K_INTERACT_BWD = 7,      /* one kernel                                                  */
  SS_K_ROW_UPDATE = 8,        /* group: chunk + stitch + long-run passes                     */
  SS_K_MLP_FWD = 9,           /* one kernel: each forward MFMA launch of the bf16 fused and
                                 layer-wise paths (a layer's GEMM, or a fused stack)         */
  SS_K_MLP_DGRAD = 10,        /* one kernel: each data-gradient MFMA launch                  */
  SS_K_MLP_WGRAD = 11,        /* one kernel: each weight-gradient MFMA launch                */
  SS_K_COUNT = 12
} ss_kernel_id;
int ss_profile_arm(ss_ctx* ctx, uint32_t kernel_mask);
int ss_profile_sample(ss_ctx* ctx, int32_t every);
/* the same for one class (a step launches some classes once and others a dozen times) */
int ss_profile_sample_class(ss_ctx* ctx, int32_t kernel_id, int32_t every);
int ss_profile_read(ss_ctx* ctx, int32_t kernel_id, int64_t* launches, double* total_ms);

#ifdef __cplusplus
}
#endif
#endif /* SHADOWSYNC_H */
