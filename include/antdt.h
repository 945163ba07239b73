/*
 * antdt.h — C boundary of the MI355X (gfx950) library for one bulk-synchronous
 * Parameter-Server training iteration of a ranking model.
 *
 * The calls follow the iteration as the AntDT paper states it (Section II,
 * Problem Formulation): given the fixed global batch B, worker i computes its
 * local gradient on its local batch B_i and pushes it (antdt_worker_step); the
 * servers aggregate the local gradients of all workers (antdt_aggregate) and
 * update the parameters (antdt_apply_update).  Which samples a worker gets is a
 * shard = (start offset, length) pair (Section V-C.1) produced by
 * antdt_assign_shard; the lengths always add up to B (constraint of Eq. 1).
 * On one device the K workers are K contiguous slices of the global batch and
 * the pull/push communication of the paper's model has no counterpart.
 *
 * Conventions
 *  - Every pointer marked DEVICE is device memory owned by the caller (for
 *    example a torch tensor's data_ptr); HOST pointers are ordinary host memory
 *    read or written before the call returns.  The library never allocates,
 *    frees or retains device memory other than the buffers handed to
 *    antdt_bind / antdt_set_batch, which must stay valid while in use.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    GPU calls enqueue their kernels on it and return without synchronising
 *    unless stated otherwise.  Calls on one context must not overlap.
 *  - Every function returns ANTDT_OK or a negative error code; a message is kept
 *    per context (antdt_last_error).  Nothing throws, nothing aborts.
 *  - Row ids outside [0, rows_per_field) and non-monotone bag offsets are caller
 *    errors with undefined results.  An empty bag pools to zeros and receives
 *    no gradient.  An empty shard (length 0) is legal and contributes nothing.
 */
#ifndef ANTDT_H_
#define ANTDT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ANTDT_MAX_LAYERS 8
#define ANTDT_MAX_FIELDS 128
#define ANTDT_MAX_SHARDS 64
#define ANTDT_STATIC_SCRATCH_BYTES (32u << 20) /* scratch of antdt_bind_static, per device */

enum {
  ANTDT_OK = 0,
  ANTDT_INVALID_ARG = -1,         /* null pointer, size out of range, sizes not summing to B ... */
  ANTDT_BAD_STATE = -2,           /* call order violated (see each call) */
  ANTDT_WORKSPACE_TOO_SMALL = -3,
  ANTDT_HIP_ERROR = -4,           /* a HIP runtime call failed; message holds hipGetErrorString */
  ANTDT_UNSUPPORTED = -5,
  ANTDT_INFEASIBLE = -6,          /* a planning problem has no solution within its bounds */
  ANTDT_EMPTY = -7                /* the shard queue holds no waiting shard */
};

enum { ANTDT_F32 = 0, ANTDT_BF16 = 1 };
enum { ANTDT_STATE_ELEMENTWISE = 0, ANTDT_STATE_ROWWISE = 1 };
enum { ANTDT_POOL_SUM = 0, ANTDT_POOL_MEAN = 1 };

typedef struct antdt_ctx antdt_ctx; /* opaque; holds host metadata only */

/*
 * Model descriptor (plain data, copied by antdt_create).
 *
 * Input vector of a sample = [pooled embedding of field 0 | ... | field F-1 |
 * dense features], width layer_sizes[0] = num_fields*dim + num_dense.  The MLP
 * has num_layers weight layers; hidden layers apply ReLU, the last layer is
 * linear with a single output (layer_sizes[num_layers] == 1, the logit of a
 * binary cross-entropy loss).
 *
 * Flat parameter layout (mlp_params, mlp_state, every dense gradient): for
 * layer l = 0..num_layers-1, W_l as [layer_sizes[l], layer_sizes[l+1]]
 * row-major, then b_l [layer_sizes[l+1]].
 */
typedef struct antdt_model {
  int32_t num_fields;       /* F, 1..ANTDT_MAX_FIELDS */
  int64_t rows_per_field;   /* R, < 2^31 */
  int32_t dim;              /* D: a power of two, 4..256, with D*sizeof(element) >= 16 bytes */
  int32_t table_dtype;      /* ANTDT_F32 or ANTDT_BF16: element type of the embedding tables */
  int32_t adagrad_state;    /* ELEMENTWISE: fp32 [F*R, D];  ROWWISE: fp32 [F*R] */
  int32_t num_dense;        /* dense features per sample (may be 0) */
  int32_t num_layers;       /* 1..ANTDT_MAX_LAYERS */
  int32_t layer_sizes[ANTDT_MAX_LAYERS + 1];
  int32_t gemm_dtype;       /* ANTDT_F32: fp32 FMA GEMMs.  ANTDT_BF16: hidden-layer GEMM operands
                               are bf16, accumulation fp32 (matrix cores); hidden widths must then
                               be multiples of 8 */
  float lr;                 /* Adagrad learning rate (tables and MLP) */
  float eps;                /* Adagrad epsilon, added to sqrt(state) */
  int32_t max_shards;       /* K_max, 1..ANTDT_MAX_SHARDS */
  int64_t max_batch;        /* largest global batch B */
  int64_t max_nnz;          /* largest total number of lookups (all fields) of one batch */
  int32_t pooling;          /* ANTDT_POOL_SUM: a bag is the sum of its rows.  ANTDT_POOL_MEAN: the sum
                               divided by the number of lookups of the bag (an empty bag is zeros);
                               each looked-up row then receives dX / bag length as its gradient */
} antdt_model;

/* Create / destroy a context.  Host work only.  INVALID_ARG on an inconsistent model. */
int antdt_create(const antdt_model* model, antdt_ctx** out);
int antdt_destroy(antdt_ctx* ctx);

/* Message of the last failed call on ctx (ctx == NULL: of the last failed antdt_create or
 * context-free call on this thread).  Never NULL. */
const char* antdt_last_error(const antdt_ctx* ctx);

/* Size in bytes of the scratch region antdt_bind needs (activations, per-shard gradients,
 * sort buffers, coalesced gradients, bf16 weight copies). */
int antdt_workspace_bytes(const antdt_ctx* ctx, size_t* bytes);

/*
 * Attach the caller's DEVICE buffers:
 *   tables      [F*R, D]  table_dtype, field f occupies rows [f*R, (f+1)*R)
 *   table_state fp32 [F*R, D] (element-wise) or [F*R] (row-wise)
 *   mlp_params  fp32, flat layout above;  mlp_state fp32, same layout
 *   workspace   256-byte aligned, >= antdt_workspace_bytes
 * Enqueues the conversion of the MLP weights to their bf16 operand copies when
 * gemm_dtype is BF16 (call again after changing mlp_params from outside).
 */
int antdt_bind(antdt_ctx* ctx, void* tables, float* table_state, float* mlp_params,
               float* mlp_state, void* workspace, size_t workspace_bytes, void* stream);

/*
 * antdt_bind for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): the same attachment of the caller's tables,
 * table_state, mlp_params and mlp_state (DEVICE, 16-byte aligned, as for antdt_bind), but the
 * workspace is a static device buffer inside the library, ANTDT_STATIC_SCRATCH_BYTES (32 MiB)
 * on every device the library is used on, held until the process ends.  The call and every later
 * call on the context allocate nothing: no hipMalloc / hipFree, no stream, no event.  All
 * kernels of the iteration are therefore enqueued on the caller's stream, one after the other
 * (antdt_bind's contexts run the sort and the weight gradients on streams of the library); the
 * results are the same.
 *   - ANTDT_WORKSPACE_TOO_SMALL when antdt_workspace_bytes(ctx) exceeds the buffer; the message
 *     names both sizes.  Nothing is touched in that case.
 *   - The buffer belongs to the device that is current at the call; the context must be used
 *     with that device current.
 *   - One buffer per device serves every context bound this way.  It keeps whatever the last
 *     user left in it; the library initialises every part before reading it, so nothing needs
 *     clearing.  Binding a second context takes the buffer away from the first: the first
 *     context's calls return ANTDT_BAD_STATE until it is bound again.  Two such contexts must
 *     not be used in overlapping calls or on streams that run concurrently: they would race
 *     on the buffer.
 *   - antdt_aggregate with a mask still waits for the stream once, antdt_validate_batch and the
 *     views still synchronise as documented; none of them allocates.
 */
int antdt_bind_static(antdt_ctx* ctx, void* tables, float* table_state, float* mlp_params,
                      float* mlp_state, void* stream);

/*
 * Present one global batch of B samples (B <= max_batch) in CSR form per field:
 *   ids       DEVICE int32 [field_ptr[F]]  lookups of field f at [field_ptr[f], field_ptr[f+1]),
 *                                          bags in sample order
 *   field_ptr HOST   int64 [F+1]           field_ptr[0] == 0, non-decreasing
 *   offsets   DEVICE int32 [F][B+1]        bag s of field f = lookups [offsets[f][s], offsets[f][s+1])
 *                                          relative to field_ptr[f]; offsets[f][B] == nnz_f
 *   dense     DEVICE fp32  [B, num_dense]  (may be NULL when num_dense == 0)
 *   labels    DEVICE fp32  [B]             0 or 1
 * Arrays without elements may be NULL (ids when there is no lookup; dense and labels when
 * B == 0, which is legal: every following call then runs and changes nothing).
 * Only pointers and sizes are recorded; nothing is copied.  Resets the iteration state.
 * Requires antdt_bind.
 */
int antdt_set_batch(antdt_ctx* ctx, const int32_t* ids, const int64_t* field_ptr,
                    const int32_t* offsets, const float* dense, const float* labels,
                    int64_t B, void* stream);

/*
 * Optional check of the batch given to antdt_set_batch (the other calls trust it: ids are
 * clamped into the table, offsets are followed as they are).  Launches a check kernel on
 * `stream` and waits for it.  ANTDT_INVALID_ARG, naming the lowest offending field, when an id
 * lies outside [0, rows_per_field) or a field's offsets do not start at 0, decrease, or do not
 * end at the field's lookup count.
 */
int antdt_validate_batch(antdt_ctx* ctx, void* stream);

/*
 * Split the global batch into K contiguous shards (start, length), worker order, lengths
 * summing to B (Section V-C.1; constraint of Eq. 1).  HOST work only.
 *   sizes != NULL : explicit B_k (>= 0, must sum to B);
 *   else speed != NULL : ADJUST_BS, Eq. 3 — integer B_k minimising max_k B_k / speed[k]
 *                   (speed[k] > 0, samples per second); ties go to the lowest k;
 *   else          : equal split B/K, the first B mod K shards one larger (Section VI-A, step 1).
 * start_out / len_out: HOST int64 [K], may be NULL.  The split is stored in ctx for the
 * following worker_step / aggregate calls.
 */
int antdt_assign_shard(antdt_ctx* ctx, int64_t B, int32_t K, const int64_t* sizes,
                       const double* speed, int64_t* start_out, int64_t* len_out);

/*
 * Worker k's local step on its shard (Section II: forward and backpropagation on B_k):
 * sum-pool the bags, MLP forward, mean binary cross-entropy over the shard, backward.
 * Produces, inside the workspace, the pooled inputs, the shard's dense gradient (mean over
 * the shard, flat layout) and d loss_k / d pooled-embedding for each of its samples — the
 * pair (ids, that gradient) is the shard's sparse gradient.  loss_out: DEVICE fp32 [1], may
 * be NULL.  Requires set_batch and assign_shard with matching B.
 * Everything is enqueued on `stream` except the weight gradients of the hidden layers, which the
 * library computes on a stream of its own, beside the rest of the backward pass or inside
 * antdt_apply_update (see antdt_set_eager_weight_gradients): the dense parameters are complete, in
 * the order of `stream`, after antdt_apply_update; antdt_view_shard_grads computes the per-shard
 * gradients if need be and waits for them on the host.
 */
int antdt_worker_step(antdt_ctx* ctx, int32_t k, float* loss_out, void* stream);

/* The same for all K shards in one batched pass of launches; loss_out DEVICE fp32 [K] or NULL.
 * Results per shard equal those of K antdt_worker_step calls. */
int antdt_worker_step_all(antdt_ctx* ctx, float* loss_out, void* stream);

/*
 * Server-side aggregation of the pushed gradients (Section II: the servers combine the
 * workers' gradients) of the included shards, weights w_k = B_k / sum of the included B_k:
 *   dense   g = sum_k w_k g_k;
 *   sparse  per field: the lookups of the included shards are sorted by row id; the distinct
 *           ids ascending (unique_ids), the start of each id's run (seg_offsets) and
 *           G[u, :] = sum over the run of w_k(sample) * d loss_k / d pooled[sample, field].
 * shard_mask: HOST uint8 [K], 0 = shard left out, as when the servers disregard the gradients
 * of the slowest workers (the backup-workers baseline, Section VII-A.3): its worker_step need
 * not have run, its lookups are not coalesced and the weights renormalise over the others;
 * NULL = all.  With a mask that leaves out a non-empty shard the call waits for `stream` once
 * (it reads the per-field lookup counts of the remaining shards back to plan the sort);
 * without one it only enqueues.
 * Requires worker_step for every included shard since the last set_batch / apply_update.
 */
int antdt_aggregate(antdt_ctx* ctx, const uint8_t* shard_mask, void* stream);

/*
 * Parameter update (Section II: the servers update the parameters): Adagrad with the aggregated
 * gradient, S += g^2 (row-wise state: S[r] += mean_d g[r,d]^2), p -= lr * g / (sqrt(S) + eps),
 * on the rows listed by the last aggregate only and on all MLP parameters; bf16 tables are
 * written back round-to-nearest-even; bf16 operand copies of the MLP weights are refreshed.
 * Requires antdt_aggregate.
 */
int antdt_apply_update(antdt_ctx* ctx, void* stream);

/*
 * Where the weight gradients of the hidden layers are computed.  By default (on == 0), with bf16
 * matrix products and a context bound by antdt_bind, antdt_worker_step leaves them out:
 * antdt_apply_update forms them inside the dense update (per shard in registers, weighted and
 * added up in shard order, then Adagrad; neither the per-shard nor the aggregated gradient is
 * written), and antdt_view_shard_grads / antdt_view_dense_grad compute the per-shard gradients
 * on request.  With on != 0 every antdt_worker_step computes its shards' weight gradients itself,
 * as K separate workers would before pushing them (Section II), and antdt_apply_update
 * aggregates what they wrote; the results agree to rounding.  Takes effect at the next
 * antdt_worker_step.  Host only.
 */
int antdt_set_eager_weight_gradients(antdt_ctx* ctx, int32_t on);

/*
 * on == 0: every kernel of the following iterations is enqueued on the caller's stream, one
 * after the other, although the context owns streams (the order a context bound by
 * antdt_bind_static always uses: per-kernel durations without overlap, captures of a whole
 * iteration on one stream).  on != 0 (the state after antdt_bind): the sort and run detection run
 * on a stream of the library beside the MLP, the weight-gradient work on another beside the
 * input-gradient product and the sparse update.  Results are the same.  To be called between
 * iterations (ANTDT_BAD_STATE while work of an iteration is outstanding).  Host only.
 */
int antdt_set_library_streams(antdt_ctx* ctx, int32_t on);

/*
 * Learning rate of the following antdt_apply_update calls (the ADJUST_LR global action of
 * Table II changes it between iterations; the optimizer state is kept).  lr finite, >= 0.
 * Host only.
 */
int antdt_set_lr(antdt_ctx* ctx, float lr);

/*
 * Per-worker factors c_k on the aggregation weights: w_k = c_k * B_k / sum_{included} B_j.  The
 * optimization-based methods of Section III (ADJUST_LR in Table II) give each worker a learning
 * rate of its own that penalises the lagging ones; with one server-side update this is a factor
 * on that worker's gradient.  The factors are not renormalised.  scale: host array of K values,
 * finite and >= 0; NULL resets all factors to 1 (the state after antdt_create).  They stay in
 * force until changed, also across antdt_set_batch and antdt_assign_shard (a worker index
 * beyond the K given here has factor 1).  May be called at any point before antdt_aggregate; when
 * it comes after antdt_worker_step_all, that aggregate rebuilds the lookup weights on its stream
 * instead of using the ones prepared beside the worker step.  Host only.
 */
int antdt_set_shard_scale(antdt_ctx* ctx, const double* scale, int32_t K);

/*
 * Plan for heterogeneous dedicated devices with gradient accumulation (Section VI-B, Eq. 4).
 * There are k device types; type i has n[i] devices of measured speed v[i] (samples per unit
 * of time).  Each device of type i computes C_i micro-batches of B_i samples in sequence
 * before the synchronisation.  Finds integers minimising  max_i C_i * B_i / v[i]  subject to
 *   sum_i n[i] * C_i * B_i = B,  bmin[i] <= B_i <= bmax[i],  cmin <= C_i <= cmax
 * (bmin: the saturation batch below which the batch time no longer falls; bmax: the memory
 * limit).  Exact: the counts are enumerated, the batch sizes found by bisection over the
 * candidate optimum values with an exact reachability table.  Among optimal plans the one
 * returned is unspecified.  All arrays HOST; B_out, C_out: [k]; z_out (optional): the optimum.
 * Limits: k <= 8, B <= 2^24, cmax <= 64, (cmax-cmin+1)^k <= 262144.
 * Returns ANTDT_INFEASIBLE when no plan satisfies the constraints.  Host only, no GPU work.
 */
int antdt_plan_accumulation(int64_t B, int32_t k, const int32_t* n, const double* v,
                            const int64_t* bmin, const int64_t* bmax, int32_t cmin, int32_t cmax,
                            int64_t* B_out, int32_t* C_out, double* z_out);

/*
 * The micro-batches of such a plan as shard sizes for antdt_assign_shard, device after device
 * (type 0's devices first), C_i consecutive shards of B_i samples per device of type i.  A
 * micro-batch is a shard: aggregating the shards with weights B_i / B equals accumulating each
 * device's micro-batch gradients and weighting the device by its share of B.
 * sizes_out, device_out (optional: index of the device a shard belongs to): HOST [cap];
 * count_out: number of shards written.  INVALID_ARG when cap is too small.
 */
int antdt_expand_accumulation(int32_t k, const int32_t* n, const int64_t* B_i, const int32_t* C_i,
                              int32_t cap, int64_t* sizes_out, int32_t* device_out,
                              int32_t* count_out);

/*
 * Shard queue with states (Section V-C, the stateful dynamic data sharding service: the shard
 * arithmetic of Section V-C.1, the states and the re-queue of Section V-C.3).  The N
 * samples of a data set are cut into K = ceil(N / (B*M)) shards of M batches, each a pair
 * (start offset, length); only the last may be short.  All shards start as TODO, in a queue in
 * index order.  antdt_dds_fetch hands the head of the queue to a worker (TODO -> DOING; EMPTY when
 * nothing waits).  antdt_dds_report_done marks a shard DONE once its worker has pushed its
 * gradients (BAD_STATE unless that worker holds the shard as DOING).  antdt_dds_release_worker is
 * for a worker that is lost (its gradients were disregarded, or its node was killed): its DOING
 * shards become TODO again and are appended to the END of the queue in index order, which gives
 * at-least-once processing.  Host only; not thread-safe.
 */
typedef struct antdt_dds antdt_dds;
enum { ANTDT_SHARD_TODO = 0, ANTDT_SHARD_DOING = 1, ANTDT_SHARD_DONE = 2 };
int antdt_dds_create(int64_t N, int64_t B, int32_t M, antdt_dds** out);
int antdt_dds_destroy(antdt_dds* dds);
int antdt_dds_num_shards(const antdt_dds* dds, int64_t* K);
int antdt_dds_fetch(antdt_dds* dds, int32_t worker, int64_t* shard, int64_t* start, int64_t* len);
int antdt_dds_report_done(antdt_dds* dds, int64_t shard, int32_t worker);
int antdt_dds_release_worker(antdt_dds* dds, int32_t worker, int64_t* requeued /* may be NULL */);
/* start, len, state, owner (worker holding it as DOING, else -1): each may be NULL */
int antdt_dds_shard(const antdt_dds* dds, int64_t shard, int64_t* start, int64_t* len,
                    int32_t* state, int32_t* owner);
int antdt_dds_counts(const antdt_dds* dds, int64_t* todo, int64_t* doing, int64_t* done);

/*
 * Iteration-level model of bulk-synchronous training under injected stragglers, to turn measured
 * batch times into job completion times.  One iteration of the present workers takes
 *   max_i T_i + t_server,   T_i = t0[i] + B_i / v[i] + delay_i,   sum_i B_i = B
 * (Eq. 1 of Section II with the server and communication terms lumped into t_server; the batch
 * time F(B_i) is affine: a latency floor t0 plus B_i / v).  Delays (Section VII-A.2): during the
 * first `duration` seconds of every `period` seconds a disturbed worker adds
 * sleep_duration * intensity to each of its iterations; the pair (window w, worker i) is
 * disturbed when fmix32(seed ^ fmix32(w * 0x9E3779B9 + i + 1)) / 2^32 < prob (fmix32:
 * MurmurHash3's 32-bit finaliser); persistent_delay[i] (may be NULL) is added from the start.
 * The job ends when N samples are processed.  Policies:
 *   BSP            equal split (first B mod n workers one more), never changed;
 *   ADJUST_BS      at the first iteration end at or after every multiple of decide_every: per
 *                  present worker the mean batch time over the iterations that ended within
 *                  the last L_trans seconds; if the largest is >= lambda * their mean, or the
 *                  smallest * lambda <= their mean, the split is re-solved (Eq. 3, the rule of
 *                  antdt_assign_shard in double precision) from v_i = mean of B_i / T_i over the
 *                  same window;
 *   BACKUP_WORKERS the backup_b slowest workers of every iteration (ties: higher index first) are
 *                  disregarded: the iteration takes the slowest remaining worker's time and only
 *                  the remaining workers' samples count as processed (Section VII-A.3);
 *   ANTDT_ND       ADJUST_BS, preceded at each decision by: mean batch times over L_per seconds;
 *                  if the slowest worker (ties: lowest index) is >= lambda * their mean it is
 *                  killed: absent for restart_cost seconds, back without its persistent delay
 *                  and with an empty history; no ADJUST_BS at that decision (Section VI-A).
 * Whenever the set of present workers changes the batch is split equally among them.
 * final_sizes: HOST int64 [n] (may be NULL), the split when the job ended.  Host only.
 */
enum { ANTDT_POLICY_BSP = 0, ANTDT_POLICY_ADJUST_BS = 1, ANTDT_POLICY_BACKUP_WORKERS = 2, ANTDT_POLICY_ANTDT_ND = 3 };
typedef struct {
  int32_t n;                      /* workers, 1..64 */
  int64_t B, N;                   /* global batch (>= n), samples of the job */
  const double* t0;               /* HOST [n] seconds */
  const double* v;                /* HOST [n] samples per second */
  double t_server;
  double period, duration, prob, sleep_duration, intensity;
  uint32_t seed;
  const double* persistent_delay; /* HOST [n] seconds, or NULL */
  int32_t policy, backup_b;
  double decide_every, L_trans, L_per, lambda, restart_cost;
  int64_t max_iterations;         /* the simulation stops there at the latest */
} antdt_sim_config;
typedef struct {
  double jct;                     /* job completion time, seconds */
  int64_t iterations, processed;
  int32_t adjust_actions, kills;
  double max_bpt, sum_bpt;        /* largest and summed batch processing time (without t_server) */
} antdt_sim_result;
int antdt_simulate_bsp(const antdt_sim_config* cfg, antdt_sim_result* result, int64_t* final_sizes);

/*
 * Dense data-parallel step on one device (Section II: the AllReduce variant drops the
 * server term): g = sum_k weights[k] * grads[k], then Adam with bias correction,
 *   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;
 *   p -= lr * (m / (1 - b1^step)) / (sqrt(v / (1 - b2^step)) + eps),
 * fused in one pass.  p, m, v: DEVICE fp32 [n], updated in place.  grads: HOST array of K
 * DEVICE pointers to fp32 [n] (1 <= K <= 16).  weights: HOST fp32 [K].  step >= 1.
 * The hyper-parameters are doubles so that 1-b1, 1-b2 and the bias corrections are formed
 * exactly before being rounded to the kernel's fp32.  All device pointers 16-byte aligned.
 * Context-free.
 */
int antdt_dense_aggregate_adam(float* p, float* m, float* v, const float* const* grads,
                               const float* weights, int32_t K, int64_t n, double lr, double beta1,
                               double beta2, double eps, int64_t step, void* stream);

/*
 * Plain streaming copy dst[i] = src[i], i < n (measurement aid, not part of the iteration): the
 * bandwidth this kernel reaches on a large buffer is the practical ceiling that the memory-bound
 * kernels of the iteration are compared with, and its known traffic (4n bytes read, 4n written)
 * calibrates the profiler's HBM byte counters.  dst, src: DEVICE, 16-byte aligned, not
 * overlapping; 0 <= n < 2^40.  Enqueues one kernel on `stream`.  Context-free.
 */
int antdt_stream_copy(float* dst, const float* src, int64_t n, void* stream);

/*
 * Fill embedding tables with their procedural initial values (input generation, not part
 * of the iteration): value(f, r, d) = scale * (u * 2^-23 - 1), u = top 24 bits of
 * fmix32(fmix32(r + 0x9E3779B9*(f+1)) ^ (0x85EBCA6B*(d+1))), fmix32 = MurmurHash3's 32-bit
 * finaliser; rounded to nearest even when dtype is BF16.  tables: DEVICE [F*R, D].
 */
int antdt_fill_tables(void* tables, int32_t dtype, int32_t num_fields, int64_t rows_per_field,
                      int32_t dim, float scale, void* stream);

/*
 * Read-only views into the workspace for checking results.  Pointers are DEVICE pointers,
 * valid until the next call that recomputes them.  These calls synchronise `stream` where
 * they need device-side counts.
 */
/* Pooled inputs of shard k: rows x ld elements of `dtype` (F32, or BF16 when gemm_dtype is
 * BF16); columns [0, F*D + num_dense) are meaningful. */
int antdt_view_pooled(antdt_ctx* ctx, int32_t k, const void** x, int64_t* rows, int64_t* ld,
                      int32_t* dtype);
/* Shard k's dense gradient (fp32, flat layout) and d loss_k / d pooled (fp32 [B_k, ld_dx]).
 * Waits (on the host) for the library's own stream that writes the weight gradients; the
 * caller still synchronises the stream it passed to antdt_worker_step before reading. */
int antdt_view_shard_grads(antdt_ctx* ctx, int32_t k, const float** dense, const float** dx,
                           int64_t* ld_dx);
/* Aggregated dense gradient (fp32, flat layout), written out on this request (apply_update
 * forms the same sum inside its optimizer kernel).  Enqueues on `stream`; valid between
 * antdt_aggregate and antdt_apply_update. */
int antdt_view_dense_grad(antdt_ctx* ctx, const float** g, void* stream);
/* Coalesced sparse gradient of field f after antdt_aggregate: unique_ids int32 [U_f] ascending,
 * seg_offsets int32 [U_f + 1], seg_samples int32 [nnz_f] (global sample index of every sorted
 * lookup; inside a run ascending), G fp32 [U_f, D]; with a mask, of the included shards'
 * lookups only.  G is written out on the first request (apply_update applies the same sums
 * without storing them).  Valid between antdt_aggregate and antdt_apply_update (BAD_STATE
 * otherwise).  Synchronises `stream`. */
int antdt_view_coalesced(antdt_ctx* ctx, int32_t f, const int32_t** unique_ids,
                         const int32_t** seg_offsets, const int32_t** seg_samples,
                         int64_t* num_unique, int64_t* nnz, const float** G, void* stream);

/*
 * Optional per-kernel timing with HIP events on the launch stream.  mode 0: off;
 * mode 1: every kernel class; mode 2: only the class `kernel_id`; mode 3: the classes whose bit
 * is set in `kernel_id` read as a mask (bit i = class i).  The matrix products of a pass that
 * are launched back to back share one pair of events.  Timings accumulate until
 * antdt_profile_read, which synchronises the recorded events and reports, per class, the
 * number of launches and their total duration in milliseconds, then resets.
 * antdt_kernel_name returns the class name (NULL past the last class).
 */
int antdt_profile(antdt_ctx* ctx, int32_t mode, int32_t kernel_id);
int antdt_profile_read(antdt_ctx* ctx, int32_t kernel_id, int64_t* launches, double* total_ms);
/*
 * What a pair of timing events adds to the time it reports: n times on `stream`, a pair with
 * nothing between its records (mean elapsed time -> *empty_ms) and a pair around the library's
 * smallest kernel, a two-word store (-> *tiny_ms), each behind such a kernel so that the stream
 * is busy as it is inside an iteration.  A class duration from antdt_profile_read contains about
 * *empty_ms per pair of events (at most *tiny_ms, which also holds that kernel's own run time).
 * Requires antdt_bind; synchronises `stream`; 1 <= n <= 4096.
 */
int antdt_profile_overhead(antdt_ctx* ctx, void* stream, int32_t n, double* empty_ms, double* tiny_ms);
const char* antdt_kernel_name(int32_t kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* ANTDT_H_ */
