// C boundary: context, workspace layout, call-order checks and the launch
// sequences of worker_step / aggregate / apply_update (see include/antdt.h).
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "common.h"

namespace antdt {

struct ProfRec {
  hipEvent_t start, stop;
  int kid;
  int n = 1;  // launches inside the bracket
  bool closed = false;
};
struct Profiler {
  int mode = 0, sel = -1;
  std::vector<ProfRec> recs;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;
  double total_ms[KID_COUNT] = {};
  int64_t launches[KID_COUNT] = {};
};

int prof_begin(Profiler* p, int kid, hipStream_t s) {
  if (p->mode == 0 || (p->mode == 2 && kid != p->sel) || (p->mode == 3 && !((p->sel >> kid) & 1))) return -1;
  ProfRec r;
  r.kid = kid;
  if (!p->pool.empty()) {
    r.start = p->pool.back().first;
    r.stop = p->pool.back().second;
    p->pool.pop_back();
  } else {
    // timing events: no cache write-back at the record (it would disturb what is being timed)
    if (hipEventCreateWithFlags(&r.start, hipEventDisableSystemFence) != hipSuccess) return -1;
    if (hipEventCreateWithFlags(&r.stop, hipEventDisableSystemFence) != hipSuccess) return -1;
  }
  (void)hipEventRecord(r.start, s);
  p->recs.push_back(r);
  return (int)p->recs.size() - 1;
}
void prof_count(Profiler* p, int idx, int launches) { p->recs[idx].n = launches; }
void prof_end(Profiler* p, int idx, hipStream_t s) {
  p->recs[idx].closed = true;
  (void)hipEventRecord(p->recs[idx].stop, s);
}

static void prof_drain(Profiler* p) {
  for (auto& r : p->recs) {
    float ms = 0.f;
    if (r.closed && hipEventSynchronize(r.stop) == hipSuccess &&
        hipEventElapsedTime(&ms, r.start, r.stop) == hipSuccess) {
      p->total_ms[r.kid] += ms;
      p->launches[r.kid] += r.n;
    }
    p->pool.push_back({r.start, r.stop});
  }
  p->recs.clear();
}

static const char* kKernelNames[KID_COUNT] = {
    "pool",        "gemm_fwd",   "gemm_dgrad",     "gemm_wgrad",  "head",
    "head_reduce", "bias_grad",  "sort_hist",      "sort_scan",   "sort_scatter",
    "seg_heads",   "seg_scan",   "seg_emit",       "seg_reduce",  "seg_reduce_long",
    "dense_agg",   "sparse_adagrad", "dense_adagrad", "adam", "transpose", "gemm_bwd", "wgrad_adagrad"};

}  // namespace antdt

using namespace antdt;

static thread_local std::string g_last_error;

namespace antdt {
void set_last_error(const std::string& msg) { g_last_error = msg; }
}

enum Stage { ST_CREATED = 0, ST_BOUND, ST_BATCH, ST_AGGREGATED };

struct antdt_ctx {
  antdt_model m;
  std::string err;
  Stage stage = ST_CREATED;
  Profiler prof;
  // derived sizes
  int L = 0, FD = 0, in0 = 0, ldx = 0;
  int act_bf16 = 0;
  size_t act_size = 4;
  int64_t P = 0, Pstride = 0;  // Pstride: P rounded up to 4 (per-shard gradient pitch)
  bool gdense_valid = false;
  int64_t w_off[ANTDT_MAX_LAYERS], b_off[ANTDT_MAX_LAYERS];
  int width[ANTDT_MAX_LAYERS + 1];  // width[l] = layer_sizes[l]
  int sort_passes = 1, radix_bits = 1;
  int64_t max_tiles_total = 0;
  // Runs of more than long_threshold lookups are summed by whole blocks, `chunk` lookups at a time (measured on
  // configurations 2-4: 32 / 1024 against 64 / 256 shortens the sparse update by 3-5 %; below 32 and above 1024 flat)
  int long_threshold = 32;
  int64_t long_cap = 0, item_cap = 0;
  int chunk = 1024;
  bool g_valid = false;
  size_t ws_bytes = 0;
  // caller's buffers
  void* tables = nullptr;
  float* table_state = nullptr;
  float* params = nullptr;
  float* pstate = nullptr;
  // workspace carve-up
  char* x = nullptr;
  char* h[ANTDT_MAX_LAYERS] = {};
  char* dh[ANTDT_MAX_LAYERS] = {};
  float *z = nullptr, *loss_s = nullptr, *dz = nullptr, *loss_k = nullptr, *dx = nullptr;
  float *shard_grads = nullptr, *g_dense = nullptr, *sample_w = nullptr, *G = nullptr;
  bf16_t* wb[ANTDT_MAX_LAYERS] = {};     // bf16 W_l as [in (padded), out]: operand of the data gradient
  bf16_t* wb0_alt = nullptr;             // second buffer for W_0: the fused dense update writes the new copy there
                                         // while the input-gradient product may still read the old one
  bf16_t* wbt[ANTDT_MAX_LAYERS] = {};    // bf16 W_l^T as [out, in (padded)]: operand of the forward product
  bf16_t* act_t[ANTDT_MAX_LAYERS] = {};  // transposed activations [width + 8, ldt], row `width` = ones
  bf16_t* dh_t[ANTDT_MAX_LAYERS] = {};   // transposed pre-activation gradients [width, ldt]
  int64_t ldt = 0;
  int32_t* lookup_sample = nullptr;
  int32_t *key[2] = {}, *pay[2] = {}, *tile_heads = nullptr, *ubase = nullptr, *uniq = nullptr;
  int32_t *segoff = nullptr, *ufield = nullptr, *segabs = nullptr, *counters = nullptr, *long_seg = nullptr, *items = nullptr, *qcnt = nullptr, *xcd_tab = nullptr;
  float* partial = nullptr;
  uint32_t *hist = nullptr, *digit_base = nullptr;
  // batch
  const int32_t* ids = nullptr;
  const int32_t* offsets = nullptr;
  const float* dense = nullptr;
  const float* labels = nullptr;
  int64_t B = 0;
  FieldPtr fp;
  TileBase tb;
  int max_tiles = 0, total_tiles = 0;
  // the lookups that the current aggregation coalesces: all of the batch (the four above), or
  // the packed lookups of the included shards when some are left out
  FieldPtr afp;
  TileBase atb;
  int amax_tiles = 0, atotal_tiles = 0;
  int64_t* cbase = nullptr;
  int32_t* vflags = nullptr;  // result of antdt_validate_batch
  // shards
  ShardTab tab;
  bool have_shards = false;
  int64_t shard_B = 0;
  bool stepped[ANTDT_MAX_SHARDS] = {};
  bool included[ANTDT_MAX_SHARDS] = {};
  double shard_scale[ANTDT_MAX_SHARDS];  // per-worker factor on the aggregation weight (1 unless set)
  bool weights_dirty = false;            // the factors changed after the weights were last formed
  bool head_weights_deferred = false;    // the last layer's weight sums of this worker step are still to be launched
  // Weight gradients formed inside the dense update (bf16 products with a weight-gradient stream):
  // the worker step only leaves their operands behind and an event (ev_dh[0]) that says they are
  // complete; per-shard gradients are computed when a view asks for them.
  bool eager_wgrad = false;              // option: the worker step computes the per-shard weight gradients itself
  bool wgrad_deferred = false;           // this worker step left the weight gradients to apply_update / the views
  bool shard_grads_done = false;         // the per-shard dense gradients of this worker step are (being) written
  HeadReduceArgs head_reduce_args;
  int sorted_buf = 0;
  // side stream on which the coalescing structure of a batch is built while the MLP runs
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  // second side stream: the weight-gradient products, which nothing needs before the dense
  // update, run there beside the data-gradient chain and the sparse reduction
  hipStream_t wside = nullptr;
  hipEvent_t ev_dh[ANTDT_MAX_LAYERS + 1] = {};  // ev_dh[l]: dH_l (and its transposed copy) is ready
  hipEvent_t ev_wgrad = nullptr;                // all weight gradients of the last worker step are written
  bool wgrad_pending = false;
  bool presorted = false;     // the coalescing structure of the current batch and split is built (or being built)
  bool side_pending = false;  // work is in flight on the side stream that no other stream has waited for yet
  // bound by antdt_bind_static: the workspace is the library's static device buffer and every
  // kernel goes to the caller's stream (no library-owned stream or event exists or is created)
  bool static_bound = false;
  bool no_streams = false;   // option: everything on the caller's stream although the library's streams exist
  int static_device = -1;
};

// The library's own streams, or none when the context works on the caller's stream only.
static inline hipStream_t side_stream(const antdt_ctx* c) { return (c->static_bound || c->no_streams) ? nullptr : c->side; }
static inline hipStream_t wgrad_stream(const antdt_ctx* c) { return (c->static_bound || c->no_streams) ? nullptr : c->wside; }

static int fail(antdt_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  g_last_error = msg;
  return code;
}
#define HIP_TRY(c, expr)                                                                   \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return fail(c, ANTDT_HIP_ERROR, std::string(#expr) + ": " + hipGetErrorString(e__)); \
  } while (0)

// Events that order the library's own streams on one device.  Without the system-scope fence a
// record does not write the caches back for the host or other devices (work on this device
// still sees everything the recorded work wrote): on the launch stream that fence costs about
// 2 us per record and evicts what the next kernel would have found in L2.
static constexpr unsigned SYNC_EVENT_FLAGS = hipEventDisableTiming | hipEventDisableSystemFence;

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline Profiler* prof_of(antdt_ctx* c) { return c->prof.mode ? &c->prof : nullptr; }

static bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

// Lays the workspace out; with base == nullptr only the size is computed.
static size_t carve(antdt_ctx* c, char* base) {
  size_t off = 0;
  auto take = [&](size_t bytes) -> char* {
    char* p = base ? base + off : nullptr;
    off = align_up(off + bytes, 256);
    return p;
  };
  const antdt_model& m = c->m;
  const int64_t Bm = m.max_batch, K = m.max_shards, N = m.max_nnz;
  c->x = take((size_t)Bm * c->ldx * c->act_size);
  for (int l = 1; l < c->L; ++l) {
    c->h[l] = take((size_t)Bm * c->width[l] * c->act_size);
    c->dh[l] = take((size_t)Bm * c->width[l] * c->act_size);
  }
  c->z = (float*)take(Bm * 4);
  c->loss_s = (float*)take(Bm * 4);
  c->dz = (float*)take(Bm * 4);
  c->sample_w = (float*)take(Bm * 4);
  c->loss_k = (float*)take(K * 4);
  c->dx = (float*)take((size_t)Bm * c->FD * 4);
  c->shard_grads = (float*)take((size_t)K * c->Pstride * 4);
  c->g_dense = (float*)take((size_t)c->P * 4);
  if (c->act_bf16) {
    for (int l = 0; l + 1 < c->L; ++l) {
      const int64_t rows = l == 0 ? c->ldx : c->width[l];
      c->wb[l] = (bf16_t*)take((size_t)rows * c->width[l + 1] * 2);
      if (l == 0) c->wb0_alt = (bf16_t*)take((size_t)rows * c->width[l + 1] * 2);
      c->wbt[l] = (bf16_t*)take((size_t)rows * c->width[l + 1] * 2);
    }
    for (int l = 0; l < c->L; ++l) {
      const int64_t rows = (l == 0 ? c->ldx : c->width[l]) + 8;
      c->act_t[l] = (bf16_t*)take((size_t)rows * c->ldt * 2);
      if (l > 0) c->dh_t[l] = (bf16_t*)take((size_t)c->width[l] * c->ldt * 2);
    }
  }
  c->lookup_sample = (int32_t*)take((size_t)N * 4);
  for (int i = 0; i < 2; ++i) {
    c->key[i] = (int32_t*)take((size_t)N * 4);
    c->pay[i] = (int32_t*)take((size_t)N * 4);
  }
  c->hist = (uint32_t*)take((size_t)(c->max_tiles_total << c->radix_bits) * 4);
  c->digit_base = (uint32_t*)take((size_t)(m.num_fields << c->radix_bits) * 4);
  c->tile_heads = (int32_t*)take((size_t)(c->max_tiles_total + 1) * 4);
  c->ubase = (int32_t*)take((size_t)(m.num_fields + 1) * 4);
  c->uniq = (int32_t*)take((size_t)N * 4);
  c->segoff = (int32_t*)take((size_t)(N + m.num_fields + 1) * 4);
  c->ufield = (int32_t*)take((size_t)N * 4);
  c->segabs = (int32_t*)take((size_t)(N + 1) * 4);
  c->counters = (int32_t*)take(8);
  c->qcnt = (int32_t*)take((size_t)(N / ANTDT_QUEUE_BLOCK_RUNS + 2) * 8);
  c->xcd_tab = (int32_t*)take(3 * 9 * 4);
  c->cbase = (int64_t*)take((size_t)(ANTDT_MAX_FIELDS + 1) * 8);
  c->vflags = (int32_t*)take(8);
  c->long_seg = (int32_t*)take((size_t)c->long_cap * 12);
  c->items = (int32_t*)take((size_t)c->item_cap * 8);
  c->partial = (float*)take((size_t)c->item_cap * m.dim * 4);
  c->G = (float*)take((size_t)N * m.dim * 4);
  return off;
}

// ----------------------------------------------------------------------------------------
// Scratch of antdt_bind_static, the entry point for callers that cannot allocate.  The array's
// name is only a host-side handle; kernels and copies get the address that
// hipGetSymbolAddress reports for the device that is current, looked up once per device (each
// device holds its own copy of the array at its own address).
static __device__ __align__(256) unsigned char scratch[ANTDT_STATIC_SCRATCH_BYTES];

static constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[MAX_DEVICES] = {};
static antdt_ctx* g_scratch_owner[MAX_DEVICES] = {};  // context whose workspace the buffer currently is

// A context that gives the static buffer up (rebound to a caller's workspace, or destroyed).
static void release_static(antdt_ctx* c) {
  if (!c->static_bound) return;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (c->static_device >= 0 && c->static_device < MAX_DEVICES && g_scratch_owner[c->static_device] == c)
    g_scratch_owner[c->static_device] = nullptr;
  c->static_bound = false;
  c->static_device = -1;
}

// Makes `s` wait for whatever the side stream is still doing (it writes the sort buffers, the run
// tables and the per-sample weights, and reads the sample index of every lookup): before anything
// rebuilds or overwrites those.  Whether that structure is still valid is a separate question.
static int join_side(antdt_ctx* c, hipStream_t s) {
  if (c->side_pending) {
    HIP_TRY(c, hipStreamWaitEvent(s, c->ev_join, 0));
    c->side_pending = false;
  }
  return ANTDT_OK;
}

// Makes `s` wait for the weight-gradient products of the last worker step (they run on their
// own stream): before anything reads the per-shard dense gradients or overwrites their operands.
static int join_wgrad(antdt_ctx* c, hipStream_t s) {
  if (c->wgrad_pending) {
    HIP_TRY(c, hipStreamWaitEvent(s, c->ev_wgrad, 0));
    c->wgrad_pending = false;
  }
  return ANTDT_OK;
}

extern "C" {

const char* antdt_last_error(const antdt_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

const char* antdt_kernel_name(int32_t kid) { return (kid >= 0 && kid < KID_COUNT) ? kKernelNames[kid] : nullptr; }

int antdt_create(const antdt_model* model, antdt_ctx** out) {
  if (!model || !out) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_create: null argument");
  const antdt_model& m = *model;
  auto bad = [&](const char* what) { return fail(nullptr, ANTDT_INVALID_ARG, std::string("antdt_create: ") + what); };
  if (m.num_fields < 1 || m.num_fields > ANTDT_MAX_FIELDS) return bad("num_fields out of range");
  if (m.rows_per_field < 1 || m.rows_per_field >= (1ll << 31)) return bad("rows_per_field out of range");
  if (m.table_dtype != ANTDT_F32 && m.table_dtype != ANTDT_BF16) return bad("table_dtype");
  if (m.gemm_dtype != ANTDT_F32 && m.gemm_dtype != ANTDT_BF16) return bad("gemm_dtype");
  if (m.adagrad_state != ANTDT_STATE_ELEMENTWISE && m.adagrad_state != ANTDT_STATE_ROWWISE) return bad("adagrad_state");
  const int64_t row_bytes = (int64_t)m.dim * (m.table_dtype == ANTDT_BF16 ? 2 : 4);
  if (m.dim < 4 || m.dim > 256 || row_bytes < 16 || !is_pow2(row_bytes))
    return bad("dim: 4..256, a power of two (a row's gradient is summed by at most one wavefront, four columns per lane)");
  if (m.num_dense < 0) return bad("num_dense");
  if (m.num_layers < 1 || m.num_layers > ANTDT_MAX_LAYERS) return bad("num_layers out of range");
  if ((int64_t)m.layer_sizes[0] != (int64_t)m.num_fields * m.dim + m.num_dense) return bad("layer_sizes[0] != num_fields*dim + num_dense");
  if (m.layer_sizes[m.num_layers] != 1) return bad("last layer must have one output");
  for (int l = 1; l < m.num_layers; ++l) {
    if (m.layer_sizes[l] < 1) return bad("layer size");
    if (m.gemm_dtype == ANTDT_BF16 && m.layer_sizes[l] % 8) return bad("bf16 GEMMs need hidden widths that are multiples of 8");
  }
  if (m.max_shards < 1 || m.max_shards > ANTDT_MAX_SHARDS) return bad("max_shards out of range");
  if (m.max_batch < 1 || m.max_batch >= (1ll << 31)) return bad("max_batch out of range");
  if (m.max_nnz < 0 || m.max_nnz >= (1ll << 31) - 4096) return bad("max_nnz out of range");
  if (m.pooling != ANTDT_POOL_SUM && m.pooling != ANTDT_POOL_MEAN) return bad("pooling: ANTDT_POOL_SUM or ANTDT_POOL_MEAN");
  if (!(m.lr >= 0.f) || !(m.eps > 0.f)) return bad("lr must be >= 0 and eps > 0");

  antdt_ctx* c = new antdt_ctx();
  c->m = m;
  for (int k = 0; k < ANTDT_MAX_SHARDS; ++k) c->shard_scale[k] = 1.0;
  c->L = m.num_layers;
  c->FD = m.num_fields * m.dim;
  c->in0 = m.layer_sizes[0];
  c->ldx = (c->in0 + 7) / 8 * 8;
  c->act_bf16 = m.gemm_dtype == ANTDT_BF16;
  c->act_size = c->act_bf16 ? 2 : 4;
  c->ldt = (m.max_batch + 63) / 64 * 64;
  int64_t off = 0;
  for (int l = 0; l <= c->L; ++l) c->width[l] = m.layer_sizes[l];
  for (int l = 0; l < c->L; ++l) {
    c->w_off[l] = off;
    off += (int64_t)c->width[l] * c->width[l + 1];
    c->b_off[l] = off;
    off += c->width[l + 1];
  }
  c->P = off;
  c->Pstride = (off + 3) / 4 * 4;
  int bits = 1;
  while ((1ll << bits) < m.rows_per_field) ++bits;
  c->sort_passes = (bits + 9) / 10;
  c->radix_bits = (bits + c->sort_passes - 1) / c->sort_passes;
  c->max_tiles_total = m.max_nnz / ANTDT_SORT_TILE + m.num_fields + 1;
  c->long_cap = m.max_nnz / c->long_threshold + 1;
  c->item_cap = m.max_nnz / c->chunk + c->long_cap + 1;
  c->ws_bytes = carve(c, nullptr);
  memset(&c->tab, 0, sizeof(c->tab));
  *out = c;
  return ANTDT_OK;
}

int antdt_destroy(antdt_ctx* ctx) {
  if (!ctx) return ANTDT_OK;
  release_static(ctx);
  prof_drain(&ctx->prof);
  if (ctx->side) {
    (void)hipStreamSynchronize(ctx->side);
    (void)hipStreamDestroy(ctx->side);
    (void)hipEventDestroy(ctx->ev_fork);
    (void)hipEventDestroy(ctx->ev_join);
  }
  if (ctx->wside) {
    (void)hipStreamSynchronize(ctx->wside);
    (void)hipStreamDestroy(ctx->wside);
    (void)hipEventDestroy(ctx->ev_wgrad);
    for (auto& e : ctx->ev_dh)
      if (e) (void)hipEventDestroy(e);
  }
  for (auto& e : ctx->prof.pool) {
    (void)hipEventDestroy(e.first);
    (void)hipEventDestroy(e.second);
  }
  delete ctx;
  return ANTDT_OK;
}

int antdt_workspace_bytes(const antdt_ctx* ctx, size_t* bytes) {
  if (!ctx || !bytes) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_workspace_bytes: null argument");
  *bytes = ctx->ws_bytes;
  return ANTDT_OK;
}

// wbt[l] = transpose of wb[l] for every hidden layer, one launch.
static int transpose_weights(antdt_ctx* c, hipStream_t s) {
  if (!c->act_bf16 || c->L < 2) return ANTDT_OK;
  TransposeArgs t;
  memset(&t, 0, sizeof(t));
  for (int l = 0; l + 1 < c->L; ++l) {
    const int rows = l == 0 ? c->ldx : c->width[l], cols = c->width[l + 1];
    t.src[l] = c->wb[l]; t.dst[l] = c->wbt[l];
    t.rows[l] = rows; t.cols[l] = cols; t.ld_src[l] = cols; t.ld_dst[l] = rows;
    t.tile_base[l + 1] = t.tile_base[l] + ((rows + 63) / 64) * ((cols + 63) / 64);
  }
  t.n = c->L - 1;
  ProfScope ps(prof_of(c), KID_TRANSPOSE, s);
  HIP_TRY(c, launch_transpose_bf16(t, s));
  return ANTDT_OK;
}

static int refresh_bf16_weights(antdt_ctx* c, hipStream_t s) {
  if (!c->act_bf16) return ANTDT_OK;
  for (int l = 0; l + 1 < c->L; ++l) {
    CastArgs a;
    a.src = c->params + c->w_off[l];
    a.dst = c->wb[l];
    a.n_src = (int64_t)c->width[l] * c->width[l + 1];
    a.n_dst = (int64_t)(l == 0 ? c->ldx : c->width[l]) * c->width[l + 1];
    HIP_TRY(c, launch_cast_bf16(a, s));
    if (l == 0) {  // (its padding rows must be zero as well)
      a.dst = c->wb0_alt;
      HIP_TRY(c, launch_cast_bf16(a, s));
    }
  }
  // constant rows of the transposed activations: a row of ones below the last feature row
  // (it turns the bias gradient into one more row of the weight-gradient product), zeros after
  for (int l = 0; l < c->L; ++l) {
    OnesRowArgs o;
    o.base = c->act_t[l];
    o.ld = c->ldt;
    o.row = c->width[l];
    o.zero_rows = (l == 0 ? c->ldx : c->width[l]) + 8 - c->width[l] - 1;
    HIP_TRY(c, launch_ones_row(o, s));
  }
  return transpose_weights(c, s);
}

int antdt_bind(antdt_ctx* c, void* tables, float* table_state, float* mlp_params, float* mlp_state,
               void* workspace, size_t workspace_bytes, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_bind: null context");
  if (!tables || !table_state || !mlp_params || !mlp_state || !workspace)
    return fail(c, ANTDT_INVALID_ARG, "antdt_bind: null buffer");
  if (workspace_bytes < c->ws_bytes) return fail(c, ANTDT_WORKSPACE_TOO_SMALL, "antdt_bind: workspace too small");
  if (((uintptr_t)workspace & 255) || ((uintptr_t)tables & 15) || ((uintptr_t)table_state & 15) ||
      ((uintptr_t)mlp_params & 15) || ((uintptr_t)mlp_state & 15))
    return fail(c, ANTDT_INVALID_ARG, "antdt_bind: misaligned buffer (workspace 256 B, others 16 B)");
  release_static(c);
  c->tables = tables;
  c->table_state = table_state;
  c->params = mlp_params;
  c->pstate = mlp_state;
  carve(c, (char*)workspace);
  if (!c->side) {
    HIP_TRY(c, hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_fork, SYNC_EVENT_FLAGS));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_join, SYNC_EVENT_FLAGS));
  }
  if (!c->wside) {
    HIP_TRY(c, hipStreamCreateWithFlags(&c->wside, hipStreamNonBlocking));
    HIP_TRY(c, hipEventCreateWithFlags(&c->ev_wgrad, SYNC_EVENT_FLAGS));
    for (int l = 0; l <= c->L; ++l) HIP_TRY(c, hipEventCreateWithFlags(&c->ev_dh[l], SYNC_EVENT_FLAGS));
  }
  c->stage = ST_BOUND;
  return refresh_bf16_weights(c, (hipStream_t)stream);
}

int antdt_bind_static(antdt_ctx* c, void* tables, float* table_state, float* mlp_params, float* mlp_state,
                      void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_bind_static: null context");
  if (!tables || !table_state || !mlp_params || !mlp_state)
    return fail(c, ANTDT_INVALID_ARG, "antdt_bind_static: null buffer");
  if (((uintptr_t)tables & 15) || ((uintptr_t)table_state & 15) || ((uintptr_t)mlp_params & 15) ||
      ((uintptr_t)mlp_state & 15))
    return fail(c, ANTDT_INVALID_ARG, "antdt_bind_static: misaligned buffer (16 B)");
  if (c->ws_bytes > (size_t)ANTDT_STATIC_SCRATCH_BYTES)
    return fail(c, ANTDT_WORKSPACE_TOO_SMALL,
                "antdt_bind_static: the model needs " + std::to_string(c->ws_bytes) +
                    " bytes of scratch, the library's static buffer holds " +
                    std::to_string((size_t)ANTDT_STATIC_SCRATCH_BYTES) + " (use antdt_bind with a workspace)");
  int dev = -1;
  HIP_TRY(c, hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(c, ANTDT_UNSUPPORTED, "antdt_bind_static: device index out of range");
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {  // once per device, with that device current
      void* p = nullptr;
      const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !p)
        return fail(c, ANTDT_HIP_ERROR, std::string("antdt_bind_static: hipGetSymbolAddress: ") + hipGetErrorString(e));
      g_scratch_ptr[dev] = p;
    }
    base = g_scratch_ptr[dev];
    // The buffer serves one context at a time: the context that held it must be bound again
    // before its next iteration (its calls fail with BAD_STATE until then).
    antdt_ctx* prev = g_scratch_owner[dev];
    if (prev && prev != c) {
      prev->stage = ST_CREATED;
      prev->static_bound = false;
      prev->static_device = -1;
    }
    g_scratch_owner[dev] = c;
  }
  if (((uintptr_t)base & 255)) return fail(c, ANTDT_HIP_ERROR, "antdt_bind_static: static buffer is not 256-byte aligned");
  // A context that was bound with antdt_bind before may still have work on its own streams.
  if (c->side) HIP_TRY(c, hipStreamSynchronize(c->side));
  if (c->wside) HIP_TRY(c, hipStreamSynchronize(c->wside));
  c->side_pending = false;
  c->wgrad_pending = false;
  c->presorted = false;
  c->static_bound = true;
  c->static_device = dev;
  c->tables = tables;
  c->table_state = table_state;
  c->params = mlp_params;
  c->pstate = mlp_state;
  carve(c, (char*)base);
  c->stage = ST_BOUND;
  c->have_shards = false;
  return refresh_bf16_weights(c, (hipStream_t)stream);
}

// Tile decomposition of per-field lookup ranges.
static void plan_tiles(int F, const FieldPtr& fp, TileBase& tb, int& max_tiles, int& total_tiles) {
  memset(&tb, 0, sizeof(tb));
  max_tiles = 0;
  for (int f = 0; f < F; ++f) {
    const int tiles = (int)((fp.p[f + 1] - fp.p[f] + ANTDT_SORT_TILE - 1) / ANTDT_SORT_TILE);
    tb.t[f + 1] = tb.t[f] + tiles;
    if (tiles > max_tiles) max_tiles = tiles;
  }
  for (int f = F + 1; f <= ANTDT_MAX_FIELDS; ++f) tb.t[f] = tb.t[F];
  total_tiles = tb.t[F];
  for (int x = 0; x < 8; ++x)
    for (int j = 0; j < ANTDT_MAX_FIELDS / 8; ++j) {
      const int f = x + 8 * j;
      tb.xcum[x][j + 1] = tb.xcum[x][j] + (f < F ? tb.t[f + 1] - tb.t[f] : 0);
    }
}

static void coalesce_whole_batch(antdt_ctx* c) {
  c->afp = c->fp;
  c->atb = c->tb;
  c->amax_tiles = c->max_tiles;
  c->atotal_tiles = c->total_tiles;
}

int antdt_set_batch(antdt_ctx* c, const int32_t* ids, const int64_t* field_ptr, const int32_t* offsets,
                    const float* dense, const float* labels, int64_t B, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_set_batch: null context");
  if (c->stage < ST_BOUND) return fail(c, ANTDT_BAD_STATE, "antdt_set_batch: call antdt_bind first");
  if (B < 0 || B > c->m.max_batch) return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: B out of range");
  if (!field_ptr || !offsets || (B > 0 && (!labels || (c->m.num_dense > 0 && !dense))))
    return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: null buffer");
  const int F = c->m.num_fields;
  if (field_ptr[0] != 0) return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: field_ptr[0] != 0");
  for (int f = 0; f < F; ++f)
    if (field_ptr[f + 1] < field_ptr[f]) return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: field_ptr decreases");
  if (field_ptr[F] > c->m.max_nnz) return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: more lookups than max_nnz");
  if (field_ptr[F] > 0 && !ids) return fail(c, ANTDT_INVALID_ARG, "antdt_set_batch: null ids");
  memset(&c->fp, 0, sizeof(c->fp));
  for (int f = 0; f < F; ++f) c->fp.p[f + 1] = field_ptr[f + 1];
  for (int f = F + 1; f <= ANTDT_MAX_FIELDS; ++f) c->fp.p[f] = c->fp.p[F];
  plan_tiles(F, c->fp, c->tb, c->max_tiles, c->total_tiles);
  coalesce_whole_batch(c);
  c->ids = ids;
  c->offsets = offsets;
  c->dense = dense;
  c->labels = labels;
  c->B = B;
  c->stage = ST_BATCH;
  {
    const int rc = join_side(c, (hipStream_t)stream);
    if (rc) return rc;
  }
  c->presorted = false;
  memset(c->stepped, 0, sizeof(c->stepped));
  return ANTDT_OK;
}

int antdt_validate_batch(antdt_ctx* c, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_validate_batch: null context");
  if (c->stage < ST_BATCH) return fail(c, ANTDT_BAD_STATE, "antdt_validate_batch: call antdt_set_batch first");
  hipStream_t s = (hipStream_t)stream;
  HIP_TRY(c, launch_validate(c->ids, c->offsets, c->fp, c->B, c->m.rows_per_field, c->m.num_fields, c->vflags, s));
  int32_t fl[2] = {0, 0};
  HIP_TRY(c, hipMemcpyAsync(fl, c->vflags, sizeof(fl), hipMemcpyDeviceToHost, s));
  HIP_TRY(c, hipStreamSynchronize(s));
  if (fl[0] == 0) return ANTDT_OK;
  std::string what = "antdt_validate_batch: field " + std::to_string(fl[1] - 1) + " (lowest offending):";
  if (fl[0] & 1) what += " an id outside [0, rows_per_field)";
  if (fl[0] & 2) what += std::string(fl[0] & 1 ? ";" : "") + " offsets that do not start at 0, decrease, or do not end at the field's lookup count";
  return fail(c, ANTDT_INVALID_ARG, what);
}

int antdt_assign_shard(antdt_ctx* c, int64_t B, int32_t K, const int64_t* sizes, const double* speed,
                       int64_t* start_out, int64_t* len_out) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_assign_shard: null context");
  if (K < 1 || K > c->m.max_shards) return fail(c, ANTDT_INVALID_ARG, "antdt_assign_shard: K out of range");
  if (B < 0 || B > c->m.max_batch) return fail(c, ANTDT_INVALID_ARG, "antdt_assign_shard: B out of range");
  std::vector<int64_t> len(K, 0);
  if (sizes) {
    int64_t tot = 0;
    for (int k = 0; k < K; ++k) {
      if (sizes[k] < 0) return fail(c, ANTDT_INVALID_ARG, "antdt_assign_shard: negative shard size");
      len[k] = sizes[k];
      tot += sizes[k];
    }
    if (tot != B) return fail(c, ANTDT_INVALID_ARG, "antdt_assign_shard: sizes do not sum to B");
  } else if (speed) {
    // Eq. 3: minimise z subject to z >= B_k / v_k, sum_k B_k = B.  Every worker can take
    // floor(B v_k / sum v) - 1 samples without exceeding the continuous optimum B / sum v;
    // the rest is handed out one sample at a time to the worker whose load after the
    // addition is smallest (ties: lowest k), which is optimal for a max of linear costs.
    long double tot_v = 0;
    for (int k = 0; k < K; ++k) {
      if (!(speed[k] > 0.0) || !isfinite(speed[k])) return fail(c, ANTDT_INVALID_ARG, "antdt_assign_shard: speed must be finite and > 0");
      tot_v += speed[k];
    }
    int64_t given = 0;
    for (int k = 0; k < K; ++k) {
      int64_t b = (int64_t)floorl((long double)B * speed[k] / tot_v) - 1;
      if (b < 0) b = 0;
      len[k] = b;
      given += b;
    }
    for (; given < B; ++given) {
      int best = 0;
      for (int k = 1; k < K; ++k) {
        // (len[k]+1)/v_k < (len[best]+1)/v_best, cross-multiplied
        const long double lhs = (long double)(len[k] + 1) * speed[best];
        const long double rhs = (long double)(len[best] + 1) * speed[k];
        if (lhs < rhs) best = k;
      }
      ++len[best];
    }
  } else {
    const int64_t q = B / K, r = B % K;
    for (int k = 0; k < K; ++k) len[k] = q + (k < r ? 1 : 0);
  }
  memset(&c->tab, 0, sizeof(c->tab));
  c->tab.K = K;
  int64_t s = 0;
  for (int k = 0; k < K; ++k) {
    c->tab.start[k] = (int32_t)s;
    c->tab.len[k] = (int32_t)len[k];
    if (start_out) start_out[k] = s;
    if (len_out) len_out[k] = len[k];
    s += len[k];
  }
  for (int k = K; k < ANTDT_MAX_SHARDS; ++k) c->tab.start[k] = (int32_t)s;
  c->have_shards = true;
  c->presorted = false;
  c->shard_B = B;
  memset(c->stepped, 0, sizeof(c->stepped));
  if (c->stage == ST_AGGREGATED) c->stage = ST_BATCH;
  return ANTDT_OK;
}

static void fill_seg_args(antdt_ctx* c, SegArgs& a) {
  const antdt_model& m = c->m;
  memset(&a, 0, sizeof(a));
  a.key = c->key[c->sorted_buf]; a.pay = c->pay[c->sorted_buf];
  a.tile_heads = c->tile_heads; a.ubase = c->ubase; a.uniq = c->uniq; a.ufield = c->ufield;
  a.segabs = c->segabs; a.segoff = c->segoff; a.sample_w = c->sample_w; a.counters = c->counters; a.qcnt = c->qcnt; a.xcd_tab = c->xcd_tab;
  a.long_seg = c->long_seg; a.items = c->items; a.partial = c->partial;
  a.G = c->G; a.dx = c->dx; a.lddx = c->FD;
  a.offsets = c->offsets; a.mean_pool = m.pooling == ANTDT_POOL_MEAN;
  a.F = m.num_fields; a.D = m.dim; a.B = (int32_t)c->B; a.max_tiles = c->amax_tiles;
  a.total_tiles = c->atotal_tiles; a.long_threshold = c->long_threshold; a.chunk = c->chunk;
  a.long_cap = (int32_t)c->long_cap; a.item_cap = (int32_t)c->item_cap;
  a.tables = c->tables; a.state = c->table_state; a.R = m.rows_per_field; a.lr = m.lr; a.eps = m.eps;
  a.table_bf16 = m.table_dtype == ANTDT_BF16; a.rowwise = m.adagrad_state == ANTDT_STATE_ROWWISE;
}

static void set_weights(antdt_ctx* c) {
  const int K = c->tab.K;
  int64_t tot = 0;
  for (int k = 0; k < K; ++k)
    if (c->included[k]) tot += c->tab.len[k];
  for (int k = 0; k < ANTDT_MAX_SHARDS; ++k)
    c->tab.w[k] = (k < K && c->included[k] && tot > 0)
                      ? (float)(c->shard_scale[k] * ((double)c->tab.len[k] / (double)tot)) : 0.0f;
  c->weights_dirty = false;
}

// Sort the lookups by row id, find the runs, and fill the per-sample weights: everything of
// the server side that depends only on the batch's ids and on the shard weights.
static int build_coalescing(antdt_ctx* c, const int32_t* ids, const int32_t* pay0, hipStream_t s) {
  Profiler* pr = prof_of(c);
  const antdt_model& m = c->m;
  SortPlan pl;
  pl.F = m.num_fields; pl.B = (int32_t)c->B; pl.passes = c->sort_passes; pl.radix_bits = c->radix_bits;
  pl.max_tiles = c->amax_tiles; pl.total_tiles = c->atotal_tiles;
  SortBuffers sb;
  sb.ids = ids; sb.offsets = c->offsets;
  sb.key[0] = c->key[0]; sb.key[1] = c->key[1]; sb.pay[0] = c->pay[0]; sb.pay[1] = c->pay[1];
  sb.hist = c->hist;
  sb.digit_base = c->digit_base;
  sb.pay0 = pay0;
  for (int p = 0; p < pl.passes; ++p) HIP_TRY(c, launch_sort_pass(pl, sb, p, c->afp, c->atb, pr, s));
  c->sorted_buf = (pl.passes - 1) & 1;
  SegArgs a;
  fill_seg_args(c, a);
  HIP_TRY(c, launch_segments(a, c->afp, c->atb, c->tab, pr, s));
  return ANTDT_OK;
}

// Per-shard weight gradient of hidden layer l for shards [k0, k1), one grouped product on `ws`.
static int shard_weight_gradient(antdt_ctx* c, int l, int k0, int k1, hipStream_t ws) {
  Profiler* pr = prof_of(c);
  GemmArgs g;
  memset(&g, 0, sizeof(g));
  if (c->act_bf16) {
    // [dW_l ; db_l][k] = [act_l ; 1]^T dh_{l+1} over the shard's samples: both operands are the
    // transposed copies (sample index contiguous); the ones row yields the bias gradient,
    // which sits right behind W_l in the flat layout.
    g.A = c->act_t[l]; g.lda = c->ldt;
    g.B = c->dh_t[l + 1]; g.ldb = c->ldt;
    g.M = c->width[l] + 1;
    g.bf16_in = 1;
  } else {  // dW_l[k] = act_l^T dh_{l+1} over the shard's samples
    g.A = l == 0 ? c->x : c->h[l]; g.lda = l == 0 ? c->ldx : c->width[l]; g.a_kc = 0;
    g.B = c->dh[l + 1]; g.ldb = c->width[l + 1]; g.b_kc = 0;
    g.M = c->width[l];
    g.bf16_in = 0;
  }
  g.C = c->shard_grads + c->w_off[l]; g.ldc = c->width[l + 1];
  g.N = c->width[l + 1]; g.K = 0;
  g.epi = EPI_PLAIN; g.bf16_out = 0;
  g.grouped = 1; g.k0 = k0; g.groups = k1 - k0; g.group_stride = c->Pstride;
  ProfScope ps(pr, KID_GEMM_WGRAD, ws);
  HIP_TRY(c, launch_gemm(g, c->tab, ws));
  return ANTDT_OK;
}

// The per-shard dense gradients of a worker step that left them to the dense update: computed
// now, on the weight-gradient stream, for a view (or the stand-alone aggregation) that wants
// them in memory.  Shards that were not stepped get whatever their rows hold (never read back).
static int compute_shard_grads(antdt_ctx* c) {
  if (!c->wgrad_deferred || c->shard_grads_done) return ANTDT_OK;
  hipStream_t ws = c->wside;
  HIP_TRY(c, hipStreamWaitEvent(ws, c->ev_dh[0], 0));
  {
    HeadReduceArgs r = c->head_reduce_args;
    r.part = 1;
    r.k_begin = 0; r.k_end = c->tab.K;
    r.loss_out = nullptr;
    ProfScope ps(prof_of(c), KID_HEAD_REDUCE, ws);
    HIP_TRY(c, launch_head_reduce(r, c->tab, ws));
  }
  for (int l = c->L - 2; l >= 0; --l) {
    const int rc = shard_weight_gradient(c, l, 0, c->tab.K, ws);
    if (rc) return rc;
  }
  HIP_TRY(c, hipEventRecord(c->ev_wgrad, ws));
  c->wgrad_pending = true;
  c->shard_grads_done = true;
  return ANTDT_OK;
}

// Forward and backward of shards [k0, k1) as one batched sequence of launches.
static int worker_range(antdt_ctx* c, int k0, int k1, float* loss_out, hipStream_t s) {
  if (c->stage < ST_BATCH) return fail(c, ANTDT_BAD_STATE, "antdt_worker_step: call antdt_set_batch first");
  if (!c->have_shards || c->shard_B != c->B)
    return fail(c, ANTDT_BAD_STATE, "antdt_worker_step: antdt_assign_shard with the batch's B is required");
  {  // an earlier batched step whose aggregate never came (or whose split was replaced): let its side work finish
    const int rc = join_side(c, s);
    if (rc) return rc;
    c->presorted = false;
  }
  {  // this step overwrites the operands of the previous step's weight-gradient products
    const int rc = join_wgrad(c, s);
    if (rc) return rc;
  }
  Profiler* pr = prof_of(c);
  const antdt_model& m = c->m;
  const ShardTab& tab = c->tab;
  const int64_t s0 = tab.start[k0];
  const int64_t ns = (int64_t)tab.start[k1 - 1] + tab.len[k1 - 1] - s0;
  const int L = c->L;
  const size_t es = c->act_size;
  {
    PoolArgs a;
    a.tables = c->tables; a.ids = c->ids; a.offsets = c->offsets; a.dense = c->dense; a.x = c->x;
    a.F = m.num_fields; a.D = m.dim; a.num_dense = m.num_dense; a.ldx = c->ldx; a.B = (int32_t)c->B;
    a.s0 = (int32_t)s0; a.ns = (int32_t)ns; a.R = m.rows_per_field;
    a.table_bf16 = m.table_dtype == ANTDT_BF16; a.x_bf16 = c->act_bf16;
    a.mean_pool = m.pooling == ANTDT_POOL_MEAN;
    a.xt = c->act_bf16 ? c->act_t[0] : nullptr; a.ldt = c->ldt; a.lookup_sample = c->lookup_sample;
    ProfScope ps(pr, KID_POOL, s);
    HIP_TRY(c, launch_pool(a, c->fp, s));
  }
  c->presorted = false;
  if (k0 == 0 && k1 == tab.K && side_stream(c)) {
    // All shards in one pass: the ids and the sample index of every lookup are known now, so
    // the sort and the run detection of the coming aggregate can run beside the MLP.
    for (int k = 0; k < tab.K; ++k) c->included[k] = true;
    set_weights(c);
    HIP_TRY(c, hipEventRecord(c->ev_fork, s));
    HIP_TRY(c, hipStreamWaitEvent(c->side, c->ev_fork, 0));
    coalesce_whole_batch(c);
    const int rc = build_coalescing(c, c->ids, c->lookup_sample, c->side);
    if (rc) return rc;
    HIP_TRY(c, hipEventRecord(c->ev_join, c->side));
    c->presorted = true;
    c->side_pending = true;
  }
  auto act = [&](int l) -> char* { return l == 0 ? c->x : c->h[l]; };
  auto ld = [&](int l) -> int64_t { return l == 0 ? c->ldx : c->width[l]; };
  auto weight = [&](int l) -> const void* {
    return c->act_bf16 ? (const void*)c->wb[l] : (const void*)(c->params + c->w_off[l]);
  };
  // the matrix products of each pass are timed as one bracket when they run back to back
  ProfScope fwd_scope(L > 1 ? pr : nullptr, KID_GEMM_FWD, s);
  fwd_scope.launches(L - 1);
  for (int l = 0; l + 1 < L; ++l) {  // hidden layers
    GemmArgs g;
    memset(&g, 0, sizeof(g));
    g.A = act(l) + s0 * ld(l) * es; g.lda = ld(l); g.a_kc = 1;
    g.C = c->h[l + 1] + s0 * c->width[l + 1] * es; g.ldc = c->width[l + 1];
    g.bias = c->params + c->b_off[l];
    g.M = (int32_t)ns; g.N = c->width[l + 1];
    if (c->act_bf16) {  // B = W_l^T [out, in padded]; the result also goes to the transposed copy
      g.K = (int32_t)ld(l);
      g.B = c->wbt[l]; g.ldb = ld(l); g.b_kc = 1;
      g.CT = c->act_t[l + 1]; g.ldct = c->ldt; g.ct_col0 = s0;
    } else {
      g.K = c->width[l];
      g.B = c->params + c->w_off[l]; g.ldb = c->width[l + 1]; g.b_kc = 0;
    }
    g.epi = EPI_BIAS_RELU; g.bf16_in = c->act_bf16; g.bf16_out = c->act_bf16;
    HIP_TRY(c, launch_gemm(g, tab, s));
  }
  fwd_scope.close();
  {
    HeadArgs a;
    memset(&a, 0, sizeof(a));
    a.h = act(L - 1); a.ldh = ld(L - 1); a.width = c->width[L - 1];
    a.w = c->params + c->w_off[L - 1]; a.b = c->params + c->b_off[L - 1];
    a.labels = c->labels; a.z = c->z; a.loss_s = c->loss_s; a.dz = c->dz;
    a.bf16_h = c->act_bf16;
    if (L > 1) {
      a.dh = c->dh[L - 1]; a.lddh = c->width[L - 1]; a.dh_cols = c->width[L - 1]; a.relu = 1; a.bf16_dh = c->act_bf16;
    } else {
      a.dh = c->dx; a.lddh = c->FD; a.dh_cols = c->FD; a.relu = 0; a.bf16_dh = 0;
    }
    a.k_begin = k0; a.k_end = k1;
    const bool head_writes_dht = c->act_bf16 && L > 1 && c->width[L - 1] <= 4096;
    if (head_writes_dht) {
      a.dht = c->dh_t[L - 1];
      a.ldt = c->ldt;
    }
    {
      ProfScope ps(pr, KID_HEAD, s);
      HIP_TRY(c, launch_head(a, tab, s));
    }
    HeadReduceArgs r;
    memset(&r, 0, sizeof(r));
    r.h = act(L - 1); r.ldh = ld(L - 1); r.width = c->width[L - 1]; r.bf16_h = c->act_bf16;
    r.dz = c->dz; r.loss_s = c->loss_s; r.grads = c->shard_grads; r.loss_k = c->loss_k; r.loss_out = loss_out;
    r.P = c->Pstride; r.w_off = c->w_off[L - 1]; r.b_off = c->b_off[L - 1]; r.k_begin = k0; r.k_end = k1;
    if (c->act_bf16 && L > 1) {
      r.ht = c->act_t[L - 1];
      r.ldt = c->ldt;
    }
    // With a weight-gradient stream, only the bias sum and the shard losses stay on the launch
    // stream (one wavefront per shard); the weight sums of the last layer, which nothing needs
    // before the dense update, are computed on that stream ahead of the other weight gradients.
    c->head_weights_deferred = r.ht != nullptr && L > 1 && wgrad_stream(c) != nullptr;  // (launched with the weight gradients)
    r.part = c->head_weights_deferred ? 2 : 0;
    {
      ProfScope ps(pr, KID_HEAD_REDUCE, s);
      HIP_TRY(c, launch_head_reduce(r, tab, s));
    }
    c->head_reduce_args = r;
    if (c->act_bf16 && L > 1 && !head_writes_dht) {  // the weight-gradient product wants dh^T
      TransposeArgs t;
      memset(&t, 0, sizeof(t));
      t.n = 1;
      t.src[0] = (const bf16_t*)c->dh[L - 1] + s0 * c->width[L - 1];
      t.dst[0] = c->dh_t[L - 1] + s0;
      t.rows[0] = (int32_t)ns; t.cols[0] = c->width[L - 1];
      t.ld_src[0] = c->width[L - 1]; t.ld_dst[0] = c->ldt;
      t.tile_base[1] = (int32_t)((ns + 63) / 64) * ((c->width[L - 1] + 63) / 64);
      ProfScope ps(pr, KID_TRANSPOSE, s);
      HIP_TRY(c, launch_transpose_bf16(t, s));
    }
  }
  // Backward.  The data-gradient chain dH_{l+1} -> dH_l stays on the launch stream; the weight
  // gradient of layer l needs dH_{l+1} but nothing needs it before the dense update, so it goes
  // to its own stream and runs beside the rest of the chain and the sparse reduction.
  hipStream_t ws = wgrad_stream(c) ? wgrad_stream(c) : s;
  // With bf16 products and a weight-gradient stream the weight gradients are not computed here
  // at all: apply_update forms them inside the dense update (aggregated over the shards in
  // registers, never written per shard), and this step only records when their operands are
  // complete.  The per-shard gradients of the contract are computed when a view asks for them.
  const bool deferred = c->act_bf16 && L > 1 && c->wside && !c->static_bound && !c->eager_wgrad;
  c->wgrad_deferred = deferred;
  c->shard_grads_done = false;
  if (deferred && L == 2) HIP_TRY(c, hipEventRecord(c->ev_dh[0], s));  // dH_1 comes from the loss kernel
  ProfScope bwd_scope(c->act_bf16 && L > 1 ? pr : nullptr, KID_GEMM_BWD, s);
  bwd_scope.launches(L - 1);
  Profiler* pr_each = c->act_bf16 ? nullptr : pr;  // the fp32 path has other kernels in between
  auto weight_gradient = [&](int l) -> int { return shard_weight_gradient(c, l, k0, k1, ws); };
  // An event record costs the launch stream about as much as a small kernel, so the weight
  // gradients are released in pairs: after the data gradient of layer l both dW_l (needs
  // dH_{l+1}) and dW_{l-1} (needs dH_l) can start.
  int next_w = L - 2;  // highest layer whose weight gradient is not launched yet
  for (int l = L - 2; l >= 0; --l) {
    if (!c->act_bf16) {
      BiasGradArgs b;
      memset(&b, 0, sizeof(b));
      b.dh = c->dh[l + 1]; b.lddh = c->width[l + 1]; b.width = c->width[l + 1]; b.bf16_dh = 0;
      b.grads = c->shard_grads; b.P = c->Pstride; b.b_off = c->b_off[l]; b.k_begin = k0; b.k_end = k1;
      ProfScope ps(pr, KID_BIAS_GRAD, s);
      HIP_TRY(c, launch_bias_grad(b, tab, s));
    }
    {  // gradient w.r.t. act_l: through W_l, then the ReLU of layer l-1 (none for the input)
      GemmArgs g;
      memset(&g, 0, sizeof(g));
      g.A = c->dh[l + 1] + s0 * c->width[l + 1] * es; g.lda = c->width[l + 1]; g.a_kc = 1;
      g.B = weight(l); g.ldb = c->width[l + 1]; g.b_kc = 1;
      g.M = (int32_t)ns; g.K = c->width[l + 1];
      g.bf16_in = c->act_bf16;
      if (l > 0) {
        g.C = c->dh[l] + s0 * c->width[l] * es; g.ldc = c->width[l]; g.N = c->width[l];
        g.mask = c->h[l] + s0 * c->width[l] * es; g.ldmask = c->width[l];
        g.epi = EPI_RELU_MASK; g.bf16_out = c->act_bf16;
        if (c->act_bf16) {
          g.CT = c->dh_t[l]; g.ldct = c->ldt; g.ct_col0 = s0;
        }
      } else {
        g.C = c->dx + s0 * c->FD; g.ldc = c->FD; g.N = c->FD;
        g.epi = EPI_PLAIN; g.bf16_out = 0;
      }
      ProfScope ps(pr_each, KID_GEMM_DGRAD, s);
      HIP_TRY(c, launch_gemm(g, tab, s));
    }
    if (deferred) {
      if (l == 1) HIP_TRY(c, hipEventRecord(c->ev_dh[0], s));  // dH_1, the last operand of the weight gradients
      continue;
    }
    const bool release = l == 0 || ((L - 2 - l) & 1) == 0;
    if (release) {
      if (ws != s) {
        if (l == 0) bwd_scope.close();
        HIP_TRY(c, hipEventRecord(c->ev_dh[l], s));
        HIP_TRY(c, hipStreamWaitEvent(ws, c->ev_dh[l], 0));
        if (c->head_weights_deferred) {  // (first release: everything the loss kernel wrote is behind this event)
          HeadReduceArgs r = c->head_reduce_args;
          r.part = 1;
          ProfScope ps(pr, KID_HEAD_REDUCE, ws);
          HIP_TRY(c, launch_head_reduce(r, tab, ws));
          c->head_weights_deferred = false;
        }
      }
      for (const int last = l > 0 ? l - 1 : 0; next_w >= last; --next_w) {
        const int rc = weight_gradient(next_w);
        if (rc) return rc;
      }
    }
  }
  bwd_scope.close();
  if (L > 1 && ws != s && !deferred) {
    HIP_TRY(c, hipEventRecord(c->ev_wgrad, ws));
    c->wgrad_pending = true;
  }
  for (int k = k0; k < k1; ++k) c->stepped[k] = true;
  if (c->stage == ST_AGGREGATED) c->stage = ST_BATCH;
  return ANTDT_OK;
}

int antdt_worker_step(antdt_ctx* c, int32_t k, float* loss_out, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_worker_step: null context");
  if (!c->have_shards || k < 0 || k >= c->tab.K) return fail(c, ANTDT_INVALID_ARG, "antdt_worker_step: shard index out of range");
  return worker_range(c, k, k + 1, loss_out, (hipStream_t)stream);
}

int antdt_worker_step_all(antdt_ctx* c, float* loss_out, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_worker_step_all: null context");
  if (!c->have_shards) return fail(c, ANTDT_BAD_STATE, "antdt_worker_step_all: call antdt_assign_shard first");
  return worker_range(c, 0, c->tab.K, loss_out, (hipStream_t)stream);
}

int antdt_aggregate(antdt_ctx* c, const uint8_t* shard_mask, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_aggregate: null context");
  if (c->stage < ST_BATCH || !c->have_shards || c->shard_B != c->B)
    return fail(c, ANTDT_BAD_STATE, "antdt_aggregate: set_batch, assign_shard and worker_step come first");
  hipStream_t s = (hipStream_t)stream;
  const int K = c->tab.K;
  for (int k = 0; k < K; ++k) {
    c->included[k] = !shard_mask || shard_mask[k];
    if (c->included[k]) {
      if (c->tab.len[k] > 0 && !c->stepped[k])
        return fail(c, ANTDT_BAD_STATE, "antdt_aggregate: an included shard has no worker_step result");
    }
  }
  bool all = true;  // leaving out an empty shard changes nothing
  for (int k = 0; k < K; ++k) all = all && (c->included[k] || c->tab.len[k] == 0);
  {  // also when the structure built there is stale (a new split): its buffers are rebuilt below
    const int rc = join_side(c, s);
    if (rc) return rc;
  }
  if (c->presorted && all && !c->weights_dirty) {
    // the batched worker step already built the structure on the side stream
  } else if (all) {
    set_weights(c);
    coalesce_whole_batch(c);
    const int rc = build_coalescing(c, c->ids, c->lookup_sample, s);
    if (rc) return rc;
  } else {
    // Some shards are left out: pack the lookups of the others (the unique-id buffers serve as
    // staging; the sort has consumed them before the runs are emitted there), fetch the
    // per-field counts (the one place where the host waits for the stream) and coalesce those.
    set_weights(c);
    const int F = c->m.num_fields;
    int32_t* ids_in = c->uniq;
    int32_t* pay_in = c->ufield;
    HIP_TRY(c, launch_mask_pack(c->ids, c->lookup_sample, c->offsets, c->B, F, c->fp, c->tab, c->cbase, ids_in,
                                pay_in, s));
    int64_t cb[ANTDT_MAX_FIELDS + 1];
    HIP_TRY(c, hipMemcpyAsync(cb, c->cbase, (size_t)(F + 1) * 8, hipMemcpyDeviceToHost, s));
    HIP_TRY(c, hipStreamSynchronize(s));
    memset(&c->afp, 0, sizeof(c->afp));
    for (int f = 0; f <= F; ++f) {
      if (cb[f] < 0 || cb[f] > c->fp.p[F] || (f > 0 && cb[f] < cb[f - 1]))
        return fail(c, ANTDT_INVALID_ARG, "antdt_aggregate: offsets of the batch are not monotone");
      c->afp.p[f] = cb[f];
    }
    for (int f = F + 1; f <= ANTDT_MAX_FIELDS; ++f) c->afp.p[f] = c->afp.p[F];
    plan_tiles(F, c->afp, c->atb, c->amax_tiles, c->atotal_tiles);
    const int rc = build_coalescing(c, ids_in, pay_in, s);
    if (rc) return rc;
  }
  c->presorted = false;
  c->g_valid = false;
  c->gdense_valid = false;  // the dense sum is formed inside the optimizer kernel (or on request)
  c->stage = ST_AGGREGATED;
  return ANTDT_OK;
}

int antdt_set_shard_scale(antdt_ctx* c, const double* scale, int32_t K) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_set_shard_scale: null context");
  if (scale && (K < 1 || K > c->m.max_shards)) return fail(c, ANTDT_INVALID_ARG, "antdt_set_shard_scale: K out of range");
  if (scale)
    for (int k = 0; k < K; ++k)
      if (!(scale[k] >= 0.0) || !isfinite(scale[k]))
        return fail(c, ANTDT_INVALID_ARG, "antdt_set_shard_scale: factors must be finite and >= 0");
  for (int k = 0; k < ANTDT_MAX_SHARDS; ++k) c->shard_scale[k] = (scale && k < K) ? scale[k] : 1.0;
  c->weights_dirty = true;  // an aggregation structure built ahead of time carries the old weights
  return ANTDT_OK;
}

int antdt_set_eager_weight_gradients(antdt_ctx* c, int32_t on) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_set_eager_weight_gradients: null context");
  c->eager_wgrad = on != 0;
  return ANTDT_OK;
}

int antdt_set_library_streams(antdt_ctx* c, int32_t on) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_set_library_streams: null context");
  bool stepped = false;
  for (int k = 0; k < ANTDT_MAX_SHARDS; ++k) stepped = stepped || c->stepped[k];
  if (c->side_pending || c->wgrad_pending || stepped)
    return fail(c, ANTDT_BAD_STATE, "antdt_set_library_streams: call it between iterations (after antdt_apply_update or antdt_bind)");
  c->no_streams = on == 0;
  return ANTDT_OK;
}

int antdt_set_lr(antdt_ctx* c, float lr) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_set_lr: null context");
  if (!(lr >= 0.f) || !isfinite(lr)) return fail(c, ANTDT_INVALID_ARG, "antdt_set_lr: lr must be finite and >= 0");
  c->m.lr = lr;
  return ANTDT_OK;
}

int antdt_apply_update(antdt_ctx* c, void* stream) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_apply_update: null context");
  if (c->stage != ST_AGGREGATED) return fail(c, ANTDT_BAD_STATE, "antdt_apply_update: call antdt_aggregate first");
  hipStream_t s = (hipStream_t)stream;
  Profiler* pr = prof_of(c);
  const antdt_model& m = c->m;
  // The dense update touches nothing the sparse update touches, so it runs on the
  // weight-gradient stream (behind those products, which it needs anyway) beside the sparse
  // update; `s` joins it before this call's work on `s` is complete.
  hipStream_t ds = wgrad_stream(c) ? wgrad_stream(c) : s;
  if (ds != s && c->L == 1) {
    // (with hidden layers every worker step ends by making this stream wait for the launch stream)
    HIP_TRY(c, hipEventRecord(c->ev_dh[c->L], s));  // everything enqueued on `s` so far (loss, last layer's gradient)
    HIP_TRY(c, hipStreamWaitEvent(ds, c->ev_dh[c->L], 0));
  }
  {  // weighted run sums with the Adagrad step of every touched row applied on the spot
    SegArgs a;
    fill_seg_args(c, a);
    a.update = 1;
    HIP_TRY(c, launch_seg_reduce(a, c->afp.p[m.num_fields], pr, s));
  }
  if (c->wgrad_deferred) {
    // Weight gradients, their aggregation over the shards and the dense update in one kernel
    // (the per-shard and the aggregated gradient stay in registers), behind the event that
    // says the worker step's activations and pre-activation gradients are complete.
    if (ds != s) {
      HIP_TRY(c, hipStreamWaitEvent(ds, c->ev_dh[0], 0));
    } else {  // (per-shard gradients that a view asked for may still be in flight on the library's stream)
      const int rcj = join_wgrad(c, s);
      if (rcj) return rcj;
    }
    const int Lh = c->L - 1;  // hidden layers
    if (!c->shard_grads_done) {  // last layer: per-shard weight sums (its bias sum is already there)
      HeadReduceArgs r = c->head_reduce_args;
      r.part = 1;
      r.k_begin = 0; r.k_end = c->tab.K;
      r.loss_out = nullptr;
      ProfScope ps(pr, KID_HEAD_REDUCE, ds);
      HIP_TRY(c, launch_head_reduce(r, c->tab, ds));
    }
    {
      DenseAdagradArgs a;  // plain range: the last layer's weights and bias
      memset(&a, 0, sizeof(a));
      a.p = c->params; a.state = c->pstate; a.grads = c->shard_grads; a.stride = c->Pstride; a.lr = m.lr; a.eps = m.eps;
      a.n_mat = 0; a.n_rng = 1;
      a.rng_off[0] = c->w_off[Lh]; a.rng_len[0] = c->P - c->w_off[Lh];
      a.rng_block[0] = 0; a.rng_block[1] = (int)((a.rng_len[0] + 255) / 256);
      ProfScope ps(pr, KID_DENSE_ADAGRAD, ds);
      HIP_TRY(c, launch_dense_adagrad(a, c->tab, ds));
    }
    WgradUpdateArgs u;
    memset(&u, 0, sizeof(u));
    u.n_layers = Lh;
    for (int l = 0; l < Lh; ++l) {
      u.A[l] = c->act_t[l]; u.B[l] = c->dh_t[l + 1];
      u.M[l] = c->width[l] + 1; u.N[l] = c->width[l + 1];
      u.w_off[l] = c->w_off[l]; u.wb[l] = l == 0 ? c->wb0_alt : c->wb[l];
    }
    u.ld = c->ldt; u.p = c->params; u.state = c->pstate; u.lr = m.lr; u.eps = m.eps;
    KSegments seg;
    memset(&seg, 0, sizeof(seg));
    for (int k = 0; k < c->tab.K; ++k) {
      const float w = c->tab.w[k];
      if (w == 0.0f || c->tab.len[k] == 0) continue;
      const int ks = c->tab.start[k], ke = ks + c->tab.len[k];
      if (seg.n > 0 && seg.w[seg.n - 1] == w && seg.ke[seg.n - 1] == ks) {
        seg.ke[seg.n - 1] = ke;  // neighbours of equal weight: one range
      } else {
        seg.ks[seg.n] = ks; seg.ke[seg.n] = ke; seg.w[seg.n] = w;
        ++seg.n;
      }
    }
    {
      ProfScope ps(pr, KID_WGRAD_ADAGRAD, ds);
      HIP_TRY(c, launch_wgrad_update(u, seg, ds));
    }
    // The input-gradient product of this step, enqueued behind the event this stream waited for,
    // may still be reading the old bf16 copy of W_0: the kernel wrote the new one to the other
    // buffer, which is the current one from here on (the products of deeper layers ran before
    // the event).
    std::swap(c->wb[0], c->wb0_alt);
    {
      const int rc = transpose_weights(c, ds);  // the forward operand copies W_l^T from the new W_l
      if (rc) return rc;
    }
    if (ds != s) {
      HIP_TRY(c, hipEventRecord(c->ev_wgrad, ds));
      HIP_TRY(c, hipStreamWaitEvent(s, c->ev_wgrad, 0));
    }
    c->wgrad_pending = false;  // `s` now waits for everything on that stream
  } else {
    DenseAdagradArgs a;
    memset(&a, 0, sizeof(a));
    a.p = c->params; a.state = c->pstate; a.grads = c->shard_grads; a.stride = c->Pstride; a.lr = m.lr; a.eps = m.eps;
    int nr = 0, rblocks = 0;
    auto add_range = [&](int64_t off, int64_t len) {
      a.rng_off[nr] = off; a.rng_len[nr] = len; a.rng_block[nr] = rblocks;
      rblocks += (int)((len + 255) / 256);
      ++nr;
    };
    if (c->act_bf16) {
      for (int l = 0; l + 1 < c->L; ++l) {
        a.w_off[l] = c->w_off[l]; a.rows[l] = c->width[l]; a.cols[l] = c->width[l + 1];
        a.rows_pad[l] = l == 0 ? c->ldx : c->width[l];
        a.wb[l] = c->wb[l]; a.wbt[l] = c->wbt[l];
        a.tile_base[l + 1] = a.tile_base[l] + ((c->width[l] + 63) / 64) * ((c->width[l + 1] + 63) / 64);
        add_range(c->b_off[l], c->width[l + 1]);
      }
      a.n_mat = c->L - 1;
      add_range(c->w_off[c->L - 1], c->P - c->w_off[c->L - 1]);
    } else {
      add_range(0, c->P);
    }
    a.n_rng = nr;
    a.rng_block[nr] = rblocks;
    {
      ProfScope ps(pr, KID_DENSE_ADAGRAD, ds);
      HIP_TRY(c, launch_dense_adagrad(a, c->tab, ds));
    }
    if (ds != s) {
      HIP_TRY(c, hipEventRecord(c->ev_wgrad, ds));
      HIP_TRY(c, hipStreamWaitEvent(s, c->ev_wgrad, 0));
      c->wgrad_pending = false;  // `s` now waits for everything on that stream
    }
  }
  c->stage = ST_BATCH;
  memset(c->stepped, 0, sizeof(c->stepped));
  return ANTDT_OK;
}

int antdt_dense_aggregate_adam(float* p, float* mm, float* v, const float* const* grads, const float* weights,
                               int32_t K, int64_t n, double lr, double beta1, double beta2, double eps,
                               int64_t step, void* stream) {
  if (K < 1 || K > 16) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_dense_aggregate_adam: K must be 1..16");
  if (n < 0 || step < 1) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_dense_aggregate_adam: n >= 0 and step >= 1 required");
  if (n == 0) return ANTDT_OK;  // nothing to do; empty buffers may be null
  if (!p || !mm || !v || !grads || !weights) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_dense_aggregate_adam: null argument");
  AdamArgs a;
  memset(&a, 0, sizeof(a));
  a.p = p; a.m = mm; a.v = v; a.K = K; a.n = n;
  uintptr_t al = (uintptr_t)p | (uintptr_t)mm | (uintptr_t)v;
  for (int k = 0; k < K; ++k) {
    if (!grads[k]) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_dense_aggregate_adam: null gradient buffer");
    a.g[k] = grads[k];
    a.w[k] = weights[k];
    al |= (uintptr_t)grads[k];
  }
  if (al & 15) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_dense_aggregate_adam: buffers must be 16-byte aligned");
  a.lr = (float)lr; a.b1 = (float)beta1; a.b2 = (float)beta2; a.eps = (float)eps;
  a.c1 = (float)(1.0 - beta1); a.c2 = (float)(1.0 - beta2);
  a.inv_bc1 = (float)(1.0 / (1.0 - pow(beta1, (double)step)));
  a.inv_bc2 = (float)(1.0 / (1.0 - pow(beta2, (double)step)));
  HIP_TRY(nullptr, launch_adam(a, (hipStream_t)stream));
  return ANTDT_OK;
}

int antdt_stream_copy(float* dst, const float* src, int64_t n, void* stream) {
  if (n < 0 || n >= (1ll << 40) || (n > 0 && (!dst || !src)) || (((uintptr_t)dst | (uintptr_t)src) & 15))
    return fail(nullptr, ANTDT_INVALID_ARG, "antdt_stream_copy: null or misaligned pointer, or n out of range");
  HIP_TRY(nullptr, launch_stream_copy(dst, src, n, (hipStream_t)stream));
  return ANTDT_OK;
}

int antdt_fill_tables(void* tables, int32_t dtype, int32_t F, int64_t R, int32_t D, float scale, void* stream) {
  if (!tables || F < 1 || R < 1 || D < 1 || (dtype != ANTDT_F32 && dtype != ANTDT_BF16))
    return fail(nullptr, ANTDT_INVALID_ARG, "antdt_fill_tables: invalid argument");
  HIP_TRY(nullptr, launch_fill_tables(tables, dtype == ANTDT_BF16, F, R, D, scale, (hipStream_t)stream));
  return ANTDT_OK;
}

int antdt_view_pooled(antdt_ctx* c, int32_t k, const void** x, int64_t* rows, int64_t* ldo, int32_t* dtype) {
  if (!c || !x || !rows || !ldo || !dtype) return fail(c, ANTDT_INVALID_ARG, "antdt_view_pooled: null argument");
  if (!c->have_shards || k < 0 || k >= c->tab.K) return fail(c, ANTDT_INVALID_ARG, "antdt_view_pooled: shard index out of range");
  if (c->stage < ST_BATCH) return fail(c, ANTDT_BAD_STATE, "antdt_view_pooled: nothing computed yet");
  *x = c->x + (int64_t)c->tab.start[k] * c->ldx * c->act_size;
  *rows = c->tab.len[k];
  *ldo = c->ldx;
  *dtype = c->act_bf16 ? ANTDT_BF16 : ANTDT_F32;
  return ANTDT_OK;
}

int antdt_view_shard_grads(antdt_ctx* c, int32_t k, const float** dense, const float** dx, int64_t* ld_dx) {
  if (!c || !dense || !dx || !ld_dx) return fail(c, ANTDT_INVALID_ARG, "antdt_view_shard_grads: null argument");
  if (!c->have_shards || k < 0 || k >= c->tab.K) return fail(c, ANTDT_INVALID_ARG, "antdt_view_shard_grads: shard index out of range");
  if (c->stage < ST_BATCH) return fail(c, ANTDT_BAD_STATE, "antdt_view_shard_grads: nothing computed yet");
  {
    const int rcg = compute_shard_grads(c);
    if (rcg) return rcg;
  }
  if (c->wgrad_pending) {  // the weight gradients are written on their own stream: wait for it here
    HIP_TRY(c, hipStreamSynchronize(c->wside));
    c->wgrad_pending = false;
  }
  *dense = c->shard_grads + (int64_t)k * c->Pstride;
  *dx = c->dx + (int64_t)c->tab.start[k] * c->FD;
  *ld_dx = c->FD;
  return ANTDT_OK;
}

int antdt_view_dense_grad(antdt_ctx* c, const float** g, void* stream) {
  if (!c || !g) return fail(c, ANTDT_INVALID_ARG, "antdt_view_dense_grad: null argument");
  if (c->stage != ST_AGGREGATED) return fail(c, ANTDT_BAD_STATE, "antdt_view_dense_grad: valid between antdt_aggregate and antdt_apply_update");
  {
    const int rcg = compute_shard_grads(c);
    if (rcg) return rcg;
    const int rcj = join_wgrad(c, (hipStream_t)stream);
    if (rcj) return rcj;
  }
  if (!c->gdense_valid) {  // written out on request only; apply_update forms the same sum on the fly
    DenseAggArgs d;
    d.grads = c->shard_grads; d.g = c->g_dense; d.P = c->P; d.stride = c->Pstride;
    ProfScope ps(prof_of(c), KID_DENSE_AGG, (hipStream_t)stream);
    HIP_TRY(c, launch_dense_agg(d, c->tab, (hipStream_t)stream));
    c->gdense_valid = true;
  }
  *g = c->g_dense;
  return ANTDT_OK;
}

int antdt_view_coalesced(antdt_ctx* c, int32_t f, const int32_t** unique_ids, const int32_t** seg_offsets,
                         const int32_t** seg_samples, int64_t* num_unique, int64_t* nnz, const float** G,
                         void* stream) {
  if (!c || !unique_ids || !seg_offsets || !seg_samples || !num_unique || !nnz || !G)
    return fail(c, ANTDT_INVALID_ARG, "antdt_view_coalesced: null argument");
  if (f < 0 || f >= c->m.num_fields) return fail(c, ANTDT_INVALID_ARG, "antdt_view_coalesced: field out of range");
  if (c->stage < ST_BATCH) return fail(c, ANTDT_BAD_STATE, "antdt_view_coalesced: call antdt_aggregate first");
  if (c->stage != ST_AGGREGATED) return fail(c, ANTDT_BAD_STATE, "antdt_view_coalesced: valid between antdt_aggregate and antdt_apply_update");
  if (!c->g_valid) {  // the coalesced sums are only written out on request
    SegArgs a;
    fill_seg_args(c, a);
    a.update = 0;
    HIP_TRY(c, launch_seg_reduce(a, c->afp.p[c->m.num_fields], prof_of(c), (hipStream_t)stream));
    c->g_valid = true;
  }
  int32_t ub[2];
  HIP_TRY(c, hipMemcpyAsync(ub, c->ubase + f, sizeof(ub), hipMemcpyDeviceToHost, (hipStream_t)stream));
  HIP_TRY(c, hipStreamSynchronize((hipStream_t)stream));
  *unique_ids = c->uniq + ub[0];
  *seg_offsets = c->segoff + ub[0] + f;
  *seg_samples = c->pay[c->sorted_buf] + c->afp.p[f];
  *num_unique = ub[1] - ub[0];
  *nnz = c->afp.p[f + 1] - c->afp.p[f];
  *G = c->G + (int64_t)ub[0] * c->m.dim;
  return ANTDT_OK;
}

int antdt_profile(antdt_ctx* c, int32_t mode, int32_t kernel_id) {
  if (!c) return fail(nullptr, ANTDT_INVALID_ARG, "antdt_profile: null context");
  if (mode < 0 || mode > 3 || (mode == 2 && (kernel_id < 0 || kernel_id >= KID_COUNT)))
    return fail(c, ANTDT_INVALID_ARG, "antdt_profile: invalid mode or kernel id");
  c->prof.mode = mode;
  c->prof.sel = kernel_id;
  return ANTDT_OK;
}

int antdt_profile_overhead(antdt_ctx* c, void* stream, int32_t n, double* empty_ms, double* tiny_ms) {
  if (!c || !empty_ms || !tiny_ms || n < 1 || n > 4096)
    return fail(c, ANTDT_INVALID_ARG, "antdt_profile_overhead: null argument or n outside 1..4096");
  if (c->stage < ST_BOUND) return fail(c, ANTDT_BAD_STATE, "antdt_profile_overhead: call antdt_bind first");
  hipStream_t s = (hipStream_t)stream;
  std::vector<hipEvent_t> ev((size_t)n * 4);
  for (auto& e : ev) HIP_TRY(c, hipEventCreateWithFlags(&e, hipEventDisableSystemFence));
  for (int i = 0; i < n; ++i) {  // the flags kernel is the smallest one the library has
    HIP_TRY(c, launch_validate_reset(c->vflags, s));
    HIP_TRY(c, hipEventRecord(ev[4 * i + 0], s));
    HIP_TRY(c, hipEventRecord(ev[4 * i + 1], s));
    HIP_TRY(c, launch_validate_reset(c->vflags, s));
    HIP_TRY(c, hipEventRecord(ev[4 * i + 2], s));
    HIP_TRY(c, launch_validate_reset(c->vflags, s));
    HIP_TRY(c, hipEventRecord(ev[4 * i + 3], s));
  }
  HIP_TRY(c, hipStreamSynchronize(s));
  double e_sum = 0.0, t_sum = 0.0;
  for (int i = 0; i < n; ++i) {
    float a = 0.f, b = 0.f;
    HIP_TRY(c, hipEventElapsedTime(&a, ev[4 * i + 0], ev[4 * i + 1]));
    HIP_TRY(c, hipEventElapsedTime(&b, ev[4 * i + 2], ev[4 * i + 3]));
    e_sum += a;
    t_sum += b;
  }
  for (auto& e : ev) (void)hipEventDestroy(e);
  *empty_ms = e_sum / n;
  *tiny_ms = t_sum / n;
  return ANTDT_OK;
}

int antdt_profile_read(antdt_ctx* c, int32_t kid, int64_t* launches, double* total_ms) {
  if (!c || !launches || !total_ms) return fail(c, ANTDT_INVALID_ARG, "antdt_profile_read: null argument");
  if (kid < 0 || kid >= KID_COUNT) return fail(c, ANTDT_INVALID_ARG, "antdt_profile_read: kernel id out of range");
  prof_drain(&c->prof);
  *launches = c->prof.launches[kid];
  *total_ms = c->prof.total_ms[kid];
  c->prof.launches[kid] = 0;
  c->prof.total_ms[kid] = 0.0;
  return ANTDT_OK;
}

}  // extern "C"
