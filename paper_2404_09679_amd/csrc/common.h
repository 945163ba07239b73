// Shared declarations of the gfx950 kernels and their host-side launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "antdt.h"

#include <string>

namespace antdt {

void set_last_error(const std::string& msg);  // message returned by antdt_last_error(NULL)

typedef uint16_t bf16_t;  // raw bfloat16 bit pattern

__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// float -> bfloat16, round to nearest even (NaN stays NaN).
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return bf2f(x); }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float x) { return f2bf(x); }

// Small tables passed to kernels by value (kernel-argument segment), so that no
// host-to-device copy is needed per call.
struct FieldPtr {
  int64_t p[ANTDT_MAX_FIELDS + 1];  // start of each field's lookups inside ids
};
struct ShardTab {
  int32_t K;
  int32_t start[ANTDT_MAX_SHARDS];
  int32_t len[ANTDT_MAX_SHARDS];
  float w[ANTDT_MAX_SHARDS];  // aggregation weight B_k / sum of included B_k (0 if excluded)
};
struct TileBase {
  int32_t t[ANTDT_MAX_FIELDS + 1];  // prefix sum of sort tiles per field
  // xcum[x][j] = tiles of the fields x, x + 8, ..., x + 8 (j - 1): the blocks with index x modulo 8 take the
  // tiles of these fields in this order (16 fields per group at most; entries past the last field repeat the total)
  int32_t xcum[8][ANTDT_MAX_FIELDS / 8 + 1];
};
static_assert(ANTDT_MAX_FIELDS % 8 == 0, "fields are dealt to eight groups");

// Kernel classes for the optional event timing.
enum KernelId {
  KID_POOL = 0,
  KID_GEMM_FWD,
  KID_GEMM_DGRAD,
  KID_GEMM_WGRAD,
  KID_HEAD,
  KID_HEAD_REDUCE,
  KID_BIAS_GRAD,
  KID_SORT_HIST,
  KID_SORT_SCAN,
  KID_SORT_SCATTER,
  KID_SEG_HEADS,
  KID_SEG_SCAN,
  KID_SEG_EMIT,
  KID_SEG_REDUCE,
  KID_SEG_REDUCE_LONG,
  KID_DENSE_AGG,
  KID_SPARSE_ADAGRAD,
  KID_DENSE_ADAGRAD,
  KID_ADAM,
  KID_TRANSPOSE,
  KID_GEMM_BWD,
  KID_WGRAD_ADAGRAD,
  KID_COUNT
};

struct Profiler;  // defined in ctx.hip
int prof_begin(Profiler* p, int kid, hipStream_t s);   // returns the bracket's index, -1 if not timed
void prof_end(Profiler* p, int idx, hipStream_t s);
void prof_count(Profiler* p, int idx, int launches);   // launches covered by the bracket (default 1)

// A pair of events on stream `s` around the launches made while the scope is open.
struct ProfScope {
  Profiler* p;
  int idx = -1;
  hipStream_t s;
  ProfScope(Profiler* p_, int kid, hipStream_t s_) : p(p_), s(s_) {
    if (p) idx = prof_begin(p, kid, s);
  }
  ~ProfScope() { close(); }
  // One bracket around several back-to-back launches: the bracket itself costs a few
  // microseconds on the stream, which would swamp kernels of 10-20 us if each had its own.
  void launches(int n) {
    if (p && idx >= 0) prof_count(p, idx, n);
  }
  void close() {  // end the bracket before the scope does
    if (p && idx >= 0) prof_end(p, idx, s);
    p = nullptr;
  }
};

// ---------------------------------------------------------------- embed.hip
struct PoolArgs {
  const void* tables;
  const int32_t* ids;
  const int32_t* offsets;
  const float* dense;
  void* x;
  bf16_t* xt;             // optional transposed copy [ldx + 8, ldt] (bf16 activations only)
  int32_t* lookup_sample; // optional [nnz]: global sample index of every lookup (sort payload)
  int32_t F, D, num_dense, ldx, B, s0, ns;
  int64_t R, ldt;
  int32_t table_bf16, x_bf16;
  int32_t mean_pool;      // divide every bag's sum by its number of lookups
};
hipError_t launch_pool(const PoolArgs& a, const FieldPtr& fp, hipStream_t s);
hipError_t launch_validate(const int32_t* ids, const int32_t* offsets, const FieldPtr& fp, int64_t B, int64_t R, int F,
                           int32_t* flags, hipStream_t s);
hipError_t launch_validate_reset(int32_t* flags, hipStream_t s);
hipError_t launch_fill_tables(void* tables, int bf16, int F, int64_t R, int D, float scale,
                              hipStream_t s);

// ----------------------------------------------------------------- gemm.hip
enum Epilogue { EPI_BIAS_RELU = 0, EPI_RELU_MASK = 1, EPI_PLAIN = 2 };

// C[m, n] = sum_k A(m, k) * B(n, k).
// fp32 path: a_kc: A(m,k) = A[m*lda + k], else A[k*lda + m]; b_kc likewise for B; with
// `grouped`, group g (blockIdx.z) contracts over rows [tab.start[k0+g], +tab.len[k0+g]) of A
// and B (both not *_kc).
// bf16 path: both operands have the contraction index contiguous (A[m*lda + k], B[n*ldb + k]);
// with `grouped`, group g contracts over k in [tab.start[k0+g], +tab.len[k0+g]).
// Grouped launches write C + (k0+g)*group_stride.  CT, when set, receives the bf16 result
// transposed: CT[n*ldct + ct_col0 + m].
struct GemmArgs {
  const void* A;
  const void* B;
  void* C;
  bf16_t* CT;
  const float* bias;   // EPI_BIAS_RELU: [N]
  const void* mask;    // EPI_RELU_MASK: activations [M, ldmask], C = acc where mask > 0 else 0
  int64_t lda, ldb, ldc, ldct, ct_col0, ldmask;
  int32_t M, N, K;
  int32_t a_kc, b_kc, epi;
  int32_t bf16_in;     // operands (and mask) are bf16, else fp32
  int32_t bf16_out;    // C is bf16, else fp32
  int32_t grouped, k0, groups;
  int64_t group_stride;
};
hipError_t launch_gemm(const GemmArgs& a, const ShardTab& tab, hipStream_t s);

// Weight gradients of all hidden layers with the server's aggregation and dense update applied
// on the spot: for layer l the tile of [dW_l ; db_l] = sum_k w_k * ([act_l ; 1]^T dH_{l+1}) over
// the samples of shard k, accumulated shard after shard in registers, then Adagrad on the matching
// tile of the flat parameters (W_l with b_l right behind it) and the bf16 copy of W_l.  Neither
// the per-shard nor the aggregated gradient goes to memory.
struct KSegments {        // sample ranges with one aggregation weight each (shards; neighbours of
  int32_t n;              // equal weight merged), in sample order
  int32_t ks[ANTDT_MAX_SHARDS], ke[ANTDT_MAX_SHARDS];
  float w[ANTDT_MAX_SHARDS];
};
struct WgradUpdateArgs {
  int32_t n_layers;
  const bf16_t* A[ANTDT_MAX_LAYERS];   // transposed activations [M (with the ones row), ld]
  const bf16_t* B[ANTDT_MAX_LAYERS];   // transposed pre-activation gradients [N, ld]
  int32_t M[ANTDT_MAX_LAYERS], N[ANTDT_MAX_LAYERS];
  int64_t w_off[ANTDT_MAX_LAYERS];     // W_l inside the flat parameters, [M - 1, N] then the bias [N]
  bf16_t* wb[ANTDT_MAX_LAYERS];        // bf16 copy of W_l, [rows padded, N]
  int32_t tile_base[ANTDT_MAX_LAYERS + 1];
  int32_t tiles_n[ANTDT_MAX_LAYERS];
  int64_t ld;
  float* p;
  float* state;
  float lr, eps;
};
hipError_t launch_wgrad_update(const WgradUpdateArgs& a, const KSegments& seg, hipStream_t s);

struct CastArgs {  // fp32 [rows, cols] -> bf16 [rows_pad, cols], extra rows zero
  const float* src;
  bf16_t* dst;
  int64_t n_src, n_dst;
};
hipError_t launch_cast_bf16(const CastArgs& a, hipStream_t s);

struct TransposeArgs {  // dst[c*ld_dst + r] = src[r*ld_src + c] for up to 8 bf16 matrices
  int32_t n;
  const bf16_t* src[ANTDT_MAX_LAYERS];
  bf16_t* dst[ANTDT_MAX_LAYERS];
  int32_t rows[ANTDT_MAX_LAYERS], cols[ANTDT_MAX_LAYERS];
  int64_t ld_src[ANTDT_MAX_LAYERS], ld_dst[ANTDT_MAX_LAYERS];
  int32_t tile_base[ANTDT_MAX_LAYERS + 1];
};
hipError_t launch_transpose_bf16(const TransposeArgs& a, hipStream_t s);

struct OnesRowArgs {    // row `row` of a bf16 matrix [.., ld] = 1, the `zero_rows` rows after it = 0
  bf16_t* base;
  int64_t ld;
  int32_t row, zero_rows;
};
hipError_t launch_ones_row(const OnesRowArgs& a, hipStream_t s);

// ----------------------------------------------------------------- head.hip
struct HeadArgs {
  const void* h;        // [B, ldh] last hidden activation (or the pooled input when there is none)
  const float* w;       // [width] last-layer weight
  const float* b;       // [1]
  const float* labels;  // [B]
  float* z;             // [B]
  float* loss_s;        // [B] per-sample loss
  float* dz;            // [B] d(mean shard loss)/dz
  void* dh;             // [B, lddh] gradient w.r.t. h (masked by h > 0 when `relu`), or fp32 dX
  bf16_t* dht;          // optional transposed bf16 copy [dh_cols, ldt]
  int64_t ldh, lddh, ldt;
  int32_t width, dh_cols, relu, bf16_h, bf16_dh;
  int32_t k_begin, k_end;
};
hipError_t launch_head(const HeadArgs& a, const ShardTab& tab, hipStream_t s);

struct HeadReduceArgs {
  const void* h;
  const float* dz;
  const float* loss_s;
  float* grads;         // [K, P] per-shard flat dense gradients
  float* loss_k;        // workspace [K]
  float* loss_out;      // caller's buffer or NULL; element (k - k_begin)
  const bf16_t* ht;     // optional transposed activation [width, ldt]: selects the coalesced kernel
  int64_t ldh, ldt, P, w_off, b_off;
  int32_t width, bf16_h, k_begin, k_end;
  int32_t part;         // transposed-activation kernel only: 0 everything, 1 the weight sums, 2 bias sum and loss
};
hipError_t launch_head_reduce(const HeadReduceArgs& a, const ShardTab& tab, hipStream_t s);

struct BiasGradArgs {   // db[k][o] = sum over the shard's samples of dh[s, o]
  const void* dh;
  float* grads;
  int64_t lddh, P, b_off;
  int32_t width, bf16_dh, k_begin, k_end;
};
hipError_t launch_bias_grad(const BiasGradArgs& a, const ShardTab& tab, hipStream_t s);

// ------------------------------------------------------------- coalesce.hip
// Keys per sort tile (one block of 512 threads, ANTDT_SORT_TILE / 512 keys per thread).
constexpr int ANTDT_SORT_TILE = 2048;
// Runs per block of the kernels that list the long runs (256 threads, 8 runs each).
constexpr int ANTDT_QUEUE_BLOCK_RUNS = 2048;

struct SortPlan {
  int32_t F, B;
  int32_t passes, radix_bits;      // digit width per pass
  int32_t max_tiles;               // max tiles of one field (grid.x)
  int32_t total_tiles;
};
struct SortBuffers {
  const int32_t* ids;
  const int32_t* offsets;          // [F][B+1]
  const int32_t* pay0;             // sample index of every lookup (payload of the first pass)
  int32_t* key[2];
  int32_t* pay[2];
  uint32_t* hist;                  // [total_tiles << radix_bits]
  uint32_t* digit_base;            // [F << radix_bits]
};
hipError_t launch_sort_pass(const SortPlan& pl, const SortBuffers& sb, int pass, const FieldPtr& fp,
                            const TileBase& tb, Profiler* prof, hipStream_t s);

struct SegArgs {
  const int32_t* key;              // sorted row ids, field-major at fp.p[f]
  const int32_t* pay;              // sample index of each sorted lookup
  int32_t* tile_heads;             // [total_tiles + 1] heads per tile -> exclusive prefix
  int32_t* ubase;                  // [F + 1] first unique of each field; ubase[F] = U
  int32_t* uniq;                   // [U] row id of each run
  int32_t* ufield;                 // [U] field of each run
  int32_t* segabs;                 // [U + 1] start of each run in the sorted arrays (all fields)
  int32_t* segoff;                 // [U + F], per-field offsets; field f's slice starts at ubase[f] + f
  float* sample_w;                 // [B]
  int32_t* counters;               // [2]: number of long runs, number of chunk work items
  int32_t* qcnt;                   // [2 * queue blocks]: long runs and chunks found by each block of the list
                                   // builder, then their exclusive prefix sums
  int32_t* xcd_tab;                // [3][9]: first run, first chunk item and first long run of each of the 8
                                   // shares into which the reduction divides its work (entry 8 = the totals)
  int32_t* long_seg;               // [long_cap][3]: run, first item, number of chunks
  int32_t* items;                  // [item_cap][2]: run, chunk index
  float* partial;                  // [item_cap, D] chunk sums of long runs
  float* G;                        // [U, D] coalesced gradient (written when not updating)
  const float* dx;                 // [B, lddx]
  int64_t lddx;
  const int32_t* offsets;          // [F][B + 1] bag boundaries of the batch (read when mean_pool)
  int32_t mean_pool;               // bags are averaged: a lookup's gradient is dX / bag length
  int32_t F, D, B, max_tiles, total_tiles, long_threshold, chunk, long_cap, item_cap;
  // parameter update fused into the reduction (update != 0)
  int32_t update, table_bf16, rowwise;
  void* tables;
  float* state;
  int64_t R;
  float lr, eps;
};
hipError_t launch_segments(const SegArgs& a, const FieldPtr& fp, const TileBase& tb,
                           const ShardTab& tab, Profiler* prof, hipStream_t s);
hipError_t launch_mask_pack(const int32_t* ids, const int32_t* lookup_sample, const int32_t* offsets, int64_t B, int F,
                            const FieldPtr& fp, const ShardTab& tab, int64_t* cbase, int32_t* ids_out,
                            int32_t* pay_out, hipStream_t s);
hipError_t launch_seg_reduce(const SegArgs& a, int64_t nnz_total, Profiler* prof, hipStream_t s);

// ---------------------------------------------------------------- optim.hip
struct DenseAggArgs {
  const float* grads;  // [K, stride] per-shard flat gradients
  float* g;            // [P]
  int64_t P, stride;
};
hipError_t launch_dense_agg(const DenseAggArgs& a, const ShardTab& tab, hipStream_t s);

// Dense Adagrad on the flat MLP parameters with the gradient aggregated on the fly
// (g = sum_k w_k grads[k]).  Hidden-layer weight matrices are walked in 64x64 tiles so that
// both bf16 operand copies (W as [in,out] and W^T as [out,in_pad]) are refreshed with
// coalesced stores in the same pass; everything else (biases, the last layer) goes through
// plain ranges.
struct DenseAdagradArgs {
  float* p;
  float* state;
  const float* grads;  // [K, stride]
  int64_t stride;
  float lr, eps;
  int32_t n_mat;
  int64_t w_off[ANTDT_MAX_LAYERS];
  int32_t rows[ANTDT_MAX_LAYERS], cols[ANTDT_MAX_LAYERS], rows_pad[ANTDT_MAX_LAYERS];
  bf16_t* wb[ANTDT_MAX_LAYERS];
  bf16_t* wbt[ANTDT_MAX_LAYERS];
  int32_t tile_base[ANTDT_MAX_LAYERS + 1];
  int32_t n_rng;
  int64_t rng_off[ANTDT_MAX_LAYERS + 1], rng_len[ANTDT_MAX_LAYERS + 1];
  int32_t rng_block[ANTDT_MAX_LAYERS + 2];  // first block of each range, relative to the first range block
};
hipError_t launch_dense_adagrad(const DenseAdagradArgs& a, const ShardTab& tab, hipStream_t s);

struct AdamArgs {
  float* p;
  float* m;
  float* v;
  const float* g[16];
  float w[16];
  int32_t K;
  int64_t n;
  float lr, b1, b2, c1, c2, eps, inv_bc1, inv_bc2;  // c = 1 - b, formed in double on the host
};
hipError_t launch_adam(const AdamArgs& a, hipStream_t s);
hipError_t launch_stream_copy(float* dst, const float* src, int64_t n, hipStream_t s);

}  // namespace antdt
