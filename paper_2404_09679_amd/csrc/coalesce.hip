// Server-side coalescing of the pushed sparse gradients (Section II: the servers combine
// the gradients of all workers): per field, a stable LSD radix
// sort of (row id, sample index) pairs, detection of the runs of equal ids
// (unique ids + segment offsets), and the weighted segmented reduction
//   G[u, :] = sum over the run of w(sample) * dX[sample, field slice].
// No floating-point atomics are used, so the sums are bitwise repeatable.  The reduction can
// apply the row-sparse Adagrad step of each row at once (the parameter update of Section II).
#include <algorithm>

#include "common.h"

namespace antdt {
namespace {

constexpr int SORT_THREADS = 512;
constexpr int SORT_WAVES = SORT_THREADS / 64;
constexpr int SORT_TILE = ANTDT_SORT_TILE;            // keys per block
constexpr int SORT_ITEMS = SORT_TILE / SORT_THREADS;
constexpr int MAX_BINS = 1024;

__device__ __forceinline__ uint64_t lanemask_lt() {
  const unsigned lane = threadIdx.x & 63;
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// Block -> (field, tile) for the kernels that walk the lookups of the fields tile by tile.  The
// hardware hands block i to XCD i mod 8, and every XCD has an L2 of its own: the blocks whose index
// is x modulo 8 take the tiles of the fields x, x + 8, x + 16, ..., so that every pass over a
// field's lookups runs on one XCD.  The scattered 4-byte stores of a sort pass are then assembled
// into full lines in that L2 (spread over eight L2s, each wrote its partial lines back: 3.7 times
// the payload), and the next pass over the field finds them there.
__device__ __forceinline__ bool field_tile_of_block(const TileBase& tb, int F, int& f, int& t) {
  constexpr int G = ANTDT_MAX_FIELDS / 8;
  const int x = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int32_t* cum = tb.xcum[x];  // (one row of the table: a single scalar load)
  if (slot >= cum[G]) return false;
  int j = 0;
#pragma unroll
  for (int i = 1; i < G; ++i) j += slot >= cum[i] ? 1 : 0;
  f = x + 8 * j;
  t = slot - cum[j];
  return f < F;
}

// ----------------------------------------------------------------- sort
// Histogram layout: hist[(tile_base[f] + tile) << rb | digit] (digits of a tile contiguous);
// digit_base[f << rb | digit] = number of the field's keys with a smaller digit.

// Digit histogram of one tile.
__global__ __launch_bounds__(SORT_THREADS) void sort_hist_kernel(const int32_t* keys, uint32_t* hist,
                                                                 FieldPtr fp, TileBase tb, int F, int shift, int rb) {
  __shared__ uint32_t h[MAX_BINS];
  int f, t;
  if (!field_tile_of_block(tb, F, f, t)) return;
  const int nb = 1 << rb;
  const int64_t base = fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - base);
  int32_t k[SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {  // all loads first (clamped), so that they overlap
    const int pos = min(t * SORT_TILE + i * SORT_THREADS + (int)threadIdx.x, nnz - 1);
    k[i] = keys[base + pos];
  }
  for (int d = threadIdx.x; d < nb; d += SORT_THREADS) h[d] = 0;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + i * SORT_THREADS + threadIdx.x;
    if (pos < nnz) atomicAdd(&h[((uint32_t)k[i] >> shift) & (nb - 1)], 1u);
  }
  __syncthreads();
  uint32_t* out = hist + ((int64_t)(tb.t[f] + t) << rb);
  for (int d = threadIdx.x; d < nb; d += SORT_THREADS) out[d] = h[d];
}

// One block per field, one thread per digit: the counts of a digit are replaced by their
// exclusive prefix over the tiles, and the digit totals by their exclusive prefix over digits.
__global__ __launch_bounds__(MAX_BINS) void sort_scan_kernel(uint32_t* hist, uint32_t* digit_base, TileBase tb, int rb) {
  __shared__ uint32_t wsum[MAX_BINS / 64];
  const int f = blockIdx.x;
  const int tiles = tb.t[f + 1] - tb.t[f];
  const int nb = 1 << rb;
  const int d = threadIdx.x;
  uint32_t run = 0;
  if (d < nb) {
    uint32_t* h = hist + ((int64_t)tb.t[f] << rb) + d;
    int t = 0;
    for (; t + 3 < tiles; t += 4) {  // four independent loads in flight
      const uint32_t c0 = h[(int64_t)t << rb], c1 = h[(int64_t)(t + 1) << rb];
      const uint32_t c2 = h[(int64_t)(t + 2) << rb], c3 = h[(int64_t)(t + 3) << rb];
      h[(int64_t)t << rb] = run;
      h[(int64_t)(t + 1) << rb] = run + c0;
      h[(int64_t)(t + 2) << rb] = run + c0 + c1;
      h[(int64_t)(t + 3) << rb] = run + c0 + c1 + c2;
      run += c0 + c1 + c2 + c3;
    }
    for (; t < tiles; ++t) {
      const uint32_t c = h[(int64_t)t << rb];
      h[(int64_t)t << rb] = run;
      run += c;
    }
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t incl = run;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[w] = incl;
  __syncthreads();
  uint32_t wbase = 0;
  for (int i = 0; i < w; ++i) wbase += wsum[i];
  if (d < nb) digit_base[((int64_t)f << rb) + d] = wbase + incl - run;
}

// Stable scatter of one tile.  Wave w owns the contiguous slice w of the tile and walks it in
// rounds of 64 keys; lanes holding equal digits find each other with one
// ballot per digit bit, the per-wave running count of the digit lives in LDS.
__global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(
    const int32_t* keys_in, const int32_t* pay_in, int32_t* keys_out, int32_t* pay_out, const uint32_t* hist,
    const uint32_t* digit_base, FieldPtr fp, TileBase tb, int F, int shift, int rb) {
  __shared__ uint32_t cnt[SORT_WAVES][MAX_BINS];
  __shared__ uint32_t gbase[MAX_BINS];
  int f, t;
  if (!field_tile_of_block(tb, F, f, t)) return;
  const int nb = 1 << rb;
  const int64_t base = fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - base);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  // first position of every digit's keys of this tile in the output (digits before it in the field +
  // the digit's keys in earlier tiles): loaded up front with coalesced loads, looked up in LDS
  const uint32_t* hb = hist + ((int64_t)(tb.t[f] + t) << rb);
  const uint32_t* db = digit_base + ((int64_t)f << rb);
  uint32_t gb[MAX_BINS / SORT_THREADS];
#pragma unroll
  for (int q = 0; q < MAX_BINS / SORT_THREADS; ++q) {
    const int d = min((int)threadIdx.x + q * SORT_THREADS, nb - 1);
    gb[q] = db[d] + hb[d];
  }
  int32_t key[SORT_ITEMS], pay[SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {  // all loads first (clamped), so that they overlap
    const int pos = min(t * SORT_TILE + w * (64 * SORT_ITEMS) + i * 64 + lane, nnz - 1);
    key[i] = keys_in[base + pos];
    pay[i] = pay_in[base + pos];
  }
  for (int d = threadIdx.x; d < SORT_WAVES * nb; d += SORT_THREADS) cnt[d >> rb][d & (nb - 1)] = 0;
#pragma unroll
  for (int q = 0; q < MAX_BINS / SORT_THREADS; ++q)
    if ((int)threadIdx.x + q * SORT_THREADS < nb) gbase[threadIdx.x + q * SORT_THREADS] = gb[q];
  __syncthreads();
  const uint64_t lt = lanemask_lt();
  volatile uint32_t* cw = cnt[w];
  uint32_t rank[SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + w * (64 * SORT_ITEMS) + i * 64 + lane;
    const bool valid = pos < nnz;
    const uint32_t d = ((uint32_t)key[i] >> shift) & (nb - 1);
    uint64_t m = __ballot(valid);
    for (int b = 0; b < rb; ++b) {
      const bool bit = (d >> b) & 1u;
      const uint64_t bal = __ballot(valid && bit);
      m &= bit ? bal : ~bal;
    }
    rank[i] = 0;
    if (valid) {
      const uint32_t prior = cw[d];
      rank[i] = prior + (uint32_t)__popcll(m & lt);
      if ((m & lt) == 0) cw[d] = prior + (uint32_t)__popcll(m);  // lowest lane of the group
    }
  }
  __syncthreads();
  // Per digit: the counts of the wavefronts become exclusive prefixes (keys of the digit in
  // earlier wavefronts of the tile), their sum the tile's count of the digit; an exclusive scan of
  // these counts in digit order gives every key its place in the tile sorted by digit.
  constexpr int DPT = MAX_BINS / SORT_THREADS;  // digits per thread: d = threadIdx.x + q * SORT_THREADS
  __shared__ uint32_t dpre[MAX_BINS];
  __shared__ uint32_t wsum[DPT][SORT_WAVES];
  uint32_t tot[DPT], incl[DPT];
#pragma unroll
  for (int q = 0; q < DPT; ++q) {
    const int d = threadIdx.x + q * SORT_THREADS;
    uint32_t run = 0;
    if (d < nb) {
#pragma unroll
      for (int ww = 0; ww < SORT_WAVES; ++ww) {
        const uint32_t c = cnt[ww][d];
        cnt[ww][d] = run;
        run += c;
      }
    }
    tot[q] = run;
    incl[q] = run;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
      const uint32_t v = __shfl_up(incl[q], o, 64);
      if (lane >= o) incl[q] += v;
    }
    if (lane == 63) wsum[q][w] = incl[q];
  }
  __syncthreads();
  {
    uint32_t before = 0;  // keys of the tile with a digit handled by an earlier (q, wavefront)
#pragma unroll
    for (int q = 0; q < DPT; ++q) {
      uint32_t mine = before;
      for (int ww = 0; ww < SORT_WAVES; ++ww) {
        if (ww < w) mine += wsum[q][ww];
        before += wsum[q][ww];
      }
      const int d = threadIdx.x + q * SORT_THREADS;
      if (d < nb) {
        const uint32_t first = mine + incl[q] - tot[q];  // place of the digit's first key in the sorted tile
        dpre[d] = first;
        gbase[d] -= first;   // output position = gbase[d] + place in the sorted tile
      }
    }
  }
  __syncthreads();
  uint32_t lp[SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const uint32_t d = ((uint32_t)key[i] >> shift) & (nb - 1);
    lp[i] = dpre[d] + cnt[w][d] + rank[i];
  }
  __syncthreads();  // the counters are dead: their memory stages the tile sorted by digit
  int32_t* skey = reinterpret_cast<int32_t*>(&cnt[0][0]);
  int32_t* spay = skey + SORT_TILE;
  static_assert(2 * SORT_TILE <= SORT_WAVES * MAX_BINS, "the staged tile must fit the counters' memory");
  const int tile_count = min(SORT_TILE, nnz - t * SORT_TILE);
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + w * (64 * SORT_ITEMS) + i * 64 + lane;
    if (pos < nnz && lp[i] < (uint32_t)SORT_TILE) {
      skey[lp[i]] = key[i];
      spay[lp[i]] = pay[i];
    }
  }
  __syncthreads();
  // Consecutive threads hold consecutive keys of the sorted tile: keys of one digit go to consecutive
  // positions of the output, so that their 4-byte stores merge into one request per run.
#pragma unroll
  for (int q = 0; q < SORT_ITEMS; ++q) {
    const int j = q * SORT_THREADS + threadIdx.x;
    if (j < tile_count) {
      const int32_t k = skey[j];
      const uint32_t d = ((uint32_t)k >> shift) & (nb - 1);
      const uint32_t dst = gbase[d] + (uint32_t)j;
      if (dst < (uint32_t)nnz) {
        keys_out[base + dst] = k;
        pay_out[base + dst] = spay[j];
      }
    }
  }
}

// ------------------------------------------------- leaving shards out
// When the servers disregard the gradients of some workers (the backup-workers baseline of
// Section VII-A.3), only the lookups of the remaining shards are coalesced.  A shard is a
// contiguous range of samples, hence a contiguous range of every field's lookups: the ranges
// of the included shards (weight != 0) are packed side by side, field after field.

// cbase[f] = number of included lookups in the fields before f (cbase[F] = their total).
__global__ __launch_bounds__(256) void mask_count_kernel(const int32_t* offsets, int64_t B, int F, ShardTab tab,
                                                         int64_t* cbase) {
  __shared__ int64_t cnt[ANTDT_MAX_FIELDS];
  for (int f = threadIdx.x; f < F; f += 256) {
    const int32_t* off = offsets + (int64_t)f * (B + 1);
    int64_t c = 0;
    for (int k = 0; k < tab.K; ++k)
      if (tab.w[k] != 0.0f) c += off[tab.start[k] + tab.len[k]] - off[tab.start[k]];
    cnt[f] = c;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int64_t run = 0;
    for (int f = 0; f < F; ++f) {
      cbase[f] = run;
      run += cnt[f];
    }
    cbase[F] = run;
  }
}

// Block (k, f) copies the ids and sample indices of shard k's lookups in field f.
__global__ __launch_bounds__(256) void mask_pack_kernel(const int32_t* ids, const int32_t* lookup_sample,
                                                        const int32_t* offsets, int64_t B, FieldPtr fp, ShardTab tab,
                                                        const int64_t* cbase, int32_t* ids_out, int32_t* pay_out) {
  const int k = blockIdx.x, f = blockIdx.y;
  if (tab.w[k] == 0.0f) return;
  const int32_t* off = offsets + (int64_t)f * (B + 1);
  int64_t dst = cbase[f];
  for (int q = 0; q < k; ++q)
    if (tab.w[q] != 0.0f) dst += off[tab.start[q] + tab.len[q]] - off[tab.start[q]];
  const int64_t src = fp.p[f] + off[tab.start[k]];
  const int n = off[tab.start[k] + tab.len[k]] - off[tab.start[k]];
  for (int i = threadIdx.x; i < n; i += 256) {
    ids_out[dst + i] = ids[src + i];
    pay_out[dst + i] = lookup_sample[src + i];
  }
}

// ------------------------------------------------------------- segments
__device__ __forceinline__ bool is_head(const int32_t* key, int pos) {
  return pos == 0 || key[pos] != key[pos - 1];
}

// Number of run heads in each tile of the sorted keys.
__global__ __launch_bounds__(SORT_THREADS) void seg_heads_kernel(SegArgs a, FieldPtr fp, TileBase tb) {
  __shared__ int wsum[SORT_WAVES];
  int f, t;
  if (!field_tile_of_block(tb, a.F, f, t)) return;
  const int32_t* key = a.key + fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - fp.p[f]);
  int c = 0;
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + i * SORT_THREADS + threadIdx.x;
    if (pos < nnz && is_head(key, pos)) ++c;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) c += __shfl_xor(c, o, 64);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int s = 0;
    for (int i = 0; i < SORT_WAVES; ++i) s += wsum[i];
    a.tile_heads[tb.t[f] + t] = s;
  }
}

// One block: exclusive prefix over all tiles (-> first unique of every tile and field),
// the terminal segment offset of every field and the per-sample aggregation weight.
__global__ __launch_bounds__(1024) void seg_scan_kernel(SegArgs a, FieldPtr fp, TileBase tb, ShardTab tab) {
  __shared__ int wsum[16];
  const int n = a.total_tiles;
  const int chunk = (n + 1023) / 1024;
  const int lo = min(n, (int)threadIdx.x * chunk), hi = min(n, lo + chunk);
  int sum = 0;
  for (int i = lo; i < hi; ++i) sum += a.tile_heads[i];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[w] = incl;
  __syncthreads();
  int wbase = 0, total = 0;
  for (int i = 0; i < 16; ++i) {
    if (i < w) wbase += wsum[i];
    total += wsum[i];
  }
  int run = wbase + incl - sum;
  for (int i = lo; i < hi; ++i) {
    const int c = a.tile_heads[i];
    a.tile_heads[i] = run;
    run += c;
  }
  if (threadIdx.x == 0) {
    a.tile_heads[n] = total;
    a.segabs[total] = (int32_t)fp.p[a.F];
  }
  __threadfence_block();
  __syncthreads();
  for (int f = threadIdx.x; f <= a.F; f += 1024) a.ubase[f] = a.tile_heads[tb.t[f]];
  for (int f = threadIdx.x; f < a.F; f += 1024)
    a.segoff[a.tile_heads[tb.t[f + 1]] + f] = (int32_t)(fp.p[f + 1] - fp.p[f]);
  for (int k = 0; k < tab.K; ++k) {
    const float wk = tab.w[k];
    for (int s = threadIdx.x; s < tab.len[k]; s += 1024) a.sample_w[tab.start[k] + s] = wk;
  }
}

// Unique ids and segment offsets.  Thread j of a tile owns 8 consecutive sorted positions.
__global__ __launch_bounds__(SORT_THREADS) void seg_emit_kernel(SegArgs a, FieldPtr fp, TileBase tb) {
  __shared__ int wsum[SORT_WAVES];
  int f, t;
  if (!field_tile_of_block(tb, a.F, f, t)) return;
  const int32_t* key = a.key + fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - fp.p[f]);
  const int p0 = t * SORT_TILE + threadIdx.x * SORT_ITEMS;
  unsigned flags = 0;
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i)
    if (p0 + i < nnz && is_head(key, p0 + i)) flags |= 1u << i;
  const int c = __popc(flags);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int incl = c;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[w] = incl;
  __syncthreads();
  int rank = a.tile_heads[tb.t[f] + t] + incl - c;
  for (int i = 0; i < w; ++i) rank += wsum[i];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i)
    if (flags & (1u << i)) {
      a.uniq[rank] = key[p0 + i];
      a.ufield[rank] = f;
      a.segabs[rank] = (int32_t)fp.p[f] + p0 + i;
      a.segoff[rank + f] = p0 + i;
      ++rank;
    }
}

// Runs longer than the threshold are cut into chunks of `chunk` lookups; the list of such runs
// and the list of their chunks are built here, beside the run table, so that the reduction
// kernel finds them ready.  Both lists are in run order (count per block of runs, prefix sum
// over the blocks, write): consecutive entries belong to the same field, which is what lets the
// reduction give each of its eight shares a contiguous piece of every list.
constexpr int QUEUE_RUNS = 8;  // runs per thread
static_assert(256 * QUEUE_RUNS == ANTDT_QUEUE_BLOCK_RUNS, "queue block size");
constexpr int SHARES = 8;      // one per XCD: blocks are handed to the XCDs round robin

// Long runs and chunks among the block's runs; lengths of the thread's runs in len[].
__device__ __forceinline__ void queue_count(const SegArgs& a, int U, int64_t u0, int (&len)[QUEUE_RUNS], int& nl, int& nc) {
  nl = 0;
  nc = 0;
#pragma unroll
  for (int i = 0; i < QUEUE_RUNS; ++i) {
    const int64_t u = u0 + i;
    len[i] = u < U ? a.segabs[u + 1] - a.segabs[u] : 0;
    if (len[i] > a.long_threshold) {
      ++nl;
      nc += (len[i] + a.chunk - 1) / a.chunk;
    }
  }
}

__global__ __launch_bounds__(256) void seg_queue_count_kernel(SegArgs a) {
  __shared__ int wl[4], wc[4];
  const int U = a.ubase[a.F];
  const int64_t u0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * QUEUE_RUNS;
  int len[QUEUE_RUNS], nl, nc;
  queue_count(a, U, u0, len, nl, nc);
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    nl += __shfl_xor(nl, o, 64);
    nc += __shfl_xor(nc, o, 64);
  }
  if ((threadIdx.x & 63) == 0) {
    wl[threadIdx.x >> 6] = nl;
    wc[threadIdx.x >> 6] = nc;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    a.qcnt[2 * blockIdx.x] = (wl[0] + wl[1]) + (wl[2] + wl[3]);
    a.qcnt[2 * blockIdx.x + 1] = (wc[0] + wc[1]) + (wc[2] + wc[3]);
  }
}

// One block: exclusive prefix sums of the per-block counts (qcnt[2 * nblocks ..] = the totals),
// the list lengths, and the table of shares: share x of the reduction owns the runs of the
// queue blocks [ceil(nq x / 8), ceil(nq (x+1) / 8)), nq = blocks that hold runs, hence a
// contiguous piece of the run table and of both lists.
__global__ __launch_bounds__(1024) void seg_queue_scan_kernel(SegArgs a, int nblocks) {
  __shared__ int wsl[16], wsc[16];
  const int per = (nblocks + 1023) / 1024;
  const int lo = min(nblocks, (int)threadIdx.x * per), hi = min(nblocks, lo + per);
  int sl = 0, sc = 0;
  for (int i = lo; i < hi; ++i) {
    sl += a.qcnt[2 * i];
    sc += a.qcnt[2 * i + 1];
  }
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int il = sl, ic = sc;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int vl = __shfl_up(il, o, 64), vc = __shfl_up(ic, o, 64);
    if (lane >= o) {
      il += vl;
      ic += vc;
    }
  }
  if (lane == 63) {
    wsl[w] = il;
    wsc[w] = ic;
  }
  __syncthreads();
  int bl = il - sl, bc = ic - sc, tl = 0, tc = 0;
  for (int i = 0; i < 16; ++i) {
    if (i < w) {
      bl += wsl[i];
      bc += wsc[i];
    }
    tl += wsl[i];
    tc += wsc[i];
  }
  for (int i = lo; i < hi; ++i) {
    const int cl = a.qcnt[2 * i], cc = a.qcnt[2 * i + 1];
    a.qcnt[2 * i] = bl;
    a.qcnt[2 * i + 1] = bc;
    bl += cl;
    bc += cc;
  }
  if (threadIdx.x == 0) {
    a.qcnt[2 * nblocks] = tl;
    a.qcnt[2 * nblocks + 1] = tc;
    a.counters[0] = tl;
    a.counters[1] = tc;
  }
  __threadfence_block();
  __syncthreads();
  if (threadIdx.x <= SHARES) {
    const int U = a.ubase[a.F];
    const int nq = (U + ANTDT_QUEUE_BLOCK_RUNS - 1) / ANTDT_QUEUE_BLOCK_RUNS;  // <= nblocks
    const int x = threadIdx.x;
    const int qb = min(nblocks, (int)(((int64_t)nq * x + SHARES - 1) / SHARES));
    a.xcd_tab[x] = (int)min((int64_t)U, (int64_t)qb * ANTDT_QUEUE_BLOCK_RUNS);
    a.xcd_tab[9 + x] = a.qcnt[2 * qb + 1];   // first chunk item
    a.xcd_tab[18 + x] = a.qcnt[2 * qb];      // first long run
  }
}

__global__ __launch_bounds__(256) void seg_queue_write_kernel(SegArgs a) {
  __shared__ int wl[4], wc[4];
  const int U = a.ubase[a.F];
  if ((int64_t)blockIdx.x * ANTDT_QUEUE_BLOCK_RUNS >= U) return;
  const int64_t u0 = ((int64_t)blockIdx.x * 256 + threadIdx.x) * QUEUE_RUNS;
  int len[QUEUE_RUNS], nl, nc;
  queue_count(a, U, u0, len, nl, nc);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int il = nl, ic = nc;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int vl = __shfl_up(il, o, 64), vc = __shfl_up(ic, o, 64);
    if (lane >= o) {
      il += vl;
      ic += vc;
    }
  }
  if (lane == 63) {
    wl[w] = il;
    wc[w] = ic;
  }
  __syncthreads();
  int slot = a.qcnt[2 * blockIdx.x] + il - nl, item = a.qcnt[2 * blockIdx.x + 1] + ic - nc;
  for (int i = 0; i < w; ++i) {
    slot += wl[i];
    item += wc[i];
  }
#pragma unroll
  for (int i = 0; i < QUEUE_RUNS; ++i) {
    if (len[i] <= a.long_threshold) continue;
    const int nch = (len[i] + a.chunk - 1) / a.chunk;
    if (slot < a.long_cap && item + nch <= a.item_cap) {  // (the capacities are upper bounds: always true)
      a.long_seg[slot * 3 + 0] = (int)(u0 + i);
      a.long_seg[slot * 3 + 1] = item;
      a.long_seg[slot * 3 + 2] = nch;
      for (int q = 0; q < nch; ++q) {
        a.items[(item + q) * 2 + 0] = (int)(u0 + i);
        a.items[(item + q) * 2 + 1] = q;
      }
    }
    ++slot;
    item += nch;
  }
}

// ------------------------------------------------- weighted run sums (+ update)
struct Row4 {
  float v[4];
};

// Weight of one lookup of sample s: the shard weight, divided by the length of the sample's bag
// in this field when the bags are mean-pooled (the bag is not empty: the lookup is in it).
template <bool MEAN>
__device__ __forceinline__ float lookup_weight(const SegArgs& a, const int32_t* off, int s) {
  const float w = a.sample_w[s];
  if (!MEAN) return w;
  return w / (float)max(off[s + 1] - off[s], 1);
}

// g += w(lookup) * dX[sample, field slice] over sorted entries [b, e) of field f taken with
// stride `step`, NF entries in flight (added in order).  The sample indices of the next NF entries
// are requested before the pooled-gradient rows of the current ones are waited for: the chain of
// dependent accesses is one round trip per NF entries instead of two.
template <bool MEAN, int NF = 4>
__device__ __forceinline__ void accumulate_run(const SegArgs& a, int f, int c, int b, int e, int step, Row4& g) {
  const float* dxcol = a.dx + f * a.D + c * 4;
  const int32_t* off = MEAN ? a.offsets + (int64_t)f * (a.B + 1) : nullptr;
  int i = b;
  int sn[NF];
#pragma unroll
  for (int q = 0; q < NF; ++q) sn[q] = i + q * step < e ? a.pay[i + q * step] : 0;
  for (; i + (NF - 1) * step < e; i += NF * step) {
    int s[NF];
#pragma unroll
    for (int q = 0; q < NF; ++q) s[q] = min(max(sn[q], 0), a.B - 1);
#pragma unroll
    for (int q = 0; q < NF; ++q) sn[q] = i + (NF + q) * step < e ? a.pay[i + (NF + q) * step] : 0;
    float w[NF];
    float4 x[NF];
#pragma unroll
    for (int q = 0; q < NF; ++q) {
      w[q] = lookup_weight<MEAN>(a, off, s[q]);
      x[q] = *reinterpret_cast<const float4*>(dxcol + (int64_t)s[q] * a.lddx);
    }
#pragma unroll
    for (int q = 0; q < NF; ++q) {
      g.v[0] = fmaf(w[q], x[q].x, g.v[0]);
      g.v[1] = fmaf(w[q], x[q].y, g.v[1]);
      g.v[2] = fmaf(w[q], x[q].z, g.v[2]);
      g.v[3] = fmaf(w[q], x[q].w, g.v[3]);
    }
  }
  // fewer than NF entries are left; their sample indices are in sn[]
  {
    float w[NF];
    float4 x[NF];
#pragma unroll
    for (int q = 0; q < NF; ++q) {
      const int s = min(max(sn[q], 0), a.B - 1);
      w[q] = 0.0f;
      x[q] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i + q * step < e) {
        w[q] = lookup_weight<MEAN>(a, off, s);
        x[q] = *reinterpret_cast<const float4*>(dxcol + (int64_t)s * a.lddx);
      }
    }
#pragma unroll
    for (int q = 0; q < NF; ++q)
      if (i + q * step < e) {
        g.v[0] = fmaf(w[q], x[q].x, g.v[0]);
        g.v[1] = fmaf(w[q], x[q].y, g.v[1]);
        g.v[2] = fmaf(w[q], x[q].z, g.v[2]);
        g.v[3] = fmaf(w[q], x[q].w, g.v[3]);
      }
  }
}

// Row-sparse Adagrad of one table row by its lane group (lane c owns columns 4c .. 4c+3):
//   element-wise: S += g^2;                 p -= lr * g / (sqrt(S) + eps)
//   row-wise:     S[r] += mean_d g[r,d]^2;  p -= lr * g / (sqrt(S[r]) + eps)
// bf16 tables are written back round-to-nearest-even.
template <typename TT, bool ROWWISE>
__device__ __forceinline__ void adagrad_row(const SegArgs& a, int64_t row, int c, int lps, const Row4& g,
                                            const float (&p0)[4], const float4& s0, float srow0) {
  float den[4], p[4];
  if (ROWWISE) {
    float sq = (g.v[0] * g.v[0] + g.v[1] * g.v[1]) + (g.v[2] * g.v[2] + g.v[3] * g.v[3]);
    for (int o = 1; o < lps; o <<= 1) sq += __shfl_xor(sq, o, 64);
    const float s1 = srow0 + sq / (float)a.D;
    if (c == 0) a.state[row] = s1;
    den[0] = den[1] = den[2] = den[3] = sqrtf(s1) + a.eps;
  } else {
    float4 sv = s0;
    sv.x = fmaf(g.v[0], g.v[0], sv.x);
    sv.y = fmaf(g.v[1], g.v[1], sv.y);
    sv.z = fmaf(g.v[2], g.v[2], sv.z);
    sv.w = fmaf(g.v[3], g.v[3], sv.w);
    *reinterpret_cast<float4*>(a.state + row * a.D + c * 4) = sv;
    den[0] = sqrtf(sv.x) + a.eps; den[1] = sqrtf(sv.y) + a.eps;
    den[2] = sqrtf(sv.z) + a.eps; den[3] = sqrtf(sv.w) + a.eps;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) p[e] = p0[e] - a.lr * g.v[e] / den[e];
  TT* prow = reinterpret_cast<TT*>(a.tables) + row * a.D + c * 4;
  if (sizeof(TT) == 4) {
    *reinterpret_cast<float4*>(prow) = make_float4(p[0], p[1], p[2], p[3]);
  } else {
    *reinterpret_cast<uint2*>(prow) = make_uint2((uint32_t)f2bf(p[0]) | ((uint32_t)f2bf(p[1]) << 16),
                                                 (uint32_t)f2bf(p[2]) | ((uint32_t)f2bf(p[3]) << 16));
  }
}

template <typename TT, bool ROWWISE>
__device__ __forceinline__ void load_row(const SegArgs& a, int64_t row, int c, float (&p0)[4], float4& s0, float& srow0) {
  const TT* prow = reinterpret_cast<const TT*>(a.tables) + row * a.D + c * 4;
  if (sizeof(TT) == 4) {
    const float4 v = *reinterpret_cast<const float4*>(prow);
    p0[0] = v.x; p0[1] = v.y; p0[2] = v.z; p0[3] = v.w;
  } else {
    const uint2 v = *reinterpret_cast<const uint2*>(prow);
    p0[0] = __uint_as_float(v.x << 16); p0[1] = __uint_as_float(v.x & 0xFFFF0000u);
    p0[2] = __uint_as_float(v.y << 16); p0[3] = __uint_as_float(v.y & 0xFFFF0000u);
  }
  if (ROWWISE) srow0 = a.state[row];
  else s0 = *reinterpret_cast<const float4*>(a.state + row * a.D + c * 4);
}

// Chunk sums of the long runs.  One block per chunk: the lane groups stride over the chunk, then
// their partial sums are added in group order (fixed order: repeatable bit for bit).
template <bool MEAN>
__device__ __forceinline__ void chunk_sums(const SegArgs& a, int first, int last, int step) {
  __shared__ float4 red[256];
  const int lps = a.D >> 2;
  const int ngroups = 256 / lps;
  const int g = threadIdx.x / lps, c = threadIdx.x - g * lps;
  const int count = min(last, a.item_cap);
  for (int idx = first; idx < count; idx += step) {
    const int u = a.items[idx * 2], q = a.items[idx * 2 + 1];
    const int b = a.segabs[u] + q * a.chunk, e = min(a.segabs[u + 1], b + a.chunk);
    const int f = a.ufield[u];
    Row4 gsum = {{0.f, 0.f, 0.f, 0.f}};
    accumulate_run<MEAN>(a, f, c, b + g, e, ngroups, gsum);
    red[threadIdx.x] = make_float4(gsum.v[0], gsum.v[1], gsum.v[2], gsum.v[3]);
    __syncthreads();
    for (int half = ngroups >> 1; half > 0; half >>= 1) {
      if (g < half) {
        const float4 o = red[(g + half) * lps + c];
        float4 m = red[g * lps + c];
        m.x += o.x; m.y += o.y; m.z += o.z; m.w += o.w;
        red[g * lps + c] = m;
      }
      __syncthreads();
    }
    if (g == 0) *reinterpret_cast<float4*>(a.partial + (int64_t)idx * a.D + c * 4) = red[c];
    __syncthreads();
  }
}

// The first `chunk_blocks` blocks take the chunks of the long runs (their sums are added up by
// the kernel after this one); the others work one group of D/4 lanes per run: short runs are
// summed in sorted (= sample) order and, when `UPDATE`, the Adagrad step of the row is applied
// at once (the coalesced gradient never goes to memory); otherwise the sum is written to G.
// The work is divided into eight shares of consecutive runs (consecutive runs belong to the same
// field), and the blocks whose index is x modulo 8, which the hardware places on XCD x, work
// on share x: the pooled-gradient slice of a field (all samples x D columns) is then fetched into
// one XCD's L2 instead of all eight.  With fewer than eight blocks there is one share.
template <typename TT, bool ROWWISE, bool UPDATE, bool MEAN>
__global__ __launch_bounds__(256) void seg_reduce_kernel(SegArgs a, int chunk_blocks) {
  const int x = blockIdx.x & (SHARES - 1);
  if ((int)blockIdx.x < chunk_blocks) {  // (chunk_blocks is a multiple of 8)
    chunk_sums<MEAN>(a, a.xcd_tab[9 + x] + (int)(blockIdx.x >> 3), a.xcd_tab[9 + x + 1], chunk_blocks >> 3);
    return;
  }
  const int64_t bid = (int64_t)blockIdx.x - chunk_blocks, nblk = (int64_t)gridDim.x - chunk_blocks;
  const int lps = a.D >> 2;
  const int groups_per_block = 256 / lps;
  const int g = threadIdx.x / lps, c = threadIdx.x - g * lps;
  int64_t lo, hi, slot, nslots;
  if (nblk >= SHARES) {
    lo = a.xcd_tab[x];
    hi = a.xcd_tab[x + 1];
    slot = bid >> 3;
    nslots = (nblk - x + SHARES - 1) >> 3;
  } else {
    lo = 0;
    hi = a.ubase[a.F];
    slot = bid;
    nslots = nblk;
  }
  // The kernel is bound by the chain of dependent accesses of a run (its description -> its row,
  // accumulators and sample indices -> the pooled-gradient rows of its samples), every wavefront
  // slot of the device being taken: the bounds, field and row id of a run are requested together,
  // and those of the group's next run while the current one is summed.
  const int64_t ustep = nslots * groups_per_block;
  int64_t u = lo + slot * groups_per_block + g;
  int nb = 0, ne = 0, nf = 0, nid = 0;
  if (u < hi) {
    nb = a.segabs[u]; ne = a.segabs[u + 1]; nf = a.ufield[u]; nid = a.uniq[u];
  }
  for (; u < hi; u += ustep) {
    const int b = nb, e = ne, f = nf, id = nid;
    if (u + ustep < hi) {
      nb = a.segabs[u + ustep]; ne = a.segabs[u + ustep + 1]; nf = a.ufield[u + ustep]; nid = a.uniq[u + ustep];
    }
    if (e - b > a.long_threshold) continue;
    const int64_t row = (int64_t)f * a.R + min(max(id, 0), (int)(a.R - 1));
    float p0[4] = {0.f, 0.f, 0.f, 0.f};
    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f);
    float srow0 = 0.f;
    if (UPDATE) load_row<TT, ROWWISE>(a, row, c, p0, s0, srow0);
    Row4 gsum = {{0.f, 0.f, 0.f, 0.f}};
    accumulate_run<MEAN>(a, f, c, b, e, 1, gsum);
    if (UPDATE) adagrad_row<TT, ROWWISE>(a, row, c, lps, gsum, p0, s0, srow0);
    else *reinterpret_cast<float4*>(a.G + u * a.D + c * 4) = make_float4(gsum.v[0], gsum.v[1], gsum.v[2], gsum.v[3]);
  }
}

// One lane group per long run: add its chunk sums in chunk order, then update or store.
template <typename TT, bool ROWWISE, bool UPDATE>
__global__ __launch_bounds__(256) void seg_finish_kernel(SegArgs a) {
  const int lps = a.D >> 2;
  const int groups_per_block = 256 / lps;
  const int g = threadIdx.x / lps, c = threadIdx.x - g * lps;
  const int count = min(a.counters[0], a.long_cap);
  for (int idx = blockIdx.x * groups_per_block + g; idx < count; idx += gridDim.x * groups_per_block) {
    const int u = a.long_seg[idx * 3], base = a.long_seg[idx * 3 + 1], nch = a.long_seg[idx * 3 + 2];
    const int f = a.ufield[u];
    const int64_t row = (int64_t)f * a.R + min(max(a.uniq[u], 0), (int)(a.R - 1));
    float p0[4] = {0.f, 0.f, 0.f, 0.f};
    float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f);
    float srow0 = 0.f;
    if (UPDATE) load_row<TT, ROWWISE>(a, row, c, p0, s0, srow0);
    Row4 gsum = {{0.f, 0.f, 0.f, 0.f}};
    const float* part = a.partial + (int64_t)base * a.D + c * 4;
    int q = 0;
    for (; q + 3 < nch; q += 4) {  // four loads in flight, added in chunk order
      float4 v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) v[j] = *reinterpret_cast<const float4*>(part + (int64_t)(q + j) * a.D);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        gsum.v[0] += v[j].x; gsum.v[1] += v[j].y; gsum.v[2] += v[j].z; gsum.v[3] += v[j].w;
      }
    }
    for (; q < nch; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(part + (int64_t)q * a.D);
      gsum.v[0] += v.x; gsum.v[1] += v.y; gsum.v[2] += v.z; gsum.v[3] += v.w;
    }
    if (UPDATE) adagrad_row<TT, ROWWISE>(a, row, c, lps, gsum, p0, s0, srow0);
    else *reinterpret_cast<float4*>(a.G + (int64_t)u * a.D + c * 4) = make_float4(gsum.v[0], gsum.v[1], gsum.v[2], gsum.v[3]);
  }
}

template <typename TT, bool ROWWISE, bool UPDATE, bool MEAN>
void launch_reduce_pooling(const SegArgs& a, unsigned blocks, unsigned finish_blocks, Profiler* prof, hipStream_t s) {
  {
    ProfScope ps(prof, UPDATE ? KID_SPARSE_ADAGRAD : KID_SEG_REDUCE, s);
    constexpr int CHUNK_BLOCKS = 2048;
    hipLaunchKernelGGL((seg_reduce_kernel<TT, ROWWISE, UPDATE, MEAN>), dim3(blocks + CHUNK_BLOCKS), dim3(256), 0, s, a,
                       CHUNK_BLOCKS);
  }
  {
    ProfScope ps(prof, KID_SEG_REDUCE_LONG, s);
    hipLaunchKernelGGL((seg_finish_kernel<TT, ROWWISE, UPDATE>), dim3(finish_blocks), dim3(256), 0, s, a);
  }
}

template <typename TT, bool ROWWISE, bool UPDATE>
void launch_reduce_variant(const SegArgs& a, unsigned blocks, unsigned finish_blocks, Profiler* prof, hipStream_t s) {
  if (a.mean_pool) launch_reduce_pooling<TT, ROWWISE, UPDATE, true>(a, blocks, finish_blocks, prof, s);
  else launch_reduce_pooling<TT, ROWWISE, UPDATE, false>(a, blocks, finish_blocks, prof, s);
}

}  // namespace

// Blocks of a launch whose block b works on tile (b / 8) of the fields b mod 8, b mod 8 + 8, ...:
// eight times the largest number of tiles any of the eight groups of fields has.
static unsigned tile_grid(const TileBase& tb, int F) {
  int most = 1;
  for (int x = 0; x < 8; ++x) most = std::max(most, (int)tb.xcum[x][ANTDT_MAX_FIELDS / 8]);
  (void)F;
  return (unsigned)(8 * most);
}

hipError_t launch_sort_pass(const SortPlan& pl, const SortBuffers& sb, int pass, const FieldPtr& fp,
                            const TileBase& tb, Profiler* prof, hipStream_t s) {
  if (pl.total_tiles == 0) return hipSuccess;
  const int shift = pass * pl.radix_bits;
  const int32_t* kin = pass == 0 ? sb.ids : sb.key[(pass - 1) & 1];
  const int32_t* pin = pass == 0 ? sb.pay0 : sb.pay[(pass - 1) & 1];
  dim3 grid(tile_grid(tb, pl.F));
  {
    ProfScope ps(prof, KID_SORT_HIST, s);
    hipLaunchKernelGGL(sort_hist_kernel, grid, dim3(SORT_THREADS), 0, s, kin, sb.hist, fp, tb, pl.F, shift, pl.radix_bits);
  }
  {
    ProfScope ps(prof, KID_SORT_SCAN, s);
    hipLaunchKernelGGL(sort_scan_kernel, dim3(pl.F), dim3(MAX_BINS), 0, s, sb.hist, sb.digit_base, tb, pl.radix_bits);
  }
  {
    ProfScope ps(prof, KID_SORT_SCATTER, s);
    hipLaunchKernelGGL(sort_scatter_kernel, grid, dim3(SORT_THREADS), 0, s, kin, pin, sb.key[pass & 1],
                       sb.pay[pass & 1], sb.hist, sb.digit_base, fp, tb, pl.F, shift, pl.radix_bits);
  }
  return hipGetLastError();
}

hipError_t launch_segments(const SegArgs& a, const FieldPtr& fp, const TileBase& tb, const ShardTab& tab,
                           Profiler* prof, hipStream_t s) {
  dim3 grid(tile_grid(tb, a.F));
  if (a.total_tiles > 0) {
    ProfScope ps(prof, KID_SEG_HEADS, s);
    hipLaunchKernelGGL(seg_heads_kernel, grid, dim3(SORT_THREADS), 0, s, a, fp, tb);
  }
  {
    ProfScope ps(prof, KID_SEG_SCAN, s);
    hipLaunchKernelGGL(seg_scan_kernel, dim3(1), dim3(1024), 0, s, a, fp, tb, tab);
  }
  if (a.total_tiles > 0) {
    ProfScope ps(prof, KID_SEG_EMIT, s);
    hipLaunchKernelGGL(seg_emit_kernel, grid, dim3(SORT_THREADS), 0, s, a, fp, tb);
  }
  {  // lists of the long runs and their chunks, and the table of shares (also when there is no lookup)
    const int64_t nnz = fp.p[a.F];
    const unsigned qb = (unsigned)((nnz + ANTDT_QUEUE_BLOCK_RUNS - 1) / ANTDT_QUEUE_BLOCK_RUNS);  // runs <= lookups
    ProfScope ps(prof, KID_SEG_EMIT, s);
    if (qb) hipLaunchKernelGGL(seg_queue_count_kernel, dim3(qb), dim3(256), 0, s, a);
    hipLaunchKernelGGL(seg_queue_scan_kernel, dim3(1), dim3(1024), 0, s, a, (int)qb);
    if (qb) hipLaunchKernelGGL(seg_queue_write_kernel, dim3(qb), dim3(256), 0, s, a);
  }
  return hipGetLastError();
}

hipError_t launch_mask_pack(const int32_t* ids, const int32_t* lookup_sample, const int32_t* offsets, int64_t B, int F,
                            const FieldPtr& fp, const ShardTab& tab, int64_t* cbase, int32_t* ids_out,
                            int32_t* pay_out, hipStream_t s) {
  hipLaunchKernelGGL(mask_count_kernel, dim3(1), dim3(256), 0, s, offsets, B, F, tab, cbase);
  hipLaunchKernelGGL(mask_pack_kernel, dim3(tab.K, F), dim3(256), 0, s, ids, lookup_sample, offsets, B, fp, tab, cbase,
                     ids_out, pay_out);
  return hipGetLastError();
}

hipError_t launch_seg_reduce(const SegArgs& a, int64_t nnz_total, Profiler* prof, hipStream_t s) {
  if (nnz_total == 0) return hipSuccess;
  const int groups_per_block = 256 / (a.D >> 2);
  int64_t nb = (nnz_total + groups_per_block - 1) / groups_per_block;
  if (nb > 256 * 32) nb = 256 * 32;
  if (nb >= SHARES) nb = (nb + SHARES - 1) / SHARES * SHARES;   // the same number of blocks for every share
  const unsigned blocks = (unsigned)nb;
  // one lane group per long run; there are at most nnz / threshold of them (blocks past the
  // actual number leave at once)
  int64_t fb = (nnz_total / (a.long_threshold > 0 ? a.long_threshold : 1) + groups_per_block) / groups_per_block;
  if (fb < 64) fb = 64;
  if (fb > 8192) fb = 8192;
  const unsigned finish_blocks = (unsigned)fb;
  if (a.update) {
    if (a.table_bf16) {
      if (a.rowwise) launch_reduce_variant<bf16_t, true, true>(a, blocks, finish_blocks, prof, s);
      else launch_reduce_variant<bf16_t, false, true>(a, blocks, finish_blocks, prof, s);
    } else {
      if (a.rowwise) launch_reduce_variant<float, true, true>(a, blocks, finish_blocks, prof, s);
      else launch_reduce_variant<float, false, true>(a, blocks, finish_blocks, prof, s);
    }
  } else {
    launch_reduce_variant<float, false, false>(a, blocks, finish_blocks, prof, s);
  }
  return hipGetLastError();
}

}  // namespace antdt
