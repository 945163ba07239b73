// Server-side coalescing of the pushed sparse gradients (Section II: "the servers
// aggregate the local gradients from all workers"): per field, a stable LSD radix
// sort of (row id, sample index) pairs, detection of the runs of equal ids
// (unique ids + segment offsets), and the weighted segmented reduction
//   G[u, :] = sum over the run of w(sample) * dX[sample, field slice].
// No floating-point atomics are used, so the sums are bitwise repeatable.
#include "common.h"

namespace antdt {
namespace {

constexpr int SORT_THREADS = 512;
constexpr int SORT_WAVES = SORT_THREADS / 64;
constexpr int SORT_ITEMS = 8;
constexpr int SORT_TILE = SORT_THREADS * SORT_ITEMS;  // keys per block
constexpr int MAX_BINS = 1024;

__device__ __forceinline__ uint64_t lanemask_lt() {
  const unsigned lane = threadIdx.x & 63;
  return lane == 0 ? 0ull : (~0ull >> (64 - lane));
}

// ----------------------------------------------------------------- sort
// Digit histogram of one tile: hist[(tile_base[f] << rb) + digit * T_f + tile].
__global__ __launch_bounds__(SORT_THREADS) void sort_hist_kernel(const int32_t* keys, uint32_t* hist,
                                                                 FieldPtr fp, TileBase tb, int shift, int rb) {
  __shared__ uint32_t h[MAX_BINS];
  const int f = blockIdx.y, t = blockIdx.x;
  const int tiles = tb.t[f + 1] - tb.t[f];
  if (t >= tiles) return;
  const int nb = 1 << rb;
  for (int d = threadIdx.x; d < nb; d += SORT_THREADS) h[d] = 0;
  __syncthreads();
  const int64_t base = fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - base);
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + i * SORT_THREADS + threadIdx.x;
    if (pos < nnz) atomicAdd(&h[(keys[base + pos] >> shift) & (nb - 1)], 1u);
  }
  __syncthreads();
  uint32_t* out = hist + ((int64_t)tb.t[f] << rb);
  for (int d = threadIdx.x; d < nb; d += SORT_THREADS) out[(int64_t)d * tiles + t] = h[d];
}

// Exclusive prefix sum, in place, over the (digit-major, tile-minor) histogram of one field.
__global__ __launch_bounds__(1024) void sort_scan_kernel(uint32_t* hist, TileBase tb, int rb) {
  __shared__ uint32_t wsum[16];
  const int f = blockIdx.x;
  const int tiles = tb.t[f + 1] - tb.t[f];
  const int n = tiles << rb;
  if (n == 0) return;
  uint32_t* h = hist + ((int64_t)tb.t[f] << rb);
  const int chunk = (n + 1023) / 1024;
  const int lo = min(n, (int)threadIdx.x * chunk), hi = min(n, lo + chunk);
  uint32_t sum = 0;
  for (int i = lo; i < hi; ++i) sum += h[i];
  // block-wide exclusive scan of the per-thread sums
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  uint32_t incl = sum;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) wsum[w] = incl;
  __syncthreads();
  uint32_t wbase = 0;
  for (int i = 0; i < w; ++i) wbase += wsum[i];
  uint32_t run = wbase + incl - sum;
  for (int i = lo; i < hi; ++i) {
    const uint32_t c = h[i];
    h[i] = run;
    run += c;
  }
}

// Stable scatter of one tile.  Wave w owns the contiguous 512-key slice w of the tile and
// walks it in 8 rounds of 64 keys; lanes holding equal digits find each other with one
// ballot per digit bit, the per-wave running count of the digit lives in LDS.
__global__ __launch_bounds__(SORT_THREADS) void sort_scatter_kernel(
    const int32_t* keys_in, const int32_t* pay_in, const int32_t* offsets, int32_t* keys_out,
    int32_t* pay_out, const uint32_t* hist, FieldPtr fp, TileBase tb, int shift, int rb, int B) {
  __shared__ uint32_t cnt[SORT_WAVES][MAX_BINS];
  const int f = blockIdx.y, t = blockIdx.x;
  const int tiles = tb.t[f + 1] - tb.t[f];
  if (t >= tiles) return;
  const int nb = 1 << rb;
  for (int d = threadIdx.x; d < SORT_WAVES * MAX_BINS; d += SORT_THREADS) (&cnt[0][0])[d] = 0;
  __syncthreads();
  const int64_t base = fp.p[f];
  const int nnz = (int)(fp.p[f + 1] - base);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const uint64_t lt = lanemask_lt();
  volatile uint32_t* cw = cnt[w];
  int32_t key[SORT_ITEMS];
  uint32_t rank[SORT_ITEMS];
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + w * (64 * SORT_ITEMS) + i * 64 + lane;
    const bool valid = pos < nnz;
    key[i] = valid ? keys_in[base + pos] : 0;
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
  for (int d = threadIdx.x; d < nb; d += SORT_THREADS) {
    uint32_t run = 0;
#pragma unroll
    for (int ww = 0; ww < SORT_WAVES; ++ww) {
      const uint32_t c = cnt[ww][d];
      cnt[ww][d] = run;
      run += c;
    }
  }
  __syncthreads();
  const uint32_t* hb = hist + ((int64_t)tb.t[f] << rb);
  const int32_t* off = offsets + (int64_t)f * (B + 1);
#pragma unroll
  for (int i = 0; i < SORT_ITEMS; ++i) {
    const int pos = t * SORT_TILE + w * (64 * SORT_ITEMS) + i * 64 + lane;
    if (pos < nnz) {
      const uint32_t d = ((uint32_t)key[i] >> shift) & (nb - 1);
      const uint32_t dst = hb[(int64_t)d * tiles + t] + cnt[w][d] + rank[i];
      int32_t pay;
      if (pay_in) {
        pay = pay_in[base + pos];
      } else {  // first pass: the sample whose bag holds lookup `pos`
        int lo = 0, hi = B;
        while (hi - lo > 1) {
          const int mid = (lo + hi) >> 1;
          if (off[mid] <= pos) lo = mid; else hi = mid;
        }
        pay = lo;
      }
      if (dst < (uint32_t)nnz) {
        keys_out[base + dst] = key[i];
        pay_out[base + dst] = pay;
      }
    }
  }
}

// ------------------------------------------------------------- segments
__device__ __forceinline__ bool is_head(const int32_t* key, int pos) {
  return pos == 0 || key[pos] != key[pos - 1];
}

// Number of run heads in each tile of the sorted keys.
__global__ __launch_bounds__(SORT_THREADS) void seg_heads_kernel(SegArgs a, FieldPtr fp, TileBase tb) {
  __shared__ int wsum[SORT_WAVES];
  const int f = blockIdx.y, t = blockIdx.x;
  if (t >= tb.t[f + 1] - tb.t[f]) return;
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
// the terminal segment offset of every field, the per-sample aggregation weight, and the
// reset of the long-segment queue.
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
    a.long_count[0] = 0;
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
  const int f = blockIdx.y, t = blockIdx.x;
  if (t >= tb.t[f + 1] - tb.t[f]) return;
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
      a.segoff[rank + f] = p0 + i;
      ++rank;
    }
}

__device__ __forceinline__ int field_of_unique(const int32_t* ubase, int F, int u) {
  int lo = 0, hi = F;  // ubase[lo] <= u < ubase[hi]
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (ubase[mid] <= u) lo = mid; else hi = mid;
  }
  return lo;
}

// One group of D/4 lanes per run; runs longer than the threshold are queued for the block kernel.
__global__ __launch_bounds__(256) void seg_reduce_kernel(SegArgs a, FieldPtr fp) {
  const int lps = a.D >> 2;
  const int U = a.ubase[a.F];
  const int groups_per_block = 256 / lps;
  const int g = threadIdx.x / lps, c = threadIdx.x - g * lps;
  for (int64_t u = (int64_t)blockIdx.x * groups_per_block + g; u < U; u += (int64_t)gridDim.x * groups_per_block) {
    const int f = field_of_unique(a.ubase, a.F, (int)u);
    const int b = a.segoff[u + f], e = a.segoff[u + f + 1];
    if (e - b > a.long_threshold) {
      if (c == 0) {
        const int slot = atomicAdd(a.long_count, 1);
        if (slot < a.long_cap) a.long_list[slot] = (int)u;
      }
      continue;
    }
    const int32_t* pay = a.pay + fp.p[f];
    const float* dx = a.dx + f * a.D + c * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = b; i < e; ++i) {
      const int s = min(max(pay[i], 0), a.B - 1);
      const float w = a.sample_w[s];
      const float4 v = *reinterpret_cast<const float4*>(dx + (int64_t)s * a.lddx);
      acc.x = fmaf(w, v.x, acc.x);
      acc.y = fmaf(w, v.y, acc.y);
      acc.z = fmaf(w, v.z, acc.z);
      acc.w = fmaf(w, v.w, acc.w);
    }
    *reinterpret_cast<float4*>(a.G + u * a.D + c * 4) = acc;
  }
}

// One block per long run: the lane groups stride over the run, then their partial sums are
// added in group order.
__global__ __launch_bounds__(256) void seg_reduce_long_kernel(SegArgs a, FieldPtr fp) {
  __shared__ float4 red[256];
  const int lps = a.D >> 2;
  const int ngroups = 256 / lps;
  const int g = threadIdx.x / lps, c = threadIdx.x - g * lps;
  const int count = min(a.long_count[0], a.long_cap);
  for (int idx = blockIdx.x; idx < count; idx += gridDim.x) {
    const int u = a.long_list[idx];
    const int f = field_of_unique(a.ubase, a.F, u);
    const int b = a.segoff[u + f], e = a.segoff[u + f + 1];
    const int32_t* pay = a.pay + fp.p[f];
    const float* dx = a.dx + f * a.D + c * 4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 4
    for (int i = b + g; i < e; i += ngroups) {
      const int s = min(max(pay[i], 0), a.B - 1);
      const float w = a.sample_w[s];
      const float4 v = *reinterpret_cast<const float4*>(dx + (int64_t)s * a.lddx);
      acc.x = fmaf(w, v.x, acc.x);
      acc.y = fmaf(w, v.y, acc.y);
      acc.z = fmaf(w, v.z, acc.z);
      acc.w = fmaf(w, v.w, acc.w);
    }
    red[threadIdx.x] = acc;
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
    if (g == 0) *reinterpret_cast<float4*>(a.G + (int64_t)u * a.D + c * 4) = red[c];
    __syncthreads();
  }
}

}  // namespace

hipError_t launch_sort_pass(const SortPlan& pl, const SortBuffers& sb, int pass, const FieldPtr& fp,
                            const TileBase& tb, Profiler* prof, hipStream_t s) {
  if (pl.total_tiles == 0) return hipSuccess;
  const int shift = pass * pl.radix_bits;
  const int32_t* kin = pass == 0 ? sb.ids : sb.key[(pass - 1) & 1];
  const int32_t* pin = pass == 0 ? sb.pay0 : sb.pay[(pass - 1) & 1];
  dim3 grid(pl.max_tiles, pl.F);
  {
    ProfScope ps(prof, KID_SORT_HIST, s);
    hipLaunchKernelGGL(sort_hist_kernel, grid, dim3(SORT_THREADS), 0, s, kin, sb.hist, fp, tb, shift, pl.radix_bits);
  }
  {
    ProfScope ps(prof, KID_SORT_SCAN, s);
    hipLaunchKernelGGL(sort_scan_kernel, dim3(pl.F), dim3(1024), 0, s, sb.hist, tb, pl.radix_bits);
  }
  {
    ProfScope ps(prof, KID_SORT_SCATTER, s);
    hipLaunchKernelGGL(sort_scatter_kernel, grid, dim3(SORT_THREADS), 0, s, kin, pin, sb.offsets,
                       sb.key[pass & 1], sb.pay[pass & 1], sb.hist, fp, tb, shift, pl.radix_bits, pl.B);
  }
  return hipGetLastError();
}

hipError_t launch_segments(const SegArgs& a, const FieldPtr& fp, const TileBase& tb, const ShardTab& tab,
                           Profiler* prof, hipStream_t s) {
  dim3 grid(a.max_tiles, a.F);
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
  return hipGetLastError();
}

hipError_t launch_seg_reduce(const SegArgs& a, const FieldPtr& fp, int64_t nnz_total, Profiler* prof,
                             hipStream_t s) {
  if (nnz_total == 0) return hipSuccess;
  const int groups_per_block = 256 / (a.D >> 2);
  int64_t blocks = (nnz_total + groups_per_block - 1) / groups_per_block;
  if (blocks > 256 * 32) blocks = 256 * 32;
  {
    ProfScope ps(prof, KID_SEG_REDUCE, s);
    hipLaunchKernelGGL(seg_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a, fp);
  }
  {
    ProfScope ps(prof, KID_SEG_REDUCE_LONG, s);
    hipLaunchKernelGGL(seg_reduce_long_kernel, dim3(1024), dim3(256), 0, s, a, fp);
  }
  return hipGetLastError();
}

}  // namespace antdt
