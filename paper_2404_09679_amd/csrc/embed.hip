// Embedding-bag gather and sum- or mean-pool (worker side of the iteration, Section II:
// the forward pass on the local batch B_k), plus the procedural table fill.
#include <algorithm>

#include "common.h"

namespace antdt {

// 16-byte vector of table elements.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 v;
  __device__ __forceinline__ float get(int i) const { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  uint4 v;
  __device__ __forceinline__ float get(int i) const {
    uint32_t w = i < 2 ? v.x : i < 4 ? v.y : i < 6 ? v.z : v.w;
    return (i & 1) ? __uint_as_float(w & 0xFFFF0000u) : __uint_as_float(w << 16);
  }
};

template <typename OT, int N> __device__ __forceinline__ void store_row(OT* dst, const float* v);
template <> __device__ __forceinline__ void store_row<float, 4>(float* dst, const float* v) {
  *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
}
template <> __device__ __forceinline__ void store_row<float, 8>(float* dst, const float* v) {
  reinterpret_cast<float4*>(dst)[0] = make_float4(v[0], v[1], v[2], v[3]);
  reinterpret_cast<float4*>(dst)[1] = make_float4(v[4], v[5], v[6], v[7]);
}
template <> __device__ __forceinline__ void store_row<bf16_t, 4>(bf16_t* dst, const float* v) {
  *reinterpret_cast<uint2*>(dst) = make_uint2((uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16),
                                              (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16));
}
template <> __device__ __forceinline__ void store_row<bf16_t, 8>(bf16_t* dst, const float* v) {
  *reinterpret_cast<uint4*>(dst) = make_uint4((uint32_t)f2bf(v[0]) | ((uint32_t)f2bf(v[1]) << 16),
                                              (uint32_t)f2bf(v[2]) | ((uint32_t)f2bf(v[3]) << 16),
                                              (uint32_t)f2bf(v[4]) | ((uint32_t)f2bf(v[5]) << 16),
                                              (uint32_t)f2bf(v[6]) | ((uint32_t)f2bf(v[7]) << 16));
}

// Dense-feature columns of 64 samples: copied behind the pooled embeddings (and into the
// transposed copy), the padding columns of the row are zeroed.
template <typename OT>
__device__ __forceinline__ void dense_columns(const PoolArgs& a, int sl0) {
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  if (sl0 + tx >= a.ns) return;
  const int64_t s = a.s0 + sl0 + tx;
  const int FD = a.F * a.D;
  OT* xrow = reinterpret_cast<OT*>(a.x) + s * a.ldx + FD;
  for (int c = ty; c < a.ldx - FD; c += 4) {
    const float v = c < a.num_dense ? a.dense[s * a.num_dense + c] : 0.0f;
    xrow[c] = from_f32<OT>(v);
    if (a.xt && c < a.num_dense) a.xt[(int64_t)(FD + c) * a.ldt + s] = f2bf(v);
  }
}

// Gather and sum-pool.  A block owns 64 consecutive samples of one field; a group of
// LPR = D*sizeof(T)/16 lanes owns one bag, so a wavefront works on 64/LPR bags at once.
// The group fetches LPR ids with one coalesced load, hands them round with lane
// shuffles and issues the LPR row loads (16 bytes per lane, one whole row per group)
// back to back before adding them, which keeps 64 rows in flight per wavefront.  The
// pooled rows are written to X and, through an LDS tile, to the transposed copy that the
// weight-gradient GEMM reads.  Every lookup's sample index is recorded for the sort.
template <typename TT, typename OT, int LPR>
__global__ __launch_bounds__(256) void pool_tile_kernel(PoolArgs a, FieldPtr fp) {
  constexpr int EV = Vec16<TT>::N;
  constexpr int G = 256 / LPR;       // bags per round
  constexpr int ROUNDS = 64 / G;
  constexpr int TP = 130;            // tile pitch (odd number of dwords: conflict-free column reads)
  __shared__ bf16_t tile[64 * TP];
  const int f = blockIdx.y, sl0 = blockIdx.x * 64;
  if (f == a.F) {
    dense_columns<OT>(a, sl0);
    return;
  }
  const int g = threadIdx.x / LPR, c = threadIdx.x % LPR;
  const int gl = (threadIdx.x & 63) - c;  // first lane of this group inside the wavefront
  const int32_t* ids = a.ids + fp.p[f];
  const TT* tab = reinterpret_cast<const TT*>(a.tables) + (int64_t)f * a.R * a.D + c * EV;
  const bool use_tile = a.xt != nullptr && a.D <= 128;
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    const int ls = r * G + g;
    const bool valid = sl0 + ls < a.ns;
    const int64_t s = a.s0 + sl0 + ls;
    int begin = 0, end = 0;
    if (valid) {
      const int32_t* off = a.offsets + (int64_t)f * (a.B + 1) + s;
      begin = off[0];
      end = off[1];
    }
    float acc[EV];
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[e] = 0.0f;
    for (int jb = begin; jb < end; jb += LPR) {
      const int my_j = jb + c;
      int my_id = 0;
      if (my_j < end) {
        my_id = ids[my_j];
        if (a.lookup_sample) a.lookup_sample[fp.p[f] + my_j] = (int32_t)s;
      }
      Vec16<TT> v[LPR];
#pragma unroll
      for (int q = 0; q < LPR; ++q) {
        const int64_t row = min(max((int64_t)__shfl(my_id, gl + q, 64), (int64_t)0), a.R - 1);
        if (jb + q < end) v[q].v = *reinterpret_cast<const decltype(v[q].v)*>(tab + row * a.D);
      }
#pragma unroll
      for (int q = 0; q < LPR; ++q)
        if (jb + q < end) {
#pragma unroll
          for (int e = 0; e < EV; ++e) acc[e] += v[q].get(e);
        }
    }
    if (a.mean_pool && end - begin > 1) {
      const float len = (float)(end - begin);
#pragma unroll
      for (int e = 0; e < EV; ++e) acc[e] /= len;
    }
    if (valid) {
      store_row<OT, EV>(reinterpret_cast<OT*>(a.x) + s * a.ldx + f * a.D + c * EV, acc);
      if (a.xt) {
        if (use_tile) {
#pragma unroll
          for (int e = 0; e < EV; ++e) tile[ls * TP + c * EV + e] = f2bf(acc[e]);
        } else {
#pragma unroll
          for (int e = 0; e < EV; ++e) a.xt[(int64_t)(f * a.D + c * EV + e) * a.ldt + s] = f2bf(acc[e]);
        }
      }
    }
  }
  if (use_tile) {
    __syncthreads();
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    if (sl0 + tx < a.ns) {
      bf16_t* dst = a.xt + (int64_t)f * a.D * a.ldt + a.s0 + sl0 + tx;
      for (int d = ty; d < a.D; d += 4) dst[(int64_t)d * a.ldt] = tile[tx * TP + d];
    }
  }
}

// Fallback for other row sizes: one wavefront per (sample, field) bag, 64/LPR rows in
// flight, partial sums combined with a butterfly over the lane groups.
template <typename TT, typename OT>
__global__ __launch_bounds__(256) void pool_kernel(PoolArgs a, FieldPtr fp) {
  constexpr int EV = Vec16<TT>::N;
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int64_t sl = item / a.F;
  if (sl >= a.ns) return;
  const int f = (int)(item - sl * a.F);
  const int64_t s = a.s0 + sl;
  OT* xrow = reinterpret_cast<OT*>(a.x) + s * a.ldx;
  const int lpr = a.D / EV;  // lanes per row, power of two
  const int rpi = 64 / lpr;  // rows in flight
  const int sub = lane / lpr;
  const int c = lane - sub * lpr;
  const int32_t* off = a.offsets + (int64_t)f * (a.B + 1) + s;
  const int begin = off[0], end = off[1];
  const int32_t* ids = a.ids + fp.p[f];
  const TT* tab = reinterpret_cast<const TT*>(a.tables) + (int64_t)f * a.R * a.D + c * EV;
  if (a.lookup_sample)
    for (int j = begin + lane; j < end; j += 64) a.lookup_sample[fp.p[f] + j] = (int32_t)s;
  float acc[EV];
#pragma unroll
  for (int e = 0; e < EV; ++e) acc[e] = 0.0f;
  for (int j = begin + sub; j < end; j += rpi) {
    const int64_t row = min(max((int64_t)ids[j], (int64_t)0), a.R - 1);  // keeps a bad id in bounds
    Vec16<TT> v;
    v.v = *reinterpret_cast<const decltype(v.v)*>(tab + row * a.D);
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[e] += v.get(e);
  }
  for (int o = lpr; o < 64; o <<= 1) {
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[e] += __shfl_xor(acc[e], o, 64);
  }
  if (a.mean_pool && end - begin > 1) {
    const float len = (float)(end - begin);
#pragma unroll
    for (int e = 0; e < EV; ++e) acc[e] /= len;
  }
  if (sub == 0) {
    store_row<OT, EV>(xrow + f * a.D + c * EV, acc);
    if (a.xt) {
#pragma unroll
      for (int e = 0; e < EV; ++e) a.xt[(int64_t)(f * a.D + c * EV + e) * a.ldt + s] = f2bf(acc[e]);
    }
  }
}

template <typename OT>
__global__ __launch_bounds__(256) void pool_dense_kernel(PoolArgs a) {
  dense_columns<OT>(a, blockIdx.x * 64);
}

template <typename TT, typename OT>
static void launch_pool_typed(const PoolArgs& a, const FieldPtr& fp, hipStream_t s) {
  const int lpr = a.D / Vec16<TT>::N;
  dim3 grid((a.ns + 63) / 64, a.F + 1), block(256);
  if (lpr == 4) hipLaunchKernelGGL((pool_tile_kernel<TT, OT, 4>), grid, block, 0, s, a, fp);
  else if (lpr == 8) hipLaunchKernelGGL((pool_tile_kernel<TT, OT, 8>), grid, block, 0, s, a, fp);
  else if (lpr == 16) hipLaunchKernelGGL((pool_tile_kernel<TT, OT, 16>), grid, block, 0, s, a, fp);
  else {
    const int64_t items = (int64_t)a.ns * a.F;
    hipLaunchKernelGGL((pool_kernel<TT, OT>), dim3((unsigned)((items + 3) / 4)), block, 0, s, a, fp);
    hipLaunchKernelGGL((pool_dense_kernel<OT>), dim3((a.ns + 63) / 64), block, 0, s, a);
  }
}

// Input check: flags[0] bit 0 = an id outside [0, R), bit 1 = offsets of a field that do not
// start at 0, decrease, or do not end at the field's lookup count; flags[1] = lowest offending
// field + 1.  Reads only what the host-side sizes cover, never through an offset.
__global__ __launch_bounds__(256) void validate_kernel(const int32_t* ids, const int32_t* offsets, FieldPtr fp,
                                                       int64_t B, int64_t R, int F, int32_t* flags) {
  const int f = blockIdx.y;
  const int64_t n = fp.p[f + 1] - fp.p[f];
  const int32_t* off = offsets + (int64_t)f * (B + 1);
  int bad = 0;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256) {
    const int32_t id = ids[fp.p[f] + i];
    if (id < 0 || id >= R) bad |= 1;
  }
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i <= B; i += (int64_t)gridDim.x * 256) {
    const int64_t v = off[i];
    if (i == 0 && v != 0) bad |= 2;
    if (i == B && v != n) bad |= 2;
    if (i > 0 && v < off[i - 1]) bad |= 2;
  }
  if (bad) {
    atomicOr(&flags[0], bad);
    atomicMin(&flags[1], f + 1);
  }
}

__global__ void validate_reset_kernel(int32_t* flags) {
  if (threadIdx.x == 0) {
    flags[0] = 0;
    flags[1] = 0x7FFFFFFF;
  }
}

hipError_t launch_validate_reset(int32_t* flags, hipStream_t s) {
  hipLaunchKernelGGL(validate_reset_kernel, dim3(1), dim3(64), 0, s, flags);
  return hipGetLastError();
}

hipError_t launch_validate(const int32_t* ids, const int32_t* offsets, const FieldPtr& fp, int64_t B, int64_t R, int F,
                           int32_t* flags, hipStream_t s) {
  hipLaunchKernelGGL(validate_reset_kernel, dim3(1), dim3(64), 0, s, flags);
  int64_t work = B + 1;
  for (int f = 0; f < F; ++f) work = std::max<int64_t>(work, fp.p[f + 1] - fp.p[f]);
  const unsigned bx = (unsigned)std::min<int64_t>((work + 255) / 256, 1024);
  hipLaunchKernelGGL(validate_kernel, dim3(bx, F), dim3(256), 0, s, ids, offsets, fp, B, R, F, flags);
  return hipGetLastError();
}

hipError_t launch_pool(const PoolArgs& a, const FieldPtr& fp, hipStream_t s) {
  if (a.ns <= 0) return hipSuccess;
  if (a.table_bf16) {
    if (a.x_bf16) launch_pool_typed<bf16_t, bf16_t>(a, fp, s);
    else launch_pool_typed<bf16_t, float>(a, fp, s);
  } else {
    if (a.x_bf16) launch_pool_typed<float, bf16_t>(a, fp, s);
    else launch_pool_typed<float, float>(a, fp, s);
  }
  return hipGetLastError();
}

// ------------------------------------------------------------------------
__device__ __forceinline__ uint32_t fmix32(uint32_t x) {
  x ^= x >> 16;
  x *= 0x85EBCA6Bu;
  x ^= x >> 13;
  x *= 0xC2B2AE35u;
  x ^= x >> 16;
  return x;
}

template <typename TT>
__global__ __launch_bounds__(256) void fill_tables_kernel(TT* tables, int F, int64_t R, int D, float scale) {
  const int64_t total = (int64_t)F * R * D;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int64_t row = i / D;
    const int d = (int)(i - row * D);
    const int64_t f = row / R;
    const uint32_t r = (uint32_t)(row - f * R);
    const uint32_t h1 = fmix32(r + 0x9E3779B9u * (uint32_t)(f + 1));
    const uint32_t h = fmix32(h1 ^ (0x85EBCA6Bu * (uint32_t)(d + 1)));
    const float t = __fsub_rn(__fmul_rn((float)(h >> 8), 1.1920928955078125e-07f), 1.0f);
    tables[i] = from_f32<TT>(__fmul_rn(scale, t));
  }
}

hipError_t launch_fill_tables(void* tables, int bf16, int F, int64_t R, int D, float scale, hipStream_t s) {
  dim3 grid(256 * 16), block(256);
  if (bf16) hipLaunchKernelGGL(fill_tables_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)tables, F, R, D, scale);
  else hipLaunchKernelGGL(fill_tables_kernel<float>, grid, block, 0, s, (float*)tables, F, R, D, scale);
  return hipGetLastError();
}

}  // namespace antdt
