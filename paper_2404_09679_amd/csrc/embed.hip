// Embedding-bag gather and sum-pool (worker side of the iteration, Section II:
// the forward pass on the local batch B_k), plus the procedural table fill.
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

// One wavefront per (sample, field) bag.  The 64 lanes are split into 64/LPR
// groups of LPR = D*sizeof(T)/16 lanes; every group streams one table row per
// step with 16-byte loads (a whole row is one contiguous, fully used request),
// so up to 64/LPR rows of the bag are in flight at once.  Partial sums are
// combined with a butterfly over the groups and group 0 writes the pooled row.
// The "field" index F stands for the dense-feature columns of the sample.
template <typename TT, typename OT>
__global__ __launch_bounds__(256) void pool_kernel(PoolArgs a, FieldPtr fp) {
  constexpr int EV = Vec16<TT>::N;
  const int lane = threadIdx.x & 63;
  const int64_t item = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int nf = a.F + 1;
  const int64_t sl = item / nf;
  if (sl >= a.ns) return;
  const int f = (int)(item - sl * nf);
  const int64_t s = a.s0 + sl;
  OT* xrow = reinterpret_cast<OT*>(a.x) + s * a.ldx;
  if (f == a.F) {
    const int ncol = a.ldx - a.F * a.D;  // dense features, then zero padding
    for (int c = lane; c < ncol; c += 64) {
      float v = c < a.num_dense ? a.dense[s * a.num_dense + c] : 0.0f;
      xrow[a.F * a.D + c] = from_f32<OT>(v);
    }
    return;
  }
  const int lpr = a.D / EV;  // lanes per row, power of two
  const int rpi = 64 / lpr;  // rows in flight
  const int sub = lane / lpr;
  const int c = lane - sub * lpr;
  const int32_t* off = a.offsets + (int64_t)f * (a.B + 1) + s;
  const int begin = off[0], end = off[1];
  const int32_t* ids = a.ids + fp.p[f];
  const TT* tab = reinterpret_cast<const TT*>(a.tables) + (int64_t)f * a.R * a.D + c * EV;
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
  if (sub == 0) {
    OT* dst = xrow + f * a.D + c * EV;
#pragma unroll
    for (int e = 0; e < EV; ++e) dst[e] = from_f32<OT>(acc[e]);
  }
}

hipError_t launch_pool(const PoolArgs& a, const FieldPtr& fp, hipStream_t s) {
  if (a.ns <= 0) return hipSuccess;
  const int64_t items = (int64_t)a.ns * (a.F + 1);
  dim3 grid((unsigned)((items + 3) / 4)), block(256);
  if (a.table_bf16) {
    if (a.x_bf16) hipLaunchKernelGGL((pool_kernel<bf16_t, bf16_t>), grid, block, 0, s, a, fp);
    else hipLaunchKernelGGL((pool_kernel<bf16_t, float>), grid, block, 0, s, a, fp);
  } else {
    if (a.x_bf16) hipLaunchKernelGGL((pool_kernel<float, bf16_t>), grid, block, 0, s, a, fp);
    else hipLaunchKernelGGL((pool_kernel<float, float>), grid, block, 0, s, a, fp);
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
