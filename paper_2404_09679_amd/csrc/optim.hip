// Server-side dense aggregation and the parameter updates (Section II: the servers
// combine the workers' gradients, then update the parameters).
// All of these stream through memory once: they are bound by HBM bandwidth.
#include "common.h"

namespace antdt {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float weighted_sum(const float* grads, int64_t stride, int64_t i, const ShardTab& tab) {
  // Every load is issued (a branch per load would serialise them); the value of a shard
  // with weight 0, which may never have been written, is replaced by 0 afterwards.
  float acc = 0.0f;
  int k = 0;
  for (; k + 3 < tab.K; k += 4) {  // four loads in flight, added in shard order
    float x[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) x[q] = grads[(int64_t)(k + q) * stride + i];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc = fmaf(tab.w[k + q], tab.w[k + q] != 0.0f ? x[q] : 0.0f, acc);
  }
  for (; k < tab.K; ++k) {
    const float x = grads[(int64_t)k * stride + i];
    acc = fmaf(tab.w[k], tab.w[k] != 0.0f ? x : 0.0f, acc);
  }
  return acc;
}

// g[i] = sum_k w_k * grads[k][i], shards added in index order.
__global__ __launch_bounds__(256) void dense_agg_kernel(DenseAggArgs a, ShardTab tab) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.P; i += stride)
    a.g[i] = weighted_sum(a.grads, a.stride, i, tab);
}

__device__ __forceinline__ float adagrad_elem(const DenseAdagradArgs& a, const ShardTab& tab, int64_t i) {
  const float g = weighted_sum(a.grads, a.stride, i, tab);
  const float s1 = fmaf(g, g, a.state[i]);
  const float p1 = a.p[i] - a.lr * g / (sqrtf(s1) + a.eps);
  a.state[i] = s1;
  a.p[i] = p1;
  return p1;
}

__global__ __launch_bounds__(256) void dense_adagrad_kernel(DenseAdagradArgs a, ShardTab tab) {
  __shared__ bf16_t tile[64][66];
  const int nt = a.tile_base[a.n_mat];
  if ((int)blockIdx.x < nt) {
    int mi = 0;
    while (mi + 1 < a.n_mat && (int)blockIdx.x >= a.tile_base[mi + 1]) ++mi;
    const int t = blockIdx.x - a.tile_base[mi];
    const int rows = a.rows[mi], cols = a.cols[mi];
    const int tc = (cols + 63) / 64;
    const int r0 = (t / tc) * 64, c0 = (t % tc) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const bool col_ok = c0 + tx < cols;
    // all loads of the thread's 16 elements first (indices clamped into the matrix), then the
    // arithmetic and the stores: loads interleaved with stores would wait for one another
    float g[16], p0[16], s0[16];
    int64_t idx[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = min(r0 + ty + 4 * q, rows - 1), cc = min(c0 + tx, cols - 1);
      idx[q] = a.w_off[mi] + (int64_t)r * cols + cc;
      p0[q] = a.p[idx[q]];
      s0[q] = a.state[idx[q]];
      g[q] = 0.0f;
    }
    for (int k = 0; k < tab.K; ++k) {  // shards in index order, 16 independent loads per shard
      const float w = tab.w[k];
      float x[16];
#pragma unroll
      for (int q = 0; q < 16; ++q) x[q] = a.grads[(int64_t)k * a.stride + idx[q]];
#pragma unroll
      for (int q = 0; q < 16; ++q) g[q] = fmaf(w, w != 0.0f ? x[q] : 0.0f, g[q]);
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int r = ty + 4 * q;
      bf16_t h = 0;
      if (r0 + r < rows && col_ok) {
        const int64_t e = (int64_t)(r0 + r) * cols + c0 + tx;
        const float s1 = fmaf(g[q], g[q], s0[q]);
        const float p1 = p0[q] - a.lr * g[q] / (sqrtf(s1) + a.eps);
        a.state[a.w_off[mi] + e] = s1;
        a.p[a.w_off[mi] + e] = p1;
        h = f2bf(p1);
        a.wb[mi][e] = h;
      }
      tile[r][tx] = h;
    }
    __syncthreads();
    for (int cidx = ty; cidx < 64; cidx += 4)
      if (c0 + cidx < cols && r0 + tx < rows)
        a.wbt[mi][(int64_t)(c0 + cidx) * a.rows_pad[mi] + r0 + tx] = tile[tx][cidx];
    return;
  }
  const int rb = blockIdx.x - nt;
  int ri = 0;
  while (ri + 1 < a.n_rng && rb >= a.rng_block[ri + 1]) ++ri;
  const int64_t i = (int64_t)(rb - a.rng_block[ri]) * 256 + threadIdx.x;
  if (i < a.rng_len[ri]) adagrad_elem(a, tab, a.rng_off[ri] + i);
}

// Weighted average of K gradient buffers fused with Adam (bias-corrected), 16 bytes per lane.
template <int K>
__global__ __launch_bounds__(256) void adam_kernel(AdamArgs a) {
  const int64_t n4 = a.n >> 2;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  const float c1 = a.c1, c2 = a.c2;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    f32x4 g = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const f32x4 x = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(a.g[k]) + i);
      g += a.w[k] * x;
    }
    f32x4 m = reinterpret_cast<f32x4*>(a.m)[i], v = reinterpret_cast<f32x4*>(a.v)[i];
    f32x4 p = reinterpret_cast<f32x4*>(a.p)[i];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      m[q] = fmaf(a.b1, m[q], c1 * g[q]);
      v[q] = fmaf(a.b2, v[q], c2 * g[q] * g[q]);
      p[q] -= a.lr * (m[q] * a.inv_bc1) / (sqrtf(v[q] * a.inv_bc2) + a.eps);
    }
    reinterpret_cast<f32x4*>(a.m)[i] = m;
    reinterpret_cast<f32x4*>(a.v)[i] = v;
    reinterpret_cast<f32x4*>(a.p)[i] = p;
  }
  // tail (n not a multiple of 4)
  if (blockIdx.x == 0) {
    for (int64_t i = (n4 << 2) + threadIdx.x; i < a.n; i += blockDim.x) {
      float g = 0.f;
#pragma unroll
      for (int k = 0; k < K; ++k) g = fmaf(a.w[k], a.g[k][i], g);
      const float m = fmaf(a.b1, a.m[i], c1 * g);
      const float v = fmaf(a.b2, a.v[i], c2 * g * g);
      a.m[i] = m;
      a.v[i] = v;
      a.p[i] -= a.lr * (m * a.inv_bc1) / (sqrtf(v * a.inv_bc2) + a.eps);
    }
  }
}

template <int K> void launch_adam_k(const AdamArgs& a, dim3 grid, hipStream_t s) {
  hipLaunchKernelGGL(adam_kernel<K>, grid, dim3(256), 0, s, a);
}

}  // namespace

hipError_t launch_dense_agg(const DenseAggArgs& a, const ShardTab& tab, hipStream_t s) {
  if (a.P <= 0) return hipSuccess;
  int64_t blocks = (a.P + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(dense_agg_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a, tab);
  return hipGetLastError();
}

hipError_t launch_dense_adagrad(const DenseAdagradArgs& a, const ShardTab& tab, hipStream_t s) {
  const int blocks = a.tile_base[a.n_mat] + a.rng_block[a.n_rng];
  if (blocks <= 0) return hipSuccess;
  hipLaunchKernelGGL(dense_adagrad_kernel, dim3(blocks), dim3(256), 0, s, a, tab);
  return hipGetLastError();
}

// Plain streaming copy, one 16-byte vector per thread: the measured bandwidth that the
// memory-bound kernels are compared with.
__global__ __launch_bounds__(256) void stream_copy_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                          int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t n4 = n >> 2;
  if (i < n4) reinterpret_cast<float4*>(dst)[i] = reinterpret_cast<const float4*>(src)[i];
  if (i < (n & 3)) dst[(n4 << 2) + i] = src[(n4 << 2) + i];
}

hipError_t launch_stream_copy(float* dst, const float* src, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int64_t blocks = ((n >> 2) + 255) / 256 + 1;
  hipLaunchKernelGGL(stream_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, s, dst, src, n);
  return hipGetLastError();
}

hipError_t launch_adam(const AdamArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  // One 16-byte vector per thread and no grid-stride loop: with 262144 blocks for 2^28 elements
  // the kernel streams at 5.6 TB/s; 4096 blocks looping over the buffers reach 4.6 TB/s.
  int64_t blocks = ((a.n >> 2) + 255) / 256;
  if (blocks > (1ll << 30)) blocks = 1ll << 30;
  if (blocks < 1) blocks = 1;
  dim3 grid((unsigned)blocks);
  switch (a.K) {
    case 1: launch_adam_k<1>(a, grid, s); break;
    case 2: launch_adam_k<2>(a, grid, s); break;
    case 3: launch_adam_k<3>(a, grid, s); break;
    case 4: launch_adam_k<4>(a, grid, s); break;
    case 5: launch_adam_k<5>(a, grid, s); break;
    case 6: launch_adam_k<6>(a, grid, s); break;
    case 7: launch_adam_k<7>(a, grid, s); break;
    case 8: launch_adam_k<8>(a, grid, s); break;
    case 9: launch_adam_k<9>(a, grid, s); break;
    case 10: launch_adam_k<10>(a, grid, s); break;
    case 11: launch_adam_k<11>(a, grid, s); break;
    case 12: launch_adam_k<12>(a, grid, s); break;
    case 13: launch_adam_k<13>(a, grid, s); break;
    case 14: launch_adam_k<14>(a, grid, s); break;
    case 15: launch_adam_k<15>(a, grid, s); break;
    case 16: launch_adam_k<16>(a, grid, s); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace antdt
