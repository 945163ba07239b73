// Server-side dense aggregation and the parameter updates (Section II: "the
// servers aggregate the local gradients ... and update the parameters").
// All of these stream through memory once: they are bound by HBM bandwidth.
#include "common.h"

namespace antdt {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

// g[i] = sum_k w_k * grads[k][i], shards added in index order.
__global__ __launch_bounds__(256) void dense_agg_kernel(DenseAggArgs a, ShardTab tab) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.P; i += stride) {
    float acc = 0.0f;
    for (int k = 0; k < tab.K; ++k) {
      const float w = tab.w[k];
      if (w != 0.0f) acc = fmaf(w, a.grads[(int64_t)k * a.P + i], acc);
    }
    a.g[i] = acc;
  }
}

// Dense Adagrad on the MLP parameters, refreshing the bf16 operand copies in the same pass.
__global__ __launch_bounds__(256) void dense_adagrad_kernel(DenseAdagradArgs a) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.P; i += stride) {
    const float g = a.g[i];
    const float s1 = fmaf(g, g, a.state[i]);
    const float p1 = a.p[i] - a.lr * g / (sqrtf(s1) + a.eps);
    a.state[i] = s1;
    a.p[i] = p1;
    for (int l = 0; l < a.n_copy; ++l) {
      const int64_t j = i - a.w_off[l];
      if (j >= 0 && j < a.w_len[l]) a.copy[l][j] = f2bf(p1);
    }
  }
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

hipError_t launch_dense_adagrad(const DenseAdagradArgs& a, hipStream_t s) {
  if (a.P <= 0) return hipSuccess;
  int64_t blocks = (a.P + 255) / 256;
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(dense_adagrad_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_adam(const AdamArgs& a, hipStream_t s) {
  if (a.n <= 0) return hipSuccess;
  int64_t blocks = ((a.n >> 2) + 255) / 256;
  if (blocks > 256 * 16) blocks = 256 * 16;
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
