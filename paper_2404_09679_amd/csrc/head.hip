// Last (single-logit) layer, binary cross-entropy and the start of the backward
// pass of the worker step, plus the per-shard reductions that are sums over the
// samples of a shard (last-layer weight gradient, bias gradients, mean loss).
// Every reduction runs in a fixed order, so results are bitwise repeatable.
#include "common.h"

namespace antdt {
namespace {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// One wavefront per sample: z = h . w + b, the sample's loss and dz, then dh = dz * w
// (zeroed where the hidden activation is not positive).
template <typename TH, typename TD>
__global__ __launch_bounds__(256) void head_kernel(HeadArgs a, ShardTab tab) {
  const int lane = threadIdx.x & 63;
  const int64_t first = tab.start[a.k_begin];
  const int64_t last = (int64_t)tab.start[a.k_end - 1] + tab.len[a.k_end - 1];
  const int64_t s = first + (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (s >= last) return;
  int k = a.k_begin;
  while (k + 1 < a.k_end && s >= (int64_t)tab.start[k] + tab.len[k]) ++k;
  const float inv_bk = 1.0f / (float)tab.len[k];
  const TH* h = reinterpret_cast<const TH*>(a.h) + s * a.ldh;
  float part = 0.0f;
  for (int j = lane; j < a.width; j += 64) part = fmaf(to_f32(h[j]), a.w[j], part);
  const float z = wave_sum(part) + a.b[0];
  const float y = a.labels[s];
  const float e = expf(-fabsf(z));
  const float loss = fmaxf(z, 0.0f) - z * y + log1pf(e);
  const float sig = z >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
  const float dz = (sig - y) * inv_bk;
  if (lane == 0) {
    a.z[s] = z;
    a.loss_s[s] = loss;
    a.dz[s] = dz;
  }
  TD* dh = reinterpret_cast<TD*>(a.dh) + s * a.lddh;
  for (int j = lane; j < a.dh_cols; j += 64) {
    float g = dz * a.w[j];
    if (a.relu && !(to_f32(h[j]) > 0.0f)) g = 0.0f;
    dh[j] = from_f32<TD>(g);
  }
}

// bf16 variant working on a tile of `spb` samples staged in LDS, so that the gradient can be
// written both row-major (dh) and transposed (dht, sample index contiguous) with coalesced
// stores; same arithmetic as head_kernel.
constexpr int HEAD_LDS_ELEMS = 16448;  // largest tile: 32 x (512 + 2) bf16
// Shared memory is sized at the launch to the tile actually used (spb x (width + 2) bf16, the
// last-layer weights, spb floats), so that small widths leave room for many blocks per
// compute unit: the kernel is a chain of dependent global round trips and needs them in flight.
__host__ __device__ inline size_t head_tile_lds_bytes(int spb, int width) {
  return (((size_t)spb * (width + 2) * 2 + 15) & ~(size_t)15) + (size_t)width * 4 + 32 * 4;
}
__global__ __launch_bounds__(256) void head_tile_kernel(HeadArgs a, ShardTab tab, int spb) {
  extern __shared__ __attribute__((aligned(16))) char head_lds[];
  const int width = a.width, pitch = width + 2, vpr = width >> 3;
  bf16_t* tile = reinterpret_cast<bf16_t*>(head_lds);
  float* wl = reinterpret_cast<float*>(head_lds + (((size_t)spb * pitch * 2 + 15) & ~(size_t)15));  // last-layer weights
  float* dzs = wl + width;
  for (int j = threadIdx.x; j < width; j += 256) wl[j] = a.w[j];
  const int64_t first = tab.start[a.k_begin];
  const int64_t last = (int64_t)tab.start[a.k_end - 1] + tab.len[a.k_end - 1];
  const int64_t s0 = first + (int64_t)blockIdx.x * spb;
  const int rows = (int)min((int64_t)spb, last - s0);
  const bf16_t* h = reinterpret_cast<const bf16_t*>(a.h);
  for (int idx = threadIdx.x; idx < rows * vpr; idx += 256) {
    const int r = idx / vpr, c8 = idx - r * vpr;
    const uint4 v = *reinterpret_cast<const uint4*>(h + (s0 + r) * a.ldh + c8 * 8);
    uint32_t* d = reinterpret_cast<uint32_t*>(tile + r * pitch + c8 * 8);
    d[0] = v.x; d[1] = v.y; d[2] = v.z; d[3] = v.w;
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int r = wave; r < rows; r += 4) {  // logits of the tile, from LDS only
    float part = 0.0f;
    for (int j = lane; j < width; j += 64) part = fmaf(bf2f(tile[r * pitch + j]), wl[j], part);
    part = wave_sum(part);
    if (lane == 0) dzs[r] = part;
  }
  __syncthreads();
  if ((int)threadIdx.x < rows) {  // one thread per sample: loss and dz, their loads side by side
    const int r = threadIdx.x;
    const int64_t s = s0 + r;
    const float z = dzs[r] + a.b[0];
    int k = a.k_begin;
    while (k + 1 < a.k_end && s >= (int64_t)tab.start[k] + tab.len[k]) ++k;
    const float y = a.labels[s];
    const float e = expf(-fabsf(z));
    const float sig = z >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
    const float dz = (sig - y) * (1.0f / (float)tab.len[k]);
    a.z[s] = z;
    a.loss_s[s] = fmaxf(z, 0.0f) - z * y + log1pf(e);
    a.dz[s] = dz;
    dzs[r] = dz;
  }
  __syncthreads();
  bf16_t* dh = reinterpret_cast<bf16_t*>(a.dh);
  for (int idx = threadIdx.x; idx < rows * vpr; idx += 256) {
    const int r = idx / vpr, c8 = idx - r * vpr;
    const float dz = dzs[r];
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int j = c8 * 8 + 2 * q;
      const float g0 = bf2f(tile[r * pitch + j]) > 0.0f ? dz * wl[j] : 0.0f;
      const float g1 = bf2f(tile[r * pitch + j + 1]) > 0.0f ? dz * wl[j + 1] : 0.0f;
      o[q] = (uint32_t)f2bf(g0) | ((uint32_t)f2bf(g1) << 16);
    }
    *reinterpret_cast<uint4*>(dh + (s0 + r) * a.lddh + c8 * 8) = make_uint4(o[0], o[1], o[2], o[3]);
  }
  const int ls = threadIdx.x % spb, jj = threadIdx.x / spb, jstep = 256 / spb;
  if (ls < rows) {
    const float dz = dzs[ls];
    for (int j = jj; j < width; j += jstep) {
      const float g = bf2f(tile[ls * pitch + j]) > 0.0f ? dz * wl[j] : 0.0f;
      a.dht[(int64_t)j * a.ldt + s0 + ls] = f2bf(g);
    }
  }
}

// Block (64 columns x 4 sample lanes) of shard k = k_begin + blockIdx.y:
//   dW_last[j] = sum_s h[s, j] * dz[s];  block 0 also: db_last = sum_s dz[s], loss_k = mean loss.
template <typename TH>
__global__ __launch_bounds__(256) void head_reduce_kernel(HeadReduceArgs a, ShardTab tab) {
  __shared__ float red[4][64];
  const int k = a.k_begin + blockIdx.y;
  const int64_t s0 = tab.start[k];
  const int n = tab.len[k];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + tx;
  float* g = a.grads + (int64_t)k * a.P;
  float acc = 0.0f;
  if (j < a.width) {
    const TH* h = reinterpret_cast<const TH*>(a.h) + s0 * a.ldh + j;
    for (int s = ty; s < n; s += 4) acc = fmaf(to_f32(h[(int64_t)s * a.ldh]), a.dz[s0 + s], acc);
  }
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && j < a.width) g[a.w_off + j] = (red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]);
  if (blockIdx.x == 0) {
    __syncthreads();
    float sdz = 0.0f, sl = 0.0f;
    for (int s = threadIdx.x; s < n; s += 256) {
      sdz += a.dz[s0 + s];
      sl += a.loss_s[s0 + s];
    }
    sdz = wave_sum(sdz);
    sl = wave_sum(sl);
    if (tx == 0) {
      red[0][ty] = sdz;
      red[1][ty] = sl;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      g[a.b_off] = (red[0][0] + red[0][1]) + (red[0][2] + red[0][3]);
      const float lk = n > 0 ? ((red[1][0] + red[1][1]) + (red[1][2] + red[1][3])) / (float)n : 0.0f;
      a.loss_k[k] = lk;
      if (a.loss_out) a.loss_out[k - a.k_begin] = lk;
    }
  }
}

// The same reductions from the transposed activation hT[j][s]: one wavefront per (j, shard)
// reads a contiguous run of samples; wavefront `width` of a shard does db and the loss.
__global__ __launch_bounds__(256) void head_reduce_t_kernel(HeadReduceArgs a, ShardTab tab) {
  const int k = a.k_begin + blockIdx.y;
  const int64_t s0 = tab.start[k];
  const int n = tab.len[k];
  const int lane = threadIdx.x & 63;
  const int j = a.part == 2 ? a.width + (int)(threadIdx.x >> 6) : blockIdx.x * 4 + (int)(threadIdx.x >> 6);
  float* g = a.grads + (int64_t)k * a.P;
  if (j < a.width) {
    const bf16_t* h = a.ht + (int64_t)j * a.ldt + s0;
    float acc = 0.0f;
#pragma unroll 4
    for (int s = lane; s < n; s += 64) acc = fmaf(bf2f(h[s]), a.dz[s0 + s], acc);
    acc = wave_sum(acc);
    if (lane == 0) g[a.w_off + j] = acc;
  } else if (j == a.width && a.part != 1) {
    float sdz = 0.0f, sl = 0.0f;
#pragma unroll 4
    for (int s = lane; s < n; s += 64) {
      sdz += a.dz[s0 + s];
      sl += a.loss_s[s0 + s];
    }
    sdz = wave_sum(sdz);
    sl = wave_sum(sl);
    if (lane == 0) {
      g[a.b_off] = sdz;
      const float lk = n > 0 ? sl / (float)n : 0.0f;
      a.loss_k[k] = lk;
      if (a.loss_out) a.loss_out[k - a.k_begin] = lk;
    }
  }
}

// db[k][o] = sum over the samples of shard k of dh[s, o].
template <typename TD>
__global__ __launch_bounds__(256) void bias_grad_kernel(BiasGradArgs a, ShardTab tab) {
  __shared__ float red[4][64];
  const int k = a.k_begin + blockIdx.y;
  const int64_t s0 = tab.start[k];
  const int n = tab.len[k];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const int j = blockIdx.x * 64 + tx;
  float acc = 0.0f;
  if (j < a.width) {
    const TD* d = reinterpret_cast<const TD*>(a.dh) + s0 * a.lddh + j;
    int s = ty;
    for (; s + 12 < n; s += 16) {
      const float v0 = to_f32(d[(int64_t)s * a.lddh]), v1 = to_f32(d[(int64_t)(s + 4) * a.lddh]);
      const float v2 = to_f32(d[(int64_t)(s + 8) * a.lddh]), v3 = to_f32(d[(int64_t)(s + 12) * a.lddh]);
      acc += (v0 + v1) + (v2 + v3);
    }
    for (; s < n; s += 4) acc += to_f32(d[(int64_t)s * a.lddh]);
  }
  red[ty][tx] = acc;
  __syncthreads();
  if (ty == 0 && j < a.width)
    a.grads[(int64_t)k * a.P + a.b_off + j] = (red[0][tx] + red[1][tx]) + (red[2][tx] + red[3][tx]);
}

}  // namespace

hipError_t launch_head(const HeadArgs& a, const ShardTab& tab, hipStream_t s) {
  const int64_t first = tab.start[a.k_begin];
  const int64_t last = (int64_t)tab.start[a.k_end - 1] + tab.len[a.k_end - 1];
  if (last <= first) return hipSuccess;
  dim3 grid((unsigned)((last - first + 3) / 4)), block(256);
  if (a.dht) {  // bf16 hidden activation with a transposed gradient copy: tile kernel
    int spb = 16;
    while (spb > 4 && spb * (a.width + 2) > HEAD_LDS_ELEMS) spb >>= 1;
    hipLaunchKernelGGL(head_tile_kernel, dim3((unsigned)((last - first + spb - 1) / spb)), block,
                       head_tile_lds_bytes(spb, a.width), s, a, tab, spb);
    return hipGetLastError();
  }
  if (a.bf16_h) {
    if (a.bf16_dh) hipLaunchKernelGGL((head_kernel<bf16_t, bf16_t>), grid, block, 0, s, a, tab);
    else hipLaunchKernelGGL((head_kernel<bf16_t, float>), grid, block, 0, s, a, tab);
  } else {
    hipLaunchKernelGGL((head_kernel<float, float>), grid, block, 0, s, a, tab);
  }
  return hipGetLastError();
}

hipError_t launch_head_reduce(const HeadReduceArgs& a, const ShardTab& tab, hipStream_t s) {
  if (a.ht) {
    const unsigned bx = a.part == 2 ? 1u : (unsigned)((a.width + (a.part == 1 ? 0 : 1) + 3) / 4);
    hipLaunchKernelGGL(head_reduce_t_kernel, dim3(bx, a.k_end - a.k_begin), dim3(256), 0, s, a, tab);
    return hipGetLastError();
  }
  dim3 grid((a.width + 63) / 64, a.k_end - a.k_begin), block(256);
  if (a.bf16_h) hipLaunchKernelGGL(head_reduce_kernel<bf16_t>, grid, block, 0, s, a, tab);
  else hipLaunchKernelGGL(head_reduce_kernel<float>, grid, block, 0, s, a, tab);
  return hipGetLastError();
}

hipError_t launch_bias_grad(const BiasGradArgs& a, const ShardTab& tab, hipStream_t s) {
  dim3 grid((a.width + 63) / 64, a.k_end - a.k_begin), block(256);
  if (a.bf16_dh) hipLaunchKernelGGL(bias_grad_kernel<bf16_t>, grid, block, 0, s, a, tab);
  else hipLaunchKernelGGL(bias_grad_kernel<float>, grid, block, 0, s, a, tab);
  return hipGetLastError();
}

}  // namespace antdt
