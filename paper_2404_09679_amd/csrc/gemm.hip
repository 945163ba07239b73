// MLP matrix products of the worker step (forward, data gradient, weight gradient).
//   bf16 operands / fp32 accumulate: LDS-tiled kernel on the gfx950 matrix cores
//   (v_mfma_f32_16x16x32_bf16, 64-wide wavefronts);
//   fp32: a plain LDS-tiled FMA kernel (small models, exactness checks).
#include "common.h"

namespace antdt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int BK = 32;          // contraction depth of one LDS tile = one MFMA
constexpr int PITCH_KC = 40;    // bf16 elements per row of a [rows][BK] tile (80 B, 16-byte aligned)
constexpr int PITCH_NK = 132;   // bf16 elements per row of a [BK][cols<=128] tile (264 B, 8-byte aligned)

__device__ __forceinline__ float epilogue_mask(const GemmArgs& p, int64_t m, int n) {
  if (p.bf16_in) return bf2f(reinterpret_cast<const bf16_t*>(p.mask)[m * p.ldmask + n]);
  return reinterpret_cast<const float*>(p.mask)[m * p.ldmask + n];
}

__device__ __forceinline__ void epilogue_store(const GemmArgs& p, void* Cbase, int64_t m, int n, float acc) {
  float v = acc;
  if (p.epi == EPI_BIAS_RELU) v = fmaxf(acc + p.bias[n], 0.0f);
  else if (p.epi == EPI_RELU_MASK) v = epilogue_mask(p, m, n) > 0.0f ? acc : 0.0f;
  if (p.bf16_out) reinterpret_cast<bf16_t*>(Cbase)[m * p.ldc + n] = f2bf(v);
  else reinterpret_cast<float*>(Cbase)[m * p.ldc + n] = v;
}

// Block tile (32*TM) x (32*TN), 4 wavefronts in a 2x2 arrangement, each owning
// TM x TN MFMA tiles of 16x16.  Operand tiles go global -> registers -> LDS
// (double buffered, one barrier per K step).  An operand whose contraction
// index is contiguous in memory is kept as [row][k] and read back with one
// 16-byte LDS load per fragment; the other kind is kept as [k][col] and its
// fragment is gathered with eight 2-byte LDS loads.
template <int TM, int TN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_mfma_kernel(GemmArgs p, ShardTab tab) {
  constexpr int BM = 32 * TM, BN = 32 * TN;
  constexpr int A_ELEMS = A_KC ? BM * PITCH_KC : BK * PITCH_NK;
  constexpr int B_ELEMS = B_KC ? BN * PITCH_KC : BK * PITCH_NK;
  __shared__ __attribute__((aligned(16))) bf16_t lds[2 * (A_ELEMS + B_ELEMS)];

  const bf16_t* A = reinterpret_cast<const bf16_t*>(p.A);
  const bf16_t* B = reinterpret_cast<const bf16_t*>(p.B);
  char* C = reinterpret_cast<char*>(p.C);
  int K = p.K;
  if (p.grouped) {
    const int k = p.k0 + blockIdx.z;
    const int64_t r0 = tab.start[k];
    K = tab.len[k];
    A += r0 * p.lda;
    B += r0 * p.ldb;
    C += (int64_t)k * p.group_stride * (p.bf16_out ? 2 : 4);
  }
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave >> 1, wc = wave & 1;
  const int fr = lane & 15, fg = lane >> 4;

  constexpr int VA = BM * BK / 8 / 256;  // 16-byte vectors per thread for the A tile
  constexpr int VB = BN * BK / 8 / 256;
  uint4 ra[VA], rb[VB];

  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + i * 256;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (A_KC) {
        const int row = v >> 2, kc = (v & 3) * 8;
        if (m0 + row < p.M && k0 + kc < K) val = *reinterpret_cast<const uint4*>(A + (int64_t)(m0 + row) * p.lda + k0 + kc);
      } else {
        constexpr int CPR = BM / 8;  // vectors per k row
        const int kk = v / CPR, cc = (v % CPR) * 8;
        if (k0 + kk < K && m0 + cc < p.M) val = *reinterpret_cast<const uint4*>(A + (int64_t)(k0 + kk) * p.lda + m0 + cc);
      }
      ra[i] = val;
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + i * 256;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (B_KC) {
        const int row = v >> 2, kc = (v & 3) * 8;
        if (n0 + row < p.N && k0 + kc < K) val = *reinterpret_cast<const uint4*>(B + (int64_t)(n0 + row) * p.ldb + k0 + kc);
      } else {
        constexpr int CPR = BN / 8;
        const int kk = v / CPR, cc = (v % CPR) * 8;
        if (k0 + kk < K && n0 + cc < p.N) val = *reinterpret_cast<const uint4*>(B + (int64_t)(k0 + kk) * p.ldb + n0 + cc);
      }
      rb[i] = val;
    }
  };
  auto store_tile = [&](int buf) {
    bf16_t* la = lds + buf * (A_ELEMS + B_ELEMS);
    bf16_t* lb = la + A_ELEMS;
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + i * 256;
      if (A_KC) {
        const int row = v >> 2, kc = (v & 3) * 8;
        *reinterpret_cast<uint4*>(la + row * PITCH_KC + kc) = ra[i];
      } else {
        constexpr int CPR = BM / 8;
        const int kk = v / CPR, cc = (v % CPR) * 8;
        uint2* d = reinterpret_cast<uint2*>(la + kk * PITCH_NK + cc);
        d[0] = make_uint2(ra[i].x, ra[i].y);
        d[1] = make_uint2(ra[i].z, ra[i].w);
      }
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + i * 256;
      if (B_KC) {
        const int row = v >> 2, kc = (v & 3) * 8;
        *reinterpret_cast<uint4*>(lb + row * PITCH_KC + kc) = rb[i];
      } else {
        constexpr int CPR = BN / 8;
        const int kk = v / CPR, cc = (v % CPR) * 8;
        uint2* d = reinterpret_cast<uint2*>(lb + kk * PITCH_NK + cc);
        d[0] = make_uint2(rb[i].x, rb[i].y);
        d[1] = make_uint2(rb[i].z, rb[i].w);
      }
    }
  };
  // Fragment of a 16-row MFMA tile starting at tile row `r0`: lane (fr, fg) supplies the
  // 8 contraction slots fg*8 .. fg*8+7 of row r0 + fr.
  auto frag = [&](const bf16_t* base, bool kc, int r0) -> bf16x8 {
    union { uint4 u; bf16x8 v; uint16_t h[8]; } x;
    if (kc) {
      x.u = *reinterpret_cast<const uint4*>(base + (r0 + fr) * PITCH_KC + fg * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) x.h[e] = base[(fg * 8 + e) * PITCH_NK + r0 + fr];
    }
    return x.v;
  };

  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nk = (K + BK - 1) / BK;
  if (nk > 0) {
    load_tile(0);
    store_tile(0);
  }
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) load_tile((kt + 1) * BK);
    const bf16_t* la = lds + buf * (A_ELEMS + B_ELEMS);
    const bf16_t* lb = la + A_ELEMS;
    bf16x8 af[TM], bfr[TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) af[i] = frag(la, A_KC, wr * (BM / 2) + i * 16);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[j] = frag(lb, B_KC, wc * (BN / 2) + j * 16);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    if (kt + 1 < nk) store_tile(buf ^ 1);
    __syncthreads();
  }

  // D fragment: lane (fr, fg) holds column fr and rows fg*4 .. fg*4+3 of each 16x16 tile.
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wc * (BN / 2) + j * 16 + fr;
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int m = m0 + wr * (BM / 2) + i * 16 + fg * 4 + v;
        if (m < p.M && n < p.N) epilogue_store(p, C, m, n, acc[i][j][v]);
      }
    }
}

// fp32 tiled FMA kernel with arbitrary operand orientation: 64x64 block tile, 4x4 per thread.
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmArgs p, ShardTab tab) {
  constexpr int T = 64, KT = 16;
  __shared__ float As[KT][T + 4];
  __shared__ float Bs[KT][T + 4];
  const float* A = reinterpret_cast<const float*>(p.A);
  const float* B = reinterpret_cast<const float*>(p.B);
  char* C = reinterpret_cast<char*>(p.C);
  int K = p.K;
  if (p.grouped) {
    const int k = p.k0 + blockIdx.z;
    const int64_t r0 = tab.start[k];
    K = tab.len[k];
    A += r0 * p.lda;
    B += r0 * p.ldb;
    C += (int64_t)k * p.group_stride * 4;
  }
  const int64_t sAm = p.a_kc ? p.lda : 1, sAk = p.a_kc ? 1 : p.lda;
  const int64_t sBn = p.b_kc ? p.ldb : 1, sBk = p.b_kc ? 1 : p.ldb;
  const int m0 = blockIdx.y * T, n0 = blockIdx.x * T;
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += KT) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int e = tid + i * 256;
      // contiguous index runs fastest across threads for either orientation
      const int kk = p.a_kc ? (e & 15) : (e >> 6), mm = p.a_kc ? (e >> 4) : (e & 63);
      As[kk][mm] = (m0 + mm < p.M && k0 + kk < K) ? A[(int64_t)(m0 + mm) * sAm + (int64_t)(k0 + kk) * sAk] : 0.0f;
      const int kb = p.b_kc ? (e & 15) : (e >> 6), nn = p.b_kc ? (e >> 4) : (e & 63);
      Bs[kb][nn] = (n0 + nn < p.N && k0 + kb < K) ? B[(int64_t)(n0 + nn) * sBn + (int64_t)(k0 + kb) * sBk] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KT; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < p.M && n < p.N) epilogue_store(p, C, m, n, acc[i][j]);
    }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(CastArgs a) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n_dst; i += stride)
    a.dst[i] = i < a.n_src ? f2bf(a.src[i]) : (bf16_t)0;
}

template <int TM, int TN>
void launch_mfma_variant(const GemmArgs& a, const ShardTab& tab, dim3 grid, hipStream_t s) {
  dim3 block(256);
  if (a.a_kc && a.b_kc) hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, true, true>), grid, block, 0, s, a, tab);
  else if (a.a_kc && !a.b_kc) hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, true, false>), grid, block, 0, s, a, tab);
  else if (!a.a_kc && !a.b_kc) hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, false, false>), grid, block, 0, s, a, tab);
  else hipLaunchKernelGGL((gemm_mfma_kernel<TM, TN, false, true>), grid, block, 0, s, a, tab);
}

}  // namespace

hipError_t launch_gemm(const GemmArgs& a, const ShardTab& tab, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  const int groups = a.grouped ? a.groups : 1;
  if (groups <= 0) return hipSuccess;
  if (!a.bf16_in) {
    dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, groups);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, s, a, tab);
    return hipGetLastError();
  }
  // Large tiles when they still give the 256 compute units enough blocks, else 64x64.
  const int64_t big = (int64_t)((a.N + 127) / 128) * ((a.M + 127) / 128) * groups;
  if (big >= 192) {
    dim3 grid((a.N + 127) / 128, (a.M + 127) / 128, groups);
    launch_mfma_variant<4, 4>(a, tab, grid, s);
  } else {
    dim3 grid((a.N + 63) / 64, (a.M + 63) / 64, groups);
    launch_mfma_variant<2, 2>(a, tab, grid, s);
  }
  return hipGetLastError();
}

hipError_t launch_cast_bf16(const CastArgs& a, hipStream_t s) {
  if (a.n_dst <= 0) return hipSuccess;
  int64_t blocks = (a.n_dst + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace antdt
