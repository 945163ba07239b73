// MLP matrix products of the worker step (forward, data gradient, weight gradient).
//   bf16 operands / fp32 accumulate: LDS-tiled kernel on the gfx950 matrix cores
//   (v_mfma_f32_32x32x16_bf16, 64-wide wavefronts; measured on MI355X it sustains ~2.2 PFLOP/s
//   where the 16x16x32 form stays near 1.3), every operand stored with the contraction
//   index contiguous so that an MFMA fragment is one 16-byte LDS read;
//   fp32: a plain LDS-tiled FMA kernel (small models, exactness checks).
#include "common.h"

namespace antdt {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int BK = 64;      // contraction depth of one LDS tile (four MFMA k-steps)
constexpr int PITCH = 72;   // bf16 elements per LDS row: 144 B puts the 16 rows of a fragment read
                            // on 16 distinct 16-byte bank groups

__device__ __forceinline__ float epilogue_value(const GemmArgs& p, int64_t m, int n, float acc) {
  if (p.epi == EPI_BIAS_RELU) return fmaxf(acc + p.bias[n], 0.0f);
  if (p.epi == EPI_RELU_MASK) {
    const float h = p.bf16_in ? bf2f(reinterpret_cast<const bf16_t*>(p.mask)[m * p.ldmask + n])
                              : reinterpret_cast<const float*>(p.mask)[m * p.ldmask + n];
    return h > 0.0f ? acc : 0.0f;
  }
  return acc;
}

// Branch-free: zero the elements of an 8-element bf16 vector starting at contraction index
// k that fall outside [ks, ke); `all` is 0 or ~0 and clears the whole vector.
__device__ __forceinline__ uint4 clip_k(uint4 v, int k, int ks, int ke, uint32_t all) {
  const int lo = ks - k, hi = ke - k;  // element e survives iff lo <= e < hi
  uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t m0 = (2 * e >= lo && 2 * e < hi) ? 0x0000FFFFu : 0u;
    const uint32_t m1 = (2 * e + 1 >= lo && 2 * e + 1 < hi) ? 0xFFFF0000u : 0u;
    w[e] &= (m0 | m1) & all;
  }
  return make_uint4(w[0], w[1], w[2], w[3]);
}

// Two packed bf16 values, each kept where the matching mask value is positive.
__device__ __forceinline__ uint32_t relu_mask2(uint32_t v, uint32_t mk) {
  const uint32_t lo = ((mk & 0x8000u) == 0 && (mk & 0x7FFFu) != 0) ? 0x0000FFFFu : 0u;
  const uint32_t hi = ((mk & 0x80000000u) == 0 && (mk & 0x7FFF0000u) != 0) ? 0xFFFF0000u : 0u;
  return v & (lo | hi);
}

// acc[i][j] += sum_{k in [ks, ke)} A[m*lda + k] * B[n*ldb + k] for the block tile at (m0, n0).
// Block tile (32*TM*WR) x (32*TN*WC): WR x WC wavefronts, each TM x TN MFMA tiles of 32x32.
// Global -> registers -> LDS with the next tile's loads in flight during the MFMAs.  CLIP: the
// range need not start or end on a multiple of 8 (a shard's samples): the elements of the first
// and last 16-byte vectors that lie outside it are zeroed.  On return every wavefront has
// passed the last barrier: the LDS tiles are free.
template <int TM, int TN, int WR, int WC, bool CLIP>
__device__ __forceinline__ void accumulate_k(const bf16_t* A, const bf16_t* B, int64_t lda, int64_t ldb, int M, int N,
                                             int m0, int n0, int ks, int ke, bf16_t* la, bf16_t* lb,
                                             f32x16 (&acc)[TM][TN]) {
  constexpr int THREADS = 64 * WR * WC;
  constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
  constexpr int VA = BM * BK / 8 / THREADS, VB = BN * BK / 8 / THREADS;  // 16-byte vectors per thread
  static_assert(VA >= 1 && VB >= 1 && VA * THREADS * 8 == BM * BK && VB * THREADS * 8 == BN * BK, "tile / thread count");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int fr = lane & 31, fg = lane >> 5;

  // Two register stages: while tile kt is multiplied out of LDS, tiles kt+1 and kt+2 are in
  // flight from L2/HBM (one block per compute unit leaves no other wavefront to hide that
  // latency behind).
  uint4 ra0[VA], rb0[VB], ra1[VA], rb1[VB];
  const int kfirst = ks & ~7;
  // Loads are unconditional (addresses clamped into the operand) so that all of a tile's
  // loads are issued back to back; rows / contraction slots outside the problem are zeroed
  // when the tile is moved to LDS.
  const int klast = (ke - 1) & ~7;
  auto load_tile = [&](int kt, uint4 (&ra)[VA], uint4 (&rb)[VB]) {
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + i * THREADS;
      const int row = min(m0 + (v >> 3), M - 1), k = min(kfirst + kt * BK + (v & 7) * 8, klast);
      ra[i] = *reinterpret_cast<const uint4*>(A + (int64_t)row * lda + k);
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + i * THREADS;
      const int row = min(n0 + (v >> 3), N - 1), k = min(kfirst + kt * BK + (v & 7) * 8, klast);
      rb[i] = *reinterpret_cast<const uint4*>(B + (int64_t)row * ldb + k);
    }
  };
  // straight-line code only: a branch here makes the compiler wait for every outstanding load
  auto fix = [&](uint4 val, bool row_ok, int k) -> uint4 {
    const uint32_t all = (row_ok && k < ke) ? 0xFFFFFFFFu : 0u;
    if (CLIP) return clip_k(val, k, ks, ke, all);
    return make_uint4(val.x & all, val.y & all, val.z & all, val.w & all);
  };
  auto store_tile = [&](int kt, const uint4 (&ra)[VA], const uint4 (&rb)[VB]) {
#pragma unroll
    for (int i = 0; i < VA; ++i) {
      const int v = tid + i * THREADS;
      const uint4 val = fix(ra[i], m0 + (v >> 3) < M, kfirst + kt * BK + (v & 7) * 8);
      *reinterpret_cast<uint4*>(la + (v >> 3) * PITCH + (v & 7) * 8) = val;
    }
#pragma unroll
    for (int i = 0; i < VB; ++i) {
      const int v = tid + i * THREADS;
      const uint4 val = fix(rb[i], n0 + (v >> 3) < N, kfirst + kt * BK + (v & 7) * 8);
      *reinterpret_cast<uint4*>(lb + (v >> 3) * PITCH + (v & 7) * 8) = val;
    }
  };
  auto multiply = [&]() {
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      // lane (fr, fg) supplies contraction slots fg*8 .. fg*8+7 of row fr of each 32-row tile
      bf16x8 af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
        af[i] = *reinterpret_cast<const bf16x8*>(la + (wr * (32 * TM) + i * 32 + fr) * PITCH + kk + fg * 8);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8*>(lb + (wc * (32 * TN) + j * 32 + fr) * PITCH + kk + fg * 8);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };

  // Slabs are processed in pairs and every load is issued unconditionally (addresses past
  // the end are clamped, the data is zeroed by `fix`): with conditional loads the compiler
  // cannot count outstanding loads and drains them all before each LDS store.
  const int nk = ke > kfirst ? (ke - kfirst + BK - 1) / BK : 0;
  if (nk > 0) {
    load_tile(0, ra0, rb0);
    load_tile(1, ra1, rb1);
  }
  for (int kt = 0; kt < nk; kt += 2) {
    store_tile(kt, ra0, rb0);
    __syncthreads();
    load_tile(kt + 2, ra0, rb0);
    multiply();
    __syncthreads();
    store_tile(kt + 1, ra1, rb1);
    __syncthreads();
    load_tile(kt + 3, ra1, rb1);
    multiply();
    __syncthreads();
  }
}

// C[m, n] = sum_{k in [ks, ke)} A[m*lda + k] * B[n*ldb + k], with the epilogue of GemmArgs.
// Blocks are numbered so that the blocks sharing an A row-panel run on the same XCD (L2).
template <int TM, int TN, int WR, int WC, bool GROUPED>
__global__ __launch_bounds__(64 * WR * WC) void gemm_bf16_kernel(GemmArgs p, ShardTab tab, int tiles_m, int tiles_n) {
  constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
  __shared__ __attribute__((aligned(16))) bf16_t lds[(BM + BN) * PITCH];
  bf16_t* la = lds;
  bf16_t* lb = lds + BM * PITCH;

  const bf16_t* A = reinterpret_cast<const bf16_t*>(p.A);
  const bf16_t* B = reinterpret_cast<const bf16_t*>(p.B);
  char* C = reinterpret_cast<char*>(p.C);
  int ks = 0, ke = p.K;
  if (GROUPED) {
    const int k = p.k0 + blockIdx.z;
    ks = tab.start[k];
    ke = ks + tab.len[k];
    C += (int64_t)k * p.group_stride * (p.bf16_out ? 2 : 4);
  }
  int pid = blockIdx.x;
  const int nblk = tiles_m * tiles_n;
  if ((nblk & 7) == 0) pid = (pid & 7) * (nblk >> 3) + (pid >> 3);
  const int m0 = (pid / tiles_n) * BM, n0 = (pid % tiles_n) * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int fr = lane & 31, fg = lane >> 5;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
  accumulate_k<TM, TN, WR, WC, GROUPED>(A, B, p.lda, p.ldb, p.M, p.N, m0, n0, ks, ke, la, lb, acc);

  // Epilogue.  In the D fragment lane (fr, fg) holds column fr and rows 8*(v/4) + 4*fg + v%4
  // (v = 0..15) of each 32x32 tile, which would mean 2-byte scattered stores.  Each wavefront instead stages its
  // tile in its own slice of the (now free) LDS and writes it out row by row in 16-byte
  // pieces; the ReLU mask is read the same way; the transposed copy is read back column-wise.
  constexpr int WM = 32 * TM, WN = 32 * TN;
  const int mw = m0 + wr * WM, nw = n0 + wc * WN;
  if (p.bf16_out) {
    // staged PTM tile rows at a time: the largest number whose slices (one per wavefront) fit the
    // operand buffer
    constexpr int SP = WN + 8;
    constexpr int CAP = (BM + BN) * PITCH / (WR * WC * 32 * SP);
    static_assert(CAP >= 1, "epilogue staging exceeds the operand buffer");
    constexpr int PTM = CAP < TM ? (TM % CAP == 0 ? CAP : 1) : TM, PM = 32 * PTM;
    bf16_t* st = lds + wave * (PM * SP);
    float bias[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = nw + j * 32 + fr;
      bias[j] = (p.epi == EPI_BIAS_RELU && n < p.N) ? p.bias[n] : 0.0f;
    }
    constexpr int CPR = WN / 8;    // 16-byte pieces per row
    constexpr int RPI = 64 / CPR;  // rows per wavefront instruction
    const int rr = lane / CPR, cc = (lane % CPR) * 8;
    bf16_t* Cb = reinterpret_cast<bf16_t*>(C);
#pragma unroll
    for (int ip = 0; ip < TM; ip += PTM) {
      if (ip) __syncthreads();
#pragma unroll
      for (int i = 0; i < PTM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float v = acc[ip + i][j][e];
            if (p.epi == EPI_BIAS_RELU) v = fmaxf(v + bias[j], 0.0f);
            st[(i * 32 + 8 * (e >> 2) + 4 * fg + (e & 3)) * SP + j * 32 + fr] = f2bf(v);
          }
      __syncthreads();
      const int mp = mw + ip * 32;  // first row of this pass
#pragma unroll
      for (int r0 = 0; r0 < PM; r0 += RPI) {
        const int r = r0 + rr, m = mp + r, n = nw + cc;
        if (m < p.M && n < p.N) {
          uint4 val = *reinterpret_cast<const uint4*>(st + r * SP + cc);
          if (p.epi == EPI_RELU_MASK) {
            const uint4 mk = *reinterpret_cast<const uint4*>(reinterpret_cast<const bf16_t*>(p.mask) + (int64_t)m * p.ldmask + n);
            val = make_uint4(relu_mask2(val.x, mk.x), relu_mask2(val.y, mk.y), relu_mask2(val.z, mk.z), relu_mask2(val.w, mk.w));
            if (p.CT) *reinterpret_cast<uint4*>(st + r * SP + cc) = val;
          }
          *reinterpret_cast<uint4*>(Cb + (int64_t)m * p.ldc + n) = val;
        }
      }
      if (p.CT) {
        __syncthreads();
        constexpr int CPI = WN < 64 ? WN : 64;  // columns per wavefront instruction
        constexpr int HV = 64 / CPI;
        const int col = lane % CPI, hv = lane / CPI;
        const int n = nw + col;
        // Groups of eight rows that start where the destination (sample index ct_col0 + row) is a
        // multiple of eight, so that a full group is one aligned 16-byte store whatever sample
        // the shard starts at; the rows before the first such boundary and past the last row of
        // the matrix go out element by element.
        const int lead = (int)((8 - ((p.ct_col0 + mp) & 7)) & 7);  // rows before the first boundary
        for (int mc = hv; mc <= PM / 8; mc += HV) {
          const int r0 = lead + (mc - 1) * 8;                     // first staged row of the group (may be < 0)
          if (n < p.N && r0 < PM && r0 + 8 > 0) {
            bf16_t h[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h[e] = st[min(max(r0 + e, 0), PM - 1) * SP + col];
            bf16_t* dst = p.CT + (int64_t)n * p.ldct + p.ct_col0 + mp + r0;
            if (r0 >= 0 && r0 + 8 <= PM && mp + r0 + 7 < p.M) {
              *reinterpret_cast<uint4*>(dst) = make_uint4((uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16),
                                                          (uint32_t)h[4] | ((uint32_t)h[5] << 16), (uint32_t)h[6] | ((uint32_t)h[7] << 16));
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (r0 + e >= 0 && r0 + e < PM && mp + r0 + e < p.M) dst[e] = h[e];
            }
          }
        }
      }
    }
  } else {
    constexpr int SPF = WN + 4;
    // rows staged per pass: one MFMA tile row, or half of one where eight wavefronts share the buffer
    constexpr int ROWS = (WR * WC * 32 * SPF * 4 <= (BM + BN) * PITCH * 2) ? 32 : 16;
    static_assert(WR * WC * ROWS * SPF * 4 <= (BM + BN) * PITCH * 2, "epilogue staging exceeds the operand buffer");
    float* stf = reinterpret_cast<float*>(lds) + wave * (ROWS * SPF);
    constexpr int CPR = WN / 4;
    constexpr int RPI = 64 / CPR;
    const int rr = lane / CPR, cc = (lane % CPR) * 4;
    float* Cf = reinterpret_cast<float*>(C);
#pragma unroll
    for (int pass = 0; pass < WM / ROWS; ++pass) {
      if (pass) __syncthreads();
      // a D fragment's element e sits in row 8*(e/4) + 4*fg + e%4 of its 32-row tile: elements
      // 0..7 are the upper 16 rows, 8..15 the lower
      constexpr int EPP = ROWS / 2;               // fragment elements per pass
      const int tile = pass * ROWS / 32, e0 = (pass * ROWS % 32) / 2;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < EPP; ++e)
          stf[(8 * (e >> 2) + 4 * fg + (e & 3)) * SPF + j * 32 + fr] = acc[tile][j][e0 + e];
      __syncthreads();
#pragma unroll
      for (int r0 = 0; r0 < ROWS; r0 += RPI) {
        const int r = r0 + rr, m = mw + pass * ROWS + r, n = nw + cc;
        if (m < p.M && n < p.N) {
          const float4 val = *reinterpret_cast<const float4*>(stf + r * SPF + cc);
          float* dst = Cf + (int64_t)m * p.ldc + n;
          if (n + 3 < p.N && (reinterpret_cast<uintptr_t>(dst) & 15) == 0) {
            *reinterpret_cast<float4*>(dst) = val;
          } else {
            dst[0] = val.x;
            if (n + 1 < p.N) dst[1] = val.y;
            if (n + 2 < p.N) dst[2] = val.z;
            if (n + 3 < p.N) dst[3] = val.w;
          }
        }
      }
    }
  }
}

// Weight gradient + aggregation + dense Adagrad of one tile (see WgradUpdateArgs).  The sums of
// the sample ranges are formed one after the other, each from zero, and added up with their
// weights in range order: g = fma(w_k, sum_k, g), the order in which the stand-alone dense
// update adds the shards' gradients.
// ONE: a single sample range (all shards of one weight, one after the other): its sum is scaled in
// place, fma(w, sum, 0) = w * sum, and the second set of accumulators is not needed (fewer registers:
// three wavefronts per SIMD instead of two, which leaves more room for the kernels running beside it).
template <int TM, int TN, int WR, int WC, bool ONE>
__global__ __launch_bounds__(64 * WR * WC) void wgrad_update_kernel(WgradUpdateArgs u, KSegments seg) {
  constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
  __shared__ __attribute__((aligned(16))) bf16_t lds[(BM + BN) * PITCH];
  bf16_t* la = lds;
  bf16_t* lb = lds + BM * PITCH;
  int li = 0;
  while (li + 1 < u.n_layers && (int)blockIdx.x >= u.tile_base[li + 1]) ++li;
  const int pid = blockIdx.x - u.tile_base[li];
  const int M = u.M[li], N = u.N[li];
  const int m0 = (pid / u.tiles_n[li]) * BM, n0 = (pid % u.tiles_n[li]) * BN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wr = wave / WC, wc = wave % WC;
  const int fr = lane & 31, fg = lane >> 5;

  f32x16 tot[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) tot[i][j][e] = 0.0f;
  if (ONE) {
    accumulate_k<TM, TN, WR, WC, true>(u.A[li], u.B[li], u.ld, u.ld, M, N, m0, n0, seg.ks[0], seg.ke[0], la, lb, tot);
    const float w = seg.w[0];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) tot[i][j][e] = fmaf(w, tot[i][j][e], 0.0f);
  } else {
    for (int q = 0; q < seg.n; ++q) {
      f32x16 acc[TM][TN];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.0f;
      accumulate_k<TM, TN, WR, WC, true>(u.A[li], u.B[li], u.ld, u.ld, M, N, m0, n0, seg.ks[q], seg.ke[q], la, lb, acc);
      const float w = seg.w[q];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int e = 0; e < 16; ++e) tot[i][j][e] = fmaf(w, acc[i][j][e], tot[i][j][e]);
    }
  }

  // Epilogue: each wavefront stages its tile through its own slice of the (free) LDS, a band of
  // rows at a time, so that a lane ends up with four consecutive columns of one row: 16-byte
  // loads of the parameters and their accumulators, the Adagrad step, 16-byte stores, and the
  // bf16 copy of the new weights (not of the bias row).
  constexpr int WM = 32 * TM, WN = 32 * TN;
  const int mw = m0 + wr * WM, nw = n0 + wc * WN;
  constexpr int SPF = WN + 4;
  constexpr int ROWS = (WR * WC * 32 * SPF * 4 <= (BM + BN) * PITCH * 2) ? 32 : 16;
  static_assert(WR * WC * ROWS * SPF * 4 <= (BM + BN) * PITCH * 2, "epilogue staging exceeds the operand buffer");
  float* stf = reinterpret_cast<float*>(lds) + wave * (ROWS * SPF);
  constexpr int CPR = WN / 4;
  constexpr int RPI = 64 / CPR;
  const int rr = lane / CPR, cc = (lane % CPR) * 4;
  float* P = u.p + u.w_off[li];
  float* S = u.state + u.w_off[li];
  bf16_t* Wb = u.wb[li];
#pragma unroll
  for (int pass = 0; pass < WM / ROWS; ++pass) {
    if (pass) __syncthreads();
    constexpr int EPP = ROWS / 2;               // fragment elements per pass
    const int tile = pass * ROWS / 32, e0 = (pass * ROWS % 32) / 2;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < EPP; ++e)
        stf[(8 * (e >> 2) + 4 * fg + (e & 3)) * SPF + j * 32 + fr] = tot[tile][j][e0 + e];
    __syncthreads();
#pragma unroll
    for (int r0 = 0; r0 < ROWS; r0 += RPI) {
      const int r = r0 + rr, m = mw + pass * ROWS + r, n = nw + cc;
      if (m < M && n < N) {   // (N is a multiple of 8: the four columns are inside together)
        const float4 g = *reinterpret_cast<const float4*>(stf + r * SPF + cc);
        const int64_t idx = (int64_t)m * N + n;
        const float4 p0 = *reinterpret_cast<const float4*>(P + idx);
        float4 s1 = *reinterpret_cast<const float4*>(S + idx);
        s1.x = fmaf(g.x, g.x, s1.x); s1.y = fmaf(g.y, g.y, s1.y);
        s1.z = fmaf(g.z, g.z, s1.z); s1.w = fmaf(g.w, g.w, s1.w);
        float4 p1;
        p1.x = p0.x - u.lr * g.x / (sqrtf(s1.x) + u.eps);
        p1.y = p0.y - u.lr * g.y / (sqrtf(s1.y) + u.eps);
        p1.z = p0.z - u.lr * g.z / (sqrtf(s1.z) + u.eps);
        p1.w = p0.w - u.lr * g.w / (sqrtf(s1.w) + u.eps);
        *reinterpret_cast<float4*>(S + idx) = s1;
        *reinterpret_cast<float4*>(P + idx) = p1;
        if (m < M - 1)
          *reinterpret_cast<uint2*>(Wb + idx) = make_uint2((uint32_t)f2bf(p1.x) | ((uint32_t)f2bf(p1.y) << 16),
                                                           (uint32_t)f2bf(p1.z) | ((uint32_t)f2bf(p1.w) << 16));
      }
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
      if (m < p.M && n < p.N) reinterpret_cast<float*>(C)[(int64_t)m * p.ldc + n] = epilogue_value(p, m, n, acc[i][j]);
    }
}

__global__ __launch_bounds__(256) void cast_bf16_kernel(CastArgs a) {
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < a.n_dst; i += stride)
    a.dst[i] = i < a.n_src ? f2bf(a.src[i]) : (bf16_t)0;
}

// 64x64 bf16 tiles transposed through LDS; one launch covers several matrices.
__global__ __launch_bounds__(256) void transpose_bf16_kernel(TransposeArgs a) {
  __shared__ bf16_t tile[64][66];
  int mi = 0;
  while (mi + 1 < a.n && (int)blockIdx.x >= a.tile_base[mi + 1]) ++mi;
  const int t = blockIdx.x - a.tile_base[mi];
  const int tc = (a.cols[mi] + 63) / 64;
  const int r0 = (t / tc) * 64, c0 = (t % tc) * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int r = ty; r < 64; r += 4)
    tile[r][tx] = (r0 + r < a.rows[mi] && c0 + tx < a.cols[mi]) ? a.src[mi][(int64_t)(r0 + r) * a.ld_src[mi] + c0 + tx]
                                                              : (bf16_t)0;
  __syncthreads();
  for (int cidx = ty; cidx < 64; cidx += 4)
    if (c0 + cidx < a.cols[mi] && r0 + tx < a.rows[mi])
      a.dst[mi][(int64_t)(c0 + cidx) * a.ld_dst[mi] + r0 + tx] = tile[tx][cidx];
}

__global__ __launch_bounds__(256) void ones_row_kernel(OnesRowArgs a) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.ld) return;
  a.base[(int64_t)a.row * a.ld + i] = 0x3F80;  // 1.0
  for (int r = 1; r <= a.zero_rows; ++r) a.base[(int64_t)(a.row + r) * a.ld + i] = 0;
}

template <int TM, int TN, int WR, int WC>
void launch_bf16_variant(const GemmArgs& a, const ShardTab& tab, int groups, hipStream_t s) {
  constexpr int BM = 32 * TM * WR, BN = 32 * TN * WC;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  dim3 grid(tiles_m * tiles_n, 1, groups), block(64 * WR * WC);
  if (a.grouped) hipLaunchKernelGGL((gemm_bf16_kernel<TM, TN, WR, WC, true>), grid, block, 0, s, a, tab, tiles_m, tiles_n);
  else hipLaunchKernelGGL((gemm_bf16_kernel<TM, TN, WR, WC, false>), grid, block, 0, s, a, tab, tiles_m, tiles_n);
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
  // The largest tile that still gives the 256 compute units more than one block each.  A
  // 128 x 128 tile moves the fewest operand bytes per compute unit and is fastest for a product
  // running alone with one block per unit, but inside the iteration (three streams sharing the
  // device) two resident blocks of 128 x 64 hide each other's load latency, barriers and
  // epilogue: measured 294 against 305 us per step with the threshold at 300 instead of 200.
  constexpr int64_t MIN_BLOCKS = 300;
  auto blocks = [&](int bm, int bn) { return (int64_t)((a.M + bm - 1) / bm) * ((a.N + bn - 1) / bn) * groups; };
  // Eight wavefronts on a 256 x 128 tile (a quarter fewer operand bytes per compute unit than
  // 128 x 128) pay off only where there are blocks enough that the last, partly filled round
  // of blocks does not matter: measured -5 % on a step whose products have thousands of
  // blocks, +1 % where they have about five hundred.
  if (blocks(256, 128) >= 4 * 256) launch_bf16_variant<2, 2, 4, 2>(a, tab, groups, s);
  else if (blocks(128, 128) >= MIN_BLOCKS) launch_bf16_variant<2, 2, 2, 2>(a, tab, groups, s);
  else if (blocks(128, 64) >= MIN_BLOCKS) launch_bf16_variant<2, 1, 2, 2>(a, tab, groups, s);
  else launch_bf16_variant<1, 1, 2, 2>(a, tab, groups, s);
  return hipGetLastError();
}

hipError_t launch_wgrad_update(const WgradUpdateArgs& a, const KSegments& seg, hipStream_t s) {
  // The largest tile that still gives about two hundred blocks: every block walks the whole batch,
  // so a large tile means few operand bytes per output but also few blocks, each pulling its
  // operands at the rate of one compute unit.  (Config-2 model at 4096 samples, running beside the
  // sparse update: 128 x 128 / 128 x 64 / 64 x 64 tiles = 102 / 204 / 396 blocks took 126 / 115 /
  // 107 us, the step 256.1 / 255.0 / 254.8 us; alone 78 / 55 / 48 us.)
  auto blocks_of = [&](int bm, int bn) {
    int n = 0;
    for (int l = 0; l < a.n_layers; ++l) n += ((a.M[l] + bm - 1) / bm) * ((a.N[l] + bn - 1) / bn);
    return n;
  };
  const int tv = blocks_of(128, 128) >= 200 ? 0 : blocks_of(128, 64) >= 200 ? 1 : 2;
  const int BM = tv == 2 ? 64 : 128, BN = tv == 0 ? 128 : 64;
  WgradUpdateArgs u = a;
  u.tile_base[0] = 0;
  for (int l = 0; l < u.n_layers; ++l) {
    if (u.M[l] <= 0 || u.N[l] <= 0 || (u.N[l] & 7)) return hipErrorInvalidValue;
    u.tiles_n[l] = (u.N[l] + BN - 1) / BN;
    u.tile_base[l + 1] = u.tile_base[l] + ((u.M[l] + BM - 1) / BM) * u.tiles_n[l];
  }
  const int blocks = u.tile_base[u.n_layers];
  if (blocks <= 0) return hipSuccess;
  const bool one = seg.n == 1;
  if (tv == 0 && one) hipLaunchKernelGGL((wgrad_update_kernel<2, 2, 2, 2, true>), dim3(blocks), dim3(256), 0, s, u, seg);
  else if (tv == 0) hipLaunchKernelGGL((wgrad_update_kernel<2, 2, 2, 2, false>), dim3(blocks), dim3(256), 0, s, u, seg);
  else if (tv == 1 && one) hipLaunchKernelGGL((wgrad_update_kernel<2, 1, 2, 2, true>), dim3(blocks), dim3(256), 0, s, u, seg);
  else if (tv == 1) hipLaunchKernelGGL((wgrad_update_kernel<2, 1, 2, 2, false>), dim3(blocks), dim3(256), 0, s, u, seg);
  else if (one) hipLaunchKernelGGL((wgrad_update_kernel<1, 1, 2, 2, true>), dim3(blocks), dim3(256), 0, s, u, seg);
  else hipLaunchKernelGGL((wgrad_update_kernel<1, 1, 2, 2, false>), dim3(blocks), dim3(256), 0, s, u, seg);
  return hipGetLastError();
}

hipError_t launch_cast_bf16(const CastArgs& a, hipStream_t s) {
  if (a.n_dst <= 0) return hipSuccess;
  int64_t blocks = (a.n_dst + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(cast_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16(const TransposeArgs& a, hipStream_t s) {
  if (a.n <= 0 || a.tile_base[a.n] <= 0) return hipSuccess;
  hipLaunchKernelGGL(transpose_bf16_kernel, dim3(a.tile_base[a.n]), dim3(256), 0, s, a);
  return hipGetLastError();
}

hipError_t launch_ones_row(const OnesRowArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(ones_row_kernel, dim3((unsigned)((a.ld + 255) / 256)), dim3(256), 0, s, a);
  return hipGetLastError();
}

}  // namespace antdt
