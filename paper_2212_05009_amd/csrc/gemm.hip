// Dense contractions of the GCN layer on the gfx950 matrix cores (fp32 MFMA 32x32x2):
//   gemm_nn : C[M x N] = A[M x K] B[K x N]   tall-skinny "features times weights"
//             (Sec. 3.1: the dense product with W^k after the sparse aggregation), with fused
//             bias / ReLU / ReLU-derivative-mask epilogues,
//   gemm_tn : C[M x N] = A[Kd x M]^T B[Kd x N] with a huge reduction length Kd = number of rows
//             (Sec. 3.1 third equation: the weight gradient), split over the grid, partial
//             tiles summed in a fixed order.
// A 256-thread block (4 wavefronts) owns a 128 x BN output tile and walks K in steps of 32,
// staging both operand tiles in LDS (double buffered); each wavefront keeps a grid of 32x32
// MFMA accumulator tiles in registers.
#include <stdlib.h>

#include "common.h"

namespace gcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));


constexpr int BM = 128;    // output rows per block (NN) / A-columns per block (TN)
constexpr int BK = 16;     // reduction step
constexpr int APAD = 1;    // As row-major [BM][BK + APAD]: bank-conflict-free MFMA operand reads
constexpr int BPAD = 4;    // Bs [BK][BN + BPAD]

// 4 consecutive elements of a row, starting at column c (multiple of 4), zero beyond `limit`.
// vec = widest aligned vector width usable on this operand (4, 2 or 1), uniform per launch.
template <typename T>
__device__ __forceinline__ void load4(const T* __restrict__ row, int64_t c, int64_t limit, int vec, float (&o)[4]) {
  if constexpr (sizeof(T) == 4) {
    if (vec == 4 && c + 3 < limit) {
      float4 v = *reinterpret_cast<const float4*>(row + c);
      o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
      return;
    }
    if (vec >= 2 && c + 3 < limit) {
      float2 v0 = *reinterpret_cast<const float2*>(row + c);
      float2 v1 = *reinterpret_cast<const float2*>(row + c + 2);
      o[0] = v0.x; o[1] = v0.y; o[2] = v1.x; o[3] = v1.y;
      return;
    }
  } else {
    if (vec == 4 && c + 3 < limit) {
      uint2 v = *reinterpret_cast<const uint2*>(row + c);
      o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
      o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
      return;
    }
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (c + i < limit) ? load_one<T>(row + c + i) : 0.f;
}

// 4 consecutive elements from a 16-byte (fp32) / 8-byte (bf16) aligned address, no bounds checks
template <typename T>
__device__ __forceinline__ void load4_fast(const T* __restrict__ p, float (&o)[4]) {
  if constexpr (sizeof(T) == 4) {
    float4 v = *reinterpret_cast<const float4*>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  } else {
    uint2 v = *reinterpret_cast<const uint2*>(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
  }
}

struct NnArgs {
  const void* A; int64_t lda; const float* B; int64_t ldb; void* C; int64_t ldc;
  int64_t M; int N; int K; int vecA; int vecB;
  const float* bias; int relu; const void* mask; int64_t ldmask; int64_t mask_rows; void* C2; int64_t ldc2;
};

// WAVES_M x WAVES_N wavefronts; each owns TM x TN accumulator tiles of 32 x 32
template <typename T, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_gemm_nn(NnArgs a) {
  static_assert(WAVES_M * WAVES_N == 4, "4 wavefronts per block");
  constexpr int TM = BM / WAVES_M / 32, TN = BN / WAVES_N / 32;
  constexpr int LDA_S = BK + APAD, LDB_S = BN + BPAD;
  constexpr int A_IT = BM * BK / 4 / 256;            // float4 groups per thread for the A tile
  constexpr int B_IT = (BK * BN / 4 + 255) / 256;    // ... for the B tile
  __shared__ float As[2][BM * LDA_S];
  __shared__ float Bs[2][BK * LDB_S];

  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wm = w / WAVES_N, wn = w % WAVES_N;
  const int64_t m0 = (int64_t)blockIdx.x * BM;
  const int n0 = blockIdx.y * BN;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float ra[A_IT][4], rb[B_IT][4];
  // interior tiles of aligned operands take plain 16-byte loads; edges go element by element
  const bool a_in = a.vecA == 4 && m0 + BM <= a.M;
  const bool b_in = a.vecB == 4 && n0 + BN <= a.N;
  auto fetch = [&](int k0) {
    const bool k_in = k0 + BK <= a.K;
    if (a_in && k_in) {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int q = it * 256 + t;
        load4_fast<T>(A + (m0 + q / (BK / 4)) * a.lda + k0 + (q % (BK / 4)) * 4, ra[it]);
      }
    } else {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int q = it * 256 + t;                 // group id: row = q / (BK/4), k-quad = q % (BK/4)
        const int64_t row = m0 + q / (BK / 4);
        const int kq = (q % (BK / 4)) * 4;
        if (row < a.M) load4<T>(A + row * a.lda, k0 + kq, a.K, a.vecA, ra[it]);
        else { ra[it][0] = ra[it][1] = ra[it][2] = ra[it][3] = 0.f; }
      }
    }
    if (b_in && k_in) {
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int q = it * 256 + t;
        if (B_IT * 256 == BK * BN / 4 || q < BK * BN / 4)
          load4_fast<float>(a.B + (int64_t)(k0 + q / (BN / 4)) * a.ldb + n0 + (q % (BN / 4)) * 4, rb[it]);
      }
    } else {
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int q = it * 256 + t;                 // group id: k = q / (BN/4), n-quad = q % (BN/4)
        const int k = q / (BN / 4);
        const int nq = (q % (BN / 4)) * 4;
        if (k < BK && k0 + k < a.K) load4<float>(a.B + (int64_t)(k0 + k) * a.ldb, n0 + nq, a.N, a.vecB, rb[it]);
        else { rb[it][0] = rb[it][1] = rb[it][2] = rb[it][3] = 0.f; }
      }
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int q = it * 256 + t;
      const int r = q / (BK / 4), kq = (q % (BK / 4)) * 4;
#pragma unroll
      for (int i = 0; i < 4; ++i) As[buf][r * LDA_S + kq + i] = ra[it][i];
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int q = it * 256 + t;
      const int k = q / (BN / 4), nq = (q % (BN / 4)) * 4;
      if (k < BK) *reinterpret_cast<float4*>(&Bs[buf][k * LDB_S + nq]) = make_float4(rb[it][0], rb[it][1], rb[it][2], rb[it][3]);
    }
  };

  const int nk = (a.K + BK - 1) / BK;
  fetch(0);
  stage(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) fetch((kt + 1) * BK);
    const float* as = &As[buf][(wm * TM * 32 + (lane & 31)) * LDA_S + (lane >> 5)];
    const float* bs = &Bs[buf][(lane >> 5) * LDB_S + wn * TN * 32 + (lane & 31)];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {                   // the tile is zero beyond K
      float av[TM], bv[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) av[i] = as[i * 32 * LDA_S + kk];
#pragma unroll
      for (int j = 0; j < TN; ++j) bv[j] = bs[kk * LDB_S + j * 32];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) stage(buf ^ 1);
    __syncthreads();
  }

  // epilogue.  32x32 accumulator layout: register r of lane l holds
  // row 8*(r/4) + 4*(l/32) + r%4, column l%32 of the tile.
  T* __restrict__ C = reinterpret_cast<T*>(a.C);
  T* __restrict__ C2 = reinterpret_cast<T*>(a.C2);
  const T* __restrict__ Mk = reinterpret_cast<const T*>(a.mask);
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + (wn * TN + j) * 32 + (lane & 31);
      if (n >= a.N) continue;
      const float bias = a.bias ? a.bias[n] : 0.f;
      // all mask values first, then all stores: the loads are in flight together
      float keep[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
        keep[r] = 1.f;
        if (Mk && m < a.mask_rows && m < a.M) keep[r] = load_one<T>(Mk + m * a.ldmask + n);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
        if (m >= a.M) continue;
        float v = acc[i][j][r] + bias;
        if (C2) store_one<T>(C2 + m * a.ldc2 + n, v);
        if (a.relu) v = v > 0.f ? v : 0.f;
        v = keep[r] > 0.f ? v : 0.f;
        store_one<T>(C + m * a.ldc + n, v);
      }
    }
}

static bool use_direct() {
  return tune().gemm_direct != 0;      // override for experiments: 0 = LDS-tiled kernels only
}

static int pick_vec(const void* p, int64_t ld, int64_t extent, size_t es) {
  int v = 4;
  while (v > 1 && !((ld % v) == 0 && ((uintptr_t)p % (v * es)) == 0)) v >>= 1;
  (void)extent;
  return v;
}

template <typename T>
static int gemm_nn_t(NnArgs& a, hipStream_t s) {
  const int64_t gm = ceil_div(a.M, BM);
  if (gm * 256 >= ((int64_t)1 << 32)) return fail(GCN_EINVAL, "gemm: too many rows for one launch");
  const double nb = (double)sizeof(T) * (double)a.M * (a.K + a.N * (a.C2 ? 2.0 : 1.0) + (a.mask ? a.N : 0)) +
                    4.0 * (double)a.K * a.N;
  ProfScope ps(GCN_K_GEMM_NN, s, a.N, sizeof(T) == 2 ? GCN_BF16 : GCN_F32, a.M, a.K, nb, nb,
               2.0 * (double)a.M * a.N * a.K);
  if (a.N <= 32) {
    k_gemm_nn<T, 32, 4, 1><<<dim3((unsigned)gm, (unsigned)ceil_div(a.N, 32)), 256, 0, s>>>(a);
  } else if (a.N <= 64) {
    k_gemm_nn<T, 64, 4, 1><<<dim3((unsigned)gm, (unsigned)ceil_div(a.N, 64)), 256, 0, s>>>(a);
  } else {
    k_gemm_nn<T, 128, 2, 2><<<dim3((unsigned)gm, (unsigned)ceil_div(a.N, 128)), 256, 0, s>>>(a);
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

// fp32 only, so the bf16-pipe kernel never competes for these shapes
bool gemm_nn_limits_blocks(const void* A, int64_t lda, int64_t M, int N, int K, int dtype) {
  return use_direct() && gemm_nn_regw_ok(A, lda, M, N, K, dtype) && ((N >= 192 && K >= 96) || tune().gemm_regw == 2);
}

int gemm_nn(const void* A, int64_t lda, const float* B, int64_t ldb, void* C, int64_t ldc, int64_t M, int N,
            int K, int dtype, const GemmEpilogue& epi, hipStream_t s) {
  if (M == 0) return GCN_OK;
  const size_t es = dtype == GCN_BF16 ? 2 : 4;
  if (dtype == GCN_BF16 && use_direct() && gemm_nn_bf16_ok(A, lda, C, ldc, M, N, K, epi)) {
    const double nb = 2.0 * (double)M * (K + N * (epi.C2 ? 2.0 : 1.0) + (epi.mask ? N : 0)) + 4.0 * (double)K * N;
    ProfScope ps(GCN_K_GEMM_NN, s, N, dtype, M, K, nb, nb, 2.0 * (double)M * N * K);
    return gemm_nn_bf16(A, lda, B, ldb, C, ldc, M, N, K, epi, s);
  }
  // Wide weight matrices are held in registers, the operand rows streamed past them through LDS.  Measured on
  // 2.45 M rows (TFLOP/s, this kernel / the LDS-resident-W kernel or, for 256 x 256, the LDS-tiled one):
  // 256 x 256: 123 / 89, 128 x 256: 108 / 74, 200 x 192: 70 / 66, 100 x 256 (13 steps of 8 k): see the profile, 128 x 128 (two of the four
  // SIMDs busy): 49 / 113.  GCN_GEMM_REGW=2 takes it wherever it applies (tests).
  if (gemm_nn_limits_blocks(A, lda, M, N, K, dtype)) {
    const double nb = (double)es * (double)M * (K + N * (epi.C2 ? 2.0 : 1.0) + (epi.mask ? N : 0)) + 4.0 * (double)K * N;
    ProfScope ps(GCN_K_GEMM_NN, s, N, dtype, M, K, nb, nb, 2.0 * (double)M * N * K);
    return gemm_nn_regw(A, lda, B, ldb, C, ldc, M, N, K, epi, s);
  }
  if (use_direct() && gemm_nn_direct_ok(N, K)) {
    const double nb = (double)es * (double)M * (K + N * (epi.C2 ? 2.0 : 1.0) + (epi.mask ? N : 0)) + 4.0 * (double)K * N;
    ProfScope ps(GCN_K_GEMM_NN, s, N, dtype, M, K, nb, nb, 2.0 * (double)M * N * K);
    return gemm_nn_direct(A, lda, B, ldb, C, ldc, M, N, K, dtype, epi, s);
  }
  NnArgs a{A, lda, B, ldb, C, ldc, M, N, K, pick_vec(A, lda, K, es), pick_vec(B, ldb, N, 4),
           epi.bias, epi.relu, epi.mask, epi.ldmask, epi.mask_rows, epi.C2, epi.ldc2};
  if (dtype == GCN_BF16 && a.vecA == 2) a.vecA = 1;
  return dtype == GCN_BF16 ? gemm_nn_t<bf16_t>(a, s) : gemm_nn_t<float>(a, s);
}

// ------------------------------------------------------------------------------------------
// TN: C = A^T B over a long reduction.  Block (split, tile_m, tile_n) reduces rows
// [split*rows_per_split, ...) into a 128 x 128 partial tile.
// ------------------------------------------------------------------------------------------
struct TnArgs {
  const void* A; int64_t lda; const void* B; int64_t ldb;
  int64_t Kd; int M; int N; int vecA; int vecB; int64_t rows_per_split; int nsplit;
  float* partial;   // [nsplit][M*N]
};

// WAVES_M x WAVES_N wavefronts, each TM x TN accumulator tiles of 32 x 32, on a 128 x BN output tile
template <typename T, int BN, int WAVES_M, int WAVES_N>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_gemm_tn(TnArgs a) {
  static_assert(WAVES_M * WAVES_N == 4, "4 wavefronts per block");
  constexpr int TM = BM / WAVES_M / 32, TN = BN / WAVES_N / 32;
  constexpr int LDA_S = BM + BPAD, LDB_S = BN + BPAD;
  __shared__ float As[2][BK * LDA_S];
  __shared__ float Bs[2][BK * LDB_S];
  const int t = threadIdx.x, lane = t & 63, w = t >> 6;
  const int wm = w / WAVES_N, wn = w % WAVES_N;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.z * BN;
  const int64_t k_lo = (int64_t)blockIdx.x * a.rows_per_split;
  const int64_t k_hi = k_lo + a.rows_per_split < a.Kd ? k_lo + a.rows_per_split : a.Kd;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);
  const T* __restrict__ B = reinterpret_cast<const T*>(a.B);

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  constexpr int A_IT = BK * BM / 4 / 256;
  constexpr int B_IT = (BK * BN / 4 + 255) / 256;
  float ra[A_IT][4], rb[B_IT][4];
  const bool a_in = a.vecA == 4 && m0 + BM <= a.M;
  const bool b_in = a.vecB == 4 && n0 + BN <= a.N;
  auto fetch = [&](int64_t k0) {
    const bool k_in = k0 + BK <= k_hi;
    if (a_in && k_in) {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int q = it * 256 + t;
        load4_fast<T>(A + (k0 + q / (BM / 4)) * a.lda + m0 + (q % (BM / 4)) * 4, ra[it]);
      }
    } else {
#pragma unroll
      for (int it = 0; it < A_IT; ++it) {
        const int q = it * 256 + t;
        const int k = q / (BM / 4), cq = (q % (BM / 4)) * 4;
        if (k0 + k < k_hi) load4<T>(A + (k0 + k) * a.lda, m0 + cq, a.M, a.vecA, ra[it]);
        else { ra[it][0] = ra[it][1] = ra[it][2] = ra[it][3] = 0.f; }
      }
    }
    if (b_in && k_in) {
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int q = it * 256 + t;
        if (B_IT * 256 == BK * BN / 4 || q < BK * BN / 4)
          load4_fast<T>(B + (k0 + q / (BN / 4)) * a.ldb + n0 + (q % (BN / 4)) * 4, rb[it]);
      }
    } else {
#pragma unroll
      for (int it = 0; it < B_IT; ++it) {
        const int q = it * 256 + t;
        const int k = q / (BN / 4), cq = (q % (BN / 4)) * 4;
        if (k < BK && k0 + k < k_hi) load4<T>(B + (k0 + k) * a.ldb, n0 + cq, a.N, a.vecB, rb[it]);
        else { rb[it][0] = rb[it][1] = rb[it][2] = rb[it][3] = 0.f; }
      }
    }
  };
  auto stage = [&](int buf) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int q = it * 256 + t;
      const int k = q / (BM / 4), cq = (q % (BM / 4)) * 4;
      *reinterpret_cast<float4*>(&As[buf][k * LDA_S + cq]) = make_float4(ra[it][0], ra[it][1], ra[it][2], ra[it][3]);
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int q = it * 256 + t;
      const int k = q / (BN / 4), cq = (q % (BN / 4)) * 4;
      if (k < BK) *reinterpret_cast<float4*>(&Bs[buf][k * LDB_S + cq]) = make_float4(rb[it][0], rb[it][1], rb[it][2], rb[it][3]);
    }
  };

  const int64_t nk = (k_hi - k_lo + BK - 1) / BK;
  if (nk > 0) {
    fetch(k_lo);
    stage(0);
  }
  __syncthreads();
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int buf = (int)(kt & 1);
    if (kt + 1 < nk) fetch(k_lo + (kt + 1) * BK);
    const float* as = &As[buf][(lane >> 5) * LDA_S + wm * TM * 32 + (lane & 31)];
    const float* bs = &Bs[buf][(lane >> 5) * LDB_S + wn * TN * 32 + (lane & 31)];
#pragma unroll
    for (int kk = 0; kk < BK; kk += 2) {
      float av[TM], bv[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) av[i] = as[kk * LDA_S + i * 32];
#pragma unroll
      for (int j = 0; j < TN; ++j) bv[j] = bs[kk * LDB_S + j * 32];
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) stage(buf ^ 1);
    __syncthreads();
  }
  float* __restrict__ P = a.partial + (int64_t)blockIdx.x * a.M * a.N;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + (wn * TN + j) * 32 + (lane & 31);
      if (n >= a.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + (wm * TM + i) * 32 + 8 * (r / 4) + 4 * (lane >> 5) + (r % 4);
        if (m < a.M) P[(int64_t)m * a.N + n] = acc[i][j][r];
      }
    }
}

// C[e] = sum over splits of partial[s][e] in fp64 with a fixed association: a block takes 16
// consecutive elements; thread (r, el) adds the splits r, r+16, ... of element el, then the 16
// partial sums of an element are added in order of r.
__global__ __launch_bounds__(256) void k_tn_reduce(const float* __restrict__ partial, int nsplit, int64_t mn, int N,
                                                   float* __restrict__ C, int64_t ldc) {
  __shared__ double red[16][17];
  const int el = threadIdx.x & 15, r = threadIdx.x >> 4;
  const int64_t e = (int64_t)blockIdx.x * 16 + el;
  double s = 0.0;
  if (e < mn) {
    int p = r;
    for (; p + 48 < nsplit; p += 64) {          // four loads in flight, added in split order
      const float v0 = partial[(int64_t)p * mn + e], v1 = partial[(int64_t)(p + 16) * mn + e];
      const float v2 = partial[(int64_t)(p + 32) * mn + e], v3 = partial[(int64_t)(p + 48) * mn + e];
      s += (double)v0; s += (double)v1; s += (double)v2; s += (double)v3;
    }
    for (; p < nsplit; p += 16) s += (double)partial[(int64_t)p * mn + e];
  }
  red[r][el] = s;
  __syncthreads();
  if (r == 0 && e < mn) {
    double t = 0.0;
#pragma unroll
    for (int q = 0; q < 16; ++q) t += red[q][el];
    C[(e / N) * ldc + (e % N)] = (float)t;
  }
}

static int tn_bn(int N) { return N <= 32 ? 32 : (N <= 64 ? 64 : 128); }

static int tn_splits(int64_t Kd, int M, int N) {
  const int64_t tiles = ceil_div(M, BM) * ceil_div(N, tn_bn(N));
  int64_t want = ceil_div(512, tiles);                 // about two blocks per compute unit
  int64_t max_by_k = ceil_div(Kd, 256);                // at least 256 rows per split
  int64_t ns = want < max_by_k ? want : max_by_k;
  return (int)(ns < 1 ? 1 : ns);
}

size_t gemm_tn_ws_bytes(int64_t Kd, int M, int N) {
  const size_t tiled = sizeof(float) * (size_t)tn_splits(Kd, M, N) * (size_t)M * (size_t)N;
  const size_t direct = gemm_tn_direct_ws_bytes(Kd, M, N);
  return tiled > direct ? tiled : direct;
}

int gemm_tn(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc, int64_t Kd, int M,
            int N, int dtype, void* ws, hipStream_t s, int max_blocks) {
  const size_t es = dtype == GCN_BF16 ? 2 : 4;
  const int64_t mn = (int64_t)M * N;
  int nsplit = 0;
  if (use_direct()) {
    const double nb = (double)es * (double)Kd * (M + N) + 4.0 * (double)mn;
    ProfScope ps(GCN_K_GEMM_TN, s, N, dtype, M, Kd, nb, nb, 2.0 * (double)Kd * M * N);
    GCN_TRY(gemm_tn_direct_partials(A, lda, B, ldb, Kd, M, N, dtype, (float*)ws, &nsplit, s, max_blocks));
  } else {
    TnArgs a{A, lda, B, ldb, Kd, M, N, pick_vec(A, lda, M, es), pick_vec(B, ldb, N, es), 0, 0, (float*)ws};
    if (dtype == GCN_BF16) { if (a.vecA == 2) a.vecA = 1; if (a.vecB == 2) a.vecB = 1; }
    a.nsplit = tn_splits(Kd, M, N);
    a.rows_per_split = round_up(ceil_div(Kd > 0 ? Kd : 1, a.nsplit), BK);
    nsplit = a.nsplit;
    const int bn = tn_bn(N);
    dim3 grid((unsigned)a.nsplit, (unsigned)ceil_div(M, BM), (unsigned)ceil_div(N, bn));
    const double nb = (double)es * (double)Kd * (M + N) + 4.0 * (double)mn;
    ProfScope ps(GCN_K_GEMM_TN, s, N, dtype, M, Kd, nb, nb, 2.0 * (double)Kd * M * N);
    if (dtype == GCN_BF16) {
      if (bn == 32) k_gemm_tn<bf16_t, 32, 4, 1><<<grid, 256, 0, s>>>(a);
      else if (bn == 64) k_gemm_tn<bf16_t, 64, 4, 1><<<grid, 256, 0, s>>>(a);
      else k_gemm_tn<bf16_t, 128, 2, 2><<<grid, 256, 0, s>>>(a);
    } else {
      if (bn == 32) k_gemm_tn<float, 32, 4, 1><<<grid, 256, 0, s>>>(a);
      else if (bn == 64) k_gemm_tn<float, 64, 4, 1><<<grid, 256, 0, s>>>(a);
      else k_gemm_tn<float, 128, 2, 2><<<grid, 256, 0, s>>>(a);
    }
  }
  {
    const double nb = 4.0 * (double)mn * (nsplit + 1);
    ProfScope ps(GCN_K_GEMM_TN_SUM, s, N, GCN_F32, M, nsplit, nb, nb, (double)mn * nsplit);
    k_tn_reduce<<<(unsigned)ceil_div(mn, 16), 256, 0, s>>>((const float*)ws, nsplit, mn, N, C, ldc);
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

bool gemm_tn_limits_blocks(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, int dtype) {
  return use_direct() && !(dtype == GCN_BF16 && gemm_tn_bf16_ok(A, lda, B, ldb, Kd, M, N)) && gemm_tn_lds_ok(A, lda, B, ldb, Kd, M, N, dtype);
}

// ------------------------------------------------------------------------------------------
__global__ void k_transpose(const float* __restrict__ W, int K, int N, float* __restrict__ Wt) {
  int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= (int64_t)K * N) return;
  int n = (int)(e / K), k = (int)(e % K);
  Wt[e] = W[(int64_t)k * N + n];
}

int transpose_f32(const float* W, int K, int N, float* Wt, hipStream_t s) {
  ProfScope ps(GCN_K_OTHER, s, N, GCN_F32, K, 0, 8.0 * K * N, 8.0 * K * N, 0.0);
  k_transpose<<<(unsigned)ceil_div((int64_t)K * N, 256), 256, 0, s>>>(W, K, N, Wt);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

// column sums: block b adds rows [b*kRows, ...) per column into partial[b][c]; then fp64 finish
constexpr int kColsumRows = 4096;
template <typename T>
__global__ __launch_bounds__(256) void k_colsum_part(const T* __restrict__ G, int64_t ldg, int64_t rows, int N,
                                                     float* __restrict__ partial) {
  const int64_t r0 = (int64_t)blockIdx.x * kColsumRows;
  const int64_t r1 = r0 + kColsumRows < rows ? r0 + kColsumRows : rows;
  for (int c = threadIdx.x; c < N; c += 256) {
    float s = 0.f;
    // 16 interleaved partial chains keep each fp32 chain short
    float ch[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) ch[i] = 0.f;
    int64_t r = r0;
    for (; r + 16 <= r1; r += 16)
#pragma unroll
      for (int i = 0; i < 16; ++i) ch[i] += load_one<T>(G + (r + i) * ldg + c);
    for (; r < r1; ++r) s += load_one<T>(G + r * ldg + c);
#pragma unroll
    for (int i = 0; i < 16; ++i) s += ch[i];
    partial[(int64_t)blockIdx.x * N + c] = s;
  }
}
__global__ void k_colsum_finish(const float* __restrict__ partial, int64_t nb, int N, float* __restrict__ out) {
  int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= N) return;
  double s = 0.0;
  for (int64_t b = 0; b < nb; ++b) s += (double)partial[b * N + c];
  out[c] = (float)s;
}
size_t colsum_ws_bytes(int64_t rows, int N) { return sizeof(float) * (size_t)ceil_div(rows > 0 ? rows : 1, kColsumRows) * (size_t)N; }
int colsum(const void* G, int64_t ldg, int64_t rows, int N, int dtype, float* out, void* ws, hipStream_t s) {
  const int64_t nb = ceil_div(rows > 0 ? rows : 1, kColsumRows);
  const double by = (dtype == GCN_BF16 ? 2.0 : 4.0) * (double)rows * N;
  ProfScope ps(GCN_K_OTHER, s, N, dtype, rows, 0, by, by, (double)rows * N);
  if (dtype == GCN_BF16) k_colsum_part<bf16_t><<<(unsigned)nb, 256, 0, s>>>((const bf16_t*)G, ldg, rows, N, (float*)ws);
  else k_colsum_part<float><<<(unsigned)nb, 256, 0, s>>>((const float*)G, ldg, rows, N, (float*)ws);
  k_colsum_finish<<<(unsigned)ceil_div(N, 256), 256, 0, s>>>((const float*)ws, nb, N, out);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

}  // namespace gcn
