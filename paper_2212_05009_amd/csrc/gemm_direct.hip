// Streaming forms of the two tall-and-skinny dense products of a GCN layer (Sec. 3.1: the product
// with W^k after the sparse aggregation, and the weight gradient), for gfx950.  The long operand
// (one row per vertex) goes from global memory straight into the MFMA operand registers: no LDS
// staging and no barrier in the main loop, so a wavefront keeps many independent loads in flight,
// which is what a product bound by HBM bandwidth needs.
//
//   nn_direct : C[M x N] = A[M x K] W[K x N], W small enough to sit in LDS for the whole kernel.
//               MFMA 16x16x4: lane (c = l%16, q = l/16) loads A[row c][k0 + 4q .. k0 + 4q + 3] with one
//               16-byte load and feeds element i of it to the i-th of four MFMAs, whose W operand is
//               W[k0 + 4q + i][col c]: every k of the 16-wide step is used exactly once, only in a
//               permuted order, which a sum does not care about.
//   tn_direct : C[M x N] = A[Kd x M]^T B[Kd x N], Kd = number of vertices.  MFMA 32x32x2: lane
//               (c = l%32, h = l/32) loads A[k + h][m0 + c] and B[k + h][n0 + c]: 128-byte coalesced
//               rows.  The four wavefronts of a block take interleaved row chunks of one output tile,
//               add their tiles through LDS and write one partial tile per block.
#include <stdlib.h>

#include <algorithm>

#include "common.h"

namespace gcn {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// 4 consecutive elements starting at column k (multiple of 4) of a row, zero beyond `limit`
template <typename T>
__device__ __forceinline__ void load_quad(const T* __restrict__ row, int k, int limit, bool vec_ok, float (&o)[4]) {
  if (vec_ok && k + 3 < limit) {
    if constexpr (sizeof(T) == 4) {
      float4 v = *reinterpret_cast<const float4*>(row + k);
      o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    } else {
      uint2 v = *reinterpret_cast<const uint2*>(row + k);
      o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
      o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) o[i] = (k + i < limit) ? load_one<T>(row + k + i) : 0.f;
}

// 4 consecutive elements starting at column n (multiple of 4) of a row, none beyond `limit`
template <typename T>
__device__ __forceinline__ void store_quad(T* __restrict__ row, int n, int limit, bool vec_ok, const float (&v)[4]) {
  if (vec_ok && n + 3 < limit) {
    if constexpr (sizeof(T) == 4) {
      *reinterpret_cast<float4*>(row + n) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
      bf16_t h[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) store_one<T>(&h[i], v[i]);
      uint2 pk;
      pk.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
      pk.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
      *reinterpret_cast<uint2*>(row + n) = pk;
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (n + i < limit) store_one<T>(row + n + i, v[i]);
}

// ------------------------------------------------------------------------------------------
struct NnDirectArgs {
  const void* A; int64_t lda; const float* W; int64_t ldw; void* C; int64_t ldc;
  int64_t M; int N; int K; int vecA; int vecC; int vecC2; int vecM;
  const float* bias; int relu; const void* mask; int64_t ldmask; int64_t mask_rows; void* C2; int64_t ldc2;
};

constexpr int kNnThreads = 512;
constexpr int kNnKU = 8;          // 16-wide k steps whose loads are issued together

// At most 128 registers for up to 8 column tiles, so that two 8-wave blocks share a compute unit
// (four wavefronts per SIMD): measured 161 -> 137 us for 2^18 x 128 x 128.
template <typename T, int NT>
__global__ __launch_bounds__(kNnThreads) __attribute__((amdgpu_waves_per_eu(NT <= 8 ? 4 : 2, 8))) void k_gemm_nn_direct(NnDirectArgs a) {
  extern __shared__ float Ws[];                      // [Kp][LDW], zero beyond K and N
  constexpr int LDW = NT * 16 + 4;                    // 4 k-rows apart land 16 banks apart
  const int Kp = (a.K + 15) & ~15;
  for (int e = threadIdx.x; e < Kp * NT * 16; e += kNnThreads) {
    const int k = e / (NT * 16), n = e % (NT * 16);
    Ws[k * LDW + n] = (k < a.K && n < a.N) ? a.W[(int64_t)k * a.ldw + n] : 0.f;
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, q = lane >> 4;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);
  T* __restrict__ C = reinterpret_cast<T*>(a.C);
  T* __restrict__ C2 = reinterpret_cast<T*>(a.C2);
  const T* __restrict__ Mk = reinterpret_cast<const T*>(a.mask);
  const bool vec_ok = a.vecA == 4;
  const int64_t ntiles = (a.M + 15) / 16;
  constexpr int WPB = kNnThreads / 64;

  // Software pipeline over the tiles of this wavefront: the operand rows (first 128 k) and the mask
  // values of the NEXT tile are requested before the current tile's MFMAs and stores, so that a
  // wavefront always has a tile's worth of loads in flight.
  constexpr int TC = NT < 8 ? NT : 8;                 // column tiles finished together (bounds registers)
  constexpr bool kPrefetchMask = NT <= 4;
  const int64_t stride = (int64_t)gridDim.x * WPB;
  auto load_a = [&](int64_t tile, int k0, float (&av)[kNnKU][4]) {
    const int64_t row = tile * 16 + c;
    const T* __restrict__ arow = A + (row < a.M ? row : a.M - 1) * a.lda;
#pragma unroll
    for (int u = 0; u < kNnKU; ++u) {
      if (k0 + 16 * u < Kp) load_quad<T>(arow, k0 + 16 * u + 4 * q, a.K, vec_ok, av[u]);
      else { av[u][0] = av[u][1] = av[u][2] = av[u][3] = 0.f; }
    }
  };
  auto load_m = [&](int64_t tile, int t0, float (&keep)[TC][4]) {
    const int64_t m = tile * 16 + c;
    const bool masked = Mk != nullptr && m < a.mask_rows && m < a.M;
#pragma unroll
    for (int t = 0; t < TC; ++t) {
      keep[t][0] = keep[t][1] = keep[t][2] = keep[t][3] = 1.f;
      if (masked && t0 + t < NT) load_quad<T>(Mk + m * a.ldmask, (t0 + t) * 16 + 4 * q, a.N, a.vecM == 4, keep[t]);
    }
  };

  int64_t tile = (int64_t)blockIdx.x * WPB + w;
  float a_nxt[kNnKU][4], m_nxt[TC][4];
  if (tile < ntiles) {
    load_a(tile, 0, a_nxt);
    if (kPrefetchMask) load_m(tile, 0, m_nxt);
  }
  for (; tile < ntiles; tile += stride) {
    float av[kNnKU][4], keep[TC][4];
#pragma unroll
    for (int u = 0; u < kNnKU; ++u)
#pragma unroll
      for (int i = 0; i < 4; ++i) av[u][i] = a_nxt[u][i];
    if (kPrefetchMask) {
#pragma unroll
      for (int t = 0; t < TC; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) keep[t][i] = m_nxt[t][i];
    }
    if (tile + stride < ntiles) {
      load_a(tile + stride, 0, a_nxt);
      if (kPrefetchMask) load_m(tile + stride, 0, m_nxt);
    }

    floatx4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = 0; k0 < Kp; k0 += 16 * kNnKU) {
      if (k0 > 0) load_a(tile, k0, av);
#pragma unroll
      for (int u = 0; u < kNnKU; ++u) {
        if (k0 + 16 * u < Kp) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float* wrow = Ws + (k0 + 16 * u + 4 * q + i) * LDW + c;
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wrow[t * 16], av[u][i], acc[t], 0, 0, 0);
          }
        }
      }
    }

    // W is the first MFMA operand, so the 16 x 16 result tile is transposed: register r of lane (c, q)
    // holds output column 16t + 4q + r of row c.  A lane owns 4 consecutive columns of its row:
    // one 16-byte store (and one 16-byte mask load) per column tile.
    const int64_t m = tile * 16 + c;
    if (m < a.M) {
      const bool masked = Mk != nullptr && m < a.mask_rows;
#pragma unroll
      for (int t0 = 0; t0 < NT; t0 += TC) {
        if (!kPrefetchMask) load_m(tile, t0, keep);
#pragma unroll
        for (int t = 0; t < TC; ++t) {
          if (t0 + t >= NT) continue;
          const int n = (t0 + t) * 16 + 4 * q;
          if (n >= a.N) continue;
          float v[4], pre[4];
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            pre[r] = acc[t0 + t][r] + ((a.bias && n + r < a.N) ? a.bias[n + r] : 0.f);
            v[r] = a.relu ? (pre[r] > 0.f ? pre[r] : 0.f) : pre[r];
            if (masked) v[r] = keep[t][r] > 0.f ? v[r] : 0.f;
          }
          if (C2) store_quad<T>(C2 + m * a.ldc2, n, a.N, a.vecC2 == 4, pre);
          store_quad<T>(C + m * a.ldc, n, a.N, a.vecC == 4, v);
        }
      }
    }
  }
}

// ---- the same product without a single data-dependent branch ----------------------------------------
// For operands whose rows are 16-byte aligned (fp32; 8-byte for bf16), K up to 128 (KU = ceil(K / 16) k steps, the
// whole row in one request batch, a tail of the row cleared by bit masks) or a multiple of 128 (KU = 8), N up to 256 and a mask that covers every row.  Every load is an
// unconditional 16-byte (bf16: 8-byte) request - rows beyond M are clamped to the last row and dropped at
// the store - so the compiler can keep the next step's operand loads in flight across the MFMAs of the
// current one instead of waiting at every join of the general kernel's bounds checks.
template <typename T> __device__ __forceinline__ void vload4(const T* __restrict__ p, float (&o)[4]) {
  if constexpr (sizeof(T) == 4) {
    const floatx4 v = *reinterpret_cast<const floatx4*>(p);
    o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
  } else {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = *reinterpret_cast<const u32x2*>(p);
    o[0] = __uint_as_float(v[0] << 16); o[1] = __uint_as_float(v[0] & 0xffff0000u);
    o[2] = __uint_as_float(v[1] << 16); o[3] = __uint_as_float(v[1] & 0xffff0000u);
  }
}
template <typename T> __device__ __forceinline__ void vstore4(T* __restrict__ p, const float (&v)[4]) {
  if constexpr (sizeof(T) == 4) {
    *reinterpret_cast<floatx4*>(p) = floatx4{v[0], v[1], v[2], v[3]};
  } else {
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    bf16_t h[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) store_one<T>(&h[i], v[i]);
    *reinterpret_cast<u32x2*>(p) = u32x2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
  }
}

// FULL: K is a multiple of 16 and N = 16 NT, so there is no tail to clear and no column group to skip
template <typename T, int NT, int KU, bool MASK, bool SAVE, bool FULL>
__global__ __launch_bounds__(kNnThreads) __attribute__((amdgpu_waves_per_eu(NT <= 8 ? 4 : 2, 8))) void k_gemm_nn_fast(NnDirectArgs a) {
  // W in LDS.  NT a multiple of 4: [k][t / 4][c][t % 4], so that the four column tiles 4 tq .. 4 tq + 3 of a
  // lane's (k, c) are one 16-byte read and the 16 lanes of a k row read 256 contiguous bytes.  Else [k][LDW].
  extern __shared__ float Ws[];
  constexpr int LDW = NT * 16 + 4;
  constexpr bool kQuad = NT % 4 == 0;
  constexpr int TQ = kQuad ? NT / 4 : 1;
  const int chunks = (a.K + 16 * KU - 1) / (16 * KU);   // k chunks per tile
  for (int e = threadIdx.x; e < chunks * 16 * KU * NT * 16; e += kNnThreads) {      // zero beyond K and N
    const int k = e / (NT * 16), n = e % (NT * 16);
    const int t = n >> 4, cc = n & 15;
    const int at = kQuad ? ((k * TQ + (t >> 2)) * 16 + cc) * 4 + (t & 3) : k * LDW + n;
    Ws[at] = (k < a.K && n < a.N) ? a.W[(int64_t)k * a.ldw + n] : 0.f;
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, q = lane >> 4;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);
  T* __restrict__ C = reinterpret_cast<T*>(a.C);
  T* __restrict__ C2 = reinterpret_cast<T*>(a.C2);
  const T* __restrict__ Mk = reinterpret_cast<const T*>(a.mask);
  constexpr int WPB = kNnThreads / 64;
  const int64_t ntiles = (a.M + 15) / 16;
  const int64_t stride = (int64_t)gridDim.x * WPB;
  // mask values of the next tile travel with its operand rows when a tile is a single chunk and they fit
  constexpr bool kPrefetchMask = MASK && KU <= 2 && NT <= 8;

  // K that is no multiple of 16: the lane's request of the very last k step may start past K (moved to column 0)
  // or reach past it (the row is padded to 4 elements); `tail` clears what is not part of the product
  const int k_last = 16 * KU * chunks - 16 + 4 * q;
  const int n_ok = a.K - k_last;
  const int last_off = n_ok > 0 ? k_last : 0;
  uint32_t tail[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) tail[i] = i < n_ok ? 0xffffffffu : 0u;
  const int n_up = FULL ? NT * 16 : (a.N + 3) & ~3;     // columns come in groups of 4; the rows are that long
  auto load_a = [&](int64_t tile, int chunk, float (&av)[KU][4]) {
    const int64_t row = tile * 16 + c;
    if constexpr (FULL) {
      const T* __restrict__ arow = A + (row < a.M ? row : a.M - 1) * a.lda + chunk * (16 * KU) + 4 * q;
#pragma unroll
      for (int u = 0; u < KU; ++u) vload4<T>(arow + 16 * u, av[u]);
    } else {
      const T* __restrict__ arow = A + (row < a.M ? row : a.M - 1) * a.lda;
      const bool last = chunk == chunks - 1;
#pragma unroll
      for (int u = 0; u < KU; ++u)
        vload4<T>(arow + ((u == KU - 1 && last) ? last_off : chunk * (16 * KU) + 16 * u + 4 * q), av[u]);
    }
  };
  auto load_m = [&](int64_t tile, float (&keep)[NT][4]) {
    const int64_t row = tile * 16 + c;
    const T* __restrict__ mrow = Mk + (row < a.M ? row : a.M - 1) * a.ldmask;
#pragma unroll
    for (int t = 0; t < NT; ++t) vload4<T>(mrow + ((FULL || 16 * t + 4 * q < n_up) ? 16 * t + 4 * q : 0), keep[t]);
  };

  int64_t tile = (int64_t)blockIdx.x * WPB + w;
  if (tile >= ntiles) return;
  float a_nxt[KU][4];
  float m_nxt[kPrefetchMask ? NT : 1][4];
  load_a(tile, 0, a_nxt);
  if constexpr (kPrefetchMask) load_m(tile, m_nxt);
  for (; tile < ntiles; tile += stride) {
    floatx4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    float keep[kPrefetchMask ? NT : 1][4];
    if constexpr (kPrefetchMask) {
#pragma unroll
      for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) keep[t][i] = m_nxt[t][i];
    }
    for (int chunk = 0; chunk < chunks; ++chunk) {
      float av[KU][4];
#pragma unroll
      for (int u = 0; u < KU; ++u)
#pragma unroll
        for (int i = 0; i < 4; ++i) av[u][i] = a_nxt[u][i];
      if constexpr (!FULL) {
        if (chunk == chunks - 1) {
#pragma unroll
          for (int i = 0; i < 4; ++i) av[KU - 1][i] = __uint_as_float(__float_as_uint(av[KU - 1][i]) & tail[i]);
        }
      }
      // the next request: this tile's next chunk, else the first chunk of the wavefront's next tile
      // (clamped to the last tile: a valid, wasted load at the very end)
      const bool same = chunk + 1 < chunks;
      const int64_t nt = same ? tile : (tile + stride < ntiles ? tile + stride : ntiles - 1);
      load_a(nt, same ? chunk + 1 : 0, a_nxt);
      if constexpr (kPrefetchMask) load_m(nt, m_nxt);
      if constexpr (kQuad) {
        // the W operands of step (u, i + 1) are read from LDS before the MFMAs of step (u, i) are issued
        const floatx4* wq = reinterpret_cast<const floatx4*>(Ws) + ((chunk * (16 * KU) + 4 * q) * TQ) * 16 + c;
        floatx4 wc[TQ], wn[TQ];
#pragma unroll
        for (int tq = 0; tq < TQ; ++tq) wc[tq] = wq[tq * 16];
#pragma unroll
        for (int st = 0; st < KU * 4; ++st) {
          const int u = st >> 2, i = st & 3;
          if (st + 1 < KU * 4) {
            const int kn = 16 * ((st + 1) >> 2) + ((st + 1) & 3);
#pragma unroll
            for (int tq = 0; tq < TQ; ++tq) wn[tq] = wq[(kn * TQ + tq) * 16];
          }
#pragma unroll
          for (int tq = 0; tq < TQ; ++tq)
#pragma unroll
            for (int r = 0; r < 4; ++r)
              acc[tq * 4 + r] = __builtin_amdgcn_mfma_f32_16x16x4f32(wc[tq][r], av[u][i], acc[tq * 4 + r], 0, 0, 0);
#pragma unroll
          for (int tq = 0; tq < TQ; ++tq) wc[tq] = wn[tq];
        }
      } else {
        const float* wbase = Ws + (chunk * (16 * KU) + 4 * q) * LDW + c;
#pragma unroll
        for (int u = 0; u < KU; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float* wrow = wbase + (16 * u + i) * LDW;
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wrow[t * 16], av[u][i], acc[t], 0, 0, 0);
          }
      }
    }
    // register r of lane (c, q) holds output column 16t + 4q + r of row c
    const int64_t m = tile * 16 + c;
    if (m < a.M) {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = t * 16 + 4 * q;
        if constexpr (!FULL) { if (n >= n_up) continue; }
        float v[4], pre[4], kp[4];
        if constexpr (MASK && !kPrefetchMask) vload4<T>(Mk + m * a.ldmask + n, kp);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          pre[r] = acc[t][r] + ((a.bias && (FULL || n + r < a.N)) ? a.bias[n + r] : 0.f);
          v[r] = a.relu ? (pre[r] > 0.f ? pre[r] : 0.f) : pre[r];
          if constexpr (MASK) v[r] = (kPrefetchMask ? keep[t][r] : kp[r]) > 0.f ? v[r] : 0.f;
        }
        if constexpr (SAVE) vstore4<T>(C2 + m * a.ldc2 + n, pre);
        vstore4<T>(C + m * a.ldc + n, v);
      }
    }
  }
}

static int nn_tiles(int N) { return N <= 16 ? 1 : N <= 32 ? 2 : N <= 48 ? 3 : N <= 64 ? 4 : N <= 128 ? 8 : 16; }

size_t gemm_nn_direct_lds_bytes(int N, int K) {
  return sizeof(float) * (size_t)((K + 15) & ~15) * (size_t)(nn_tiles(N) * 16 + 4);
}

bool gemm_nn_direct_ok(int N, int K) { return N <= 256 && gemm_nn_direct_lds_bytes(N, K) <= 128 * 1024; }

template <typename T, int NT>
static int nn_launch(const NnDirectArgs& a, hipStream_t s) {
  const size_t lds = gemm_nn_direct_lds_bytes(a.N, a.K);
  auto kern = k_gemm_nn_direct<T, NT>;
  GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
  const int64_t ntiles = ceil_div(a.M, 16);
  const int per_cu = lds > 80 * 1024 ? 1 : 2;         // blocks that fit one compute unit's LDS
  int64_t blocks = ceil_div(ntiles, kNnThreads / 64);
  if (blocks > 256 * per_cu) blocks = 256 * per_cu;
  kern<<<dim3((unsigned)blocks), dim3(kNnThreads), lds, s>>>(a);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

template <typename T, int NT, int KU>
static int nn_launch_fast(const NnDirectArgs& a, hipStream_t s) {
  const size_t lds = gemm_nn_direct_lds_bytes(a.N, a.K);
  const int64_t ntiles = ceil_div(a.M, 16);
  const int per_cu = lds > 80 * 1024 ? 1 : 2;
  int64_t blocks = ceil_div(ntiles, kNnThreads / 64);
  if (blocks > 256 * per_cu) blocks = 256 * per_cu;
  auto go = [&](auto kern) -> int {
    GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<dim3((unsigned)blocks), dim3(kNnThreads), lds, s>>>(a);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  };
  if constexpr (KU == 1 || KU == 2 || KU == 4 || KU == 8) {
    if ((a.K % 16) == 0 && a.N == NT * 16) {
      if (a.mask) return go(k_gemm_nn_fast<T, NT, KU, true, false, true>);
      return a.C2 ? go(k_gemm_nn_fast<T, NT, KU, false, true, true>) : go(k_gemm_nn_fast<T, NT, KU, false, false, true>);
    }
  }
  if (a.mask) return go(k_gemm_nn_fast<T, NT, KU, true, false, false>);
  return a.C2 ? go(k_gemm_nn_fast<T, NT, KU, false, true, false>) : go(k_gemm_nn_fast<T, NT, KU, false, false, false>);
}

// the branch-free kernel serves aligned rows with K up to 128 or a multiple of 128
template <typename T>
static bool nn_fast(const NnDirectArgs& a, hipStream_t s, int* rc) {
  const bool off = tune().gemm_fast == 0;
  const int NT = nn_tiles(a.N);
  if (off || a.vecA != 4 || a.vecC != 4 || (a.C2 && a.vecC2 != 4)) return false;
  if (a.mask && (a.vecM != 4 || a.mask_rows < a.M || a.C2)) return false;
  const int ku = a.K % 128 == 0 ? 8 : a.K < 128 ? (a.K + 15) / 16 : 0;
  if (ku == 0) return false;
#define GCN_NN_FAST(NTV)                                              \
  {                                                                   \
    switch (ku) {                                                     \
      case 1: *rc = nn_launch_fast<T, NTV, 1>(a, s); break;           \
      case 2: *rc = nn_launch_fast<T, NTV, 2>(a, s); break;           \
      case 3: *rc = nn_launch_fast<T, NTV, 3>(a, s); break;           \
      case 4: *rc = nn_launch_fast<T, NTV, 4>(a, s); break;           \
      case 5: *rc = nn_launch_fast<T, NTV, 5>(a, s); break;           \
      case 6: *rc = nn_launch_fast<T, NTV, 6>(a, s); break;           \
      case 7: *rc = nn_launch_fast<T, NTV, 7>(a, s); break;           \
      default: *rc = nn_launch_fast<T, NTV, 8>(a, s); break;          \
    }                                                                 \
    return true;                                                      \
  }
  switch (NT) {
    case 1: GCN_NN_FAST(1)
    case 2: GCN_NN_FAST(2)
    case 3: GCN_NN_FAST(3)
    case 4: GCN_NN_FAST(4)
    case 8: GCN_NN_FAST(8)
    default: GCN_NN_FAST(16)
  }
#undef GCN_NN_FAST
}

template <typename T>
static int nn_dispatch(const NnDirectArgs& a, hipStream_t s) {
  int rc = GCN_OK;
  if (nn_fast<T>(a, s, &rc)) return rc;
  switch (nn_tiles(a.N)) {
    case 1: return nn_launch<T, 1>(a, s);
    case 2: return nn_launch<T, 2>(a, s);
    case 3: return nn_launch<T, 3>(a, s);
    case 4: return nn_launch<T, 4>(a, s);
    case 8: return nn_launch<T, 8>(a, s);
    default: return nn_launch<T, 16>(a, s);
  }
}

int gemm_nn_direct(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N,
                   int K, int dtype, const GemmEpilogue& epi, hipStream_t s) {
  if (M == 0) return GCN_OK;
  const size_t es = dtype == GCN_BF16 ? 2 : 4;
  auto vec_of = [&](const void* p, int64_t ld) { return (p && (ld % 4) == 0 && ((uintptr_t)p % (4 * es)) == 0) ? 4 : 1; };
  NnDirectArgs a{A, lda, W, ldw, C, ldc, M, N, K, vec_of(A, lda), vec_of(C, ldc), vec_of(epi.C2, epi.ldc2),
                 vec_of(epi.mask, epi.ldmask),
                 epi.bias, epi.relu, epi.mask, epi.ldmask, epi.mask_rows, epi.C2, epi.ldc2};
  return dtype == GCN_BF16 ? nn_dispatch<bf16_t>(a, s) : nn_dispatch<float>(a, s);
}

// ------------------------------------------------------------------------------------------
struct TnDirectArgs {
  const void* A; int64_t lda; const void* B; int64_t ldb;
  int64_t Kd; int M; int N; int64_t rows_per_split; int nsplit;
  float* partial;   // [nsplit][M*N]
};

constexpr int kTnMaxUK = 8;       // most row pairs whose loads are issued together

template <typename T, int TM, int TN, int kTnUK>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 8))) void k_gemm_tn_direct(TnDirectArgs a) {
  __shared__ float red[2][TM * TN * 16 * 64];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 31, h = lane >> 5;
  const int m0 = blockIdx.y * (32 * TM), n0 = blockIdx.z * (32 * TN);
  const int64_t k_lo = (int64_t)blockIdx.x * a.rows_per_split;
  const int64_t k_hi = k_lo + a.rows_per_split < a.Kd ? k_lo + a.rows_per_split : a.Kd;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);
  const T* __restrict__ B = reinterpret_cast<const T*>(a.B);

  // per-lane column offsets (clamped into the row so that every address is valid) and validity
  int64_t aoff[TM], boff[TN];
  bool aok[TM], bok[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) { const int m = m0 + 32 * i + c; aok[i] = m < a.M; aoff[i] = (int64_t)h * a.lda + (aok[i] ? m : 0); }
#pragma unroll
  for (int j = 0; j < TN; ++j) { const int n = n0 + 32 * j + c; bok[j] = n < a.N; boff[j] = (int64_t)h * a.ldb + (bok[j] ? n : 0); }

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // wavefront w takes the chunks w, w + 4, ... of 2 * kTnUK rows
  constexpr int CH = 2 * kTnUK;
  for (int64_t k = k_lo + (int64_t)w * CH; k < k_hi; k += 4 * CH) {
    float av[kTnUK][TM], bv[kTnUK][TN];
    if (k + CH <= k_hi) {
#pragma unroll
      for (int u = 0; u < kTnUK; ++u) {
        const T* __restrict__ ar = A + (k + 2 * u) * a.lda;
        const T* __restrict__ br = B + (k + 2 * u) * a.ldb;
#pragma unroll
        for (int i = 0; i < TM; ++i) av[u][i] = load_one<T>(ar + aoff[i]);
#pragma unroll
        for (int j = 0; j < TN; ++j) bv[u][j] = load_one<T>(br + boff[j]);
      }
    } else {
#pragma unroll
      for (int u = 0; u < kTnUK; ++u) {
        const int64_t kr = k + 2 * u + h;
        const bool rok = kr < k_hi;
        const int64_t kc = rok ? k + 2 * u : k_lo - h;       // kc + h stays inside [k_lo, k_hi)
        const T* __restrict__ ar = A + kc * a.lda;
        const T* __restrict__ br = B + kc * a.ldb;
#pragma unroll
        for (int i = 0; i < TM; ++i) { const float v = load_one<T>(ar + aoff[i]); av[u][i] = rok ? v : 0.f; }
#pragma unroll
        for (int j = 0; j < TN; ++j) { const float v = load_one<T>(br + boff[j]); bv[u][j] = rok ? v : 0.f; }
      }
    }
#pragma unroll
    for (int u = 0; u < kTnUK; ++u) {
#pragma unroll
      for (int i = 0; i < TM; ++i) { if (!aok[i]) av[u][i] = 0.f; }
#pragma unroll
      for (int j = 0; j < TN; ++j) { if (!bok[j]) bv[u][j] = 0.f; }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][i], bv[u][j], acc[i][j], 0, 0, 0);
    }
  }

  // add the four wavefronts' tiles: (2,3) -> LDS -> (0,1) add; 1 -> LDS -> 0 adds
  auto dump = [&](float* buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) buf[((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  };
  auto take = [&](const float* buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] += buf[((i * TN + j) * 16 + r) * 64 + lane];
  };
  if (w >= 2) dump(red[w - 2]);
  __syncthreads();
  if (w < 2) take(red[w]);
  __syncthreads();
  if (w == 1) dump(red[0]);
  __syncthreads();
  if (w != 0) return;
  take(red[0]);
  float* __restrict__ P = a.partial + (int64_t)blockIdx.x * a.M * a.N;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + 32 * j + c;
      if (n >= a.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + 32 * i + 8 * (r / 4) + 4 * h + (r % 4);
        if (m < a.M) P[(int64_t)m * a.N + n] = acc[i][j][r];
      }
    }
}

// ---- the same contraction with vector requests ------------------------------------------------------------
// The texture path takes as long for a 4-byte request per lane as for a 16-byte one, and the kernel above
// issues one 4-byte request per MFMA: it is bound by that path, not by the matrix pipe or by memory.  Here a
// lane asks for 4 consecutive columns of A at once (and TN consecutive columns of B): component i of the
// request is the lane's operand for column tile i, so tile i holds the columns {4 c + i} and the 32 lanes of a
// row half read 512 contiguous bytes.  The MFMA never sees the permutation; it is undone when the partial tile
// is stored.  One request per four (TN = 1) or four requests per sixteen (TN = 2) MFMAs.  The next chunk's
// requests are issued before the MFMAs of the current one; scheduling barriers keep them there.
// Needs rows of A aligned to 4 elements and, for TN = 2, rows of B aligned to 2.
template <typename T, int N> struct RawVec;
template <> struct RawVec<float, 4> { typedef floatx4 type; };
template <> struct RawVec<float, 2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct RawVec<float, 1> { typedef float type; };
template <> struct RawVec<bf16_t, 4> { typedef uint32_t type __attribute__((ext_vector_type(2))); };
template <> struct RawVec<bf16_t, 2> { typedef uint32_t type; };
template <> struct RawVec<bf16_t, 1> { typedef uint16_t type; };

template <typename T, int N>
__device__ __forceinline__ void raw_to_f32(const typename RawVec<T, N>::type& v, uint32_t (&o)[N]) {
  if constexpr (sizeof(T) == 4) {
    if constexpr (N == 1) o[0] = __float_as_uint(v);
    else {
#pragma unroll
      for (int i = 0; i < N; ++i) o[i] = __float_as_uint(v[i]);
    }
  } else {
    if constexpr (N == 1) o[0] = (uint32_t)v << 16;
    else if constexpr (N == 2) { o[0] = v << 16; o[1] = v & 0xffff0000u; }
    else { o[0] = v[0] << 16; o[1] = v[0] & 0xffff0000u; o[2] = v[1] << 16; o[3] = v[1] & 0xffff0000u; }
  }
}

template <typename T, int TN, int UK, int WN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8))) void k_gemm_tn_wide(TnDirectArgs a) {
  // the four wavefronts of a block: WN column tiles of B side by side (all of them read the same rows of A,
  // which then come from HBM once) times WK = 4 / WN interleaved sets of row chunks, added up at the end
  constexpr int TM = 4, CH = 2 * UK, WK = 4 / WN;
  typedef typename RawVec<T, TM>::type AV;
  typedef typename RawVec<T, TN>::type BV;
  __shared__ float red[2][TM * TN * 16 * 64];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 31, h = lane >> 5;
  const int wn = w % WN, kw = w / WN;
  const int m0 = blockIdx.y * (32 * TM), n0 = (blockIdx.z * WN + wn) * (32 * TN);
  const int64_t k_lo = (int64_t)blockIdx.x * a.rows_per_split;
  const int64_t k_hi = k_lo + a.rows_per_split < a.Kd ? k_lo + a.rows_per_split : a.Kd;
  const T* __restrict__ A = reinterpret_cast<const T*>(a.A);
  const T* __restrict__ B = reinterpret_cast<const T*>(a.B);

  // the lane's columns; a request that starts past the operand is moved to column 0 and cleared
  const int ma = m0 + TM * c, nb = n0 + TN * c;
  uint32_t amask[TM], bmask[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) amask[i] = ma + i < a.M ? 0xffffffffu : 0u;
#pragma unroll
  for (int j = 0; j < TN; ++j) bmask[j] = nb + j < a.N ? 0xffffffffu : 0u;
  // a request is (row pair, uniform over the wavefront) + (lane half and column, 32 bits per lane).  Where the
  // split ends on the first row of a pair both lane halves read that row, and a pair past the end reads the
  // first rows of the split; what is not part of the product is cleared when the values are used.
  const bool two_rows = k_lo + 1 < k_hi;
  const uint32_t acol = (uint32_t)((ma < a.M ? ma : 0) * (int64_t)sizeof(T));      // bytes
  const uint32_t bcol = (uint32_t)((nb < a.N ? nb : 0) * (int64_t)sizeof(T));
  const uint32_t aoff = acol + (uint32_t)(h * a.lda * (int64_t)sizeof(T));
  const uint32_t boff = bcol + (uint32_t)(h * a.ldb * (int64_t)sizeof(T));

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  auto load = [&](int64_t k, AV (&av)[UK], BV (&bv)[UK]) {
#pragma unroll
    for (int u = 0; u < UK; ++u) {
      const int64_t kp = k + 2 * u;
      const int64_t kc = kp < k_hi ? kp : k_lo;
      const bool both = kp + 1 < k_hi || (kp >= k_hi && two_rows);          // rows kc and kc + 1 both lie in the split
      av[u] = *reinterpret_cast<const AV*>(reinterpret_cast<const char*>(A + kc * a.lda) + (both ? aoff : acol));
      bv[u] = *reinterpret_cast<const BV*>(reinterpret_cast<const char*>(B + kc * a.ldb) + (both ? boff : bcol));
    }
  };
  int64_t k = k_lo + (int64_t)kw * CH;
  AV an[UK]; BV bn[UK];
  if (k < k_hi) load(k, an, bn);
  for (; k < k_hi; k += WK * CH) {
    float av[UK][TM], bv[UK][TN];
#pragma unroll
    for (int u = 0; u < UK; ++u) {
      const uint32_t rmask = k + 2 * u + h < k_hi ? 0xffffffffu : 0u;   // cleared by a bit mask, never by a branch
      uint32_t ra[TM], rb[TN];
      raw_to_f32<T, TM>(an[u], ra);
      raw_to_f32<T, TN>(bn[u], rb);
#pragma unroll
      for (int i = 0; i < TM; ++i) av[u][i] = __uint_as_float(ra[i] & (amask[i] & rmask));
#pragma unroll
      for (int j = 0; j < TN; ++j) bv[u][j] = __uint_as_float(rb[j] & (bmask[j] & rmask));
    }
    __builtin_amdgcn_sched_barrier(0);
    const int64_t kn = k + WK * CH;
    load(kn < k_hi ? kn : k, an, bn);                      // past the end: the current chunk again, unused
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UK; ++u)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[u][i], bv[u][j], acc[i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }

  // add up the row sets of a column tile
  auto dump = [&](float* buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) buf[((i * TN + j) * 16 + r) * 64 + lane] = acc[i][j][r];
  };
  auto take = [&](const float* buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] += buf[((i * TN + j) * 16 + r) * 64 + lane];
  };
  if constexpr (WK == 4) {               // (2, 3) -> LDS -> (0, 1) add; 1 -> LDS -> 0 adds
    if (kw >= 2) dump(red[kw - 2]);
    __syncthreads();
    if (kw < 2) take(red[kw]);
    __syncthreads();
    if (kw == 1) dump(red[0]);
    __syncthreads();
    if (kw != 0) return;
    take(red[0]);
  } else if constexpr (WK == 2) {        // the second row set of each column tile -> LDS -> the first adds
    if (kw == 1) dump(red[wn]);
    __syncthreads();
    if (kw != 0) return;
    take(red[wn]);
  }
  // register r of lane (c, h) holds the product of A's lane 8 (r / 4) + 4 h + r % 4 and B's lane c
  float* __restrict__ P = a.partial + (int64_t)blockIdx.x * a.M * a.N;
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = nb + j;
      if (n >= a.N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + TM * (8 * (r / 4) + 4 * h + (r % 4)) + i;
        if (m < a.M) P[(int64_t)m * a.N + n] = acc[i][j][r];
      }
    }
}

constexpr int kWideUK1 = 8, kWideUK2 = 8;   // row pairs per request batch (TN = 1, TN = 2)

static bool tn_wide_ok(const void* A, int64_t lda, const void* B, int64_t ldb, int N, int dtype) {
  const bool off = tune().gemm_tn_wide == 0;
  const size_t es = dtype == GCN_BF16 ? 2 : 4;
  if (off || (lda % 4) != 0 || ((uintptr_t)A % (4 * es)) != 0) return false;
  if (lda >= (1 << 28) || ldb >= (1 << 28)) return false;      // a lane's offset (one row + a column, in bytes) is kept in 32 bits
  if (N > 32 && ((ldb % 2) != 0 || ((uintptr_t)B % (2 * es)) != 0)) return false;
  return true;
}

// column tiles of B per block in the vector variant: all of B for up to 256 columns
int tn_wide_wn(int N) { return N <= 64 ? 1 : N <= 128 ? 2 : 4; }

// splits of the vector variant: about two blocks per compute unit
int tn_wide_splits(int64_t Kd, int M, int N) {
  const int blocks = tune().gemm_tn_blocks;
  const int64_t tiles = ceil_div(M, 128) * ceil_div(N, (N <= 32 ? 32 : 64) * tn_wide_wn(N));
  int64_t want = ceil_div(blocks, tiles);
  int64_t max_by_k = ceil_div(Kd, 512);
  int64_t ns = want < max_by_k ? want : max_by_k;
  return (int)(ns < 1 ? 1 : ns);
}

static int tn_direct_tn(int N) { return N <= 32 ? 1 : 2; }

static int tn_direct_splits(int64_t Kd, int M, int N) {
  const int64_t tiles = ceil_div(M, 64) * ceil_div(N, 32 * tn_direct_tn(N));
  int64_t want = ceil_div(1024, tiles);                // about four blocks per compute unit
  int64_t max_by_k = ceil_div(Kd, 512);                // at least 512 rows per block
  int64_t ns = want < max_by_k ? want : max_by_k;
  return (int)(ns < 1 ? 1 : ns);
}

size_t gemm_tn_direct_ws_bytes(int64_t Kd, int M, int N) {
  const int ns = std::max(tn_direct_splits(Kd, M, N), tn_wide_splits(Kd, M, N));
  return std::max(sizeof(float) * (size_t)ns * (size_t)M * (size_t)N, gemm_tn_lds_ws_bytes(Kd, M, N));
}

int gemm_tn_direct_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, int dtype,
                            float* partial, int* nsplit_out, hipStream_t s, int max_blocks) {
  if (dtype == GCN_BF16 && gemm_tn_bf16_ok(A, lda, B, ldb, Kd, M, N))
    return gemm_tn_bf16_partials(A, lda, B, ldb, Kd, M, N, partial, nsplit_out, s);
  if (gemm_tn_lds_ok(A, lda, B, ldb, Kd, M, N, dtype)) return gemm_tn_lds_partials(A, lda, B, ldb, Kd, M, N, partial, nsplit_out, s, max_blocks);
  TnDirectArgs a{A, lda, B, ldb, Kd, M, N, 0, 0, partial};
  if (tn_wide_ok(A, lda, B, ldb, N, dtype)) {
    a.nsplit = tn_wide_splits(Kd, M, N);
    a.rows_per_split = round_up(ceil_div(Kd > 0 ? Kd : 1, a.nsplit), 2 * kTnMaxUK);
    *nsplit_out = a.nsplit;
    const int tnw = N <= 32 ? 1 : 2, wnw = tn_wide_wn(N);
    dim3 grid((unsigned)a.nsplit, (unsigned)ceil_div(M, 128), (unsigned)ceil_div(N, 32 * tnw * wnw));
#define GCN_TN_WIDE(TT)                                                                   \
    if (tnw == 1) k_gemm_tn_wide<TT, 1, kWideUK1, 1><<<grid, 256, 0, s>>>(a);               \
    else if (wnw == 1) k_gemm_tn_wide<TT, 2, kWideUK2, 1><<<grid, 256, 0, s>>>(a);          \
    else if (wnw == 2) k_gemm_tn_wide<TT, 2, kWideUK2, 2><<<grid, 256, 0, s>>>(a);          \
    else k_gemm_tn_wide<TT, 2, kWideUK2, 4><<<grid, 256, 0, s>>>(a);
    if (dtype == GCN_BF16) { GCN_TN_WIDE(bf16_t) } else { GCN_TN_WIDE(float) }
#undef GCN_TN_WIDE
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  }
  a.nsplit = tn_direct_splits(Kd, M, N);
  a.rows_per_split = round_up(ceil_div(Kd > 0 ? Kd : 1, a.nsplit), 2 * kTnMaxUK);
  *nsplit_out = a.nsplit;
  const int tn = tn_direct_tn(N);
  dim3 grid((unsigned)a.nsplit, (unsigned)ceil_div(M, 64), (unsigned)ceil_div(N, 32 * tn));
  if (dtype == GCN_BF16) {
    if (tn == 1) k_gemm_tn_direct<bf16_t, 2, 1, 8><<<grid, 256, 0, s>>>(a);
    else k_gemm_tn_direct<bf16_t, 2, 2, 4><<<grid, 256, 0, s>>>(a);
  } else {
    if (tn == 1) k_gemm_tn_direct<float, 2, 1, 8><<<grid, 256, 0, s>>>(a);
    else k_gemm_tn_direct<float, 2, 2, 4><<<grid, 256, 0, s>>>(a);
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

}  // namespace gcn
