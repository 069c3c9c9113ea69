// Dense product C = epilogue(A W) for bf16 features on the bf16 matrix pipe (gfx950).
//
// The bf16 variant keeps features, activations and gradients in bf16 and the weights in fp32; the
// products accumulate in fp32.  Feeding the fp32 MFMA with widened values (gemm_direct.hip) runs at
// the fp32 matrix rate; here W is rounded to bf16 once per launch, when it is placed in LDS, and the
// product runs on v_mfma_f32_16x16x32_bf16 (16x16x16 for K = 16).  One more rounding of W (2^-9
// relative per term) stays far inside the bf16 tolerance of the products, 2e-2 * sum |terms|.  At
// sixteen times the fp32 matrix rate the kernel is a streaming kernel: it is bound by reading A and
// writing C.
//
// Shapes: N = 16 NT <= 256, K = 16, 32, 64, 128 or 256, rows of A / C / mask aligned to 16 bytes
// (8 for K = 16), W (as bf16) within 128 KB of LDS.  Everything else stays on the fp32 path.
#include <stdlib.h>

#include "common.h"

namespace gcn {

namespace {

typedef uint16_t bf16_t;
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct NnBf16Args {
  const bf16_t* A; int64_t lda; const float* W; int64_t ldw; bf16_t* C; int64_t ldc;
  int64_t M; int N; int K;
  const float* bias; int relu; const bf16_t* mask; int64_t ldmask; bf16_t* C2; int64_t ldc2;
};

constexpr int kThreads = 512;

__device__ __forceinline__ bf16_t to_bf16(float f) {   // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// LV bf16 values per lane and k step: 8 -> one 16-byte request and a 16x16x32 MFMA, 4 -> 8 bytes and 16x16x16
template <int LV> struct Frag;
template <> struct Frag<8> { typedef u32x4 raw; };
template <> struct Frag<4> { typedef u32x2 raw; };

template <int LV>
__device__ __forceinline__ floatx4 mfma(const typename Frag<LV>::raw& w, const typename Frag<LV>::raw& x, floatx4 acc) {
  if constexpr (LV == 8) {
    bf16x8 a, b;
    __builtin_memcpy(&a, &w, 16); __builtin_memcpy(&b, &x, 16);
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc, 0, 0, 0);
  } else {
    short4v a, b;
    __builtin_memcpy(&a, &w, 8); __builtin_memcpy(&b, &x, 8);
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a, b, acc, 0, 0, 0);
  }
}

__device__ __forceinline__ void unpack4(const u32x2& v, float (&o)[4]) {
  o[0] = __uint_as_float(v[0] << 16); o[1] = __uint_as_float(v[0] & 0xffff0000u);
  o[2] = __uint_as_float(v[1] << 16); o[3] = __uint_as_float(v[1] & 0xffff0000u);
}

// One wavefront per tile of 16 rows.  Lane (c, q) = (lane % 16, lane / 16) supplies row c of the tile as the
// second MFMA operand (k = KS s + LV q .. + LV - 1 of k step s, KS = 4 LV) and the column 16 t + c of W as the
// first, so register r of its accumulator t is column 16 t + 4 q + r of row c: four consecutive outputs.
// KL = K / KS k steps per tile; the next tile's rows are requested before the current tile's MFMAs.
template <int NT, int KL, int LV, bool MASK, bool SAVE>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(2, 8))) void k_gemm_nn_bf16(NnBf16Args a) {
  typedef typename Frag<LV>::raw Raw;
  constexpr int KS = 4 * LV;
  // With an even number of column tiles the columns are dealt to the tiles so that a lane's results of the
  // tiles 2 j and 2 j + 1 are 8 consecutive columns, 32 j + 8 q .. + 7: one 16-byte store (and mask load) per
  // pair, and the four lanes of a row write 64 contiguous bytes.  (The MFMA only sees a permuted W.)
  constexpr bool kPair = NT % 2 == 0;
  extern __shared__ u32x4 lds_bf16[];                 // [k step][column tile][lane]: LV values of W as bf16
  Raw* Wl = reinterpret_cast<Raw*>(lds_bf16);
  {
    bf16_t* wl = reinterpret_cast<bf16_t*>(lds_bf16);
    for (int e = threadIdx.x; e < a.K * NT * 16; e += kThreads) {
      const int k = e / (NT * 16), n = e % (NT * 16);
      const int s = k / KS, q = (k % KS) / LV, el = k % LV;
      int t = n >> 4, cc = n & 15;
      if constexpr (kPair) {           // column n is entry 4 (n % 32 / 8) + n % 4 of tile 2 (n / 32) + (n % 8) / 4
        t = 2 * (n >> 5) + ((n & 7) >> 2);
        cc = 4 * ((n & 31) >> 3) + (n & 3);
      }
      wl[(((s * NT + t) * 64 + q * 16 + cc) * LV) + el] = to_bf16(a.W[(int64_t)k * a.ldw + n]);
    }
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, q = lane >> 4;
  constexpr int WPB = kThreads / 64;
  const int64_t ntiles = (a.M + 15) / 16;
  const int64_t stride = (int64_t)gridDim.x * WPB;

  auto load_a = [&](int64_t tile, Raw (&av)[KL]) {
    const int64_t row = tile * 16 + c;
    const bf16_t* __restrict__ arow = a.A + (row < a.M ? row : a.M - 1) * a.lda + LV * q;
#pragma unroll
    for (int s = 0; s < KL; ++s) av[s] = *reinterpret_cast<const Raw*>(arow + KS * s);
  };

  int64_t tile = (int64_t)blockIdx.x * WPB + w;
  if (tile >= ntiles) return;
  Raw a_nxt[KL];
  load_a(tile, a_nxt);
  for (; tile < ntiles; tile += stride) {
    Raw av[KL];
#pragma unroll
    for (int s = 0; s < KL; ++s) av[s] = a_nxt[s];
    load_a(tile + stride < ntiles ? tile + stride : ntiles - 1, a_nxt);     // past the end: a valid, unused request
    u32x2 keep[MASK ? NT : 1];
    const int64_t m = tile * 16 + c;
    const int64_t mc = m < a.M ? m : a.M - 1;
    if constexpr (MASK) {
      if constexpr (kPair) {
#pragma unroll
        for (int j = 0; j < NT / 2; ++j) {
          const u32x4 kv = *reinterpret_cast<const u32x4*>(a.mask + mc * a.ldmask + 32 * j + 8 * q);
          keep[2 * j] = u32x2{kv[0], kv[1]}; keep[2 * j + 1] = u32x2{kv[2], kv[3]};
        }
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) keep[t] = *reinterpret_cast<const u32x2*>(a.mask + mc * a.ldmask + 16 * t + 4 * q);
      }
    }
    floatx4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
    // the fragments of W for up to 8 column tiles are read, then used; scheduling barriers keep the compiler
    // from hoisting all K / KS x NT reads to the top, which needs more registers than there are
    constexpr int TB = NT < 8 ? NT : 8;
#pragma unroll
    for (int s = 0; s < KL; ++s)
#pragma unroll
      for (int t0 = 0; t0 < NT; t0 += TB) {
        Raw wf[TB];
#pragma unroll
        for (int t = 0; t < TB; ++t) wf[t] = Wl[(s * NT + t0 + t) * 64 + lane];
#pragma unroll
        for (int t = 0; t < TB; ++t) acc[t0 + t] = mfma<LV>(wf[t], av[s], acc[t0 + t]);
        __builtin_amdgcn_sched_barrier(0);
      }

    if (m < a.M) {
      u32x2 out[NT], out2[SAVE ? NT : 1];
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        const int n = kPair ? 32 * (t / 2) + 8 * q + 4 * (t % 2) : t * 16 + 4 * q;
        float v[4], pre[4], kp[4];
        if constexpr (MASK) unpack4(keep[t], kp);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          pre[r] = acc[t][r] + (a.bias ? a.bias[n + r] : 0.f);
          v[r] = a.relu ? (pre[r] > 0.f ? pre[r] : 0.f) : pre[r];
          if constexpr (MASK) v[r] = kp[r] > 0.f ? v[r] : 0.f;
        }
        out[t] = u32x2{(uint32_t)to_bf16(v[0]) | ((uint32_t)to_bf16(v[1]) << 16), (uint32_t)to_bf16(v[2]) | ((uint32_t)to_bf16(v[3]) << 16)};
        if constexpr (SAVE)
          out2[t] = u32x2{(uint32_t)to_bf16(pre[0]) | ((uint32_t)to_bf16(pre[1]) << 16), (uint32_t)to_bf16(pre[2]) | ((uint32_t)to_bf16(pre[3]) << 16)};
      }
      if constexpr (kPair) {
#pragma unroll
        for (int j = 0; j < NT / 2; ++j) {
          const int n = 32 * j + 8 * q;
          if constexpr (SAVE)
            *reinterpret_cast<u32x4*>(a.C2 + m * a.ldc2 + n) = u32x4{out2[2 * j][0], out2[2 * j][1], out2[2 * j + 1][0], out2[2 * j + 1][1]};
          *reinterpret_cast<u32x4*>(a.C + m * a.ldc + n) = u32x4{out[2 * j][0], out[2 * j][1], out[2 * j + 1][0], out[2 * j + 1][1]};
        }
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int n = t * 16 + 4 * q;
          if constexpr (SAVE) *reinterpret_cast<u32x2*>(a.C2 + m * a.ldc2 + n) = out2[t];
          *reinterpret_cast<u32x2*>(a.C + m * a.ldc + n) = out[t];
        }
      }
    }
  }
}

template <int NT, int KL, int LV>
int launch(const NnBf16Args& a, hipStream_t s) {
  const size_t lds = (size_t)a.K * NT * 16 * sizeof(bf16_t);
  const int64_t ntiles = ceil_div(a.M, 16);
  const int per_cu = lds > 64 * 1024 ? 1 : 2;
  int64_t blocks = ceil_div(ntiles, kThreads / 64);
  if (blocks > 256 * per_cu) blocks = 256 * per_cu;
  auto go = [&](auto kern) -> int {
    GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    kern<<<dim3((unsigned)blocks), dim3(kThreads), lds, s>>>(a);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  };
  if (a.mask) return go(k_gemm_nn_bf16<NT, KL, LV, true, false>);
  return a.C2 ? go(k_gemm_nn_bf16<NT, KL, LV, false, true>) : go(k_gemm_nn_bf16<NT, KL, LV, false, false>);
}

template <int NT>
int launch_k(const NnBf16Args& a, hipStream_t s) {
  switch (a.K) {
    case 16: return launch<NT, 1, 4>(a, s);
    case 32: return launch<NT, 1, 8>(a, s);
    case 64: return launch<NT, 2, 8>(a, s);
    case 128: return launch<NT, 4, 8>(a, s);
    default: return launch<NT, 8, 8>(a, s);
  }
}

bool aligned_rows(const void* p, int64_t ld, int bytes) {
  return p == nullptr || (((uintptr_t)p % bytes) == 0 && ((ld * 2) % bytes) == 0);
}

}  // namespace

bool gemm_nn_bf16_ok(const void* A, int64_t lda, void* C, int64_t ldc, int64_t M, int N, int K, const GemmEpilogue& epi) {
  static const bool off = getenv("GCN_GEMM_BF16") && atoi(getenv("GCN_GEMM_BF16")) == 0;
  if (off || M < 1 || N < 16 || N > 256 || (N % 16) != 0 || N / 16 == 5 || N / 16 == 6 || N / 16 == 7 || (N > 128 && N != 256)) return false;
  if (K != 16 && K != 32 && K != 64 && K != 128 && K != 256) return false;
  if ((size_t)K * N * 2 > 128 * 1024) return false;
  const int ob = (N / 16) % 2 == 0 ? 16 : 8;          // bytes per store / mask load
  if (!aligned_rows(A, lda, K == 16 ? 8 : 16) || !aligned_rows(C, ldc, ob) || !aligned_rows(epi.C2, epi.ldc2, ob)) return false;
  if (epi.mask && (!aligned_rows(epi.mask, epi.ldmask, ob) || epi.mask_rows < M || epi.C2)) return false;
  return true;
}

int gemm_nn_bf16(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N, int K,
                 const GemmEpilogue& epi, hipStream_t s) {
  NnBf16Args a{(const bf16_t*)A, lda, W, ldw, (bf16_t*)C, ldc, M, N, K,
               epi.bias, epi.relu, (const bf16_t*)epi.mask, epi.ldmask, (bf16_t*)epi.C2, epi.ldc2};
  switch (N / 16) {
    case 1: return launch_k<1>(a, s);
    case 2: return launch_k<2>(a, s);
    case 3: return launch_k<3>(a, s);
    case 4: return launch_k<4>(a, s);
    case 8: return launch_k<8>(a, s);
    default: return launch_k<16>(a, s);
  }
}

}  // namespace gcn
