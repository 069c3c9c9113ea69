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
// Shapes: N <= 256 (N not a multiple of 16 only where the rows of C are padded to the store width), K = 32, 64,
// 128, 256 with 16-byte requests or any K <= 128 with 8-byte requests (rows of A aligned accordingly), W (as bf16)
// within 128 KB of LDS.  Everything else stays on the fp32 path.
#include <stdlib.h>

#include "common.h"

namespace gcn {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct NnBf16Args {
  const bf16_t* A; int64_t lda; const float* W; int64_t ldw; bf16_t* C; int64_t ldc;
  int64_t M; int N; int K;
  const float* bias; int relu; const bf16_t* mask; int64_t ldmask; bf16_t* C2; int64_t ldc2;
  int wide_requests;      // rows of A aligned to 16 bytes and K in {32, 64, 128, 256}: 16-byte requests, 16x16x32 MFMA
};

constexpr int kThreads = 512;

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
  // columns are stored (and mask values read) in groups of 8 (pairs) or 4; groups that start at or past N rounded
  // up to the group width are skipped, the last kept group may reach into the padding of the row (the host checks
  // that the rows are that long)
  const int n_up = kPair ? (a.N + 7) & ~7 : (a.N + 3) & ~3;
  extern __shared__ u32x4 lds_bf16[];                 // [k step][column tile][lane]: LV values of W as bf16
  Raw* Wl = reinterpret_cast<Raw*>(lds_bf16);
  {
    bf16_t* wl = reinterpret_cast<bf16_t*>(lds_bf16);
    for (int e = threadIdx.x; e < KL * KS * NT * 16; e += kThreads) {      // zero beyond K and N
      const int k = e / (NT * 16), n = e % (NT * 16);
      const int s = k / KS, q = (k % KS) / LV, el = k % LV;
      int t = n >> 4, cc = n & 15;
      if constexpr (kPair) {           // column n is entry 4 (n % 32 / 8) + n % 4 of tile 2 (n / 32) + (n % 8) / 4
        t = 2 * (n >> 5) + ((n & 7) >> 2);
        cc = 4 * ((n & 31) >> 3) + (n & 3);
      }
      wl[(((s * NT + t) * 64 + q * 16 + cc) * LV) + el] = (k < a.K && n < a.N) ? f32_to_bf16(a.W[(int64_t)k * a.ldw + n]) : (bf16_t)0;
    }
  }
  __syncthreads();

  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int c = lane & 15, q = lane >> 4;
  constexpr int WPB = kThreads / 64;
  const int64_t ntiles = (a.M + 15) / 16;
  const int64_t stride = (int64_t)gridDim.x * WPB;

  // K that is no multiple of the k step (8-byte requests only): the lane's request of the last step may start
  // past K (moved to column 0) or reach past it; `tail` clears what is not part of the product when it is used
  const int k_last = KS * (KL - 1) + LV * q;                    // first k of the lane's request in the last step
  const int n_ok = a.K - k_last;                                // elements of it below K
  const int last_off = n_ok > 0 ? k_last : 0;
  u32x2 tail = u32x2{0xffffffffu, 0xffffffffu};
  if (n_ok < 4) tail = u32x2{n_ok >= 2 ? 0xffffffffu : n_ok == 1 ? 0x0000ffffu : 0u, n_ok == 3 ? 0x0000ffffu : 0u};
  auto load_a = [&](int64_t tile, Raw (&av)[KL]) {
    const int64_t row = tile * 16 + c;
    const bf16_t* __restrict__ arow = a.A + (row < a.M ? row : a.M - 1) * a.lda;
#pragma unroll
    for (int s = 0; s < KL; ++s) av[s] = *reinterpret_cast<const Raw*>(arow + (s == KL - 1 ? last_off : KS * s + LV * q));
  };

  int64_t tile = (int64_t)blockIdx.x * WPB + w;
  if (tile >= ntiles) return;
  Raw a_nxt[KL];
  load_a(tile, a_nxt);
  for (; tile < ntiles; tile += stride) {
    Raw av[KL];
#pragma unroll
    for (int s = 0; s < KL; ++s) av[s] = a_nxt[s];
    if constexpr (LV == 4) av[KL - 1] = u32x2{av[KL - 1][0] & tail[0], av[KL - 1][1] & tail[1]};
    load_a(tile + stride < ntiles ? tile + stride : ntiles - 1, a_nxt);     // past the end: a valid, unused request
    u32x2 keep[MASK ? NT : 1];
    const int64_t m = tile * 16 + c;
    const int64_t mc = m < a.M ? m : a.M - 1;
    if constexpr (MASK) {
      if constexpr (kPair) {
#pragma unroll
        for (int j = 0; j < NT / 2; ++j) {
          const int n = 32 * j + 8 * q;
          const u32x4 kv = *reinterpret_cast<const u32x4*>(a.mask + mc * a.ldmask + (n < n_up ? n : 0));
          keep[2 * j] = u32x2{kv[0], kv[1]}; keep[2 * j + 1] = u32x2{kv[2], kv[3]};
        }
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int n = 16 * t + 4 * q;
          keep[t] = *reinterpret_cast<const u32x2*>(a.mask + mc * a.ldmask + (n < n_up ? n : 0));
        }
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
          pre[r] = acc[t][r] + ((a.bias && n + r < a.N) ? a.bias[n + r] : 0.f);
          v[r] = a.relu ? (pre[r] > 0.f ? pre[r] : 0.f) : pre[r];
          if constexpr (MASK) v[r] = kp[r] > 0.f ? v[r] : 0.f;
        }
        out[t] = u32x2{(uint32_t)f32_to_bf16(v[0]) | ((uint32_t)f32_to_bf16(v[1]) << 16), (uint32_t)f32_to_bf16(v[2]) | ((uint32_t)f32_to_bf16(v[3]) << 16)};
        if constexpr (SAVE)
          out2[t] = u32x2{(uint32_t)f32_to_bf16(pre[0]) | ((uint32_t)f32_to_bf16(pre[1]) << 16), (uint32_t)f32_to_bf16(pre[2]) | ((uint32_t)f32_to_bf16(pre[3]) << 16)};
      }
      if constexpr (kPair) {
#pragma unroll
        for (int j = 0; j < NT / 2; ++j) {
          const int n = 32 * j + 8 * q;
          if (n >= n_up) continue;
          if constexpr (SAVE)
            *reinterpret_cast<u32x4*>(a.C2 + m * a.ldc2 + n) = u32x4{out2[2 * j][0], out2[2 * j][1], out2[2 * j + 1][0], out2[2 * j + 1][1]};
          *reinterpret_cast<u32x4*>(a.C + m * a.ldc + n) = u32x4{out[2 * j][0], out[2 * j][1], out[2 * j + 1][0], out[2 * j + 1][1]};
        }
      } else {
#pragma unroll
        for (int t = 0; t < NT; ++t) {
          const int n = t * 16 + 4 * q;
          if (n >= n_up) continue;
          if constexpr (SAVE) *reinterpret_cast<u32x2*>(a.C2 + m * a.ldc2 + n) = out2[t];
          *reinterpret_cast<u32x2*>(a.C + m * a.ldc + n) = out[t];
        }
      }
    }
  }
}

template <int NT, int KL, int LV>
int launch(const NnBf16Args& a, hipStream_t s) {
  const size_t lds = (size_t)KL * 4 * LV * NT * 16 * sizeof(bf16_t);
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
  if (a.wide_requests) {
    switch (a.K) {
      case 32: return launch<NT, 1, 8>(a, s);
      case 64: return launch<NT, 2, 8>(a, s);
      case 128: return launch<NT, 4, 8>(a, s);
      default: return launch<NT, 8, 8>(a, s);
    }
  }
  switch ((a.K + 15) / 16) {
    case 1: return launch<NT, 1, 4>(a, s);
    case 2: return launch<NT, 2, 4>(a, s);
    case 3: return launch<NT, 3, 4>(a, s);
    case 4: return launch<NT, 4, 4>(a, s);
    case 5: return launch<NT, 5, 4>(a, s);
    case 6: return launch<NT, 6, 4>(a, s);
    case 7: return launch<NT, 7, 4>(a, s);
    default: return launch<NT, 8, 4>(a, s);
  }
}

bool aligned_rows(const void* p, int64_t ld, int bytes) {
  return p == nullptr || (((uintptr_t)p % bytes) == 0 && ((ld * 2) % bytes) == 0);
}

// ---- dW = A^T B ---------------------------------------------------------------------------------------------
// The bf16 MFMA takes 4 consecutive k (rows of A and B) per lane, the operands are stored with the columns
// contiguous: a lane reads 4 columns of 4 rows (rows k + 4 h .. + 3 of an 8-row group for lane half h) and
// transposes the 4 x 4 block in registers with byte permutes.  As in the fp32 vector-request kernel, component i
// of a request is the operand of column tile i (tile i holds the columns {4 c + i} of A, {TN c + j} of B), the
// four wavefronts of a block take WN column tiles of B side by side times 4 / WN interleaved sets of row chunks,
// and the next chunk of 32 rows is requested before the MFMAs of the current one.
struct TnBf16Args {
  const bf16_t* A; int64_t lda; const bf16_t* B; int64_t ldb;
  int64_t Kd; int M; int N; int64_t rows_per_split; float* partial;
};

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <int TN> struct BRaw;
template <> struct BRaw<2> { typedef uint32_t type; };
template <> struct BRaw<1> { typedef uint16_t type; };

template <int TN, int WN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 8))) void k_gemm_tn_bf16(TnBf16Args a) {
  constexpr int TM = 4, UK = 4, CH = 8 * UK, WK = 4 / WN;
  typedef typename BRaw<TN>::type BR;
  __shared__ float red[2][TM * TN * 16 * 64];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 31, h = lane >> 5;
  const int wn = w % WN, kw = w / WN;
  const int m0 = blockIdx.y * (32 * TM), n0 = (blockIdx.z * WN + wn) * (32 * TN);
  const int64_t k_lo = (int64_t)blockIdx.x * a.rows_per_split;
  const int64_t k_hi = k_lo + a.rows_per_split < a.Kd ? k_lo + a.rows_per_split : a.Kd;
  // a request = (first row of the split: uniform) + (row inside the split and column: 32 bits per lane); columns
  // past the operand are moved to column 0: they only reach results that are never stored
  const int ma = m0 + TM * c, nb = n0 + TN * c;
  const uint32_t acol = (uint32_t)((ma < a.M ? ma : 0) * 2), bcol = (uint32_t)((nb < a.N ? nb : 0) * 2);
  const uint32_t lda_b = (uint32_t)(a.lda * 2), ldb_b = (uint32_t)(a.ldb * 2);
  const char* __restrict__ Ab = reinterpret_cast<const char*>(a.A + k_lo * a.lda);
  const char* __restrict__ Bb = reinterpret_cast<const char*>(a.B + k_lo * a.ldb);
  const uint32_t n_rows = k_hi > k_lo ? (uint32_t)(k_hi - k_lo) : 0u;

  floatx16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // rows r0 + 8 u + 4 h + r of the split (r0 relative to k_lo); a row past the split repeats its last row
  auto load = [&](uint32_t r0, u32x2 (&ar)[UK][4], BR (&br)[UK][4]) {
#pragma unroll
    for (int u = 0; u < UK; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t row = r0 + 8 * u + 4 * h + r;
        const uint32_t rc = row < n_rows ? row : n_rows - 1;
        ar[u][r] = *reinterpret_cast<const u32x2*>(Ab + rc * lda_b + acol);
        br[u][r] = *reinterpret_cast<const BR*>(Bb + rc * ldb_b + bcol);
      }
  };
  uint32_t r0 = (uint32_t)kw * CH;
  u32x2 an[UK][4]; BR bn[UK][4];
  if (r0 < n_rows) load(r0, an, bn);
  for (; r0 < n_rows; r0 += WK * CH) {
    u32x2 ac[UK][4]; uint32_t bc[UK][4];
#pragma unroll
    for (int u = 0; u < UK; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const uint32_t rm = r0 + 8 * u + 4 * h + r < n_rows ? 0xffffffffu : 0u;   // cleared by a bit mask, never by a branch
        ac[u][r] = u32x2{an[u][r][0] & rm, an[u][r][1] & rm};
        bc[u][r] = (uint32_t)bn[u][r] & rm;
      }
    __builtin_amdgcn_sched_barrier(0);
    const uint32_t rn = r0 + WK * CH;
    load(rn < n_rows ? rn : r0, an, bn);                    // past the end: the current chunk again, unused
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int u = 0; u < UK; ++u) {
      // 4 x 4 transposes: operand of tile i = column i of the block, rows 0..3 as 4 bf16
      u32x2 ao[TM], bo[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const uint32_t sel = (i & 1) ? 0x07060302u : 0x05040100u;
        ao[i] = u32x2{__builtin_amdgcn_perm(ac[u][1][i >> 1], ac[u][0][i >> 1], sel),
                      __builtin_amdgcn_perm(ac[u][3][i >> 1], ac[u][2][i >> 1], sel)};
      }
      if constexpr (TN == 2) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const uint32_t sel = (j & 1) ? 0x07060302u : 0x05040100u;
          bo[j] = u32x2{__builtin_amdgcn_perm(bc[u][1], bc[u][0], sel), __builtin_amdgcn_perm(bc[u][3], bc[u][2], sel)};
        }
      } else {
        bo[0] = u32x2{bc[u][0] | (bc[u][1] << 16), bc[u][2] | (bc[u][3] << 16)};
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          short4v x, y;
          __builtin_memcpy(&x, &ao[i], 8); __builtin_memcpy(&y, &bo[j], 8);
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(x, y, acc[i][j], 0, 0, 0);
        }
    }
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

}  // namespace

static int nn_tiles_bf16(int N) { return N <= 16 ? 1 : N <= 32 ? 2 : N <= 48 ? 3 : N <= 64 ? 4 : N <= 128 ? 8 : 16; }
static bool wide_requests(const void* A, int64_t lda, int K) {
  return (K == 32 || K == 64 || K == 128 || K == 256) && aligned_rows(A, lda, 16);
}

bool gemm_nn_bf16_ok(const void* A, int64_t lda, void* C, int64_t ldc, int64_t M, int N, int K, const GemmEpilogue& epi) {
  const bool off = tune().gemm_bf16 == 0;
  if (off || M < 1 || N < 1 || N > 256 || K < 1) return false;
  const int NT = nn_tiles_bf16(N);
  const bool wide = wide_requests(A, lda, K);
  if (!wide && (K > 128 || !aligned_rows(A, lda, 8) || lda < ((K + 3) & ~3))) return false;
  const int kpad = wide ? K : ((K + 15) & ~15);
  if ((size_t)kpad * NT * 16 * 2 > 128 * 1024) return false;
  // stores and mask loads come in groups of 8 (even tile count) or 4 columns: the rows must hold whole groups
  const int g = NT % 2 == 0 ? 8 : 4;
  const int64_t n_up = (N + g - 1) / g * g;
  if (!aligned_rows(C, ldc, 2 * g) || ldc < n_up) return false;
  if (epi.C2 && (!aligned_rows(epi.C2, epi.ldc2, 2 * g) || epi.ldc2 < n_up)) return false;
  if (epi.mask && (!aligned_rows(epi.mask, epi.ldmask, 2 * g) || epi.ldmask < n_up || epi.mask_rows < M || epi.C2)) return false;
  return true;
}

int gemm_nn_bf16(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N, int K,
                 const GemmEpilogue& epi, hipStream_t s) {
  NnBf16Args a{(const bf16_t*)A, lda, W, ldw, (bf16_t*)C, ldc, M, N, K,
               epi.bias, epi.relu, (const bf16_t*)epi.mask, epi.ldmask, (bf16_t*)epi.C2, epi.ldc2,
               wide_requests(A, lda, K) ? 1 : 0};
  switch (nn_tiles_bf16(N)) {
    case 1: return launch_k<1>(a, s);
    case 2: return launch_k<2>(a, s);
    case 3: return launch_k<3>(a, s);
    case 4: return launch_k<4>(a, s);
    case 8: return launch_k<8>(a, s);
    default: return launch_k<16>(a, s);
  }
}

bool gemm_tn_bf16_ok(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N) {
  const bool off = tune().gemm_bf16 == 0;
  if (off || Kd < 1 || M < 1 || N < 1) return false;
  if ((lda % 4) != 0 || ((uintptr_t)A % 8) != 0) return false;
  if (N > 32 && ((ldb % 2) != 0 || ((uintptr_t)B % 4) != 0)) return false;
  // 32-bit byte offsets inside a row split
  const int64_t rows = round_up(ceil_div(Kd, tn_wide_splits(Kd, M, N)), 32);
  return (double)rows * (double)(lda > ldb ? lda : ldb) * 2.0 < 4.0e9;
}

int gemm_tn_bf16_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, float* partial,
                          int* nsplit_out, hipStream_t s) {
  TnBf16Args a{(const bf16_t*)A, lda, (const bf16_t*)B, ldb, Kd, M, N, 0, partial};
  const int ns = tn_wide_splits(Kd, M, N);
  a.rows_per_split = round_up(ceil_div(Kd, ns), 32);
  *nsplit_out = ns;
  const int tnw = N <= 32 ? 1 : 2, wnw = tn_wide_wn(N);
  dim3 grid((unsigned)ns, (unsigned)ceil_div(M, 128), (unsigned)ceil_div(N, 32 * tnw * wnw));
  if (tnw == 1) k_gemm_tn_bf16<1, 1><<<grid, 256, 0, s>>>(a);
  else if (wnw == 1) k_gemm_tn_bf16<2, 1><<<grid, 256, 0, s>>>(a);
  else if (wnw == 2) k_gemm_tn_bf16<2, 2><<<grid, 256, 0, s>>>(a);
  else k_gemm_tn_bf16<2, 4><<<grid, 256, 0, s>>>(a);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

}  // namespace gcn
