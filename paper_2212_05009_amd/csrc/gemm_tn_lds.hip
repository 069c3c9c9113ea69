// Partial products of C[M x N] = A[Kd x M]^T B[Kd x N] (Sec. 3.2: the weight gradient (A^ H)^T G, a sum over all
// rows of the block) for wide fp32 operands: the whole output of a workgroup lives in registers, both operands
// stream through LDS.
//
// A workgroup of four wavefronts owns up to 256 x 256 elements of C for one range of rows (a split of the sum).
// Its wavefronts form a WM x WN grid; each accumulates TMW x TNW tiles of 32 x 32 (at 4 x 4: 256 registers per
// lane, the accumulator half of the register file).  Chunks of 32 rows of both operands are copied from global
// memory straight into LDS (global_load_lds, 16 bytes per lane, one instruction per row), a whole chunk ahead of
// their use, into the other half of a double buffer; the wavefronts meet once per chunk.  The inner loop is LDS
// reads and MFMAs only: a pair of rows costs TMW + TNW four-byte LDS reads per lane for TMW TNW MFMAs.
//
// Operand layout of v_mfma_f32_32x32x2f32: lane l supplies A^T[m = l % 32][k = l / 32] and B[k = l / 32][n = l % 32],
// i.e. both operands are read along a row of the chunk, consecutive lanes at consecutive addresses: no transposition
// anywhere.  The two halves of a wavefront read rows k and k + 1, 1 KB apart; odd rows are stored with their
// 32-column tiles swapped in pairs (the copy fetches quad q ^ 8), so the halves fall on different banks.
#include "common.h"

namespace gcn {

typedef float floatx16 __attribute__((ext_vector_type(16)));

struct TnLdsArgs {
  const float* A; int64_t lda; const float* B; int64_t ldb;
  int64_t Kd; int M; int N; int64_t rows_per_split;
  int wm, wn;          // wavefront grid, wm * wn = 4
  int mblocks;         // blocks of 256 columns of A
  float* partial;      // [nsplit][M * N]
};

constexpr int kTnlKC = 32;                               // rows per chunk
constexpr int kTnlOpFloats = kTnlKC * 256;               // one operand's chunk: 32 rows of 64 quads
constexpr int kTnlBufFloats = 2 * kTnlOpFloats;          // A's chunk, then B's
constexpr size_t kTnlLdsBytes = 2 * sizeof(float) * kTnlBufFloats;

template <int TMW, int TNW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_tn_lds(TnLdsArgs a) {
  extern __shared__ float S[];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 31, h = lane >> 5;
  const int mb = (int)blockIdx.y % a.mblocks, nb = (int)blockIdx.y / a.mblocks;
  const int m0 = 256 * mb, n0 = 256 * nb;
  const int mwid = a.M - m0 < 256 ? a.M - m0 : 256, nwid = a.N - n0 < 256 ? a.N - n0 : 256;
  const int64_t k_lo = (int64_t)blockIdx.x * a.rows_per_split;
  const int64_t k_hi = k_lo + a.rows_per_split < a.Kd ? k_lo + a.rows_per_split : a.Kd;
  const int mt0 = (w / a.wn) * TMW, nt0 = (w % a.wn) * TNW;      // this wavefront's first tiles
  const float* __restrict__ A = a.A + m0;
  const float* __restrict__ B = a.B + n0;

  // wavefront w copies rows w, w + 4, ... of both operands' chunks; rows past the end repeat the last row (they are
  // cleared in LDS before use), quads past the width repeat the first (they only meet columns that are not stored)
  const int q = lane ^ (8 * (w & 1));                 // rows w + 4 t all have the parity of w
  const int colA = 4 * q < mwid ? 4 * q : 0, colB = 4 * q < nwid ? 4 * q : 0;
  auto copy_chunk = [&](int64_t k, int b) {
    float* dst = S + b * kTnlBufFloats + w * 256;
#pragma unroll
    for (int t = 0; t < kTnlKC / 4; ++t) {
      const int64_t row = k + w + 4 * t < a.Kd ? k + w + 4 * t : a.Kd - 1;
      __builtin_amdgcn_global_load_lds(A + row * a.lda + colA, dst + t * 1024, 16, 0, 0);
    }
#pragma unroll
    for (int t = 0; t < kTnlKC / 4; ++t) {
      const int64_t row = k + w + 4 * t < a.Kd ? k + w + 4 * t : a.Kd - 1;
      __builtin_amdgcn_global_load_lds(B + row * a.ldb + colB, dst + kTnlOpFloats + t * 1024, 16, 0, 0);
    }
  };

  floatx16 acc[TMW][TNW];
#pragma unroll
  for (int i = 0; i < TMW; ++i)
#pragma unroll
    for (int j = 0; j < TNW; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // a lane's element of tile t in the row of its half: the row (h), the tile as stored in a row of that parity, c
  int offA[TMW], offB[TNW];
#pragma unroll
  for (int i = 0; i < TMW; ++i) offA[i] = h * 256 + 32 * ((mt0 + i) ^ h) + c;
#pragma unroll
  for (int j = 0; j < TNW; ++j) offB[j] = kTnlOpFloats + h * 256 + 32 * ((nt0 + j) ^ h) + c;

  if (k_lo < k_hi) {
    copy_chunk(k_lo, 0);
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    int b = 0;
    for (int64_t k = k_lo; k < k_hi; k += kTnlKC, b ^= 1) {
      if (k + kTnlKC < k_hi) copy_chunk(k + kTnlKC, b ^ 1);
      float* sb = S + b * kTnlBufFloats;
      if (k + kTnlKC > k_hi) {                       // the last, shorter chunk of the sum: rows past the end count as zero
        const int valid = (int)(k_hi - k);
        for (int r = valid + w; r < kTnlKC; r += 4) {
          *reinterpret_cast<float4*>(sb + r * 256 + 4 * lane) = float4{0.f, 0.f, 0.f, 0.f};
          *reinterpret_cast<float4*>(sb + kTnlOpFloats + r * 256 + 4 * lane) = float4{0.f, 0.f, 0.f, 0.f};
        }
        __syncthreads();
      }
      float av[TMW], bv[TNW], an[TMW], bn[TNW];
#pragma unroll
      for (int i = 0; i < TMW; ++i) an[i] = sb[offA[i]];
#pragma unroll
      for (int j = 0; j < TNW; ++j) bn[j] = sb[offB[j]];
#pragma unroll
      for (int p = 0; p < kTnlKC / 2; ++p) {
#pragma unroll
        for (int i = 0; i < TMW; ++i) av[i] = an[i];
#pragma unroll
        for (int j = 0; j < TNW; ++j) bv[j] = bn[j];
        if (p + 1 < kTnlKC / 2) {
#pragma unroll
          for (int i = 0; i < TMW; ++i) an[i] = sb[offA[i] + 512 * (p + 1)];
#pragma unroll
          for (int j = 0; j < TNW; ++j) bn[j] = sb[offB[j] + 512 * (p + 1)];
        }
#pragma unroll
        for (int i = 0; i < TMW; ++i)
#pragma unroll
          for (int j = 0; j < TNW; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
      }
      __builtin_amdgcn_s_waitcnt(0);
      __syncthreads();
    }
  }

  // register r of lane (c, h) holds C[m = 8 (r / 4) + 4 h + r % 4][n = c] of its tile
  float* __restrict__ P = a.partial + (int64_t)blockIdx.x * a.M * a.N;
#pragma unroll
  for (int i = 0; i < TMW; ++i)
#pragma unroll
    for (int j = 0; j < TNW; ++j) {
      const int n = n0 + 32 * (nt0 + j) + c;
      if (32 * (nt0 + j) + c >= nwid) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int ml = 32 * (mt0 + i) + 8 * (r / 4) + 4 * h + (r % 4);
        if (ml < mwid) P[(int64_t)(m0 + ml) * a.N + n] = acc[i][j][r];
      }
    }
}

namespace {

struct TnLdsShape { int wm, wn, tm, tn; };

int up124(int v) { return v <= 1 ? 1 : v <= 2 ? 2 : 4; }

// wavefront grid and tiles per wavefront for a block of mw x nw columns: fewest MFMAs per wavefront
bool tn_lds_shape(int mw, int nw, TnLdsShape* out) {
  const int MT = (int)ceil_div(mw, 32), NT = (int)ceil_div(nw, 32);
  static const int grids[3][2] = {{2, 2}, {1, 4}, {4, 1}};
  int best = 1 << 30;
  for (auto& g : grids) {
    const int tm = (int)ceil_div(MT, g[0]), tn = (int)ceil_div(NT, g[1]);
    if (tm > 4 || tn > 4) continue;
    if (up124(tm) * up124(tn) == 4 && up124(tm) != up124(tn)) continue;      // not instantiated, never the cheapest
    const int cost = 64 * up124(tm) * up124(tn) + up124(tm) + up124(tn);
    if (cost < best) { best = cost; *out = TnLdsShape{g[0], g[1], up124(tm), up124(tn)}; }
  }
  return best != (1 << 30);
}

int tn_lds_blocks_mn(int M, int N) { return (int)(ceil_div(M, 256) * ceil_div(N, 256)); }

}  // namespace

// fp32 operands with 16-byte aligned rows; pays once a wavefront has at least 4 tiles to accumulate and neither operand
// is narrow.  On 2.4 M rows, vector-request kernel against this one: 256 x 256 2.97 / 2.57 ms, 100 x 256 1.47 / 1.33,
// 128 x 128 0.97 / 0.85 (with the final sum), but 256 x 47 0.77 / 0.82 and 128 x 16 0.29 / 0.44: there the product is
// bound by memory and one chunk of lookahead leaves the memory pipe idle around each meeting of the wavefronts.
bool gemm_tn_lds_ok(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, int dtype) {
  const int mode = tune().gemm_tn_lds;
  if (mode == 0 || dtype != GCN_F32 || Kd < 1 || M < 1 || N < 1) return false;
  if ((lda % 4) != 0 || (ldb % 4) != 0 || ((uintptr_t)A % 16) != 0 || ((uintptr_t)B % 16) != 0) return false;
  TnLdsShape sh;
  if (!tn_lds_shape(M < 256 ? M : 256, N < 256 ? N : 256, &sh)) return false;
  if (mode == 2) return true;
  return sh.tm * sh.tn >= 4 && M >= 64 && N >= 64;
}

static int tn_lds_splits(int64_t Kd, int M, int N, int max_blocks = 0) {
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
      return p.multiProcessorCount;
    return 256;
  }();
  // one workgroup per compute unit (its LDS is taken whole), or fewer: the rest is left to a concurrent kernel
  int lim = tune().gemm_tn_lds_blocks > 0 && tune().gemm_tn_lds_blocks < cus ? tune().gemm_tn_lds_blocks : cus;
  if (max_blocks > 0 && max_blocks < lim) lim = max_blocks;
  int64_t want = lim / tn_lds_blocks_mn(M, N);
  const int64_t max_by_k = ceil_div(Kd, 4 * kTnlKC);
  if (want > max_by_k) want = max_by_k;
  return (int)(want < 1 ? 1 : want);
}

size_t gemm_tn_lds_ws_bytes(int64_t Kd, int M, int N) {
  return sizeof(float) * (size_t)tn_lds_splits(Kd, M, N) * (size_t)M * (size_t)N;
}

int gemm_tn_lds_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, float* partial,
                         int* nsplit_out, hipStream_t s, int max_blocks) {
  TnLdsShape sh;
  if (!tn_lds_shape(M < 256 ? M : 256, N < 256 ? N : 256, &sh)) return fail(GCN_EINVAL, "gemm_tn_lds: shape");
  const int want = tn_lds_splits(Kd, M, N, max_blocks);
  const int64_t rps = round_up(ceil_div(Kd, want), kTnlKC);
  const int nsplit = (int)ceil_div(Kd, rps);            // every split holds at least one row
  *nsplit_out = nsplit;
  TnLdsArgs a{(const float*)A, lda, (const float*)B, ldb, Kd, M, N, rps, sh.wm, sh.wn, (int)ceil_div(M, 256), partial};
  dim3 grid((unsigned)nsplit, (unsigned)tn_lds_blocks_mn(M, N));
#define GCN_TNL(TM_, TN_)                                                                                       \
  if (sh.tm == TM_ && sh.tn == TN_) {                                                                           \
    auto kern = k_gemm_tn_lds<TM_, TN_>;                                                                        \
    GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)kTnlLdsBytes));                                                            \
    kern<<<grid, 256, kTnlLdsBytes, s>>>(a);                                                                    \
  }
  // (1, 4) and (4, 1) never win: the 1 x 4 and 4 x 1 wavefront grids cover those shapes with fewer tiles each
  GCN_TNL(1, 1) GCN_TNL(1, 2) GCN_TNL(2, 1) GCN_TNL(2, 2) GCN_TNL(2, 4) GCN_TNL(4, 2) GCN_TNL(4, 4)
#undef GCN_TNL
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

}  // namespace gcn
