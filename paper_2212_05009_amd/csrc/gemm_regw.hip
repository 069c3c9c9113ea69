// C[M x N] = A[M x K] W[K x N] for weight matrices too large for LDS but small enough for the register file
// (Sec. 3.1: the dense product with W^k; here 64 < K <= 256 and N = 64, 128, 192 or 256, fp32).
//
// The four SIMDs of a compute unit hold 512 KB of vector registers, three times its LDS.  A workgroup has one
// wavefront per 64 output columns; wavefront w keeps its column panel W[:, 64 w .. 64 w + 64) in registers for
// the whole launch, already arranged as operands of the 32x32x2 fp32 MFMA (K / 2 x 2 registers per lane), and
// the row tiles of A (64 rows x K) stream past it through LDS: while one tile is multiplied, the next one is
// copied from global memory straight into the other half of LDS (global_load_lds, 16 bytes per lane, no
// registers involved), a whole tile time (about 14 us) ahead of its use.  The inner loop is then MFMAs and LDS
// reads only; the wavefronts meet once per tile.
//
// Operand layout of v_mfma_f32_32x32x2f32: lane l supplies A[row l % 32][k = l / 32] and B[k = l / 32][col l % 32];
// register r of lane l receives C[row 8 (r / 4) + 4 (l / 32) + r % 4][col l % 32].  Within a step of 8 k values,
// lane half h reads k0 + 4 h + i (i = 0 .. 3) as component i of one 16-byte LDS read, so MFMA i of the step
// multiplies rows {k0 + i, k0 + 4 + i} of W: the order of the k sum inside a step is permuted, nothing else.
//
// LDS layout.  A direct copy puts lane l's 16 bytes at (uniform base) + 16 l, so one instruction fills one row
// of 64 quads (1 KB).  The 32 lanes of a half wavefront later read the same quad of 32 different rows, 1 KB
// apart: one bank.  Therefore lane l of the copy of row r fetches quad l ^ (r % 32) from global memory, i.e.
// quad q of row r sits in slot q ^ (r % 32), and the 32 readers of a quad hit 32 different slots.
#include "common.h"

namespace gcn {

typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

struct RegwArgs {
  const float* A; int64_t lda; const float* W; int64_t ldw; float* C; int64_t ldc;
  int64_t M; int N; int K;
  const float* bias; int relu; const float* mask; int64_t ldmask; int64_t mask_rows; float* C2; int64_t ldc2;
};

constexpr int kRegwTileFloats = 64 * 256;             // one tile of A in LDS: 64 rows of 64 quads
constexpr size_t kRegwLdsBytes = 2 * sizeof(float) * kRegwTileFloats;

// KS: steps of 8 k values (K <= 8 KS; rows of W beyond K are zero in the registers).  TAIL: K < 8 KS, so some
// quads of a row are placeholders (the copy fetches the row's first quad instead) and are cleared before use.
template <int KS, bool MASK, bool SAVE, bool TAIL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void k_gemm_nn_regw(RegwArgs a) {
  extern __shared__ float As[];
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int nw = (int)(blockDim.x >> 6);
  const int c = lane & 31, h = lane >> 5;
  const int n0 = 64 * w;
  const float* __restrict__ A = a.A;
  const float* __restrict__ Wg = a.W;

  // this wavefront's panel of W as MFMA operands
  float wr[KS][4][2];
#pragma unroll
  for (int s = 0; s < KS; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int k = 8 * s + 4 * h + i;
#pragma unroll
      for (int ct = 0; ct < 2; ++ct) wr[s][i][ct] = k < a.K ? Wg[(int64_t)k * a.ldw + n0 + 32 * ct + c] : 0.f;
    }

  float bias[2];
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) bias[ct] = a.bias ? a.bias[n0 + 32 * ct + c] : 0.f;

  const int64_t ntiles = (a.M + 63) / 64;
  // wavefront w copies the rows w, w + nw, ... of a tile into buffer b
  auto copy_tile = [&](int64_t tile, int b) {
    for (int r = w; r < 64; r += nw) {
      const int64_t row = tile * 64 + r;
      const int q = lane ^ (r & 31);
      const float* src = A + (row < a.M ? row : a.M - 1) * a.lda + (4 * q < a.K ? 4 * q : 0);
      __builtin_amdgcn_global_load_lds(src, As + b * kRegwTileFloats + r * 256, 16, 0, 0);
    }
  };

  int64_t tile = blockIdx.x;
  if (tile >= ntiles) return;              // (whole workgroup)
  copy_tile(tile, 0);
  __builtin_amdgcn_s_waitcnt(0);
  __syncthreads();

  const int x = h ^ c;                     // slot of quad 2 s + h in rows c and 32 + c: (2 s) ^ x
  for (int b = 0; tile < ntiles; tile += gridDim.x, b ^= 1) {
    if (tile + gridDim.x < ntiles) copy_tile(tile + gridDim.x, b ^ 1);
    floatx16 acc[2][2];
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[rt][ct][r] = 0.f;
    const float* t0 = As + b * kRegwTileFloats + c * 256;
    const float* t1 = t0 + 32 * 256;
    floatx4 nxt[2] = {*reinterpret_cast<const floatx4*>(t0 + 4 * x), *reinterpret_cast<const floatx4*>(t1 + 4 * x)};
#pragma unroll
    for (int s = 0; s < KS; ++s) {
      floatx4 av[2] = {nxt[0], nxt[1]};
      if (s + 1 < KS) {
        const int slot = (2 * (s + 1)) ^ x;
        nxt[0] = *reinterpret_cast<const floatx4*>(t0 + 4 * slot);
        nxt[1] = *reinterpret_cast<const floatx4*>(t1 + 4 * slot);
      }
      if constexpr (TAIL) {
        if (8 * s + 4 * h >= a.K) { av[0] = floatx4{0.f, 0.f, 0.f, 0.f}; av[1] = floatx4{0.f, 0.f, 0.f, 0.f}; }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
            acc[rt][ct] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[rt][i], wr[s][i][ct], acc[rt][ct], 0, 0, 0);
    }
    // The next tile has landed in the other buffer and nobody reads this one any more: meet here, before the stores
    // of the epilogue, so that those drain while the next tile is multiplied instead of being waited for.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    // epilogue: a register row of a tile is 32 consecutive columns, one 128-byte store per half wavefront.
    // Whole tiles take straight-line code: all mask values are requested first, then come the 64 stores with
    // nothing to wait for in between (a wait for a load inside a conditional store also waits for the stores
    // before it, one store round trip each).
    const int64_t mbase = tile * 64 + 4 * h;
    if (tile * 64 + 64 <= a.M && (!MASK || tile * 64 + 64 <= a.mask_rows)) {
      float keep[MASK ? 2 : 1][MASK ? 2 : 1][MASK ? 16 : 1];
      if constexpr (MASK) {
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              keep[rt][ct][r] = a.mask[(mbase + 32 * rt + 8 * (r / 4) + (r % 4)) * a.ldmask + n0 + 32 * ct + c];
      }
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t m = mbase + 32 * rt + 8 * (r / 4) + (r % 4);
            const int n = n0 + 32 * ct + c;
            float v = acc[rt][ct][r] + bias[ct];
            if constexpr (SAVE) a.C2[m * a.ldc2 + n] = v;
            if (a.relu) v = v > 0.f ? v : 0.f;
            if constexpr (MASK) v = keep[rt][ct][r] > 0.f ? v : 0.f;
            a.C[m * a.ldc + n] = v;
          }
    } else {
#pragma unroll
      for (int rt = 0; rt < 2; ++rt)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int64_t m = mbase + 32 * rt + 8 * (r / 4) + (r % 4);
            const int n = n0 + 32 * ct + c;
            if (m >= a.M) continue;
            float v = acc[rt][ct][r] + bias[ct];
            if constexpr (SAVE) a.C2[m * a.ldc2 + n] = v;
            if (a.relu) v = v > 0.f ? v : 0.f;
            if constexpr (MASK) { if (m < a.mask_rows) v = a.mask[m * a.ldmask + n] > 0.f ? v : 0.f; }
            a.C[m * a.ldc + n] = v;
          }
    }
  }
}

// fp32 operands with 16-byte aligned rows, K a multiple of 4 in (64, 256], N a multiple of 64 up to 256
bool gemm_nn_regw_ok(const void* A, int64_t lda, int64_t M, int N, int K, int dtype) {
  if (tune().gemm_regw == 0 || dtype != GCN_F32) return false;
  if (N < 64 || N > 256 || N % 64 != 0 || K % 4 != 0 || K > 256 || K <= 64) return false;
  if ((lda % 4) != 0 || ((uintptr_t)A % 16) != 0 || M < 1) return false;
  return true;
}

template <int KS>
static int regw_launch(const RegwArgs& a, unsigned blocks, hipStream_t s) {
  const unsigned threads = 64u * (unsigned)(a.N / 64);
  const bool mask = a.mask != nullptr, save = a.C2 != nullptr, tail = a.K < 8 * KS;
#define GCN_REGW_GO(MK, SV, TL)                                                                                 \
  do {                                                                                                         \
    auto kern = k_gemm_nn_regw<KS, MK, SV, TL>;                                                                \
    GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, \
                                (int)kRegwLdsBytes));                                                          \
    kern<<<blocks, threads, kRegwLdsBytes, s>>>(a);                                                            \
  } while (0)
#define GCN_REGW(MK, SV)                      \
  do {                                        \
    if (tail) GCN_REGW_GO(MK, SV, true);      \
    else GCN_REGW_GO(MK, SV, false);          \
  } while (0)
  if (mask && save) GCN_REGW(true, true);
  else if (mask) GCN_REGW(true, false);
  else if (save) GCN_REGW(false, true);
  else GCN_REGW(false, false);
#undef GCN_REGW
#undef GCN_REGW_GO
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

int gemm_nn_regw(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N, int K,
                 const GemmEpilogue& epi, hipStream_t s) {
  RegwArgs a{(const float*)A, lda, W, ldw, (float*)C, ldc, M, N, K, epi.bias, epi.relu, (const float*)epi.mask,
             epi.ldmask, epi.mask_rows, (float*)epi.C2, epi.ldc2};
  static const int cus = [] {
    int dev = 0;
    hipDeviceProp_t p;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&p, dev) == hipSuccess && p.multiProcessorCount > 0)
      return p.multiProcessorCount;
    return 256;
  }();
  const int64_t ntiles = ceil_div(M, 64);
  int64_t lim = epi.max_blocks > 0 && epi.max_blocks < cus ? epi.max_blocks : cus;
  if (tune().gemm_regw_blocks > 0 && tune().gemm_regw_blocks < lim) lim = tune().gemm_regw_blocks;
  const unsigned blocks = (unsigned)(ntiles < lim ? ntiles : lim);
  const int ks = (int)ceil_div(K, 8);
  if (ks <= 13) return regw_launch<13>(a, blocks, s);
  if (ks <= 16) return regw_launch<16>(a, blocks, s);
  if (ks <= 24) return regw_launch<24>(a, blocks, s);
  return regw_launch<32>(a, blocks, s);
}

}  // namespace gcn
