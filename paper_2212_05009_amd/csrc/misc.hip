// Error bookkeeping, the halo gather and the softmax cross-entropy of the gfx950 GCN library.
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>

#include "common.h"

namespace gcn {

static thread_local char g_err[512] = {0};

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}
void clear_error() { g_err[0] = 0; }

// most blocks in the x dimension of a launch: 2^22 blocks of up to 1024 threads stay below 2^32 threads
static std::atomic<int64_t> g_max_grid_x{(int64_t)1 << 22};
int64_t max_grid_x() { return g_max_grid_x.load(std::memory_order_relaxed); }

// ------------------------------------------------------------------------------------------
// Halo gather (Sec. 4.1: the rows of H selected by an index set are copied into the buffer of
// received rows).  A row is moved as n_vec units of VB bytes; a group of LPR lanes owns a row,
// so that one request covers a whole feature row whenever it fits.
// ------------------------------------------------------------------------------------------
template <int VB> struct Unit;
template <> struct Unit<16> { typedef uint4 type; };
template <> struct Unit<8> { typedef uint2 type; };
template <> struct Unit<4> { typedef uint32_t type; };
template <> struct Unit<2> { typedef uint16_t type; };

template <int VB, int LPR>
__global__ __launch_bounds__(256) void k_gather(const char* __restrict__ table, int64_t ld_bytes,
                                                int64_t n_table_rows, int n_vec,
                                                const int32_t* __restrict__ idx, int64_t n_idx,
                                                char* __restrict__ recv, int64_t ldr_bytes) {
  typedef typename Unit<VB>::type U;
  constexpr int G = 256 / LPR;
  const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
  const int64_t s = block_id() * G + g;
  if (s >= n_idx) return;
  const int64_t j = idx[s];
  const bool ok = j >= 0 && j < n_table_rows;
  const U* __restrict__ src = reinterpret_cast<const U*>(table + (ok ? j : 0) * ld_bytes);
  U* __restrict__ dst = reinterpret_cast<U*>(recv + s * ldr_bytes);
  for (int u = l; u < n_vec; u += LPR) {
    U v;
    if (ok) v = src[u];
    else memset(&v, 0, sizeof(U));
    dst[u] = v;
  }
}

// The same copy for a table in host memory: the link to the host, not the GPU, sets the pace, and a
// few hundred rows in flight saturate it (measured: 16 workgroups reach the rate of a full grid, 8
// do not).  A few workgroups (32; GCN_GATHER_HOST_BLOCKS overrides) walk the index list with
// kGatherRows rows in flight per lane group; the rest of the GPU stays free for kernels of other
// streams, which a full grid of waiting wavefronts slows down several times over (the product with
// the owned columns runs meanwhile, Algorithm 1).
constexpr int kGatherRows = 4;
template <int VB, int LPR>
__global__ __launch_bounds__(256) void k_gather_host(const char* __restrict__ table, int64_t ld_bytes,
                                                     int64_t n_table_rows, int n_vec,
                                                     const int32_t* __restrict__ idx, int64_t n_idx,
                                                     char* __restrict__ recv, int64_t ldr_bytes) {
  typedef typename Unit<VB>::type U;
  constexpr int G = 256 / LPR;
  const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
  const int64_t stride = (int64_t)gridDim.x * G;
  for (int64_t s0 = (int64_t)blockIdx.x * G + g; s0 < n_idx; s0 += stride * kGatherRows) {
    const U* src[kGatherRows]; bool ok[kGatherRows];
#pragma unroll
    for (int r = 0; r < kGatherRows; ++r) {
      const int64_t s = s0 + r * stride;
      const int64_t j = s < n_idx ? (int64_t)idx[s] : -1;
      ok[r] = j >= 0 && j < n_table_rows;
      src[r] = reinterpret_cast<const U*>(table + (ok[r] ? j : 0) * ld_bytes);
    }
    for (int u = l; u < n_vec; u += LPR) {
      U v[kGatherRows];
#pragma unroll
      for (int r = 0; r < kGatherRows; ++r) {
        if (ok[r]) v[r] = src[r][u];
        else memset(&v[r], 0, sizeof(U));
      }
#pragma unroll
      for (int r = 0; r < kGatherRows; ++r) {
        const int64_t s = s0 + r * stride;
        if (s < n_idx) reinterpret_cast<U*>(recv + s * ldr_bytes)[u] = v[r];
      }
    }
  }
}

static bool is_host_memory(const void* p) {
  hipPointerAttribute_t at;
  if (hipPointerGetAttributes(&at, p) != hipSuccess) { (void)hipGetLastError(); return false; }
  return at.type == hipMemoryTypeHost;
}

template <int VB>
static int gather_v(const char* table, int64_t ldb, int64_t nt, int n_vec, const int32_t* idx, int64_t n_idx,
                    char* recv, int64_t ldrb, int d, int dtype, hipStream_t s) {
  auto grid = [&](int lpr) { return fold_grid(ceil_div(n_idx, 256 / lpr)); };
  const double by = 2.0 * (double)n_idx * n_vec * VB + 4.0 * (double)n_idx;
  ProfScope ps(GCN_K_GATHER, s, d, dtype, n_idx, 0, by, by, 0.0);
  if (is_host_memory(table)) {
    const int host_blocks = tune().gather_host_blocks;
    const unsigned nb = (unsigned)std::min<int64_t>(host_blocks, ceil_div(n_idx, 8));
    if (n_vec <= 4) k_gather_host<VB, 4><<<nb, 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
    else if (n_vec <= 8) k_gather_host<VB, 8><<<nb, 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
    else if (n_vec <= 16) k_gather_host<VB, 16><<<nb, 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
    else if (n_vec <= 32) k_gather_host<VB, 32><<<nb, 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
    else k_gather_host<VB, 64><<<nb, 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  }
  if (n_vec <= 4) k_gather<VB, 4><<<grid(4), 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
  else if (n_vec <= 8) k_gather<VB, 8><<<grid(8), 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
  else if (n_vec <= 16) k_gather<VB, 16><<<grid(16), 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
  else if (n_vec <= 32) k_gather<VB, 32><<<grid(32), 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
  else k_gather<VB, 64><<<grid(64), 256, 0, s>>>(table, ldb, nt, n_vec, idx, n_idx, recv, ldrb);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

// ------------------------------------------------------------------------------------------
// Softmax cross-entropy (Sec. 3.1, the output-layer gradient, with identity activation on the
// last layer): one group of LPR lanes per row.  The loss terms are added in fp64: per thread,
// then per block in a fixed tree, then over the blocks in block order.
// ------------------------------------------------------------------------------------------
constexpr int kLossBlocks = 4096;
// Per-block partial sums of the loss.  Every call takes the next of kLossSlots rows (a host-side counter), so
// calls that overlap in time on different streams do not share partials unless more than kLossSlots are in flight.
constexpr int kLossSlots = 64;
__device__ double g_loss_partial[kLossSlots][kLossBlocks];
static std::atomic<unsigned> g_loss_slot{0};

template <typename T, int LPR>
__global__ __launch_bounds__(256) void k_softmax_xent(const T* __restrict__ Z, int64_t ldz, int64_t nr, int C,
                                                      const int32_t* __restrict__ y, float scale,
                                                      T* __restrict__ G, int64_t ldg, int slot) {
  constexpr int GR = 256 / LPR;
  const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
  double local = 0.0;
  for (int64_t row = (int64_t)blockIdx.x * GR + g; row < nr; row += (int64_t)gridDim.x * GR) {
    const T* z = Z + row * ldz;
    T* go = G + row * ldg;
    const int label = y[row];
    if (label < 0 || label >= C) {                 // no label: no loss term, zero gradient
      for (int c = l; c < C; c += LPR) store_one<T>(go + c, 0.f);
      continue;
    }
    float mx = -INFINITY, se = 0.f;
    if (C <= LPR) {                      // one element per lane: one load, one exponential, one store
      const bool in = l < C;
      const float zv = in ? load_one<T>(z + l) : -INFINITY;
      mx = zv;
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      const float ev = in ? expf(zv - mx) : 0.f;
      se = ev;
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) se += __shfl_xor(se, off, 64);
      if (in) store_one<T>(go + l, scale * (ev * (1.0f / se) - (l == label ? 1.f : 0.f)));
      // the label's logit sits in lane `label` of this row's lane group: no second, dependent load
      const float zl = __shfl(zv, g * LPR + label, 64);
      if (l == 0) local += (double)(mx + logf(se)) - (double)zl;
      continue;
    } else {
      for (int c = l; c < C; c += LPR) mx = fmaxf(mx, load_one<T>(z + c));
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
      for (int c = l; c < C; c += LPR) se += expf(load_one<T>(z + c) - mx);
#pragma unroll
      for (int off = 1; off < LPR; off <<= 1) se += __shfl_xor(se, off, 64);
      const float inv = 1.0f / se;
      for (int c = l; c < C; c += LPR) {
        float p = expf(load_one<T>(z + c) - mx) * inv;
        store_one<T>(go + c, scale * (p - (c == label ? 1.f : 0.f)));
      }
    }
    if (l == 0) local += (double)(mx + logf(se)) - (double)load_one<T>(z + label);
  }
  // block sum in a fixed tree
  __shared__ double red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) g_loss_partial[slot][blockIdx.x] = red[0];
}

// The same for rows of 4 LPR >= C classes with 16-byte (fp32) / 8-byte (bf16) aligned rows and C a multiple of 4:
// a lane holds 4 classes, so a row is one vector load and one vector store per lane and two or three shuffle steps.
template <typename T, int LPR>
__global__ __launch_bounds__(256) void k_softmax_xent_v4(const T* __restrict__ Z, int64_t ldz, int64_t nr, int C,
                                                         const int32_t* __restrict__ y, float scale,
                                                         T* __restrict__ G, int64_t ldg, int slot) {
  constexpr int GR = 256 / LPR;
  const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
  const bool in = 4 * l < C;
  double local = 0.0;
  for (int64_t row = (int64_t)blockIdx.x * GR + g; row < nr; row += (int64_t)gridDim.x * GR) {
    const int label = y[row];
    float z[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    if (in) {
      if constexpr (sizeof(T) == 4) {
        const float4 v = *reinterpret_cast<const float4*>(Z + row * ldz + 4 * l);
        z[0] = v.x; z[1] = v.y; z[2] = v.z; z[3] = v.w;
      } else {
        const uint2 v = *reinterpret_cast<const uint2*>(Z + row * ldz + 4 * l);
        z[0] = __uint_as_float(v.x << 16); z[1] = __uint_as_float(v.x & 0xffff0000u);
        z[2] = __uint_as_float(v.y << 16); z[3] = __uint_as_float(v.y & 0xffff0000u);
      }
    }
    const bool labelled = label >= 0 && label < C;
    float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float e[4], se = 0.f, zl = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      e[i] = in ? expf(z[i] - mx) : 0.f;
      se += e[i];
      if (4 * l + i == label) zl = z[i];               // the label's logit, in one lane of the row
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) { se += __shfl_xor(se, off, 64); zl += __shfl_xor(zl, off, 64); }
    if (in) {
      const float inv = 1.0f / se;
      float o[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) o[i] = labelled ? scale * (e[i] * inv - (4 * l + i == label ? 1.f : 0.f)) : 0.f;
      if constexpr (sizeof(T) == 4) {
        *reinterpret_cast<float4*>(G + row * ldg + 4 * l) = make_float4(o[0], o[1], o[2], o[3]);
      } else {
        T h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) store_one<T>(&h[i], o[i]);
        uint2 pk;
        pk.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
        pk.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
        *reinterpret_cast<uint2*>(G + row * ldg + 4 * l) = pk;
      }
    }
    if (l == 0 && labelled) local += (double)(mx + logf(se)) - (double)zl;
  }
  __shared__ double red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) g_loss_partial[slot][blockIdx.x] = red[0];
}

// Rows of up to 4 LPR classes that the vector form above cannot take (C no multiple of 4, or rows not aligned): a lane
// holds the classes l, l + LPR, l + 2 LPR, l + 3 LPR, so a row is still read once and written once, and 64 / LPR rows
// share a wavefront (C = 47: four rows per wavefront instead of one).
template <typename T, int LPR>
__global__ __launch_bounds__(256) void k_softmax_xent_s4(const T* __restrict__ Z, int64_t ldz, int64_t nr, int C,
                                                         const int32_t* __restrict__ y, float scale,
                                                         T* __restrict__ G, int64_t ldg, int slot) {
  constexpr int GR = 256 / LPR;
  const int g = threadIdx.x / LPR, l = threadIdx.x % LPR;
  double local = 0.0;
  for (int64_t row = (int64_t)blockIdx.x * GR + g; row < nr; row += (int64_t)gridDim.x * GR) {
    const int label = y[row];
    const bool labelled = label >= 0 && label < C;
    const T* zr = Z + row * ldz;
    float z[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) z[i] = l + LPR * i < C ? load_one<T>(zr + l + LPR * i) : -INFINITY;
    float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float e[4], se = 0.f, zl = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      e[i] = l + LPR * i < C ? expf(z[i] - mx) : 0.f;
      se += e[i];
      if (l + LPR * i == label) zl = z[i];             // the label's logit, in one lane of the row
    }
#pragma unroll
    for (int off = 1; off < LPR; off <<= 1) { se += __shfl_xor(se, off, 64); zl += __shfl_xor(zl, off, 64); }
    const float inv = 1.0f / se;
    T* gr = G + row * ldg;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int c = l + LPR * i;
      if (c < C) store_one<T>(gr + c, labelled ? scale * (e[i] * inv - (c == label ? 1.f : 0.f)) : 0.f);
    }
    if (l == 0 && labelled) local += (double)(mx + logf(se)) - (double)zl;
  }
  __shared__ double red[256];
  red[threadIdx.x] = local;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) g_loss_partial[slot][blockIdx.x] = red[0];
}

// one block: thread t adds the partials t, t+256, ... in order, then a fixed tree over the threads
__global__ __launch_bounds__(256) void k_loss_finish(int nblocks, float scale, float* __restrict__ loss, int slot) {
  __shared__ double red[256];
  double s = 0.0;
  int b = threadIdx.x;
  for (; b + 768 < nblocks; b += 1024) {           // four loads in flight, added in block order
    const double* part = g_loss_partial[slot];
    const double v0 = part[b], v1 = part[b + 256], v2 = part[b + 512], v3 = part[b + 768];
    s += v0; s += v1; s += v2; s += v3;
  }
  for (; b < nblocks; b += 256) s += g_loss_partial[slot][b];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int off = 128; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = (float)((double)scale * red[0]);
}

template <typename T>
static int softmax_t(const T* Z, int64_t ldz, int64_t nr, int C, const int32_t* y, float scale, float* loss, T* G,
                     int64_t ldg, hipStream_t s) {
  const int slot = (int)(g_loss_slot.fetch_add(1u, std::memory_order_relaxed) % (unsigned)kLossSlots);
  const size_t vb = 4 * sizeof(T);
  if (C % 4 == 0 && C <= 256 && (ldz % 4) == 0 && (ldg % 4) == 0 && ((uintptr_t)Z % vb) == 0 && ((uintptr_t)G % vb) == 0) {
    int lpr4 = 1;
    while (4 * lpr4 < C) lpr4 <<= 1;
    int64_t want4 = ceil_div(nr > 0 ? nr : 1, 256 / lpr4);
    const int nb4 = (int)(want4 < kLossBlocks ? want4 : kLossBlocks);
    const double by4 = (double)nr * (2.0 * sizeof(T) * C + 4.0);
    ProfScope ps(GCN_K_SOFTMAX_XENT, s, C, sizeof(T) == 2 ? GCN_BF16 : GCN_F32, nr, 0, by4, by4, 0.0);
    switch (lpr4) {
      case 1: k_softmax_xent_v4<T, 1><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 2: k_softmax_xent_v4<T, 2><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 4: k_softmax_xent_v4<T, 4><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 8: k_softmax_xent_v4<T, 8><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 16: k_softmax_xent_v4<T, 16><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 32: k_softmax_xent_v4<T, 32><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      default: k_softmax_xent_v4<T, 64><<<nb4, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    }
    k_loss_finish<<<1, 256, 0, s>>>(nb4, scale, loss, slot);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  }
  if (C > 4 && C <= 256) {
    int lp = 4;
    while (4 * lp < C) lp <<= 1;
    int64_t want_s = ceil_div(nr > 0 ? nr : 1, 256 / lp);
    const int nbs = (int)(want_s < kLossBlocks ? want_s : kLossBlocks);
    const double bys = (double)nr * (2.0 * sizeof(T) * C + 4.0);
    ProfScope ps(GCN_K_SOFTMAX_XENT, s, C, sizeof(T) == 2 ? GCN_BF16 : GCN_F32, nr, 0, bys, bys, 0.0);
    switch (lp) {
      case 4: k_softmax_xent_s4<T, 4><<<nbs, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 8: k_softmax_xent_s4<T, 8><<<nbs, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 16: k_softmax_xent_s4<T, 16><<<nbs, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      case 32: k_softmax_xent_s4<T, 32><<<nbs, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
      default: k_softmax_xent_s4<T, 64><<<nbs, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    }
    k_loss_finish<<<1, 256, 0, s>>>(nbs, scale, loss, slot);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  }
  int lpr = 4;
  while (lpr < 64 && lpr < C) lpr <<= 1;
  int64_t want = ceil_div(nr > 0 ? nr : 1, 256 / lpr);
  int nb = (int)(want < kLossBlocks ? want : kLossBlocks);
  const double by = (double)nr * (2.0 * sizeof(T) * C + 4.0);
  ProfScope ps(GCN_K_SOFTMAX_XENT, s, C, sizeof(T) == 2 ? GCN_BF16 : GCN_F32, nr, 0, by, by, 0.0);
  switch (lpr) {
    case 4: k_softmax_xent<T, 4><<<nb, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    case 8: k_softmax_xent<T, 8><<<nb, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    case 16: k_softmax_xent<T, 16><<<nb, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    case 32: k_softmax_xent<T, 32><<<nb, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
    default: k_softmax_xent<T, 64><<<nb, 256, 0, s>>>(Z, ldz, nr, C, y, scale, G, ldg, slot); break;
  }
  k_loss_finish<<<1, 256, 0, s>>>(nb, scale, loss, slot);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

// dst[r][0 .. ld_dst) = src[r][0 .. d) followed by zeros: a copy with a padded leading dimension.  One thread moves
// one unit of UB bytes; the widest unit that divides both pitches and the row length is used.
template <typename U>
__global__ __launch_bounds__(256) void k_pad_rows(const char* __restrict__ src, int64_t pitch_src, char* __restrict__ dst,
                                                  int64_t pitch_dst, int64_t rows, int units_row, int units_dst) {
  const int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= rows * units_dst) return;
  const int64_t r = i / units_dst; const int c = (int)(i - r * units_dst);
  U v;
  if (c < units_row) v = reinterpret_cast<const U*>(src + r * pitch_src)[c];
  else memset(&v, 0, sizeof(U));
  reinterpret_cast<U*>(dst + r * pitch_dst)[c] = v;
}

// The same with 16-byte units for rows whose length is no multiple of 16 bytes but whose pitch is: the last unit of a
// row reads into the source row's padding (which exists for every row but the buffer's last, copied separately) and
// keeps only its first tail_bytes bytes.
__global__ __launch_bounds__(256) void k_pad_rows_tail(const char* __restrict__ src, int64_t pitch_src, char* __restrict__ dst,
                                                       int64_t pitch_dst, int64_t rows, int units_row, int units_dst,
                                                       int tail_bytes) {
  const int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= rows * units_dst) return;
  const int64_t r = i / units_dst; const int c = (int)(i - r * units_dst);
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (c < units_row) {
    v = reinterpret_cast<const uint4*>(src + r * pitch_src)[c];
    if (c == units_row - 1) {
      uint16_t* h = reinterpret_cast<uint16_t*>(&v);
#pragma unroll
      for (int b = 0; b < 8; ++b) if (2 * b >= tail_bytes) h[b] = 0;
    }
  }
  reinterpret_cast<uint4*>(dst + r * pitch_dst)[c] = v;
}

// the same for 2-byte elements whose source rows are only 2-byte aligned (odd pitch): a thread reads two elements
// and writes one 4-byte word of the destination, whose pitch is even
__global__ __launch_bounds__(256) void k_pad_rows_pairs(const uint16_t* __restrict__ src, int64_t ld_src, uint32_t* __restrict__ dst,
                                                        int64_t words_dst, int64_t rows, int d) {
  const int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= rows * words_dst) return;
  const int64_t r = i / words_dst; const int c = 2 * (int)(i - r * words_dst);
  const uint16_t* sr = src + r * ld_src;
  const uint32_t lo = c < d ? sr[c] : 0u, hi = c + 1 < d ? sr[c + 1] : 0u;
  dst[i] = lo | (hi << 16);
}

// One wavefront that sleeps for a fixed number of rounds (about 3.7 us each) and ends.
__global__ void k_pause(int rounds) {
#pragma unroll 1
  for (int i = 0; i < rounds; ++i) __builtin_amdgcn_s_sleep(127);
}

int stream_pause(hipStream_t s) {
  k_pause<<<1, 64, 0, s>>>(tune().pause_rounds);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

int pad_rows(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int d, int dtype, hipStream_t s) {
  if (rows <= 0) return GCN_OK;
  const int64_t es = dtype == GCN_BF16 ? 2 : 4;
  const int64_t ps = ld_src * es, pd = ld_dst * es, len = (int64_t)d * es;
  int ub = 16;
  while (ub > es && !((ps % ub) == 0 && (pd % ub) == 0 && (len % ub) == 0 && ((uintptr_t)src % ub) == 0 &&
                      ((uintptr_t)dst % ub) == 0)) ub >>= 1;
  const double by = (double)es * (double)rows * (double)(d + ld_dst);
  ProfScope ps_(GCN_K_OTHER, s, d, dtype, rows, 0, by, by, 0.0);
  const char* sp = (const char*)src; char* dp = (char*)dst;
  const int64_t len16 = round_up(len, 16);
  if (ub < 16 && rows > 1 && (ps % 16) == 0 && (pd % 16) == 0 && ((uintptr_t)src % 16) == 0 && ((uintptr_t)dst % 16) == 0 &&
      len16 <= ps && len16 <= pd) {
    // all rows but the last with 16-byte units (a unit may read the padding of its source row), the last row exactly
    const int64_t n16 = (rows - 1) * (pd / 16);
    k_pad_rows_tail<<<fold_grid(ceil_div(n16, 256)), 256, 0, s>>>(sp, ps, dp, pd, rows - 1, (int)(len16 / 16), (int)(pd / 16),
                                                                 (int)(len % 16));
    sp += (rows - 1) * ps; dp += (rows - 1) * pd;
    rows = 1;
  }
  const int units_row = (int)(len / ub), units_dst = (int)(pd / ub);
  const int64_t n = rows * units_dst;
  if (ub == 2 && (ld_dst % 2) == 0 && ((uintptr_t)dst % 4) == 0) {
    const int64_t words = ld_dst / 2;
    k_pad_rows_pairs<<<fold_grid(ceil_div(rows * words, 256)), 256, 0, s>>>((const uint16_t*)sp, ld_src, (uint32_t*)dp, words, rows, d);
    GCN_CHECK_LAUNCH();
    return GCN_OK;
  }
  const dim3 grid = fold_grid(ceil_div(n, 256));
  switch (ub) {
    case 16: k_pad_rows<uint4><<<grid, 256, 0, s>>>(sp, ps, dp, pd, rows, units_row, units_dst); break;
    case 8: k_pad_rows<uint2><<<grid, 256, 0, s>>>(sp, ps, dp, pd, rows, units_row, units_dst); break;
    case 4: k_pad_rows<uint32_t><<<grid, 256, 0, s>>>(sp, ps, dp, pd, rows, units_row, units_dst); break;
    default: k_pad_rows<uint16_t><<<grid, 256, 0, s>>>(sp, ps, dp, pd, rows, units_row, units_dst); break;
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

__global__ __launch_bounds__(256) void k_sgd(float* __restrict__ W, const float* __restrict__ dW, int64_t n, float lr) {
  const int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n) W[i] = fmaf(-lr, dW[i], W[i]);
}

}  // namespace gcn

using namespace gcn;

extern "C" const char* gcn_last_error(void) { return g_err; }

namespace gcn {
namespace {
struct TuneField { const char* name; int Tuning::*field; int lo, hi; };
const TuneField kTuneFields[] = {
    {"GCN_SPMM_PANEL", &Tuning::spmm_panel, -1, 1},         {"GCN_PANEL_NARROW", &Tuning::panel_narrow, 0, 1},
    {"GCN_PANEL_NOSYNC", &Tuning::panel_nosync, 0, 1},      {"GCN_PANEL_VERBOSE", &Tuning::panel_verbose, 0, 1},
    {"GCN_SPMM_SLICES", &Tuning::spmm_slices, 0, 8},        {"GCN_SPMM_EPG", &Tuning::spmm_epg, 0, 1 << 20},
    {"GCN_SPMM_WIDE", &Tuning::spmm_wide, 0, 1},            {"GCN_GEMM_DIRECT", &Tuning::gemm_direct, 0, 1},
    {"GCN_GEMM_FAST", &Tuning::gemm_fast, 0, 1},            {"GCN_GEMM_TN_WIDE", &Tuning::gemm_tn_wide, 0, 1},
    {"GCN_GEMM_BF16", &Tuning::gemm_bf16, 0, 1},            {"GCN_GEMM_REGW", &Tuning::gemm_regw, 0, 2},
    {"GCN_GEMM_TN_LDS", &Tuning::gemm_tn_lds, 0, 2},        {"GCN_GEMM_TN_BLOCKS", &Tuning::gemm_tn_blocks, 1, 1 << 16},
    {"GCN_GATHER_HOST_BLOCKS", &Tuning::gather_host_blocks, 1, 4096}, {"GCN_GEMM_TN_LDS_BLOCKS", &Tuning::gemm_tn_lds_blocks, 0, 4096}, {"GCN_GEMM_REGW_BLOCKS", &Tuning::gemm_regw_blocks, 0, 4096},
    {"GCN_OVERLAP", &Tuning::overlap, 0, 2},               {"GCN_OVERLAP_CUS", &Tuning::overlap_cus, 1, 4096},
    {"GCN_OVERLAP_CHUNKS", &Tuning::overlap_chunks, 0, 8},
    {"GCN_PAUSE_ROUNDS", &Tuning::pause_rounds, 0, 64},
};
Tuning& tuning_storage() {
  static Tuning t = [] {
    Tuning v;
    for (const TuneField& f : kTuneFields) {
      const char* e = getenv(f.name);
      if (!e || !*e) continue;
      const long x = strtol(e, nullptr, 10);
      if (x >= f.lo && x <= f.hi) v.*(f.field) = (int)x;
    }
    return v;
  }();
  return t;
}
}  // namespace
const Tuning& tune() { return tuning_storage(); }
}  // namespace gcn

extern "C" int gcn_debug_set_tuning(const char* name, int value) {
  clear_error();
  if (!name) return fail(GCN_EINVAL, "gcn_debug_set_tuning: NULL name");
  for (const TuneField& f : kTuneFields) {
    if (strcmp(name, f.name) != 0) continue;
    if (value == GCN_TUNE_DEFAULT) { tuning_storage().*(f.field) = Tuning().*(f.field); return GCN_OK; }
    if (value < f.lo || value > f.hi) return fail(GCN_EINVAL, "gcn_debug_set_tuning: %s takes %d .. %d", f.name, f.lo, f.hi);
    tuning_storage().*(f.field) = value;
    return GCN_OK;
  }
  return fail(GCN_EINVAL, "gcn_debug_set_tuning: unknown name %s", name);
}

extern "C" int64_t gcn_feature_ld(int d, int dtype) {
  if (d < 1 || (dtype != GCN_F32 && dtype != GCN_BF16)) return -1;
  const int64_t es = dtype == GCN_BF16 ? 2 : 4;
  const int64_t lines = ceil_div((int64_t)d * es, 128);
  if (lines < 2) return d;
  return (lines | 1) * (128 / es);
}

extern "C" int gcn_debug_max_grid_x(int64_t blocks) {
  clear_error();
  if (blocks != 0 && (blocks < 1 || blocks > ((int64_t)1 << 22))) return fail(GCN_EINVAL, "gcn_debug_max_grid_x: need 0 (default) or 1 .. 2^22");
  g_max_grid_x.store(blocks == 0 ? (int64_t)1 << 22 : blocks, std::memory_order_relaxed);
  return GCN_OK;
}

extern "C" int gcn_sgd_update(float* W, const float* dW, int64_t n, float lr, void* stream) {
  clear_error();
  if (n < 0) return fail(GCN_EINVAL, "gcn_sgd_update: negative size");
  if (n == 0) return GCN_OK;
  if (!W || !dW) return fail(GCN_EINVAL, "gcn_sgd_update: NULL pointer");
  if (!grid_fits(ceil_div(n, 256))) return fail(GCN_EINVAL, "gcn_sgd_update: too many elements");
  hipStream_t s = (hipStream_t)stream;
  const double by = 12.0 * (double)n;
  ProfScope ps(GCN_K_OTHER, s, 1, GCN_F32, n, 0, by, by, 2.0 * (double)n);
  k_sgd<<<fold_grid(ceil_div(n, 256)), 256, 0, s>>>(W, dW, n, lr);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

extern "C" int gcn_halo_gather(const void* table, int64_t ld, int64_t n_table_rows, int d, int dtype,
                               const int32_t* d_idx, int64_t n_idx, void* recv, int64_t ldr, void* stream) {
  clear_error();
  if (n_idx < 0 || n_table_rows < 0) return fail(GCN_EINVAL, "gcn_halo_gather: negative size");
  if (d < 1 || ld < d || ldr < d) return fail(GCN_EINVAL, "gcn_halo_gather: need 1 <= d <= ld, ldr");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_halo_gather: unknown dtype");
  if (n_idx == 0) return GCN_OK;
  if (!table || !d_idx || !recv) return fail(GCN_EINVAL, "gcn_halo_gather: NULL pointer");
  if (!grid_fits(ceil_div(n_idx, 4))) return fail(GCN_EINVAL, "gcn_halo_gather: index list too long");
  const int64_t es = dtype == GCN_BF16 ? 2 : 4;
  const int64_t row_bytes = d * es, ldb = ld * es, ldrb = ldr * es;
  int vb = 16;
  while (vb > es && !((row_bytes % vb) == 0 && (ldb % vb) == 0 && (ldrb % vb) == 0 &&
                      ((uintptr_t)table % vb) == 0 && ((uintptr_t)recv % vb) == 0)) vb >>= 1;
  const int n_vec = (int)(row_bytes / vb);
  hipStream_t s = (hipStream_t)stream;
  switch (vb) {
    case 16: return gather_v<16>((const char*)table, ldb, n_table_rows, n_vec, d_idx, n_idx, (char*)recv, ldrb, d, dtype, s);
    case 8: return gather_v<8>((const char*)table, ldb, n_table_rows, n_vec, d_idx, n_idx, (char*)recv, ldrb, d, dtype, s);
    case 4: return gather_v<4>((const char*)table, ldb, n_table_rows, n_vec, d_idx, n_idx, (char*)recv, ldrb, d, dtype, s);
    default: return gather_v<2>((const char*)table, ldb, n_table_rows, n_vec, d_idx, n_idx, (char*)recv, ldrb, d, dtype, s);
  }
}

extern "C" int gcn_softmax_xent(const void* Z, int64_t ldz, int64_t nr, int C, int dtype, const int32_t* y,
                                float scale, float* loss, void* G, int64_t ldg, void* stream) {
  clear_error();
  if (nr < 0 || C < 1) return fail(GCN_EINVAL, "gcn_softmax_xent: need nr >= 0 and C >= 1");
  if (ldz < C || ldg < C) return fail(GCN_EINVAL, "gcn_softmax_xent: leading dimension smaller than C");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_softmax_xent: unknown dtype");
  if (!loss || (nr > 0 && (!Z || !y || !G))) return fail(GCN_EINVAL, "gcn_softmax_xent: NULL pointer");
  hipStream_t s = (hipStream_t)stream;
  if (dtype == GCN_BF16)
    return softmax_t<bf16_t>((const bf16_t*)Z, ldz, nr, C, y, scale, loss, (bf16_t*)G, ldg, s);
  return softmax_t<float>((const float*)Z, ldz, nr, C, y, scale, loss, (float*)G, ldg, s);
}
