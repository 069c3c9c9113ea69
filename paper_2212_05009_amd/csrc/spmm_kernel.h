// Device templates of the sparse-times-dense kernels (included by spmm.hip, spmm_f32.hip, spmm_bf16.hip).
#pragma once
#include <stdlib.h>

#include "common.h"

namespace gcn {

template <typename T, int V> struct Vec;
template <> struct Vec<float, 1> { typedef float type; };
template <> struct Vec<float, 2> { typedef float2 type; };
template <> struct Vec<float, 4> { typedef float4 type; };
template <> struct Vec<bf16_t, 1> { typedef uint16_t type; };
template <> struct Vec<bf16_t, 2> { typedef uint32_t type; };
template <> struct Vec<bf16_t, 4> { typedef uint2 type; };
template <> struct Vec<bf16_t, 8> { typedef uint4 type; };

template <typename T, int V>
__device__ __forceinline__ void load_vec(const T* __restrict__ p, float (&out)[V]) {
  typename Vec<T, V>::type raw = *reinterpret_cast<const typename Vec<T, V>::type*>(p);
  const T* e = reinterpret_cast<const T*>(&raw);
#pragma unroll
  for (int i = 0; i < V; ++i) {
    if constexpr (sizeof(T) == 4) out[i] = (float)e[i];
    else out[i] = bf16_to_f32((bf16_t)e[i]);
  }
}

template <typename T, int V>
__device__ __forceinline__ void store_vec(T* __restrict__ p, const float (&v)[V]) {
  typename Vec<T, V>::type raw;
  T* e = reinterpret_cast<T*>(&raw);
#pragma unroll
  for (int i = 0; i < V; ++i) {
    if constexpr (sizeof(T) == 4) e[i] = v[i];
    else e[i] = f32_to_bf16(v[i]);
  }
  *reinterpret_cast<typename Vec<T, V>::type*>(p) = raw;
}

constexpr int kMaxBins = 34;

struct SpmmK {
  const int64_t* ptr; const int32_t* idx; const float* val;
  // entries of row r that take part: [lo[r], hi[r]); the whole row is lo = ptr, hi = ptr + 1
  const int64_t* lo; const int64_t* hi;
  int accumulate;     // 1: the result is added to what Y holds (a product split in two column ranges)
  const int32_t* wave_rows;
  const int32_t* hub_rows; const int64_t* hub_chunk_ptr; const int32_t* chunk_hub; int64_t n_chunks;
  int64_t n_hub_rows;
  int64_t chunk_lo, hub_lo;   // a launch on a range of rows: first chunk of entries and first hub row it covers (else 0)
  const void* X; int64_t ldx;
  void* Y; int64_t ldy;
  void* Y2; int64_t ldy2;
  const float* bias; const void* Zprev; int64_t ldz; int64_t n_mask_rows;
  float* partial;     // [n_chunks x d] partial rows of hub chunks
  int d; int epilogue;
  uint32_t row_bytes; // ldx in bytes (used by the 32-bit addressing variant)
  int S;              // feature slices; block b works on slice b % S (one slice per XCD group)
  int nvec, vps;      // V-wide vectors per row / per slice
  int y_vec;          // Y (and Y2) rows may be written with V-wide stores
  // ordinary rows: bin b holds the rows wave_rows[bin_row_begin[b] .. bin_row_end[b]) of one length
  // class; 2^bin_log2gr[b] lane groups share a row, so a wavefront takes G >> bin_log2gr[b] rows and
  // the bin's wavefronts are numbered from bin_wave_begin[b].
  int n_bins;
  int64_t bin_wave_begin[kMaxBins + 1];
  int64_t bin_row_begin[kMaxBins];
  int64_t bin_row_end[kMaxBins];
  int bin_log2gr[kMaxBins];
};

// One gathered feature vector: X[j, c0 .. c0+V) with c0b = c0 in bytes.  NARROW: 24-bit row index
// times 24-bit row pitch into a 32-bit byte offset from the (uniform) base pointer.
template <typename T, int V, bool NARROW>
__device__ __forceinline__ void gather_vec(const SpmmK& a, int32_t j, uint32_t c0b, float (&x)[V]) {
  if constexpr (NARROW) {
    const uint32_t off = __umul24((uint32_t)j, a.row_bytes) + c0b;
    load_vec<T, V>(reinterpret_cast<const T*>(reinterpret_cast<const char*>(a.X) + off), x);
  } else {
    load_vec<T, V>(reinterpret_cast<const T*>(reinterpret_cast<const char*>(a.X) +
                                             ((int64_t)j * a.ldx * (int64_t)sizeof(T) + c0b)), x);
  }
}

__device__ __forceinline__ int32_t lane_read(int byte_addr, int32_t v) { return __builtin_amdgcn_ds_bpermute(byte_addr, v); }
__device__ __forceinline__ float lane_read(int byte_addr, float v) {
  return __int_as_float(__builtin_amdgcn_ds_bpermute(byte_addr, __float_as_int(v)));
}

// A "team" of 2^lgr lane groups (TL = LPR << lgr consecutive lanes starting at wave lane team_lane0)
// adds up the entries [s, e) of one sparse row:  acc += sum_k val[k] * X[idx[k], c0 .. c0+V).
// The team reads idx/val TL entries at a time with one coalesced load (team lane t takes entry
// base + t, the next batch is requested before the current one is used); group gg then takes entries
// gg, gg + groups, ... of the batch, fetching index and value from the owning lane by a cross-lane
// read, and keeps U gathered feature vectors in flight.  When every team of the wavefront holds a
// full batch no entry needs a validity check (the common case for long rows); otherwise loads are
// predicated.  Lanes without a feature vector in this slice (active == false) are handed the slice's
// first vector by the caller (c0) - a valid address in a line the slice reads anyway - and never store.  Different teams of a wavefront may hold rows of
// different length: every cross-lane operation sits outside divergent code and loop exits are
// taken on wave-wide votes.  LGR >= 0 fixes lgr at compile time.
template <typename T, int V, int LPR, int U, bool NARROW, int LGR>
__device__ __forceinline__ void team_accumulate(const SpmmK& a, int64_t s, int64_t e, int lgr_rt, int team_lane0,
                                                int gg, int t, int64_t c0, bool active, float (&acc)[V]) {
  constexpr int UE = U < LPR ? U : LPR;
  const int lgr = LGR >= 0 ? LGR : lgr_rt;
  const int groups = 1 << lgr;
  const int TL = LPR << lgr;
  const uint32_t c0b = (uint32_t)(c0 * (int64_t)sizeof(T));
  (void)active;
  const int src0 = (team_lane0 + gg) << 2;          // byte address of the lane holding entry gg
  int64_t base = s;
  int32_t jreg = 0; float wreg = 0.f;
  if (base + t < e) { jreg = a.idx[base + t]; wreg = a.val[base + t]; }
  while (__any(base < e)) {
    const int64_t nb = base + TL;
    int32_t jn = 0; float wn = 0.f;
    if (nb + t < e) { jn = a.idx[nb + t]; wn = a.val[nb + t]; }
    const int64_t left = e - base;
    const int cnt = left <= 0 ? 0 : (left < TL ? (int)left : TL);
    if (__all(cnt == TL)) {
#pragma unroll 1
      for (int i0 = 0; i0 < LPR; i0 += UE) {
        int32_t j[UE]; float w[UE]; float x[UE][V];
#pragma unroll
        for (int u = 0; u < UE; ++u) {
          const int src = src0 + ((i0 + u) << (lgr + 2));
          j[u] = lane_read(src, jreg);
          w[u] = lane_read(src, wreg);
        }
#pragma unroll
        for (int u = 0; u < UE; ++u) gather_vec<T, V, NARROW>(a, j[u], c0b, x[u]);
#pragma unroll
        for (int u = 0; u < UE; ++u)
#pragma unroll
          for (int v = 0; v < V; ++v) acc[v] = fmaf(w[u], x[u][v], acc[v]);
      }
    } else {
#pragma unroll 1
      for (int i0 = 0; i0 < LPR; i0 += UE) {
        if (!__any(i0 * groups < cnt)) break;
        int32_t j[UE]; float w[UE]; float x[UE][V]; bool ok[UE];
#pragma unroll
        for (int u = 0; u < UE; ++u) {
          const int ei = (i0 + u) * groups + gg;
          const int src = src0 + ((i0 + u) << (lgr + 2));
          j[u] = lane_read(src, jreg);
          w[u] = lane_read(src, wreg);
          ok[u] = ei < cnt;
        }
#pragma unroll
        for (int u = 0; u < UE; ++u) {
          if (ok[u]) gather_vec<T, V, NARROW>(a, j[u], c0b, x[u]);
          else {
#pragma unroll
            for (int v = 0; v < V; ++v) x[u][v] = 0.f;
          }
        }
#pragma unroll
        for (int u = 0; u < UE; ++u)
          if (ok[u]) {
#pragma unroll
            for (int v = 0; v < V; ++v) acc[v] = fmaf(w[u], x[u][v], acc[v]);
          }
      }
    }
    jreg = jn; wreg = wn; base = nb;
  }
}

// butterfly over the `groups` (power of two) lane groups of LPR lanes that share a row
template <int V, int LPR>
__device__ __forceinline__ void reduce_groups(float (&acc)[V], int groups) {
  for (int off = LPR; off < LPR * groups; off <<= 1)
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
}

// epilogue on one element of output row `row`, feature c
template <typename T>
__device__ __forceinline__ void finish_element(const SpmmK& a, int64_t row, int64_t c, float v) {
  if (a.accumulate) v += load_one<T>(reinterpret_cast<const T*>(a.Y) + row * a.ldy + c);
  if (a.bias) v += a.bias[c];
  if (a.Y2) store_one<T>(reinterpret_cast<T*>(a.Y2) + row * a.ldy2 + c, v);
  if (a.epilogue == GCN_EPI_RELU) v = v > 0.f ? v : 0.f;
  else if (a.epilogue == GCN_EPI_MASK && row < a.n_mask_rows) {
    float z = load_one<T>(reinterpret_cast<const T*>(a.Zprev) + row * a.ldz + c);
    v = z > 0.f ? v : 0.f;
  }
  store_one<T>(reinterpret_cast<T*>(a.Y) + row * a.ldy + c, v);
}

// the same on V consecutive elements, written with one vector store per output
template <typename T, int V>
__device__ __forceinline__ void finish_vector(const SpmmK& a, int64_t row, int64_t c0, float (&v)[V]) {
  if (a.accumulate) {
    float old[V];
    load_vec<T, V>(reinterpret_cast<const T*>(a.Y) + row * a.ldy + c0, old);
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] += old[i];
  }
  if (a.bias) {
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] += a.bias[c0 + i];
  }
  if (a.Y2) store_vec<T, V>(reinterpret_cast<T*>(a.Y2) + row * a.ldy2 + c0, v);
  if (a.epilogue == GCN_EPI_RELU) {
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] = v[i] > 0.f ? v[i] : 0.f;
  } else if (a.epilogue == GCN_EPI_MASK && row < a.n_mask_rows) {
    const T* z = reinterpret_cast<const T*>(a.Zprev) + row * a.ldz + c0;
#pragma unroll
    for (int i = 0; i < V; ++i) v[i] = load_one<T>(z + i) > 0.f ? v[i] : 0.f;
  }
  store_vec<T, V>(reinterpret_cast<T*>(a.Y) + row * a.ldy + c0, v);
}

template <typename T, int V, int LPR, int U, bool NARROW>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(4, 8))) void k_spmm(SpmmK a) {
  constexpr int G = 64 / LPR;
  constexpr int kLog2G = G == 1 ? 0 : G == 2 ? 1 : G == 4 ? 2 : G == 8 ? 3 : 4;
  constexpr int TW = LPR * V;       // feature tile covered by one group
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int g = lane / LPR, l = lane % LPR;
  int slice; int64_t item;
  if (gridDim.y == 1) {       // the usual case: 32-bit division
    slice = (int)(blockIdx.x % (unsigned)a.S); item = blockIdx.x / (unsigned)a.S;
  } else {
    const int64_t bid = block_id();
    slice = (int)(bid % a.S); item = bid / a.S;
  }
  const int v_lo = slice * a.vps;
  const int v_hi = v_lo + a.vps < a.nvec ? v_lo + a.vps : a.nvec;
  __shared__ float part[4][TW];

  if (item < a.n_chunks) {
    // ---- hub chunk: the whole block works on kHubChunkNnz entries of one long row
    const int64_t c = a.chunk_lo + item;
    const int32_t h = a.chunk_hub[c];
    const int64_t row = a.hub_rows[h];
    const int64_t cs = a.ptr[row] + (c - a.hub_chunk_ptr[h]) * kHubChunkNnz;      // chunks are cut from the whole row
    const int64_t row_lo = a.lo[row], row_hi = a.hi[row];
    const int64_t s = cs > row_lo ? cs : row_lo;
    const int64_t e = cs + kHubChunkNnz < row_hi ? cs + kHubChunkNnz : row_hi;
    const int64_t ws = s + (int64_t)w * (kHubChunkNnz / 4);
    const int64_t we = ws + kHubChunkNnz / 4 < e ? ws + kHubChunkNnz / 4 : e;
    for (int t0 = v_lo; t0 < v_hi; t0 += LPR) {
      const int vi = t0 + l;
      const bool active = vi < v_hi;
      const int64_t c0 = (int64_t)(active ? vi : v_lo) * V;
      float acc[V];
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = 0.f;
      team_accumulate<T, V, LPR, U, NARROW, kLog2G>(a, ws, ws < we ? we : ws, kLog2G, 0, g, lane, c0, active, acc);
      reduce_groups<V, LPR>(acc, G);
      if (g == 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) part[w][l * V + v] = acc[v];
      }
      __syncthreads();
      const int64_t f0 = (int64_t)t0 * V;
      const int64_t f_end = (int64_t)v_hi * V < a.d ? (int64_t)v_hi * V : a.d;
      for (int f = threadIdx.x; f < TW && f0 + f < f_end; f += 256)
        a.partial[c * a.d + f0 + f] = (part[0][f] + part[1][f]) + (part[2][f] + part[3][f]);
      __syncthreads();
    }
    return;
  }

  // ---- ordinary rows: a wavefront takes R = G >> lgr rows of one length class
  const int64_t wi = (item - a.n_chunks) * 4 + w;
  if (wi >= a.bin_wave_begin[a.n_bins]) return;
  int b = 0;
  while (b + 1 < a.n_bins && wi >= a.bin_wave_begin[b + 1]) ++b;
  const int lgr = a.bin_log2gr[b];
  const int groups = 1 << lgr;
  const int q = g >> lgr, gg = g & (groups - 1);
  const int64_t ri = a.bin_row_begin[b] + (wi - a.bin_wave_begin[b]) * (G >> lgr) + q;
  const bool has_row = ri < a.bin_row_end[b];
  int64_t row = 0, s = 0, e = 0;
  if (has_row) { row = a.wave_rows[ri]; s = a.lo[row]; e = a.hi[row]; }
  for (int t0 = v_lo; t0 < v_hi; t0 += LPR) {
    const int vi = t0 + l;
    const bool active = vi < v_hi;
    const int64_t c0 = (int64_t)(active ? vi : v_lo) * V;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    if (lgr == kLog2G) team_accumulate<T, V, LPR, U, NARROW, kLog2G>(a, s, e, lgr, 0, g, lane, c0, active, acc);
    else team_accumulate<T, V, LPR, U, NARROW, -1>(a, s, e, lgr, q * (LPR << lgr), gg, lane - q * (LPR << lgr), c0, active, acc);
    reduce_groups<V, LPR>(acc, groups);
    if (gg == 0 && has_row && active) {
      if (a.y_vec && c0 + V <= a.d) {
        finish_vector<T, V>(a, row, c0, acc);
      } else {
#pragma unroll
        for (int v = 0; v < V; ++v)
          if (c0 + v < a.d) finish_element<T>(a, row, c0 + v, acc[v]);
      }
    }
  }
}

// one wavefront per (hub row, 64 features): add the chunk partials in chunk order, apply the epilogue
template <typename T>
__global__ __launch_bounds__(256) void k_spmm_hub_finish(SpmmK a) {
  const int lane = threadIdx.x & 63;
  const int64_t tiles = (a.d + 63) / 64;
  const int64_t wi = block_id() * 4 + (threadIdx.x >> 6);
  if (wi >= a.n_hub_rows * tiles) return;
  const int64_t h = a.hub_lo + wi / tiles;
  const int64_t f = (wi % tiles) * 64 + lane;
  if (f >= a.d) return;
  const int64_t row = a.hub_rows[h];
  const int64_t c_lo = a.hub_chunk_ptr[h], c_hi = a.hub_chunk_ptr[h + 1];
  // chunk order, eight loads in flight at a time (a hub of a power-law graph has dozens of chunks)
  float v = 0.f;
  int64_t c = c_lo;
  for (; c + 8 <= c_hi; c += 8) {
    float p[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) p[u] = a.partial[(c + u) * a.d + f];
#pragma unroll
    for (int u = 0; u < 8; ++u) v += p[u];
  }
  for (; c < c_hi; ++c) v += a.partial[c * a.d + f];
  finish_element<T>(a, row, f, v);
}

struct SpmmProf {
  int kind; int dtype; int64_t rows, nnz; double alg, touched, flops;
  int row_chunk = -1, row_chunk_n = 1;   // rows Schedule::chunk_row[row_chunk .. row_chunk + row_chunk_n); -1: all rows
};

// Entries each lane group should get before a row is shared by more groups (GCN_SPMM_EPG overrides, for
// experiments).  Measured on an R-MAT graph with 45 entries per row: 4 / 8 / 16 / 32 / 64 entries per group
// give 460 / 441 / 431 / 427 / 427 us at width 128 and 122 / 113 / 108 / 107 / 110 us at width 16: a
// wavefront that holds more rows keeps more gathers in flight per round trip of its dependent loads.
constexpr int kEntriesPerGroup = 32;

static inline int pow2_ceil_i(int x) { int p = 1; while (p < x) p <<= 1; return p; }

template <typename T, int V, int LPR>
static int launch_l(SpmmK& k, const Schedule* sc, const SpmmProf& pf, bool narrow, hipStream_t s) {
  constexpr int G = 64 / LPR;
  // bins of the ordinary rows: class c holds lengths in [2^(31-c), 2^(32-c)), class 32 empty rows
  k.n_bins = 0;
  int64_t waves = 0;
  for (int c = 0; c <= 32; ++c) {
    const int64_t row_begin = pf.row_chunk < 0 ? sc->class_begin[c] : sc->chunk_class_begin[pf.row_chunk][c];
    const int64_t row_end = pf.row_chunk < 0 ? sc->class_begin[c + 1] : sc->chunk_class_begin[pf.row_chunk + pf.row_chunk_n][c];
    const int64_t cnt = row_end - row_begin;
    if (cnt <= 0) continue;
    const int64_t len_hi = c >= 32 ? 0 : ((int64_t)1 << (32 - c)) - 1;
    const int epg = tune().spmm_epg > 0 ? tune().spmm_epg : kEntriesPerGroup;
    const int64_t want = ceil_div(len_hi > 0 ? len_hi : 1, epg);
    int groups = pow2_ceil_i((int)(want < G ? want : G));
    if (groups > G) groups = G;
    int lg = 0; while ((1 << lg) < groups) ++lg;
    const int b = k.n_bins++;
    k.bin_wave_begin[b] = waves;
    k.bin_row_begin[b] = row_begin;
    k.bin_row_end[b] = row_end;
    k.bin_log2gr[b] = lg;
    waves += ceil_div(cnt, G >> lg);
  }
  if (k.n_bins == 0) { k.n_bins = 1; k.bin_wave_begin[0] = 0; k.bin_row_begin[0] = k.bin_row_end[0] = 0; k.bin_log2gr[0] = 0; }
  k.bin_wave_begin[k.n_bins] = waves;
  const int64_t blocks = (k.n_chunks + ceil_div(waves, 4)) * k.S;
  if (!grid_fits(blocks)) return fail(GCN_EINVAL, "spmm: too many rows for one launch");
  if (blocks > 0) {
    ProfScope ps(pf.kind, s, k.d, pf.dtype, pf.rows, pf.nnz, pf.alg, pf.touched, pf.flops);
    // gathered vectors in flight per lane: 16 bytes each, 64 bytes in all
    constexpr int U = (int)(sizeof(T) * V) >= 16 ? 4 : 8;
    if (narrow) k_spmm<T, V, LPR, U, true><<<fold_grid(blocks), dim3(256), 0, s>>>(k);
    else k_spmm<T, V, LPR, U, false><<<fold_grid(blocks), dim3(256), 0, s>>>(k);
  }
  if (k.n_hub_rows > 0) {
    const double fb = 4.0 * (double)k.n_chunks * k.d + (double)sizeof(T) * (double)k.n_hub_rows * k.d;
    ProfScope ps(GCN_K_SPMM_FINISH, s, k.d, pf.dtype, k.n_hub_rows, k.n_chunks, fb, fb, (double)k.n_chunks * k.d);
    const int64_t fw = k.n_hub_rows * ceil_div(k.d, 64);
    k_spmm_hub_finish<T><<<fold_grid(ceil_div(fw, 4)), dim3(256), 0, s>>>(k);
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

template <typename T, int V>
static int launch_v(SpmmK& k, const Schedule* sc, const SpmmProf& pf, bool narrow, hipStream_t s) {
  k.nvec = (int)ceil_div(k.d, V);
  if (k.vps <= 0) k.vps = (int)ceil_div(k.nvec, k.S);     // else: whole lines per slice, set by the caller
  if (k.vps <= 4) return launch_l<T, V, 4>(k, sc, pf, narrow, s);
  if (k.vps <= 8) return launch_l<T, V, 8>(k, sc, pf, narrow, s);
  if (k.vps <= 16) return launch_l<T, V, 16>(k, sc, pf, narrow, s);
  if (k.vps <= 32) return launch_l<T, V, 32>(k, sc, pf, narrow, s);
  return launch_l<T, V, 64>(k, sc, pf, narrow, s);
}

// implemented in spmm_f32.hip / spmm_bf16.hip
int spmm_dispatch_f32(SpmmK& k, const Schedule* sc, const SpmmProf& pf, int V, bool narrow, hipStream_t s);
int spmm_dispatch_bf16(SpmmK& k, const Schedule* sc, const SpmmProf& pf, int V, bool narrow, hipStream_t s);

}  // namespace gcn
