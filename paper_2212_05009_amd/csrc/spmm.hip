// Y = epilogue(A X): sparse (CSR or CSC arrays) times dense row-major features, gfx950.
//
// Sec. 4.1 defines the per-row task  sum_{j in cols(A(i,:))} A(i,j) X(j,:)  and Sec. 4.3 notes
// that its cost is proportional to the row's entry count, so rows are binned by length:
//   * ordinary rows: one 64-lane wavefront per row.  The lanes are split into G = 64 / LPR groups
//     of LPR lanes; a group covers the feature dimension with V-wide vector loads (a whole
//     feature row is one coalesced request) and the G groups walk the row's entries G at a
//     time; a butterfly over the groups finishes the row.
//   * hub rows (more than kHubRowNnz entries): cut into chunks of kHubChunkNnz entries, one
//     4-wave block per chunk; the waves' partial rows meet in LDS and the chunk's partial row
//     goes to a workspace, which a finalisation kernel adds up in chunk order.
// Every sum has a fixed association, so results are bitwise reproducible.
#include "common.h"

namespace gcn {

typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {   // round to nearest even; NaN stays NaN
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

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

template <typename T> __device__ __forceinline__ float load_one(const T* p) {
  if constexpr (sizeof(T) == 4) return (float)*p;
  else return bf16_to_f32((bf16_t)*p);
}
template <typename T> __device__ __forceinline__ void store_one(T* p, float v) {
  if constexpr (sizeof(T) == 4) *p = v;
  else *p = f32_to_bf16(v);
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

struct SpmmK {
  const int64_t* ptr; const int32_t* idx; const float* val;
  const int32_t* wave_rows; int64_t n_wave_rows;
  const int32_t* hub_rows; const int64_t* hub_chunk_ptr; const int32_t* chunk_hub; int64_t n_chunks;
  int64_t n_hub_rows;
  const void* X; int64_t ldx;
  void* Y; int64_t ldy;
  void* Y2; int64_t ldy2;
  const float* bias; const void* Zprev; int64_t ldz; int64_t n_mask_rows;
  float* partial;     // [n_chunks x d] partial rows of hub chunks
  int d; int epilogue;
};

// accumulate  sum_{k in [s,e), k = s+g (mod G)} val[k] * X[idx[k], c0 .. c0+V)  into acc
template <typename T, int V, int LPR>
__device__ __forceinline__ void accumulate_run(const SpmmK& a, int64_t s, int64_t e, int g, int64_t c0,
                                               bool active, float (&acc)[V]) {
  constexpr int G = 64 / LPR;
  constexpr int U = 4;
  const T* __restrict__ X = reinterpret_cast<const T*>(a.X);
  int64_t k = s + g;
  for (; k + (U - 1) * G < e; k += U * G) {
    int32_t j[U]; float w[U]; float x[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u) { j[u] = a.idx[k + u * G]; w[u] = a.val[k + u * G]; }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (active) load_vec<T, V>(X + (int64_t)j[u] * a.ldx + c0, x[u]);
      else {
#pragma unroll
        for (int v = 0; v < V; ++v) x[u][v] = 0.f;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = fmaf(w[u], x[u][v], acc[v]);
  }
  for (; k < e; k += G) {
    int32_t j = a.idx[k]; float w = a.val[k]; float x[V];
    if (active) {
      load_vec<T, V>(X + (int64_t)j * a.ldx + c0, x);
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = fmaf(w, x[v], acc[v]);
    }
  }
}

template <int V, int LPR>
__device__ __forceinline__ void reduce_groups(float (&acc)[V]) {
#pragma unroll
  for (int off = LPR; off < 64; off <<= 1)
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] += __shfl_xor(acc[v], off, 64);
}

// epilogue on one element of output row `row`, feature c
template <typename T>
__device__ __forceinline__ void finish_element(const SpmmK& a, int64_t row, int64_t c, float v) {
  if (a.bias) v += a.bias[c];
  if (a.Y2) store_one<T>(reinterpret_cast<T*>(a.Y2) + row * a.ldy2 + c, v);
  if (a.epilogue == GCN_EPI_RELU) v = v > 0.f ? v : 0.f;
  else if (a.epilogue == GCN_EPI_MASK && row < a.n_mask_rows) {
    float z = load_one<T>(reinterpret_cast<const T*>(a.Zprev) + row * a.ldz + c);
    v = z > 0.f ? v : 0.f;
  }
  store_one<T>(reinterpret_cast<T*>(a.Y) + row * a.ldy + c, v);
}

template <typename T, int V, int LPR>
__global__ __launch_bounds__(256) void k_spmm(SpmmK a) {
  constexpr int TW = LPR * V;       // feature tile covered by one group
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int g = lane / LPR, l = lane % LPR;
  __shared__ float part[4][TW];

  if ((int64_t)blockIdx.x < a.n_chunks) {
    // ---- hub chunk: the whole block works on kHubChunkNnz entries of one long row
    const int64_t c = blockIdx.x;
    const int32_t h = a.chunk_hub[c];
    const int64_t row = a.hub_rows[h];
    const int64_t s = a.ptr[row] + (c - a.hub_chunk_ptr[h]) * kHubChunkNnz;
    const int64_t row_end = a.ptr[row + 1];
    const int64_t e = s + kHubChunkNnz < row_end ? s + kHubChunkNnz : row_end;
    const int64_t ws = s + (int64_t)w * (kHubChunkNnz / 4);
    const int64_t we = ws + kHubChunkNnz / 4 < e ? ws + kHubChunkNnz / 4 : e;
    for (int64_t t0 = 0; t0 < a.d; t0 += TW) {
      const int64_t c0 = t0 + (int64_t)l * V;
      float acc[V];
#pragma unroll
      for (int v = 0; v < V; ++v) acc[v] = 0.f;
      if (ws < we) accumulate_run<T, V, LPR>(a, ws, we, g, c0, c0 < a.d, acc);
      reduce_groups<V, LPR>(acc);
      if (g == 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) part[w][l * V + v] = acc[v];
      }
      __syncthreads();
      for (int f = threadIdx.x; f < TW && t0 + f < a.d; f += 256)
        a.partial[c * a.d + t0 + f] = (part[0][f] + part[1][f]) + (part[2][f] + part[3][f]);
      __syncthreads();
    }
    return;
  }

  // ---- ordinary rows: one wavefront per row
  const int64_t wi = ((int64_t)blockIdx.x - a.n_chunks) * 4 + w;
  if (wi >= a.n_wave_rows) return;
  const int64_t row = a.wave_rows[wi];
  const int64_t s = a.ptr[row], e = a.ptr[row + 1];
  for (int64_t t0 = 0; t0 < a.d; t0 += TW) {
    const int64_t c0 = t0 + (int64_t)l * V;
    const bool active = c0 < a.d;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = 0.f;
    accumulate_run<T, V, LPR>(a, s, e, g, c0, active, acc);
    reduce_groups<V, LPR>(acc);
    if (g == 0 && active) {
      const bool plain = !a.bias && !a.Y2 && a.epilogue == GCN_EPI_NONE;
      if (plain && c0 + V <= a.d) {
        store_vec<T, V>(reinterpret_cast<T*>(a.Y) + row * a.ldy + c0, acc);
      } else {
#pragma unroll
        for (int v = 0; v < V; ++v)
          if (c0 + v < a.d) finish_element<T>(a, row, c0 + v, acc[v]);
      }
    }
  }
}

// one wavefront per hub row: add the chunk partials in chunk order, apply the epilogue
template <typename T>
__global__ __launch_bounds__(256) void k_spmm_hub_finish(SpmmK a) {
  const int lane = threadIdx.x & 63;
  const int64_t h = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (h >= a.n_hub_rows) return;
  const int64_t row = a.hub_rows[h];
  const int64_t c_lo = a.hub_chunk_ptr[h], c_hi = a.hub_chunk_ptr[h + 1];
  for (int64_t f = lane; f < a.d; f += 64) {
    float v = 0.f;
    for (int64_t c = c_lo; c < c_hi; ++c) v += a.partial[c * a.d + f];
    finish_element<T>(a, row, f, v);
  }
}

size_t spmm_ws_bytes(const Schedule* sc, int d) {
  return sizeof(float) * (size_t)(sc->n_chunks > 0 ? sc->n_chunks : 1) * (size_t)d;
}

struct SpmmProf { int kind; int dtype; int64_t rows, nnz; double alg, touched, flops; };

template <typename T, int V>
static int launch_v(const SpmmK& k, const SpmmProf& pf, hipStream_t s) {
  const int per_row = (int)ceil_div(k.d, V);
  const int64_t blocks = k.n_chunks + ceil_div(k.n_wave_rows, 4);
  if (blocks > 0x7fffffffLL) return fail(GCN_EINVAL, "spmm: too many rows for one launch");
  if (blocks > 0) {
    ProfScope ps(pf.kind, s, k.d, pf.dtype, pf.rows, pf.nnz, pf.alg, pf.touched, pf.flops);
    dim3 grid((unsigned)blocks), block(256);
    if (per_row <= 4) k_spmm<T, V, 4><<<grid, block, 0, s>>>(k);
    else if (per_row <= 8) k_spmm<T, V, 8><<<grid, block, 0, s>>>(k);
    else if (per_row <= 16) k_spmm<T, V, 16><<<grid, block, 0, s>>>(k);
    else if (per_row <= 32) k_spmm<T, V, 32><<<grid, block, 0, s>>>(k);
    else k_spmm<T, V, 64><<<grid, block, 0, s>>>(k);
  }
  if (k.n_hub_rows > 0) {
    const double fb = 4.0 * (double)k.n_chunks * k.d + (double)sizeof(T) * (double)k.n_hub_rows * k.d;
    ProfScope ps(GCN_K_SPMM_FINISH, s, k.d, pf.dtype, k.n_hub_rows, k.n_chunks, fb, fb, (double)k.n_chunks * k.d);
    k_spmm_hub_finish<T><<<dim3((unsigned)ceil_div(k.n_hub_rows, 4)), dim3(256), 0, s>>>(k);
  }
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

static bool aligned(const void* p, size_t a) { return p == nullptr || ((uintptr_t)p % a) == 0; }

int spmm_launch(const SpmmArgs& a, void* ws, hipStream_t s) {
  SpmmK k;
  k.ptr = a.ptr; k.idx = a.idx; k.val = a.val;
  k.wave_rows = a.sched->wave_rows; k.n_wave_rows = a.sched->n_wave_rows;
  k.hub_rows = a.sched->hub_rows; k.hub_chunk_ptr = a.sched->hub_chunk_ptr;
  k.chunk_hub = a.sched->chunk_hub; k.n_chunks = a.sched->n_chunks; k.n_hub_rows = a.sched->n_hub_rows;
  k.X = a.X; k.ldx = a.ldx; k.Y = a.Y; k.ldy = a.ldy; k.Y2 = a.Y2; k.ldy2 = a.ldy2;
  k.bias = a.bias; k.Zprev = a.Zprev; k.ldz = a.ldz; k.n_mask_rows = a.n_mask_rows;
  k.partial = (float*)ws; k.d = a.d; k.epilogue = a.epilogue;
  if (a.n_rows == 0) return GCN_OK;
  const size_t es = a.dtype == GCN_BF16 ? 2 : 4;
  // widest vector such that every feature row start stays aligned to it
  int V = a.dtype == GCN_BF16 ? 8 : 4;
  while (V > 1 && !((a.ldx % V) == 0 && (a.ldy % V) == 0 && aligned(a.X, V * es) && aligned(a.Y, V * es) &&
                    ((a.d % V) == 0 || a.x_rows_padded))) V >>= 1;
  SpmmProf pf;
  pf.kind = a.transposed ? GCN_K_SPMM_T : GCN_K_SPMM; pf.dtype = a.dtype; pf.rows = a.n_rows; pf.nnz = a.nnz;
  const double csr = 8.0 * (double)a.nnz + 8.0 * (double)(a.n_rows + 1), fe = (double)es * a.d;
  pf.alg = csr + fe * (double)(a.n_cols + a.n_rows);
  pf.touched = csr + fe * (double)(a.nnz + a.n_rows);
  pf.flops = 2.0 * (double)a.nnz * a.d;
  if (a.dtype == GCN_BF16) {
    switch (V) {
      case 8: return launch_v<bf16_t, 8>(k, pf, s);
      case 4: return launch_v<bf16_t, 4>(k, pf, s);
      case 2: return launch_v<bf16_t, 2>(k, pf, s);
      default: return launch_v<bf16_t, 1>(k, pf, s);
    }
  }
  switch (V) {
    case 4: return launch_v<float, 4>(k, pf, s);
    case 2: return launch_v<float, 2>(k, pf, s);
    default: return launch_v<float, 1>(k, pf, s);
  }
}

}  // namespace gcn

using namespace gcn;

static int check_dense(const char* fn, const void* X, int64_t ldx, const void* Y, int64_t ldy, int d, int dtype) {
  if (!X || !Y) return fail(GCN_EINVAL, "%s: NULL feature buffer", fn);
  if (d < 1) return fail(GCN_EINVAL, "%s: d must be >= 1", fn);
  if (ldx < d || ldy < d) return fail(GCN_EINVAL, "%s: leading dimension smaller than d", fn);
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "%s: unknown dtype", fn);
  if (X == Y) return fail(GCN_EINVAL, "%s: X and Y must not alias", fn);
  return GCN_OK;
}

extern "C" int gcn_spmm(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y, int64_t ldy,
                        int epilogue, const float* bias, const void* Zprev, int64_t ldz, void* stream) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_spmm: NULL handle");
  GCN_TRY(check_dense("gcn_spmm", X, ldx, Y, ldy, d, dtype));
  if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_EINVAL, "gcn_spmm: unknown epilogue");
  if (epilogue == GCN_EPI_MASK && (!Zprev || ldz < d)) return fail(GCN_EINVAL, "gcn_spmm: mask epilogue needs Zprev with ldz >= d");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  GCN_TRY(ensure_workspace(Am, spmm_ws_bytes(&A->sched, d)));
  SpmmArgs a{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, X, ldx, Y, ldy, nullptr, 0,
             d, dtype, epilogue, bias, Zprev, ldz};
  return spmm_launch(a, Am->ws, (hipStream_t)stream);
}

extern "C" int gcn_spmm_t(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y, int64_t ldy,
                          int epilogue, const void* Zprev, int64_t ldz, void* stream) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_spmm_t: NULL handle");
  if (!A->colptr) return fail(GCN_EINVAL, "gcn_spmm_t: handle was built without GCN_BUILD_CSC");
  GCN_TRY(check_dense("gcn_spmm_t", X, ldx, Y, ldy, d, dtype));
  if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_EINVAL, "gcn_spmm_t: unknown epilogue");
  if (epilogue == GCN_EPI_MASK && (!Zprev || ldz < d)) return fail(GCN_EINVAL, "gcn_spmm_t: mask epilogue needs Zprev with ldz >= d");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  GCN_TRY(ensure_workspace(Am, spmm_ws_bytes(&A->sched_t, d)));
  SpmmArgs a{A->colptr, A->rowidx, A->val_t, &A->sched_t, A->nc, A->nr, A->nnz, true, A->nr, X, ldx, Y, ldy, nullptr, 0,
             d, dtype, epilogue, nullptr, Zprev, ldz};
  return spmm_launch(a, Am->ws, (hipStream_t)stream);
}
