// Column-sweep variant of Y = epilogue(A X) for matrices whose dense operand is re-read many
// times but does not fit the 4 MB L2 of an XCD (gfx950: 8 XCDs x 32 CUs, 160 KB LDS per CU).
//
// Sec. 4.1 defines the row task  Y(i,:) = sum_j A(i,j) X(j,:).  The row-per-wavefront kernel of
// spmm_kernel.h gathers the rows X(j,:) in whatever order the rows i come, so most gathers of a
// large X miss L2 and the kernel runs at the speed of the fabric behind L2.  Here the roles are
// swapped: the OUTPUT rows of a panel (about a thousand rows, one 32-feature slice) stay in the
// LDS of one workgroup, and the workgroup walks the panel's entries sorted by column block, so
// at any time all 32 workgroups of an XCD gather from the same few column blocks of one feature
// slice, which L2 holds.  A persistent grid (one workgroup per CU) takes (slice, panel) units
// from one list per XCD; the k-th unit of a list starts when all units before round k / 32 are
// done, which keeps the sweeps of an XCD in step (a bounded wait: only speed depends on it).
//
// Rows longer than part_len entries are dealt round-robin to several "virtual rows", each with
// its own LDS accumulator, so that no row is a load-balance problem; the parts are added in
// order when the panel is written out.  Every virtual row is owned by one lane group of one
// wavefront: the group adds a run of entries in registers and then into the accumulator with a
// plain read-add-write, no atomics, so results are bitwise reproducible.
#include <stdio.h>
#include <stdlib.h>

#include <algorithm>
#include <cmath>
#include <new>
#include <queue>
#include <utility>
#include <vector>

#include "spmm_kernel.h"

namespace gcn {

namespace {

constexpr int kLidBits = 8;                // index of a virtual row among those of its lane group
constexpr int kMaxLid = 254;
constexpr int kColBits = 24;               // column id
constexpr uint32_t kNoEntry = 0xffffffffu;
constexpr int kPanelThreads = 64 * kPanelWaves;
constexpr int kLdsBudget = 152 * 1024;     // accumulator bytes per workgroup (of 160 KB)
constexpr int kMaxVrows = 2047;
constexpr int kMaxSpins = 20000;
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct PanelK {
  SpmmK k;                       // X, Y and epilogue fields
  const uint2* ent; const int64_t* wb; const int32_t* nfull; const int32_t* cbend; const int32_t* obase;
  const int32_t* panel_row0; const int32_t* row_v; const int32_t* vlds; const int32_t* order;
  uint32_t* ctr;                 // [0, kPanelLists): next unit of each list; [kPanelLists, 2 kPanelLists): units done
  int n_panels, ns, n_cb;
  int soft_sync;                 // 0: no column-block barriers (experiments)
  int q;                         // > 0: q lists share a slice (list = slice * q + a takes panels a, a + q, ...)
  int list_begin[kPanelLists];   // q == 0: list i holds the units [list_begin[i], list_begin[i] + list_len[i]) of the
  int list_len[kPanelLists];     //         slice-major enumeration unit = slice * n_panels + position
  int wg_per_list;
};

__global__ void k_panel_reset(uint32_t* ctr) {
  if (threadIdx.x < 2 * kPanelLists) ctr[threadIdx.x] = 0u;
}

// ---- plan construction kernels ---------------------------------------------------------------
// key = owner << (cbbits + 8) | column block << 8 | index of the virtual row in its owner
__global__ void k_plan_keys(const int64_t* __restrict__ ptr, int64_t n_rows, int64_t nnz,
                            const int32_t* __restrict__ idx, int part_len, const int32_t* __restrict__ row_v,
                            const uint32_t* __restrict__ vinfo, int cb_shift, int cbbits,
                            uint64_t* __restrict__ keys, uint32_t* __restrict__ pay) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= nnz) return;
  int64_t lo = 0, hi = n_rows;             // last row r with ptr[r] <= p
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (ptr[mid] <= p) lo = mid; else hi = mid;
  }
  const int64_t r = lo;
  const int64_t s = ptr[r], len = ptr[r + 1] - s;
  const int64_t parts = len <= part_len ? 1 : (len + part_len - 1) / part_len;
  const uint32_t info = vinfo[row_v[r] + (p - s) % parts];      // owner << 8 | index in owner
  const uint64_t cb = (uint64_t)(idx[p] >> cb_shift);
  keys[p] = ((uint64_t)(info >> kLidBits) << (cbbits + kLidBits)) | (cb << kLidBits) | (uint64_t)(info & 0xffu);
  pay[p] = (uint32_t)p;
}

// batches of each wavefront: enough for its longest group stream; nfull = batches every group fills.
// epb = entries per group and batch.
__global__ void k_plan_waves(const int64_t* __restrict__ oseg, int64_t n_waves, int groups, int epb,
                             uint32_t* __restrict__ nb, int32_t* __restrict__ nfull) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= n_waves) return;
  int64_t mx = 0, mn = INT64_MAX;
  for (int g = 0; g < groups; ++g) {
    const int64_t len = oseg[w * groups + g + 1] - oseg[w * groups + g];
    mx = len > mx ? len : mx; mn = len < mn ? len : mn;
  }
  nb[w] = (uint32_t)((mx + epb - 1) / epb);
  nfull[w] = (int32_t)(mn / epb);
}

// cbend[w * n_cb + cb] = batches of wavefront w after which all of its groups are past column block cb
// (seg[] = boundaries of the (owner, column block) runs of the sorted entries, id = owner << cbbits | cb)
__global__ void k_plan_cbend(const int64_t* __restrict__ seg, int64_t n_waves, int groups, int epb, int n_cb, int cbbits,
                             int32_t* __restrict__ cbend) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_waves * n_cb) return;
  const int64_t w = i / n_cb; const int cb = (int)(i % n_cb);
  int64_t mx = 0;
  for (int g = 0; g < groups; ++g) {
    const int64_t o = w * groups + g;
    const int64_t upto = seg[(o << cbbits) + cb + 1] - seg[o << cbbits];
    mx = upto > mx ? upto : mx;
  }
  cbend[i] = (int32_t)((mx + epb - 1) / epb);
}

__global__ void k_plan_fill_pad(uint2* __restrict__ ent, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) ent[i] = make_uint2(kNoEntry, 0u);
}

__global__ void k_plan_scatter(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ pay,
                               const int32_t* __restrict__ idx, const float* __restrict__ val, int64_t nnz,
                               int shift, int groups, int epb, const int64_t* __restrict__ oseg,
                               const int64_t* __restrict__ wb, uint2* __restrict__ ent) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (q >= nnz) return;
  const uint64_t key = keys[q];
  const int64_t o = (int64_t)(key >> shift);
  const int64_t k = q - oseg[o];
  const int64_t w = o / groups, g = o % groups;
  const int64_t pos = (wb[w] + k / epb) * ((int64_t)epb * groups) + g * epb + k % epb;
  const uint32_t p = pay[q];
  ent[pos] = make_uint2(((uint32_t)(key & 0xffu) << kColBits) | (uint32_t)idx[p], __float_as_uint(val[p]));
}

// ---- the product kernel --------------------------------------------------------------------------
template <int EPL>
__device__ __forceinline__ void load_entries(const uint2* __restrict__ ent, int64_t batch, int batch_entries, int lane,
                                             uint32_t (&e)[2 * EPL]) {
  const uint2* p = ent + batch * batch_entries + lane * EPL;
  if constexpr (EPL == 1) {
    const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
    e[0] = t.x; e[1] = t.y;
  } else {
#pragma unroll
    for (int i = 0; i < EPL / 2; ++i) {
      const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p) + i);
      e[4 * i] = t.x; e[4 * i + 1] = t.y; e[4 * i + 2] = t.z; e[4 * i + 3] = t.w;
    }
  }
}

// entry i of lane group g of the batch held in e (every lane of the group gets it)
template <int LPG>
__device__ __forceinline__ uint32_t group_entry(const uint32_t (&e)[2 * (8 / LPG)], int g, int i, int word) {
  constexpr int EPL = 8 / LPG;
  return (uint32_t)__builtin_amdgcn_ds_bpermute((g * LPG + i / EPL) << 2, (int)e[2 * (i % EPL) + word]);
}

// puts the 8 gathers of this lane group's entries in flight (kept as loaded: 16 bytes each)
template <typename T, int V, int LPG, bool CHECK>
__device__ __forceinline__ void issue_batch(const uint32_t (&e)[2 * (8 / LPG)], int g, const char* xb, uint32_t row_bytes,
                                            uint32_t xoff, typename Vec<T, V>::type (&x)[8]) {
  uint32_t c[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) c[i] = group_entry<LPG>(e, g, i, 0);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    if (CHECK) c[i] = c[i] == kNoEntry ? 0u : c[i];     // padding gathers row 0 (a valid address), and is dropped later
    const uint32_t off = __umul24(c[i], row_bytes) + xoff;
    x[i] = *reinterpret_cast<const typename Vec<T, V>::type*>(xb + off);
  }
}

template <int V>
__device__ __forceinline__ void add_to_row(float* __restrict__ row, const float (&av)[V]) {
#pragma unroll
  for (int v0 = 0; v0 < V; v0 += 4) {
    float4 t = *reinterpret_cast<float4*>(row + v0);
    t.x += av[v0]; t.y += av[v0 + 1]; t.z += av[v0 + 2]; t.w += av[v0 + 3];
    *reinterpret_cast<float4*>(row + v0) = t;
  }
}

// e: the entries the batch was issued from (index and value are fetched from the owning lanes again)
template <typename T, int V, int LPG, bool CHECK>
__device__ __forceinline__ void consume_batch(const uint32_t (&e)[2 * (8 / LPG)], int g,
                                              const typename Vec<T, V>::type (&x)[8], float* __restrict__ myacc,
                                              bool active, int& cur, float (&av)[V]) {
  constexpr int SW = V * LPG;
  // all sixteen cross-lane reads go out before the first is used: one LDS round trip per batch, not per entry
  uint32_t pks[8]; float ws[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { pks[i] = group_entry<LPG>(e, g, i, 0); ws[i] = __uint_as_float(group_entry<LPG>(e, g, i, 1)); }
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t pk = pks[i];
    const float w = ws[i];
    const bool valid = !CHECK || pk != kNoEntry;
    const int lid = (int)(pk >> kColBits);
    if (valid && lid != cur) {
      if (cur >= 0 && active) add_to_row<V>(myacc + cur * SW, av);
#pragma unroll
      for (int v = 0; v < V; ++v) av[v] = 0.f;
      cur = lid;
    }
    float xf[V];
    if constexpr (sizeof(T) == 4) {
      xf[0] = x[i].x; xf[1] = x[i].y; xf[2] = x[i].z; xf[3] = x[i].w;
    } else {                       // two bf16 per 32-bit word, the lower-indexed one in the low half
      const uint32_t wd[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
#pragma unroll
      for (int k = 0; k < 4; ++k) { xf[2 * k] = __uint_as_float(wd[k] << 16); xf[2 * k + 1] = __uint_as_float(wd[k] & 0xffff0000u); }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) {
      const float xv = CHECK ? (valid ? xf[v] : 0.f) : xf[v];
      av[v] = fmaf(CHECK ? (valid ? w : 0.f) : w, xv, av[v]);
    }
  }
}

// Soft column-block barrier.  Left alone, the wavefronts of a workgroup drift several column blocks
// apart (the instruction arbiter prefers the older ones) and the blocks in use no longer fit L2.  So
// all wavefronts meet after every column block: wavefront w reaches the barrier of block cb when it
// has done cbend[cb] batches.  Every wavefront passes exactly n_cb barriers per unit; where exactly it
// passes them only changes speed, never results.
struct SweepSync {
  const int32_t* cbend;     // this wavefront's row of the table
  int n_cb;
  int k;                    // barriers passed so far
  int next;                 // batches after which barrier k is due
  int vals;                 // lane i: cbend[(k & ~63) + i]
  int lane;
  __device__ __forceinline__ void load_chunk() {     // only called with 0 <= k < n_cb
    const int i = (k & ~63) + lane;
    vals = cbend[i < n_cb ? i : n_cb - 1];
  }
  __device__ __forceinline__ void init(const int32_t* p, int n, int ln) {
    cbend = p; n_cb = n > 0 ? n : 0; k = 0; lane = ln; vals = 0; next = 0;
    if (n_cb > 0) {
      load_chunk();
      next = __shfl(vals, 0, 64);
    }
  }
  // call with the number of batches done; wave-uniform
  __device__ __forceinline__ void arrive(int done) {
    while (k < n_cb && done >= next) {
      __syncthreads();
      ++k;
      if (k < n_cb) {
        if ((k & 63) == 0) load_chunk();
        next = __shfl(vals, k & 63, 64);
      }
    }
  }
  __device__ __forceinline__ void finish() {
    while (k < n_cb) { __syncthreads(); ++k; }
  }
};

// batches [b0, b1) of one wavefront, two batches of gathers in flight.  Inside the loop there is no
// conditional load between the gathers of a batch and their use, so the compiler's wait counts are
// exact (the entries two batches ahead are always fetched, those of the last batch again at the end).
template <typename T, int V, int LPG, bool CHECK>
__device__ __forceinline__ void sweep(const uint2* __restrict__ ent, int64_t wave_b0, int64_t b0, int64_t b1, int lane, int g,
                                      const char* xb, uint32_t row_bytes, uint32_t xoff, float* __restrict__ myacc,
                                      bool active, int& cur, float (&av)[V], SweepSync& sync) {
  constexpr int EPL = 8 / LPG, G = 64 / LPG, BATCH = 8 * G;
  typedef typename Vec<T, V>::type XV;
  if (b0 >= b1) return;
  const int64_t last = b1 - 1;
  uint32_t eA[2 * EPL], eB[2 * EPL], eC[2 * EPL];
  XV xA[8], xB[8];
  load_entries<EPL>(ent, b0, BATCH, lane, eA);
  load_entries<EPL>(ent, b0 + 1 < last ? b0 + 1 : last, BATCH, lane, eB);
  issue_batch<T, V, LPG, CHECK>(eA, g, xb, row_bytes, xoff, xA);
  int64_t b = b0;
  while (b + 2 <= last) {
    sync.arrive((int)(b - wave_b0));
    // xA: gathers of batch b (entries eA) in flight; eB: entries of batch b + 1
    load_entries<EPL>(ent, b + 2, BATCH, lane, eC);
    issue_batch<T, V, LPG, CHECK>(eB, g, xb, row_bytes, xoff, xB);
    consume_batch<T, V, LPG, CHECK>(eA, g, xA, myacc, active, cur, av);
    load_entries<EPL>(ent, b + 3 < last ? b + 3 : last, BATCH, lane, eA);
    issue_batch<T, V, LPG, CHECK>(eC, g, xb, row_bytes, xoff, xA);
    consume_batch<T, V, LPG, CHECK>(eB, g, xB, myacc, active, cur, av);
    b += 2;
    // xA: gathers of batch b (entries eC) in flight; eA: entries of batch b + 1
#pragma unroll
    for (int i = 0; i < 2 * EPL; ++i) { const uint32_t t = eA[i]; eA[i] = eC[i]; eB[i] = t; }
  }
  if (b < last) issue_batch<T, V, LPG, CHECK>(eB, g, xb, row_bytes, xoff, xB);
  consume_batch<T, V, LPG, CHECK>(eA, g, xA, myacc, active, cur, av);
  if (b < last) consume_batch<T, V, LPG, CHECK>(eB, g, xB, myacc, active, cur, av);
}

// ---- wide variant: a lane group is half a wavefront, 32 lanes x 4 fp32 = 128 features of a row ----
// The two groups' entries of a batch sit in lanes [0, 32) and [32, 64) of the entry registers.  What
// decides control flow (which accumulator row an entry belongs to) is read into scalar registers, so
// the run bookkeeping costs no vector instructions and no divergence; per entry a lane does one
// address multiply-add, one 16-byte gather and four multiply-adds.  Eight gathers per lane are kept
// in flight in a ring that runs on across batch boundaries.
constexpr int kWideDepth = 8;

template <bool CHECK>
__device__ __forceinline__ void sweep_wide(const uint2* __restrict__ ent, int64_t wave_b0, int64_t b0, int64_t b1, int lane,
                                           const char* xb, uint32_t row_bytes, uint32_t xoff, float* __restrict__ myacc,
                                           bool active, int (&cur)[2], float (&av)[4], SweepSync& sync) {
  if (b0 >= b1) return;
  const int half = lane >> 5;
  const int64_t last = b1 - 1;
  const u32x2* ep = reinterpret_cast<const u32x2*>(ent);
  auto load_batch = [&](int64_t bq, uint32_t& pk, uint32_t& wt) {
    const u32x2 t = __builtin_nontemporal_load(ep + (bq <= last ? bq : last) * 64 + lane);
    pk = bq <= last ? t.x : kNoEntry; wt = bq <= last ? t.y : 0u;
  };
  auto gather = [&](uint32_t src_pk, int i, bool clamp) -> float4 {
    uint32_t c = (uint32_t)__builtin_amdgcn_ds_bpermute((half * 32 + i) << 2, (int)src_pk);
    if (clamp) c = c == kNoEntry ? 0u : c;         // padding gathers row 0 (a valid address) and is dropped later
    return *reinterpret_cast<const float4*>(xb + (__umul24(c, row_bytes) + xoff));
  };
  uint32_t e_pk, e_w, n_pk, n_w;
  load_batch(b0, e_pk, e_w);
  load_batch(b0 + 1, n_pk, n_w);
  float4 x[kWideDepth];
#pragma unroll
  for (int i = 0; i < kWideDepth; ++i) x[i] = gather(e_pk, i, CHECK);
  for (int64_t b = b0; b < b1; ++b) {
    sync.arrive((int)(b - wave_b0));
    uint32_t nn_pk, nn_w;
    load_batch(b + 2, nn_pk, nn_w);
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      // ---- use entry i of both groups
      const uint32_t s0 = (uint32_t)__builtin_amdgcn_readlane((int)e_pk, i);
      const uint32_t s1 = (uint32_t)__builtin_amdgcn_readlane((int)e_pk, 32 + i);
      float w = __int_as_float(__builtin_amdgcn_ds_bpermute((half * 32 + i) << 2, (int)e_w));
      const bool ok0 = !CHECK || s0 != kNoEntry, ok1 = !CHECK || s1 != kNoEntry;
      const int lid0 = (int)(s0 >> kColBits), lid1 = (int)(s1 >> kColBits);
      if (ok0 && lid0 != cur[0]) {                                   // wave-uniform
        if (cur[0] >= 0 && half == 0) {
          if (active) add_to_row<4>(myacc + cur[0] * 128, av);
          av[0] = av[1] = av[2] = av[3] = 0.f;
        }
        cur[0] = lid0;
      }
      if (ok1 && lid1 != cur[1]) {
        if (cur[1] >= 0 && half == 1) {
          if (active) add_to_row<4>(myacc + cur[1] * 128, av);
          av[0] = av[1] = av[2] = av[3] = 0.f;
        }
        cur[1] = lid1;
      }
      float4 xv = x[i % kWideDepth];
      if (CHECK) {
        const bool ok = half ? ok1 : ok0;
        w = ok ? w : 0.f;
        xv.x = ok ? xv.x : 0.f; xv.y = ok ? xv.y : 0.f; xv.z = ok ? xv.z : 0.f; xv.w = ok ? xv.w : 0.f;
      }
      av[0] = fmaf(w, xv.x, av[0]); av[1] = fmaf(w, xv.y, av[1]); av[2] = fmaf(w, xv.z, av[2]); av[3] = fmaf(w, xv.w, av[3]);
      // ---- put the gather of entry i + depth in flight (from the next batch near the end of this one)
      const int j = i + kWideDepth;
      if (j < 32) x[i % kWideDepth] = gather(e_pk, j, CHECK);
      else x[i % kWideDepth] = gather(n_pk, j - 32, true);
    }
    e_pk = n_pk; e_w = n_w; n_pk = nn_pk; n_w = nn_w;
  }
}

// common tail of a unit: add the parts of each row in order, apply the epilogue, write the rows.  A
// wavefront takes 64 rows at a time: lane i fetches the description of row i, then the lanes walk
// the rows, SW features of a row at a step (64 / SW rows per step when SW < 64).
template <typename T, int SW>
__device__ __forceinline__ void write_panel(const PanelK& a, const float* __restrict__ acc, int row0, int row1, int slice,
                                            int w, int lane) {
  constexpr int RPS = SW >= 64 ? 1 : 64 / SW;          // rows per step
  constexpr int PASSES = SW >= 64 ? SW / 64 : 1;       // steps per row
  for (int rb = row0 + w * 64; rb < row1; rb += kPanelWaves * 64) {
    const int mine = rb + lane < row1 ? rb + lane : row1 - 1;
    const int v0 = a.row_v[mine], v1 = a.row_v[mine + 1];
    const int first = a.vlds[v0];
    const int n_here = row1 - rb < 64 ? row1 - rb : 64;
    for (int j = 0; j < n_here; j += RPS) {
      const int rr = j + (SW >= 64 ? 0 : lane / SW);
      const int src = (rr < n_here ? rr : n_here - 1) << 2;
      const int p0 = __builtin_amdgcn_ds_bpermute(src, v0), p1 = __builtin_amdgcn_ds_bpermute(src, v1);
      const int l0 = __builtin_amdgcn_ds_bpermute(src, first);
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) {
        const int f = SW >= 64 ? lane + 64 * ps : lane % SW;
        const int c = slice * SW + f;
        if (rr < n_here && c < a.k.d) {
          float sum = acc[l0 * SW + f];
          for (int vg = p0 + 1; vg < p1; ++vg) sum += acc[a.vlds[vg] * SW + f];
          finish_element<T>(a.k, rb + rr, c, sum);
        }
      }
    }
  }
}

template <typename T, int V, int LPG>
__global__ __launch_bounds__(kPanelThreads) void k_spmm_panel(PanelK a) {
  constexpr int G = 64 / LPG;
  constexpr int SW = V * LPG;                // features of a slice = accumulator floats per virtual row
  static_assert(G * LPG == 64 && (LPG == 32 || 8 % LPG == 0) && V % 4 == 0, "lane groups must tile the wavefront");
  static_assert(LPG != 32 || (V == 4 && sizeof(T) == 4), "the half-wavefront variant is fp32 only");
  extern __shared__ __align__(16) float acc[];
  __shared__ int s_unit[2];
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane / LPG, l = lane % LPG;
  uint32_t xcc;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
  int li = (int)(xcc & 15u) % kPanelLists;   // thread 0's list cursor
  int tried = 0;

  for (;;) {
    if (tid == 0) {
      int unit = -1, from = 0;
      while (tried < kPanelLists) {
        const int kk = (int)atomicAdd(&a.ctr[li], 1u);
        if (kk < a.list_len[li]) { unit = kk; from = li; break; }
        li = (li + 1) % kPanelLists;
        ++tried;
      }
      if (unit >= 0) {
        // start in step with the other workgroups of this list
        const uint32_t target = (uint32_t)(unit / a.wg_per_list) * (uint32_t)a.wg_per_list;
        const uint32_t* done = a.ctr + kPanelLists + from;
        for (int spins = 0; spins < kMaxSpins; ++spins) {
          if (__hip_atomic_load(done, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= target) break;
          __builtin_amdgcn_s_sleep(16);
        }
      }
      s_unit[0] = unit; s_unit[1] = from;
    }
    __syncthreads();
    const int unit = s_unit[0], from = s_unit[1];
    if (unit < 0) break;
    int slice, pos;
    if (a.q > 0) { slice = from / a.q; pos = unit * a.q + from % a.q; }
    else { const int u = a.list_begin[from] + unit; slice = u / a.n_panels; pos = u - slice * a.n_panels; }
    const int panel = a.order[pos];
    const int row0 = a.panel_row0[panel], row1 = a.panel_row0[panel + 1];
    const int pv0 = a.row_v[row0];
    const int nv = a.row_v[row1] - pv0;
    for (int i = tid * 4; i < nv * SW; i += kPanelThreads * 4) *reinterpret_cast<float4*>(acc + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    // ---- this wavefront's batches; lane group g adds into its own accumulator rows
    {
      const int64_t gw = (int64_t)panel * kPanelWaves + w;
      const int64_t bb = a.wb[gw], be = a.wb[gw + 1];
      const int64_t bf = bb + a.nfull[gw];
      const int c0 = slice * SW + l * V;
      const bool active = c0 < a.k.d;
      const uint32_t xoff = (uint32_t)((active ? c0 : slice * SW) * (int)sizeof(T));
      const char* xb = reinterpret_cast<const char*>(a.k.X);
      float* myacc = acc + a.obase[gw * G + g] * SW + l * V;
      SweepSync sync;
      sync.init(a.cbend + gw * a.n_cb, a.soft_sync ? a.n_cb : 0, lane);
      float av[V];
#pragma unroll
      for (int v = 0; v < V; ++v) av[v] = 0.f;
      if constexpr (LPG == 32) {
        int cur[2] = {-1, -1};
        sweep_wide<false>(a.ent, bb, bb, bf, lane, xb, a.k.row_bytes, xoff, myacc, active, cur, av, sync);
        sweep_wide<true>(a.ent, bb, bf, be, lane, xb, a.k.row_bytes, xoff, myacc, active, cur, av, sync);
        const int mycur = g ? cur[1] : cur[0];
        if (mycur >= 0 && active) add_to_row<4>(myacc + mycur * SW, av);
      } else {
        int cur = -1;
        sweep<T, V, LPG, false>(a.ent, bb, bb, bf, lane, g, xb, a.k.row_bytes, xoff, myacc, active, cur, av, sync);
        sweep<T, V, LPG, true>(a.ent, bb, bf, be, lane, g, xb, a.k.row_bytes, xoff, myacc, active, cur, av, sync);
        if (cur >= 0 && active) add_to_row<V>(myacc + cur * SW, av);
      }
      sync.finish();
    }
    __syncthreads();
    if (tid == 0) __hip_atomic_fetch_add(a.ctr + kPanelLists + from, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    write_panel<T, SW>(a, acc, row0, row1, slice, w, lane);
    __syncthreads();
  }
}

template <typename T, int V, int LPG>
int launch_panel(const PanelK& k, int n_wg, size_t lds_bytes, hipStream_t s) {
  static bool attr_set = false;
  if (!attr_set) {
    GCN_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_spmm_panel<T, V, LPG>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget));
    attr_set = true;
  }
  k_spmm_panel<T, V, LPG><<<dim3((unsigned)n_wg), dim3(kPanelThreads), lds_bytes, s>>>(k);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

int device_cus() {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
    if (cus <= 0) cus = 256;
  }
  return cus;
}

void free_plan(PanelPlan* p) {
  if (!p) return;
  void* ptrs[] = {p->ent, p->wb, p->nfull, p->cbend, p->obase, p->panel_row0, p->row_v, p->vlds, p->order, p->ctr};
  for (void* q : ptrs) if (q) (void)hipFree(q);
  delete p;
}

int bits_for_count(int64_t n) { int b = 1; while ((1LL << b) < n) ++b; return b; }

// Builds the layout for products with `ns` feature slices, `sw` accumulator floats per virtual
// row and lane groups of `lpg` lanes.  *out stays null when the matrix does not fit the format.
static int build_plan_impl(gcn_csr* A, bool transposed, int ns, int sw, int lpg, int cb_shift, hipStream_t s, PanelPlan** out) {
  *out = nullptr;
  const int64_t n = transposed ? A->nc : A->nr;
  const int64_t nnz = A->nnz;
  const int64_t* d_ptr = transposed ? A->colptr : A->rowptr;
  const int32_t* d_idx = transposed ? A->rowidx : A->col;
  const float* d_val = transposed ? A->val_t : A->val;
  const int64_t n_cols = transposed ? A->nr : A->nc;
  const int n_wg = device_cus();
  const int groups = 64 / lpg;
  const int epb = lpg >= 32 ? 32 : 8;              // entries per group and batch
  const int n_own = kPanelWaves * groups;          // owners (lane groups) per panel

  std::vector<int64_t> ptr((size_t)n + 1);
  GCN_HIP(hipMemcpyAsync(ptr.data(), d_ptr, sizeof(int64_t) * (size_t)(n + 1), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));

  // ---- virtual rows and the panel size
  const int cap = std::min(kMaxVrows, kLdsBudget / (sw * 4));
  int64_t max_len = 0;
  for (int64_t r = 0; r < n; ++r) max_len = std::max(max_len, ptr[r + 1] - ptr[r]);
  // a part should be well below a lane group's share of a panel, or the groups cannot be balanced
  int part_len = nnz / std::max<int64_t>(n, 1) < 128 ? 256 : 512;
  if (lpg >= 32) {       // few lane groups per panel: parts of about a quarter of a group's share
    const double share = (double)nnz / (double)std::max<int64_t>(n, 1) * cap / n_own / 4.0;
    part_len = 32;
    while (part_len < 512 && part_len * 2 <= share) part_len *= 2;
  }
  int nv = cap;
  int64_t total_v = 0;
  for (;;) {
    total_v = 0;
    for (int64_t r = 0; r < n; ++r) {
      const int64_t len = ptr[r + 1] - ptr[r];
      total_v += len <= part_len ? 1 : ceil_div(len, part_len);
    }
    const int64_t max_parts = std::max<int64_t>(1, ceil_div(max_len, part_len));
    // whole rounds of n_wg units: the fewest rounds whose panels fit the LDS, then the smallest
    // panels that still need no more rounds
    const int64_t rounds = std::max<int64_t>(1, ceil_div(total_v * ns * 103, (int64_t)n_wg * cap * 100));
    const int64_t want_panels = std::max<int64_t>(1, (int64_t)n_wg * rounds / ns);
    nv = (int)std::min<int64_t>(cap, ceil_div(total_v * 102, want_panels * 100) + 1);
    if (max_parts * 2 <= nv || max_parts <= 1) break;
    part_len *= 2;
  }
  if (total_v >= 0x7fffffffLL) return GCN_OK;

  std::vector<int32_t> row_v((size_t)n + 1), panel_row0;
  {
    int64_t v = 0; int in_panel = 0;
    panel_row0.push_back(0);
    for (int64_t r = 0; r < n; ++r) {
      const int64_t len = ptr[r + 1] - ptr[r];
      const int parts = (int)(len <= part_len ? 1 : ceil_div(len, part_len));
      if (in_panel + parts > nv && in_panel > 0) { panel_row0.push_back((int32_t)r); in_panel = 0; }
      row_v[(size_t)r] = (int32_t)v;
      v += parts; in_panel += parts;
    }
    row_v[(size_t)n] = (int32_t)v;
    panel_row0.push_back((int32_t)n);
  }
  const int n_panels = (int)panel_row0.size() - 1;
  if ((int64_t)n_panels * n_own >= (1LL << 24)) return GCN_OK;      // owner ids must fit 24 bits
  int nv_max = 0;
  for (int p = 0; p < n_panels; ++p)
    nv_max = std::max(nv_max, row_v[(size_t)panel_row0[(size_t)p + 1]] - row_v[(size_t)panel_row0[(size_t)p]]);
  if (nv_max > cap) return fail(GCN_EHIP, "panel plan: internal error (panel of %d virtual rows)", nv_max);

  // ---- owner of each virtual row: longest first onto the least loaded lane group of the panel
  std::vector<uint32_t> vinfo((size_t)total_v);
  std::vector<int32_t> vlds((size_t)total_v), obase((size_t)n_panels * n_own);
  std::vector<int64_t> panel_nnz((size_t)n_panels);
  {
    typedef std::pair<int64_t, int32_t> Load;           // (entries, virtual row) or (entries so far, owner)
    std::vector<Load> vr;
    std::vector<int32_t> cnt((size_t)n_own), owner_of;
    for (int p = 0; p < n_panels; ++p) {
      const int64_t r0 = panel_row0[(size_t)p], r1 = panel_row0[(size_t)p + 1];
      const int32_t pv0 = row_v[(size_t)r0];
      panel_nnz[(size_t)p] = ptr[r1] - ptr[r0];
      vr.clear();
      for (int64_t r = r0; r < r1; ++r) {
        const int64_t len = ptr[r + 1] - ptr[r];
        const int64_t parts = row_v[(size_t)r + 1] - row_v[(size_t)r];
        for (int64_t j = 0; j < parts; ++j)
          vr.emplace_back(j < len ? (len - j + parts - 1) / parts : 0, (int32_t)(row_v[(size_t)r] + j));
      }
      std::stable_sort(vr.begin(), vr.end(), [](const Load& x, const Load& y) { return x.first > y.first; });
      std::priority_queue<Load, std::vector<Load>, std::greater<Load>> heap;
      for (int o = 0; o < n_own; ++o) heap.emplace(0, o);
      std::fill(cnt.begin(), cnt.end(), 0);
      owner_of.assign(vr.size(), 0);
      for (size_t i = 0; i < vr.size(); ++i) {
        if (heap.empty()) return fail(GCN_EHIP, "panel plan: internal error (no lane group left)");
        Load t = heap.top(); heap.pop();
        owner_of[(size_t)(vr[i].second - pv0)] = t.second;
        const int lid = cnt[(size_t)t.second]++;
        vinfo[(size_t)vr[i].second] = (((uint32_t)p * (uint32_t)n_own + (uint32_t)t.second) << kLidBits) | (uint32_t)lid;
        if (lid + 1 <= kMaxLid) heap.emplace(t.first + vr[i].first, t.second);
      }
      int32_t run = 0;
      for (int o = 0; o < n_own; ++o) { obase[(size_t)p * n_own + o] = run; run += cnt[(size_t)o]; }
      for (size_t i = 0; i < vr.size(); ++i) {
        const int32_t vg = pv0 + (int32_t)i;
        vlds[(size_t)vg] = obase[(size_t)p * n_own + owner_of[i]] + (int32_t)(vinfo[(size_t)vg] & 0xffu);
      }
    }
  }
  std::vector<int32_t> order((size_t)n_panels);
  for (int p = 0; p < n_panels; ++p) order[(size_t)p] = p;
  std::stable_sort(order.begin(), order.end(), [&](int32_t x, int32_t y) { return panel_nnz[(size_t)x] > panel_nnz[(size_t)y]; });

  // ---- device side: sort the entries into the interleaved group streams
  PanelPlan* P = new (std::nothrow) PanelPlan();
  if (!P) return fail(GCN_ENOMEM, "panel plan: host allocation failed");
  struct Guard { PanelPlan* p; ~Guard() { if (p) free_plan(p); } } guard{P};
  P->transposed = transposed; P->ns = ns; P->sw = sw; P->lpg = lpg; P->cb_shift = cb_shift; P->part_len = part_len;
  P->nv_max = nv_max; P->n_panels = n_panels; P->n_rows = n; P->total_vrows = total_v;
  auto dev_alloc = [&](void** p, size_t bytes) -> int {
    hipError_t e = hipMalloc(p, bytes ? bytes : 256);
    if (e != hipSuccess) { *p = nullptr; return fail(GCN_ENOMEM, "panel plan: hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e)); }
    return GCN_OK;
  };
  const int64_t n_waves = (int64_t)n_panels * kPanelWaves, n_owners = (int64_t)n_panels * n_own;
  GCN_TRY(dev_alloc((void**)&P->wb, sizeof(int64_t) * ((size_t)n_waves + 1)));
  GCN_TRY(dev_alloc((void**)&P->nfull, sizeof(int32_t) * (size_t)n_waves));
  const int n_cb = (int)ceil_div(n_cols, (int64_t)1 << cb_shift);
  const int cbbits = bits_for_count(n_cb);
  const int64_t n_seg = n_owners << cbbits;
  if (n_seg > (1LL << 26) || n_waves * n_cb > (1LL << 26)) return GCN_OK;     // too many column blocks for this layout
  P->n_cb = n_cb;
  GCN_TRY(dev_alloc((void**)&P->cbend, sizeof(int32_t) * (size_t)(n_waves * n_cb)));
  GCN_TRY(dev_alloc((void**)&P->obase, sizeof(int32_t) * (size_t)n_owners));
  GCN_TRY(dev_alloc((void**)&P->panel_row0, sizeof(int32_t) * ((size_t)n_panels + 1)));
  GCN_TRY(dev_alloc((void**)&P->row_v, sizeof(int32_t) * ((size_t)n + 1)));
  GCN_TRY(dev_alloc((void**)&P->vlds, sizeof(int32_t) * (size_t)total_v));
  GCN_TRY(dev_alloc((void**)&P->order, sizeof(int32_t) * (size_t)n_panels));
  GCN_TRY(dev_alloc((void**)&P->ctr, sizeof(uint32_t) * 2 * kPanelLists));
  DevBuf d_vinfo, keys_a, keys_b, pay_a, pay_b, tmp, oseg, nb, seg;
  GCN_TRY(d_vinfo.alloc(sizeof(uint32_t) * (size_t)total_v));
  GCN_TRY(keys_a.alloc(sizeof(uint64_t) * (size_t)nnz));
  GCN_TRY(keys_b.alloc(sizeof(uint64_t) * (size_t)nnz));
  GCN_TRY(pay_a.alloc(sizeof(uint32_t) * (size_t)nnz));
  GCN_TRY(pay_b.alloc(sizeof(uint32_t) * (size_t)nnz));
  GCN_TRY(oseg.alloc(sizeof(int64_t) * ((size_t)n_owners + 1)));
  GCN_TRY(seg.alloc(sizeof(int64_t) * ((size_t)n_seg + 1)));
  GCN_TRY(nb.alloc(sizeof(uint32_t) * (size_t)n_waves));
  size_t tb = sort_tmp_bytes(nnz);
  if (scan_tmp_bytes(n_waves) > tb) tb = scan_tmp_bytes(n_waves);
  GCN_TRY(tmp.alloc(tb));
  GCN_HIP(hipMemcpyAsync(P->panel_row0, panel_row0.data(), sizeof(int32_t) * ((size_t)n_panels + 1), hipMemcpyHostToDevice, s));
  GCN_HIP(hipMemcpyAsync(P->row_v, row_v.data(), sizeof(int32_t) * ((size_t)n + 1), hipMemcpyHostToDevice, s));
  GCN_HIP(hipMemcpyAsync(P->order, order.data(), sizeof(int32_t) * (size_t)n_panels, hipMemcpyHostToDevice, s));
  GCN_HIP(hipMemcpyAsync(P->vlds, vlds.data(), sizeof(int32_t) * (size_t)total_v, hipMemcpyHostToDevice, s));
  GCN_HIP(hipMemcpyAsync(P->obase, obase.data(), sizeof(int32_t) * (size_t)n_owners, hipMemcpyHostToDevice, s));
  GCN_HIP(hipMemcpyAsync(d_vinfo.p, vinfo.data(), sizeof(uint32_t) * (size_t)total_v, hipMemcpyHostToDevice, s));
  const int ownbits = bits_for_count(n_owners);
  if (kLidBits + cbbits + ownbits > 64) return GCN_OK;
  const unsigned grid = (unsigned)ceil_div(nnz, 256);
  k_plan_keys<<<grid, 256, 0, s>>>(d_ptr, n, nnz, d_idx, part_len, P->row_v, d_vinfo.as<uint32_t>(), cb_shift, cbbits,
                                   keys_a.as<uint64_t>(), pay_a.as<uint32_t>());
  GCN_CHECK_LAUNCH();
  uint64_t* sorted = nullptr; uint32_t* spay = nullptr;
  GCN_TRY(radix_sort_u64(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), pay_a.as<uint32_t>(), pay_b.as<uint32_t>(), nnz, 0,
                         kLidBits + cbbits + ownbits, tmp.p, s, &sorted, &spay));
  GCN_TRY(segment_boundaries(sorted, nnz, kLidBits + cbbits, n_owners, oseg.as<int64_t>(), s));
  GCN_TRY(segment_boundaries(sorted, nnz, kLidBits, n_seg, seg.as<int64_t>(), s));
  k_plan_waves<<<(unsigned)ceil_div(n_waves, 256), 256, 0, s>>>(oseg.as<int64_t>(), n_waves, groups, epb, nb.as<uint32_t>(), P->nfull);
  k_plan_cbend<<<(unsigned)ceil_div(n_waves * n_cb, 256), 256, 0, s>>>(seg.as<int64_t>(), n_waves, groups, epb, n_cb, cbbits, P->cbend);
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(nb.as<uint32_t>(), P->wb, n_waves, tmp.p, s));
  int64_t n_batches = 0;
  GCN_HIP(hipMemcpyAsync(&n_batches, P->wb + n_waves, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  P->n_batches = n_batches;
  const int64_t n_ent = n_batches * epb * groups;
  if (n_ent >= 0xffffff00LL) return GCN_OK;        // one thread per padded entry below: stay under 2^32 threads
  GCN_TRY(dev_alloc((void**)&P->ent, sizeof(uint2) * (size_t)n_ent));
  if (n_ent > 0) k_plan_fill_pad<<<(unsigned)ceil_div(n_ent, 256), 256, 0, s>>>(P->ent, n_ent);
  k_plan_scatter<<<grid, 256, 0, s>>>(sorted, spay, d_idx, d_val, nnz, kLidBits + cbbits, groups, epb, oseg.as<int64_t>(), P->wb, P->ent);
  GCN_CHECK_LAUNCH();
  GCN_HIP(hipStreamSynchronize(s));      // host vectors and temporaries go out of scope
  if (tune().panel_verbose)
    fprintf(stderr, "[panel plan] rows %lld nnz %lld ns %d sw %d lpg %d cb_shift %d part_len %d vrows %lld panels %d nv_max %d batches %lld (padding %.1f%%)\n",
            (long long)n, (long long)nnz, ns, sw, lpg, cb_shift, part_len, (long long)total_v, n_panels, nv_max,
            (long long)n_batches, 100.0 * ((double)n_ent / (double)nnz - 1.0));
  guard.p = nullptr;
  *out = P;
  return GCN_OK;
}

}  // namespace

// The host side works with std::vector; nothing may throw through the C boundary.
int build_plan(gcn_csr* A, bool transposed, int ns, int sw, int lpg, int cb_shift, hipStream_t s, PanelPlan** out) {
  try {
    return build_plan_impl(A, transposed, ns, sw, lpg, cb_shift, s, out);
  } catch (const std::bad_alloc&) {
    *out = nullptr;
    return fail(GCN_ENOMEM, "panel plan: host allocation failed");
  }
}

void free_panel_plans(gcn_csr* A) {
  for (PanelPlan* p : A->plans) free_plan(p);
  A->plans.clear();
}

// Whether the column sweep serves this product, and in which shape: lane-group width sw (features), lanes per
// group, feature slices ns, and the column-block size 2^cb_shift.
static bool panel_shape(const SpmmArgs& a, int* sw_out, int* lpg_out, int* ns_out, int* cb_shift_out) {
  const int force = tune().spmm_panel;                   // 0: never, 1: whenever the limits allow
  if (force == 0 || !a.owner || a.n_rows < 1 || a.nnz < 1 || a.part != 0) return false;
  const size_t es = a.dtype == GCN_BF16 ? 2 : 4;
  // limits of the packed entry format and of 32-bit addressing of X
  const double xspan = (double)a.n_cols * (double)a.ldx * (double)es;
  if (a.n_cols >= (1 << kColBits) - 1 || a.ldx * (int64_t)es >= (1 << 24) || xspan >= 4294967296.0 || a.nnz >= 0xffffff00LL)      // (one thread per entry in the plan kernels: below 2^32 threads)
    return false;
  // the gathers are 16-byte vector loads
  auto aligned = [](const void* p, size_t al) { return ((uintptr_t)p % al) == 0; };
  const int V = a.dtype == GCN_BF16 ? 8 : 4;
  if (!((a.ldx % V) == 0 && aligned(a.X, 16) && ((a.d % V) == 0 || a.x_rows_padded))) return false;
  // lane-group shape: half a wavefront per row (128 fp32 features) for wide fp32 products, else 32
  // features per group (16 for products no wider than that)
  const bool wide = a.dtype == GCN_F32 && a.d >= 64 && !tune().panel_narrow;
  const int sw = wide ? 128 : a.d <= 16 ? 16 : 32;
  const int ns = (int)ceil_div(a.d, sw);
  // bytes of L2 one row of the operand occupies in an XCD that works on one slice
  const double foot = ns == 1 ? (double)a.d * (double)es : std::max(128.0, (double)sw * (double)es);
  int cb_shift = 10;
  while (cb_shift < 20 && (double)(2LL << cb_shift) * foot <= 2.0 * 1024 * 1024) ++cb_shift;
  if (force != 1) {
    // Worth it when (1) the operand is large enough to spill L2 and the gathers of one round re-read it
    // several times, and (2) a virtual row has several entries per column block, so that most entries
    // extend a run in registers instead of starting a new read-add-write of an accumulator row.
    // Measured, fp32, 233 k rows with 490 entries each (runs of 8.6 / 32 entries): width 128, half-wavefront
    // groups 3.2 ms, 8-lane groups 4.1 ms, row-per-wavefront kernel 7.3 ms; width 41: 2.6 against 3.4 ms.
    // 262 k rows with 45 entries each (runs of 0.7 / 2.8): 1.17 ms and 0.56 ms against 0.48 ms.  The bf16
    // instances do not beat the row-per-wavefront kernel (they are bound by instruction issue, not bytes).
    const int cap = std::min(kMaxVrows, kLdsBudget / (sw * 4));
    const double avg = (double)a.nnz / (double)a.n_rows;
    const double reuse = (double)(device_cus() / kPanelLists) * cap * avg / (double)a.n_cols;
    const double n_cb = std::ceil((double)a.n_cols / (double)(1LL << cb_shift));
    const double run = std::min(avg, 512.0) / n_cb;
    if (a.dtype != GCN_F32 || a.nnz < (1 << 20) || (double)a.n_cols * foot < 6.0 * 1024 * 1024 || reuse < 3.0 ||
        run < (wide ? 3.0 : 8.0))
      return false;
  }
  *sw_out = sw; *lpg_out = sw / V; *ns_out = ns; *cb_shift_out = cb_shift;
  return true;
}

bool spmm_panel_wanted(const SpmmArgs& a) {
  int sw, lpg, ns, cb_shift;
  return panel_shape(a, &sw, &lpg, &ns, &cb_shift);
}

int spmm_panel_try(const SpmmArgs& a, hipStream_t s, bool* used) {
  *used = false;
  int sw, lpg, ns, cb_shift;
  if (!panel_shape(a, &sw, &lpg, &ns, &cb_shift)) return GCN_OK;
  const size_t es = a.dtype == GCN_BF16 ? 2 : 4;
  const int n_wg = device_cus();

  PanelPlan* P = nullptr;
  for (PanelPlan* p : a.owner->plans)
    if (p->transposed == a.transposed && p->ns == ns && p->sw == sw && p->lpg == lpg && p->cb_shift == cb_shift) { P = p; break; }
  if (!P) {
    GCN_TRY(build_plan(a.owner, a.transposed, ns, sw, lpg, cb_shift, s, &P));
    if (!P) {
      // the matrix does not fit the packed format: remember that, so that later products of this shape fall back
      // at once instead of repeating the host pass over the rows
      P = new (std::nothrow) PanelPlan();
      if (!P) return GCN_OK;
      P->transposed = a.transposed; P->ns = ns; P->sw = sw; P->lpg = lpg; P->cb_shift = cb_shift; P->unusable = true;
    }
    try {
      a.owner->plans.push_back(P);
    } catch (const std::bad_alloc&) {
      free_plan(P);
      return fail(GCN_ENOMEM, "panel plan: host allocation failed");
    }
  }
  if (P->unusable) return GCN_OK;

  PanelK k{};                // (zeroes the fields of the embedded SpmmK that this kernel does not use)
  k.k.X = a.X; k.k.ldx = a.ldx; k.k.Y = a.Y; k.k.ldy = a.ldy; k.k.Y2 = a.Y2; k.k.ldy2 = a.ldy2;
  k.k.bias = a.bias; k.k.Zprev = a.Zprev; k.k.ldz = a.ldz; k.k.n_mask_rows = a.n_mask_rows;
  k.k.d = a.d; k.k.epilogue = a.epilogue; k.k.row_bytes = (uint32_t)(a.ldx * (int64_t)es);
  k.ent = P->ent; k.wb = P->wb; k.nfull = P->nfull; k.cbend = P->cbend; k.obase = P->obase;
  k.panel_row0 = P->panel_row0; k.row_v = P->row_v; k.vlds = P->vlds; k.order = P->order;
  k.ctr = P->ctr; k.n_panels = P->n_panels; k.ns = ns; k.n_cb = P->n_cb;
  k.soft_sync = tune().panel_nosync ? 0 : 1;      // experiment switch
  k.wg_per_list = std::max(1, n_wg / kPanelLists);
  const int64_t units = (int64_t)ns * P->n_panels;
  if (kPanelLists % ns == 0) {
    k.q = kPanelLists / ns;
    for (int i = 0; i < kPanelLists; ++i) {
      const int aoff = i % k.q;
      k.list_begin[i] = 0;
      k.list_len[i] = P->n_panels > aoff ? (int)ceil_div(P->n_panels - aoff, k.q) : 0;
    }
  } else {
    k.q = 0;
    for (int i = 0; i < kPanelLists; ++i) {
      const int64_t b = units * i / kPanelLists, e = units * (i + 1) / kPanelLists;
      k.list_begin[i] = (int)b; k.list_len[i] = (int)(e - b);
    }
  }
  const size_t lds = (size_t)((P->nv_max * sw + 3) & ~3) * sizeof(float);

  const double csr = 8.0 * (double)a.nnz + 8.0 * (double)(a.n_rows + 1), fe = (double)es * a.d;
  ProfScope ps(a.transposed ? GCN_K_SPMM_T : GCN_K_SPMM, s, a.d, a.dtype, a.n_rows, a.nnz,
               csr + fe * (double)(a.n_cols + a.n_rows), csr + fe * (double)(a.nnz + a.n_rows), 2.0 * (double)a.nnz * a.d);
  k_panel_reset<<<1, 64, 0, s>>>(P->ctr);
  int rc;
  if (a.dtype == GCN_BF16) rc = sw == 32 ? launch_panel<bf16_t, 8, 4>(k, n_wg, lds, s) : launch_panel<bf16_t, 8, 2>(k, n_wg, lds, s);
  else if (sw == 128) rc = launch_panel<float, 4, 32>(k, n_wg, lds, s);
  else rc = sw == 32 ? launch_panel<float, 4, 8>(k, n_wg, lds, s) : launch_panel<float, 4, 4>(k, n_wg, lds, s);
  GCN_TRY(rc);
  *used = true;
  return GCN_OK;
}

}  // namespace gcn
