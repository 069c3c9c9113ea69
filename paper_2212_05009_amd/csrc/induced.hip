// gcn_csr_induced: the normalised adjacency of the subgraph induced by a vertex list, built on the
// device from a whole-graph handle (Sec. 4.3.3: a mini-batch is a subgraph G' = (V', E') of the input
// graph, and convolutions run on it as they do on the whole graph in full-batch training).
//
// The subgraph is a graph of its own: vertex k is vertices[k], its edges are the stored entries
// (vertices[a], vertices[b]) of the parent, and degrees, self-loops and D^-1/2 (A'+I) D^-1/2 are
// those of the subgraph.  The entries of the selected rows are turned into an edge list in
// subgraph numbering - an entry whose column is not selected becomes a self-loop, which the
// builder drops like any other - and that list goes through gcn_csr_build, so sorting,
// normalisation and the column-major copy are the builder's.
#include "common.h"

namespace gcn {

constexpr int kIndThreads = 256;
static inline dim3 ind_grid(int64_t n) { return fold_grid(ceil_div(n > 0 ? n : 1, kIndThreads)); }

__global__ void k_ind_fill(int32_t* __restrict__ a, int64_t n, int32_t v) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n) a[i] = v;
}

// lid[vertices[k]] = k; ids out of range are reported, never used as an index
__global__ void k_ind_scatter(const int32_t* __restrict__ vertices, int64_t n_sub, int64_t n,
                              int32_t* __restrict__ lid, int* __restrict__ bad) {
  int64_t k = block_id() * blockDim.x + threadIdx.x;
  if (k >= n_sub) return;
  const int32_t v = vertices[k];
  if (v < 0 || v >= n) { *bad = 1; return; }
  lid[v] = (int32_t)k;
}

// a vertex listed twice keeps one of its two positions in lid: the other one sees a mismatch.
// Also the number of stored entries of each selected row.
__global__ void k_ind_rows(const int32_t* __restrict__ vertices, int64_t n_sub, const int32_t* __restrict__ lid,
                           const int64_t* __restrict__ rowptr, uint32_t* __restrict__ len, int* __restrict__ bad) {
  int64_t k = block_id() * blockDim.x + threadIdx.x;
  if (k >= n_sub) return;
  const int32_t v = vertices[k];
  if (lid[v] != (int32_t)k) *bad = 2;
  len[k] = (uint32_t)(rowptr[v + 1] - rowptr[v]);
}

__global__ void k_ind_edges(const int32_t* __restrict__ vertices, int64_t n_sub, const int64_t* __restrict__ off,
                            int64_t total, const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col,
                            const int32_t* __restrict__ lid, int32_t* __restrict__ src, int32_t* __restrict__ dst) {
  int64_t t = block_id() * blockDim.x + threadIdx.x;
  if (t >= total) return;
  int64_t lo = 0, hi = n_sub;                 // selected row k: the last one with off[k] <= t
  while (hi - lo > 1) {
    const int64_t m = (lo + hi) >> 1;
    if (off[m] <= t) lo = m; else hi = m;
  }
  const int64_t e = rowptr[vertices[lo]] + (t - off[lo]);
  const int32_t l = lid[col[e]];
  src[t] = (int32_t)lo;
  dst[t] = l >= 0 ? l : (int32_t)lo;
}

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_csr_induced(const gcn_csr_t* A, const int32_t* d_vertices, int64_t n_sub, int flags, void* stream,
                               gcn_csr_t** out) {
  clear_error();
  if (out) *out = nullptr;
  if (!A || !d_vertices || !out) return fail(GCN_EINVAL, "gcn_csr_induced: NULL argument");
  if (A->nh != 0 || A->nr != A->n_global)
    return fail(GCN_EINVAL, "gcn_csr_induced: needs the handle of a whole graph (every row, no halo columns)");
  if (n_sub < 1 || n_sub > A->nr) return fail(GCN_EINVAL, "gcn_csr_induced: need 1 <= n_sub <= number of vertices");
  hipStream_t s = (hipStream_t)stream;
  const int64_t n = A->nr;

  DevBuf lid, len, off, tmp, bad;
  GCN_TRY(lid.alloc(sizeof(int32_t) * (size_t)n));
  GCN_TRY(len.alloc(sizeof(uint32_t) * (size_t)n_sub));
  GCN_TRY(off.alloc(sizeof(int64_t) * (size_t)(n_sub + 1)));
  GCN_TRY(tmp.alloc(scan_tmp_bytes(n_sub)));
  GCN_TRY(bad.alloc(sizeof(int)));
  GCN_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), s));
  k_ind_fill<<<ind_grid(n), kIndThreads, 0, s>>>(lid.as<int32_t>(), n, -1);
  k_ind_scatter<<<ind_grid(n_sub), kIndThreads, 0, s>>>(d_vertices, n_sub, n, lid.as<int32_t>(), bad.as<int>());
  GCN_CHECK_LAUNCH();
  int h_bad = 0;
  GCN_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  if (h_bad) return fail(GCN_EINVAL, "gcn_csr_induced: a vertex id lies outside the graph");
  k_ind_rows<<<ind_grid(n_sub), kIndThreads, 0, s>>>(d_vertices, n_sub, lid.as<int32_t>(), A->rowptr,
                                                    len.as<uint32_t>(), bad.as<int>());
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(len.as<uint32_t>(), off.as<int64_t>(), n_sub, tmp.p, s));
  int64_t total = 0;
  GCN_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipMemcpyAsync(&total, off.as<int64_t>() + n_sub, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  if (h_bad) return fail(GCN_EINVAL, "gcn_csr_induced: a vertex is listed twice");

  DevBuf src, dst;
  GCN_TRY(src.alloc(sizeof(int32_t) * (size_t)total));
  GCN_TRY(dst.alloc(sizeof(int32_t) * (size_t)total));
  k_ind_edges<<<ind_grid(total), kIndThreads, 0, s>>>(d_vertices, n_sub, off.as<int64_t>(), total, A->rowptr, A->col,
                                                     lid.as<int32_t>(), src.as<int32_t>(), dst.as<int32_t>());
  GCN_CHECK_LAUNCH();
  return gcn_csr_build(src.as<int32_t>(), dst.as<int32_t>(), total, n_sub, 0, n_sub, nullptr, flags, stream, out);
}
