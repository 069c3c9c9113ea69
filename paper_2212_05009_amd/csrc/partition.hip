// gcn_partition_stats: what a 1D row partition costs in communication, counted on the device.
//
// Sec. 4.3.2 (hypergraph model): column j of A^ is a net that joins the rows with a stored entry
// in that column; the part that owns vertex j sends row j of H (and of G) once to every other part
// in the net's connectivity set, so the rows moved per sparse product are sum_j (lambda(n_j) - 1).
// Sec. 5 reports, per processor, the volume and the number of messages sent.
//
// One key per stored entry (i, j) whose ends lie in different parts:
//     key = (part[j] * p + part[i]) << jbits | j          (sender, receiver, row)
// Equal keys are the same transfer needed by several rows of the receiver: after a sort, the
// distinct keys are the transfers, and the runs of equal (sender, receiver) are the messages.
#include <algorithm>

#include "common.h"

namespace gcn {

constexpr int kPsThreads = 256;
static inline dim3 ps_grid(int64_t n) { return fold_grid(ceil_div(n > 0 ? n : 1, kPsThreads)); }

__global__ void k_ps_zero(int64_t* __restrict__ a, int64_t n) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n) a[i] = 0;
}

__global__ void k_ps_check(const int32_t* __restrict__ part, int64_t n, int p, int* __restrict__ bad) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n && (part[i] < 0 || part[i] >= p)) *bad = 1;
}

__global__ void k_ps_load(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ part, int64_t n,
                          int64_t* __restrict__ load) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= n) return;
  atomicAdd(reinterpret_cast<unsigned long long*>(load + part[i]), (unsigned long long)(rowptr[i + 1] - rowptr[i]));
}

// entries whose ends share a part get the key of the pair id p*p, which sorts behind every real pair
__global__ void k_ps_keys(const int64_t* __restrict__ rowptr, const int32_t* __restrict__ col, int64_t nnz, int64_t n,
                          const int32_t* __restrict__ part, int p, int jbits, uint64_t* __restrict__ keys) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  int64_t lo = 0, hi = n;                  // row i: the last one with rowptr[i] <= e
  while (hi - lo > 1) {
    const int64_t m = (lo + hi) >> 1;
    if (rowptr[m] <= e) lo = m; else hi = m;
  }
  const int64_t j = col[e];
  const uint64_t ps = (uint64_t)part[j], pr = (uint64_t)part[lo];
  const uint64_t pair = ps != pr ? ps * (uint64_t)p + pr : (uint64_t)p * (uint64_t)p;
  keys[e] = (pair << jbits) | (uint64_t)j;
}

__global__ void k_ps_flags(const uint64_t* __restrict__ keys, int64_t nnz, uint64_t first_invalid,
                           uint32_t* __restrict__ flag) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const uint64_t k = keys[e];
  flag[e] = k < first_invalid && (e == 0 || keys[e - 1] != k) ? 1u : 0u;
}

// pos[e] = distinct transfers before position e.  A run of one (sender, receiver) pair spans [a, b]: it
// holds pos[b + 1] - pos[a] transfers, added as two terms by the threads at its two ends.
__global__ void k_ps_pairs(const uint64_t* __restrict__ keys, const int64_t* __restrict__ pos, int64_t nnz, int p,
                           int jbits, uint64_t first_invalid, int64_t* __restrict__ send_rows,
                           int64_t* __restrict__ recv_rows, int64_t* __restrict__ send_msgs,
                           int64_t* __restrict__ recv_msgs, int64_t* __restrict__ totals) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const uint64_t k = keys[e];
  if (k >= first_invalid) return;
  const uint64_t pair = k >> jbits;
  const int ps = (int)(pair / (uint64_t)p), pr = (int)(pair % (uint64_t)p);
  typedef unsigned long long u64;
  const bool first = e == 0 || (keys[e - 1] >> jbits) != pair;
  const bool last = e == nnz - 1 || (keys[e + 1] >> jbits) != pair;
  if (first) {
    atomicAdd(reinterpret_cast<u64*>(send_rows + ps), (u64)(-pos[e]));
    atomicAdd(reinterpret_cast<u64*>(recv_rows + pr), (u64)(-pos[e]));
    atomicAdd(reinterpret_cast<u64*>(send_msgs + ps), (u64)1);
    atomicAdd(reinterpret_cast<u64*>(recv_msgs + pr), (u64)1);
  }
  if (last) {
    atomicAdd(reinterpret_cast<u64*>(send_rows + ps), (u64)pos[e + 1]);
    atomicAdd(reinterpret_cast<u64*>(recv_rows + pr), (u64)pos[e + 1]);
  }
  if (e == nnz - 1 || keys[e + 1] >= first_invalid) {      // the last entry that crosses parts
    totals[0] = pos[e + 1];
    totals[1] = e + 1;
  }
}

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_partition_stats(const gcn_csr_t* A, const int32_t* d_part, int p, int64_t* d_load,
                                   int64_t* d_send_rows, int64_t* d_recv_rows, int64_t* d_send_msgs,
                                   int64_t* d_recv_msgs, int64_t* d_totals, void* stream) {
  clear_error();
  if (!A || !d_part) return fail(GCN_EINVAL, "gcn_partition_stats: NULL argument");
  if (A->nh != 0 || A->nr != A->n_global)
    return fail(GCN_EINVAL, "gcn_partition_stats: needs the handle of a whole graph (every row, no halo columns)");
  if (p < 1 || p > 32768) return fail(GCN_EINVAL, "gcn_partition_stats: the number of parts must be in [1, 32768]");
  hipStream_t s = (hipStream_t)stream;
  const int64_t n = A->nr, nnz = A->nnz;

  // results the caller does not ask for still have to land somewhere
  DevBuf spare;
  GCN_TRY(spare.alloc(sizeof(int64_t) * (size_t)(5 * (int64_t)p + 2)));
  int64_t* sp = spare.as<int64_t>();
  int64_t* load = d_load ? d_load : sp;
  int64_t* send_rows = d_send_rows ? d_send_rows : sp + p;
  int64_t* recv_rows = d_recv_rows ? d_recv_rows : sp + 2 * (int64_t)p;
  int64_t* send_msgs = d_send_msgs ? d_send_msgs : sp + 3 * (int64_t)p;
  int64_t* recv_msgs = d_recv_msgs ? d_recv_msgs : sp + 4 * (int64_t)p;
  int64_t* totals = d_totals ? d_totals : sp + 5 * (int64_t)p;
  for (int64_t* a : {load, send_rows, recv_rows, send_msgs, recv_msgs}) k_ps_zero<<<ps_grid(p), kPsThreads, 0, s>>>(a, p);
  k_ps_zero<<<1, kPsThreads, 0, s>>>(totals, 2);
  GCN_CHECK_LAUNCH();

  DevBuf bad;
  GCN_TRY(bad.alloc(sizeof(int)));
  GCN_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), s));
  k_ps_check<<<ps_grid(n), kPsThreads, 0, s>>>(d_part, n, p, bad.as<int>());
  GCN_CHECK_LAUNCH();
  int h_bad = 0;
  GCN_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  if (h_bad) return fail(GCN_EINVAL, "gcn_partition_stats: a part id lies outside [0, p)");

  k_ps_load<<<ps_grid(n), kPsThreads, 0, s>>>(A->rowptr, d_part, n, load);
  GCN_CHECK_LAUNCH();
  if (nnz == 0) { GCN_HIP(hipStreamSynchronize(s)); return GCN_OK; }

  int jbits = 1;
  while (((int64_t)1 << jbits) < n) ++jbits;
  int pair_bits = 1;
  while (((uint64_t)1 << pair_bits) <= (uint64_t)p * (uint64_t)p) ++pair_bits;
  const uint64_t first_invalid = ((uint64_t)p * (uint64_t)p) << jbits;

  DevBuf ka, kb, tmp, flag, pos;
  GCN_TRY(ka.alloc(sizeof(uint64_t) * (size_t)nnz));
  GCN_TRY(kb.alloc(sizeof(uint64_t) * (size_t)nnz));
  GCN_TRY(tmp.alloc(std::max(sort_tmp_bytes(nnz), scan_tmp_bytes(nnz))));
  GCN_TRY(flag.alloc(sizeof(uint32_t) * (size_t)nnz));
  GCN_TRY(pos.alloc(sizeof(int64_t) * (size_t)(nnz + 1)));
  k_ps_keys<<<ps_grid(nnz), kPsThreads, 0, s>>>(A->rowptr, A->col, nnz, n, d_part, p, jbits, ka.as<uint64_t>());
  GCN_CHECK_LAUNCH();
  uint64_t* sorted = nullptr; uint32_t* unused = nullptr;
  GCN_TRY(radix_sort_u64(ka.as<uint64_t>(), kb.as<uint64_t>(), nullptr, nullptr, nnz, 0, jbits + pair_bits, tmp.p, s,
                         &sorted, &unused));
  k_ps_flags<<<ps_grid(nnz), kPsThreads, 0, s>>>(sorted, nnz, first_invalid, flag.as<uint32_t>());
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(flag.as<uint32_t>(), pos.as<int64_t>(), nnz, tmp.p, s));
  k_ps_pairs<<<ps_grid(nnz), kPsThreads, 0, s>>>(sorted, pos.as<int64_t>(), nnz, p, jbits, first_invalid, send_rows,
                                               recv_rows, send_msgs, recv_msgs, totals);
  GCN_CHECK_LAUNCH();
  GCN_HIP(hipStreamSynchronize(s));      // the temporaries are released on return
  return GCN_OK;
}
