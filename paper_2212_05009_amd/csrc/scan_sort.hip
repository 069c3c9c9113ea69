// Device-wide exclusive scan and stable LSD radix sort for gfx950 (64-wide wavefronts).
// These are the integer building blocks of the CSR / CSC / halo-list construction; all of
// their results are order-deterministic (no floating point, no order-dependent atomics).
#include "common.h"

namespace gcn {

// ------------------------------------------------------------------------------------------
// Exclusive scan, uint32 in -> int64 out, reduce-then-scan in three launches.
// ------------------------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

__device__ __forceinline__ int64_t wave_inclusive_scan(int64_t v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int64_t o = __shfl_up(v, off, 64);
    if (lane >= off) v += o;
  }
  return v;
}

// exclusive prefix of `v` over the 256 threads of the block; *total = block sum
__device__ __forceinline__ int64_t block_exclusive_scan(int64_t v, int64_t* total) {
  __shared__ int64_t wave_tot[kScanThreads / 64];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  int64_t inc = wave_inclusive_scan(v, lane);
  if (lane == 63) wave_tot[w] = inc;
  __syncthreads();
  int64_t base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < kScanThreads / 64; ++i) {
    int64_t t = wave_tot[i];
    if (i < w) base += t;
    tot += t;
  }
  __syncthreads();
  *total = tot;
  return base + inc - v;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_reduce(const uint32_t* __restrict__ in,
                                                              int64_t n, int64_t* __restrict__ sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int64_t s = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i)
    if (base + i < n) s += in[base + i];
  int64_t tot;
  block_exclusive_scan(s, &tot);
  if (threadIdx.x == 0) sums[blockIdx.x] = tot;
}

// one block: in-place exclusive scan of sums[0..m); writes the grand total to *total_out
__global__ __launch_bounds__(kScanThreads) void k_scan_sums(int64_t* __restrict__ sums, int64_t m,
                                                            int64_t* __restrict__ total_out) {
  int64_t carry = 0;
  for (int64_t c0 = 0; c0 < m; c0 += kScanThreads) {
    int64_t i = c0 + threadIdx.x;
    int64_t v = i < m ? sums[i] : 0;
    int64_t tot;
    int64_t ex = block_exclusive_scan(v, &tot);
    if (i < m) sums[i] = carry + ex;
    carry += tot;
  }
  if (threadIdx.x == 0) *total_out = carry;
}

__global__ __launch_bounds__(kScanThreads) void k_scan_apply(const uint32_t* __restrict__ in,
                                                             int64_t n, const int64_t* __restrict__ sums,
                                                             int64_t* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  int64_t s = 0;
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    v[i] = (base + i < n) ? in[base + i] : 0u;
    s += v[i];
  }
  int64_t tot;
  int64_t run = sums[blockIdx.x] + block_exclusive_scan(s, &tot);
#pragma unroll
  for (int i = 0; i < kScanItems; ++i) {
    if (base + i < n) out[base + i] = run;
    run += v[i];
  }
}

size_t scan_tmp_bytes(int64_t n) { return sizeof(int64_t) * (size_t)(ceil_div(n > 0 ? n : 1, kScanTile) + 1); }

int exclusive_scan_u32(const uint32_t* in, int64_t* out, int64_t n, void* tmp, hipStream_t s) {
  if (n < 0) return fail(GCN_EINVAL, "scan: negative size");
  if (n == 0) {
    GCN_HIP(hipMemsetAsync(out, 0, sizeof(int64_t), s));
    return GCN_OK;
  }
  const int64_t nb = ceil_div(n, kScanTile);
  if (nb * kScanThreads >= ((int64_t)1 << 32)) return fail(GCN_EINVAL, "scan: input too large for one launch");
  int64_t* sums = (int64_t*)tmp;
  k_scan_reduce<<<dim3((unsigned)nb), dim3(kScanThreads), 0, s>>>(in, n, sums);
  k_scan_sums<<<dim3(1), dim3(kScanThreads), 0, s>>>(sums, nb, out + n);
  k_scan_apply<<<dim3((unsigned)nb), dim3(kScanThreads), 0, s>>>(in, n, sums, out);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

// ------------------------------------------------------------------------------------------
// Stable LSD radix sort, 8 bits per pass.
// Per pass: (1) per-block digit histogram, (2) exclusive scan of the digit-major histogram
// table gives each (digit, block) its output offset, (3) every block ranks its keys stably
// and scatters them.  Stability inside a block: a wavefront owns a contiguous run of keys and
// walks it 64 keys at a time; keys with equal digits inside one step are ordered by lane
// (ballot match + popcount of lower lanes), steps are ordered by a running per-wave counter,
// waves are ordered by a prefix over the per-wave counters.
// ------------------------------------------------------------------------------------------
constexpr int kSortThreads = 256;
constexpr int kSortItems = 8;
constexpr int kSortTile = kSortThreads * kSortItems;
constexpr int kSortWaveRun = 64 * kSortItems;

__global__ __launch_bounds__(kSortThreads) void k_sort_hist(const uint64_t* __restrict__ keys,
                                                            int64_t n, int shift, int64_t nblocks,
                                                            uint32_t* __restrict__ hist) {
  __shared__ uint32_t h[256];
  h[threadIdx.x] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
#pragma unroll
  for (int i = 0; i < kSortItems; ++i) {
    int64_t idx = base + (int64_t)i * kSortThreads + threadIdx.x;
    if (idx < n) atomicAdd(&h[(uint32_t)(keys[idx] >> shift) & 255u], 1u);
  }
  __syncthreads();
  hist[(int64_t)threadIdx.x * nblocks + blockIdx.x] = h[threadIdx.x];
}

__global__ __launch_bounds__(kSortThreads) void k_sort_scatter(
    const uint64_t* __restrict__ keys_in, uint64_t* __restrict__ keys_out,
    const uint32_t* __restrict__ pay_in, uint32_t* __restrict__ pay_out, int64_t n, int shift,
    int64_t nblocks, const int64_t* __restrict__ offsets) {
  __shared__ uint32_t wave_cnt[kSortThreads / 64][256];
  __shared__ int64_t digit_base[256];
  const int t = threadIdx.x, w = t >> 6, lane = t & 63;
#pragma unroll
  for (int i = 0; i < kSortThreads / 64; ++i) wave_cnt[i][t] = 0;
  __syncthreads();

  const int64_t wave_base = (int64_t)blockIdx.x * kSortTile + (int64_t)w * kSortWaveRun;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  uint64_t key[kSortItems];
  uint32_t pay[kSortItems];
  uint32_t rank[kSortItems];
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const int64_t idx = wave_base + (int64_t)it * 64 + lane;
    const bool valid = idx < n;
    key[it] = valid ? keys_in[idx] : 0ull;
    pay[it] = (valid && pay_in) ? pay_in[idx] : 0u;
    const uint32_t dg = (uint32_t)(key[it] >> shift) & 255u;
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < 8; ++b) {
      const bool bit = (dg >> b) & 1u;
      const uint64_t bal = __ballot(valid && bit);
      peers &= bit ? bal : ~bal;
    }
    // peers: valid lanes of this step with the same digit (includes this lane when valid)
    const int leader = valid ? (__ffsll((unsigned long long)peers) - 1) : 0;
    uint32_t base = 0;
    if (valid && lane == leader) {
      base = wave_cnt[w][dg];
      wave_cnt[w][dg] = base + (uint32_t)__popcll(peers);
    }
    base = __shfl(base, leader, 64);
    rank[it] = base + (uint32_t)__popcll(peers & lt_mask);
  }
  __syncthreads();
  {
    uint32_t run = 0;
#pragma unroll
    for (int i = 0; i < kSortThreads / 64; ++i) {
      uint32_t c = wave_cnt[i][t];
      wave_cnt[i][t] = run;
      run += c;
    }
    digit_base[t] = offsets[(int64_t)t * nblocks + blockIdx.x];
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < kSortItems; ++it) {
    const int64_t idx = wave_base + (int64_t)it * 64 + lane;
    if (idx < n) {
      const uint32_t dg = (uint32_t)(key[it] >> shift) & 255u;
      const int64_t dst = digit_base[dg] + wave_cnt[w][dg] + rank[it];
      keys_out[dst] = key[it];
      if (pay_out) pay_out[dst] = pay[it];
    }
  }
}

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t sort_tmp_bytes(int64_t n) {
  const int64_t nb = ceil_div(n > 0 ? n : 1, kSortTile);
  const int64_t m = 256 * nb;
  return align256(sizeof(uint32_t) * (size_t)m) + align256(sizeof(int64_t) * (size_t)(m + 1)) +
         align256(scan_tmp_bytes(m));
}

int radix_sort_u64(uint64_t* keys_a, uint64_t* keys_b, uint32_t* pay_a, uint32_t* pay_b, int64_t n,
                   int bit_lo, int bit_hi, void* tmp, hipStream_t s, uint64_t** keys_out,
                   uint32_t** pay_out) {
  if (n < 0 || bit_lo < 0 || bit_hi > 64 || bit_hi < bit_lo) return fail(GCN_EINVAL, "sort: bad arguments");
  uint64_t* kin = keys_a; uint64_t* kout = keys_b;
  uint32_t* pin = pay_a;  uint32_t* pout = pay_b;
  if (n > 0) {
    const int64_t nb = ceil_div(n, kSortTile);
    if (nb * kSortThreads >= ((int64_t)1 << 32)) return fail(GCN_EINVAL, "sort: input too large for one launch");
    const int64_t m = 256 * nb;
    char* p = (char*)tmp;
    uint32_t* hist = (uint32_t*)p;          p += align256(sizeof(uint32_t) * (size_t)m);
    int64_t* offsets = (int64_t*)p;         p += align256(sizeof(int64_t) * (size_t)(m + 1));
    void* scan_tmp = p;
    for (int shift = bit_lo; shift < bit_hi; shift += 8) {
      k_sort_hist<<<dim3((unsigned)nb), dim3(kSortThreads), 0, s>>>(kin, n, shift, nb, hist);
      GCN_TRY(exclusive_scan_u32(hist, offsets, m, scan_tmp, s));
      k_sort_scatter<<<dim3((unsigned)nb), dim3(kSortThreads), 0, s>>>(kin, kout, pin, pay_a ? pout : nullptr,
                                                                        n, shift, nb, offsets);
      GCN_CHECK_LAUNCH();
      uint64_t* tk = kin; kin = kout; kout = tk;
      uint32_t* tp = pin; pin = pout; pout = tp;
    }
  }
  *keys_out = kin;
  if (pay_out) *pay_out = pin;
  return GCN_OK;
}

}  // namespace gcn
