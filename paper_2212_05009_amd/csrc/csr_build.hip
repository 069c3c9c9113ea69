// gcn_csr_build: normalised adjacency block in CSR (+CSC), halo index list, degree counts and
// the row-binned execution schedules, all built on the device (Sec. 3.1: A^ = D^-1/2 (A+I) D^-1/2;
// Sec. 4.1: the non-owned columns of the block are the rows to receive, each listed once).
#include <new>

#include "common.h"

namespace gcn {

constexpr int kThreads = 256;
static inline dim3 grid_for(int64_t n) { return fold_grid(ceil_div(n > 0 ? n : 1, kThreads)); }

// ---- step 1: id validation ------------------------------------------------------------------
__global__ void k_validate(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                           int64_t n_edges, int64_t n_global, int* __restrict__ bad) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  int32_t s = src[e], t = dst[e];
  if (s < 0 || s >= n_global || t < 0 || t >= n_global) atomicOr(bad, 1);
}

__global__ void k_validate_deg(const int32_t* __restrict__ deg, int64_t n, int* __restrict__ bad) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n && deg[i] < 1) atomicOr(bad, 2);
}

// ---- step 2: halo set as a bitmap over global ids -------------------------------------------
__global__ void k_mark_halo(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                            int64_t n_edges, int64_t row_lo, int64_t row_hi,
                            uint32_t* __restrict__ bitmap) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  int64_t s = src[e], t = dst[e];
  if (s >= row_lo && s < row_hi && (t < row_lo || t >= row_hi))
    atomicOr(&bitmap[t >> 5], 1u << (t & 31));
}

__global__ void k_popc(const uint32_t* __restrict__ bitmap, int64_t words, uint32_t* __restrict__ cnt) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < words) cnt[i] = (uint32_t)__popc(bitmap[i]);
}

__global__ void k_halo_list(const uint32_t* __restrict__ bitmap, const int64_t* __restrict__ wprefix,
                            int64_t words, int32_t* __restrict__ halo_gid) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= words) return;
  uint32_t w = bitmap[i];
  int64_t p = wprefix[i];
  while (w) {
    int b = __ffs(w) - 1;
    halo_gid[p++] = (int32_t)(i * 32 + b);
    w &= w - 1;
  }
}

// ---- step 3: (row, local column) keys ---------------------------------------------------------
constexpr uint64_t kInvalidKey = ~0ull;

__global__ void k_make_keys(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                            int64_t n_edges, int64_t row_lo, int64_t row_hi, int64_t nr, int colbits,
                            const uint32_t* __restrict__ bitmap, const int64_t* __restrict__ wprefix,
                            uint64_t* __restrict__ keys) {
  int64_t e = block_id() * blockDim.x + threadIdx.x;
  if (e >= n_edges + nr) return;
  if (e >= n_edges) {                      // the diagonal of I, one entry per owned row
    uint64_t i = (uint64_t)(e - n_edges);
    keys[e] = (i << colbits) | i;
    return;
  }
  int64_t s = src[e], t = dst[e];
  uint64_t k = kInvalidKey;
  if (s >= row_lo && s < row_hi && s != t) {
    uint64_t lc;
    if (t >= row_lo && t < row_hi) {
      lc = (uint64_t)(t - row_lo);
    } else {
      uint32_t w = bitmap[t >> 5];
      lc = (uint64_t)(nr + wprefix[t >> 5] + __popc(w & ((1u << (t & 31)) - 1u)));
    }
    k = ((uint64_t)(s - row_lo) << colbits) | lc;
  }
  keys[e] = k;
}

// ---- step 4: duplicate removal ------------------------------------------------------------------
__global__ void k_flag_unique(const uint64_t* __restrict__ keys, int64_t m, uint32_t* __restrict__ flag) {
  int64_t k = block_id() * blockDim.x + threadIdx.x;
  if (k >= m) return;
  uint64_t v = keys[k];
  flag[k] = (v != kInvalidKey && (k == 0 || keys[k - 1] != v)) ? 1u : 0u;
}

__global__ void k_compact(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ flag,
                          const int64_t* __restrict__ pos, int64_t m, int colbits,
                          uint64_t* __restrict__ ukeys, int32_t* __restrict__ col) {
  int64_t k = block_id() * blockDim.x + threadIdx.x;
  if (k >= m || !flag[k]) return;
  uint64_t v = keys[k];
  int64_t p = pos[k];
  ukeys[p] = v;
  col[p] = (int32_t)(v & ((1ull << colbits) - 1ull));
}

// ptr[q] = first position whose segment id is >= q, for q in [0, n_seg]; seg ids are the bits
// of key[k] from `shift` upwards and are non-decreasing in k.  Requires n >= 1.
__global__ void k_boundaries(const uint64_t* __restrict__ key, int64_t n, int shift, int64_t n_seg,
                             int64_t* __restrict__ ptr) {
  int64_t k = block_id() * blockDim.x + threadIdx.x;
  if (k >= n) return;
  int64_t s = (int64_t)(key[k] >> shift);
  int64_t sp = k == 0 ? -1 : (int64_t)(key[k - 1] >> shift);
  for (int64_t q = sp + 1; q <= s; ++q) ptr[q] = k;
  if (k == n - 1)
    for (int64_t q = s + 1; q <= n_seg; ++q) ptr[q] = n;
}

__global__ void k_row_lengths(const int64_t* __restrict__ ptr, int64_t n, int32_t* __restrict__ len) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n) len[i] = (int32_t)(ptr[i + 1] - ptr[i]);
}

// first entry of each row whose (local) column is >= nr: columns are ascending, so the owned columns come first
__global__ void k_row_mid(const int64_t* __restrict__ ptr, const int32_t* __restrict__ col, int64_t nr,
                          int64_t* __restrict__ mid) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= nr) return;
  int64_t lo = ptr[i], hi = ptr[i + 1];
  while (lo < hi) {
    const int64_t m = (lo + hi) >> 1;
    if (col[m] < nr) lo = m + 1; else hi = m;
  }
  mid[i] = lo;
}

// ---- step 5: values ---------------------------------------------------------------------------------
// val(i,j) = fl(1/sqrt(d_i)) * fl(1/sqrt(d_j)), each operation correctly rounded in fp32.
// Both steps go through fp64: an fp64 square root or quotient rounded once more to fp32 equals the
// correctly rounded fp32 result (53 >= 2*24 + 2 bits), whatever the fp32 code generation options are.
__device__ __forceinline__ float inv_sqrt_deg(int32_t d) {
  const float r = (float)sqrt((double)(float)d);
  return (float)(1.0 / (double)r);
}

__global__ void k_values(const uint64_t* __restrict__ ukeys, int64_t nnz, int colbits, int64_t nr,
                         int64_t row_lo, const int32_t* __restrict__ deg_local,
                         const int32_t* __restrict__ deg_global, const int32_t* __restrict__ halo_gid,
                         float* __restrict__ val) {
  int64_t p = block_id() * blockDim.x + threadIdx.x;
  if (p >= nnz) return;
  uint64_t v = ukeys[p];
  int64_t i = (int64_t)(v >> colbits);
  int64_t c = (int64_t)(v & ((1ull << colbits) - 1ull));
  // an owned vertex's degree is the entry count of its row, which the block holds whole (Sec. 4.1); a halo
  // vertex's row lives elsewhere: its degree comes from the caller's global array
  (void)row_lo;
  const int32_t di = deg_local[i];
  const int32_t dj = c < nr ? deg_local[c] : deg_global[halo_gid[c - nr]];
  val[p] = __fmul_rn(inv_sqrt_deg(di), inv_sqrt_deg(dj));
}

// ---- step 6: column-major copy ------------------------------------------------------------------------
__global__ void k_make_tkeys(const uint64_t* __restrict__ ukeys, int64_t nnz, int colbits,
                             uint64_t* __restrict__ tkeys, uint32_t* __restrict__ pay) {
  int64_t p = block_id() * blockDim.x + threadIdx.x;
  if (p >= nnz) return;
  uint64_t v = ukeys[p];
  uint64_t i = v >> colbits, c = v & ((1ull << colbits) - 1ull);
  tkeys[p] = (c << 32) | i;
  pay[p] = (uint32_t)p;
}

__global__ void k_finish_csc(const uint64_t* __restrict__ tkeys, const uint32_t* __restrict__ pay,
                             const float* __restrict__ val, int64_t nnz, int32_t* __restrict__ rowidx,
                             float* __restrict__ val_t) {
  int64_t q = block_id() * blockDim.x + threadIdx.x;
  if (q >= nnz) return;
  rowidx[q] = (int32_t)(tkeys[q] & 0xffffffffull);
  val_t[q] = val[pay[q]];
}

// ---- schedules ------------------------------------------------------------------------------------------
__global__ void k_sched_keys(const int64_t* __restrict__ ptr, int64_t n, uint64_t* __restrict__ keys,
                             uint32_t* __restrict__ hub_flag, uint32_t* __restrict__ hub_chunks) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= n) return;
  int64_t len = ptr[i + 1] - ptr[i];
  bool hub = len > kHubRowNnz;
  hub_flag[i] = hub ? 1u : 0u;
  hub_chunks[i] = hub ? (uint32_t)((len + kHubChunkNnz - 1) / kHubChunkNnz) : 0u;
  // longest rows first: class 0 holds lengths in [2^31, ..), class 31 length 1, class 32 empty rows
  uint32_t cls = len > 0 ? (uint32_t)__clzll((unsigned long long)len) - 32u : 32u;
  keys[i] = hub ? kInvalidKey : (((uint64_t)cls << 32) | (uint64_t)i);
}

__global__ void k_take_low32(const uint64_t* __restrict__ keys, int64_t n, int32_t* __restrict__ out) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i < n) out[i] = (int32_t)(keys[i] & 0xffffffffull);
}

__global__ void k_hub_lists(const uint32_t* __restrict__ hub_flag, const int64_t* __restrict__ hub_pos,
                            const uint32_t* __restrict__ hub_chunks, const int64_t* __restrict__ chunk_pos,
                            int64_t n, int64_t n_hub, int32_t* __restrict__ hub_rows,
                            int64_t* __restrict__ hub_chunk_ptr, int32_t* __restrict__ chunk_hub) {
  int64_t i = block_id() * blockDim.x + threadIdx.x;
  if (i >= n || !hub_flag[i]) return;
  int64_t h = hub_pos[i];
  hub_rows[h] = (int32_t)i;
  int64_t c0 = chunk_pos[i];
  hub_chunk_ptr[h] = c0;
  if (h == n_hub - 1) hub_chunk_ptr[n_hub] = c0 + hub_chunks[i];
  for (uint32_t c = 0; c < hub_chunks[i]; ++c) chunk_hub[c0 + c] = (int32_t)h;
}

// Row boundaries in the schedule's lists.  For boundary j (row bound[j]): out[j * 35 + c], c < 33, = first position
// of class c (list positions cb[c] .. cb[c + 1], rows ascending) whose row is >= bound[j]; out[j * 35 + 33] = first
// hub row (ascending list of n_hub rows) >= bound[j]; out[j * 35 + 34] = that hub row's first chunk of entries.
__global__ void k_chunk_bounds(const int32_t* __restrict__ wave_rows, const int64_t* __restrict__ cb,
                               const int32_t* __restrict__ hub_rows, int64_t n_hub,
                               const int64_t* __restrict__ hub_chunk_ptr, const int64_t* __restrict__ bound,
                               int n_bounds, int64_t* __restrict__ out) {
  const int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_bounds * 34) return;
  const int j = t / 34, c = t % 34;
  const int32_t* list = c < 33 ? wave_rows : hub_rows;
  int64_t lo = c < 33 ? cb[c] : 0, hi = c < 33 ? cb[c + 1] : n_hub;
  const int64_t r = bound[j];
  while (lo < hi) {
    const int64_t mid = lo + (hi - lo) / 2;
    if ((int64_t)list[mid] < r) lo = mid + 1; else hi = mid;
  }
  out[j * 35 + c] = lo;
  if (c == 33) out[j * 35 + 34] = hub_chunk_ptr[lo];
}

void free_schedule(Schedule* sc) {
  if (sc->wave_rows) (void)hipFree(sc->wave_rows);
  if (sc->hub_rows) (void)hipFree(sc->hub_rows);
  if (sc->hub_chunk_ptr) (void)hipFree(sc->hub_chunk_ptr);
  if (sc->chunk_hub) (void)hipFree(sc->chunk_hub);
  *sc = Schedule();
}

int build_schedule(const int64_t* ptr, int64_t n, hipStream_t s, Schedule* out) {
  *out = Schedule();
  DevBuf keys_a, keys_b, hub_flag, hub_chunks, hub_pos, chunk_pos, tmp;
  GCN_TRY(keys_a.alloc(sizeof(uint64_t) * (size_t)n));
  GCN_TRY(keys_b.alloc(sizeof(uint64_t) * (size_t)n));
  GCN_TRY(hub_flag.alloc(sizeof(uint32_t) * (size_t)n));
  GCN_TRY(hub_chunks.alloc(sizeof(uint32_t) * (size_t)n));
  GCN_TRY(hub_pos.alloc(sizeof(int64_t) * (size_t)(n + 1)));
  GCN_TRY(chunk_pos.alloc(sizeof(int64_t) * (size_t)(n + 1)));
  size_t tb = sort_tmp_bytes(n);
  if (scan_tmp_bytes(n) > tb) tb = scan_tmp_bytes(n);
  GCN_TRY(tmp.alloc(tb));

  k_sched_keys<<<grid_for(n), kThreads, 0, s>>>(ptr, n, keys_a.as<uint64_t>(), hub_flag.as<uint32_t>(),
                                                 hub_chunks.as<uint32_t>());
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(hub_flag.as<uint32_t>(), hub_pos.as<int64_t>(), n, tmp.p, s));
  GCN_TRY(exclusive_scan_u32(hub_chunks.as<uint32_t>(), chunk_pos.as<int64_t>(), n, tmp.p, s));
  int64_t n_hub = 0, n_chunks = 0;
  GCN_HIP(hipMemcpyAsync(&n_hub, hub_pos.as<int64_t>() + n, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipMemcpyAsync(&n_chunks, chunk_pos.as<int64_t>() + n, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));

  uint64_t* sorted = nullptr;
  GCN_TRY(radix_sort_u64(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), nullptr, nullptr, n, 32, 40, tmp.p, s,
                         &sorted, nullptr));
  DevBuf wave_rows, hub_rows, hub_chunk_ptr, chunk_hub;
  const int64_t n_wave = n - n_hub;
  GCN_TRY(wave_rows.alloc(sizeof(int32_t) * (size_t)(n_wave > 0 ? n_wave : 1)));
  GCN_TRY(hub_rows.alloc(sizeof(int32_t) * (size_t)(n_hub > 0 ? n_hub : 1)));
  GCN_TRY(hub_chunk_ptr.alloc(sizeof(int64_t) * (size_t)(n_hub + 1)));
  GCN_TRY(chunk_hub.alloc(sizeof(int32_t) * (size_t)(n_chunks > 0 ? n_chunks : 1)));
  DevBuf class_begin;
  GCN_TRY(class_begin.alloc(sizeof(int64_t) * 34));
  GCN_HIP(hipMemsetAsync(class_begin.p, 0, sizeof(int64_t) * 34, s));
  if (n_wave > 0) {
    k_take_low32<<<grid_for(n_wave), kThreads, 0, s>>>(sorted, n_wave, wave_rows.as<int32_t>());
    k_boundaries<<<grid_for(n_wave), kThreads, 0, s>>>(sorted, n_wave, 32, 33, class_begin.as<int64_t>());
  }
  GCN_HIP(hipMemcpyAsync(out->class_begin, class_begin.p, sizeof(int64_t) * 34, hipMemcpyDeviceToHost, s));
  GCN_HIP(hipMemsetAsync(hub_chunk_ptr.p, 0, sizeof(int64_t) * (size_t)(n_hub + 1), s));
  if (n_hub > 0)
    k_hub_lists<<<grid_for(n), kThreads, 0, s>>>(hub_flag.as<uint32_t>(), hub_pos.as<int64_t>(),
                                                  hub_chunks.as<uint32_t>(), chunk_pos.as<int64_t>(), n, n_hub,
                                                  hub_rows.as<int32_t>(), hub_chunk_ptr.as<int64_t>(),
                                                  chunk_hub.as<int32_t>());
  GCN_CHECK_LAUNCH();
  // the class lists and the hub list cut at kRowChunks row boundaries (multiples of 64 rows)
  DevBuf chunk_bound, chunk_cb;
  constexpr int kChunkTable = (kRowChunks + 1) * 35;
  GCN_TRY(chunk_bound.alloc(sizeof(int64_t) * (kRowChunks + 1)));
  GCN_TRY(chunk_cb.alloc(sizeof(int64_t) * kChunkTable));
  int64_t chunk_table[kChunkTable];
  for (int j = 0; j <= kRowChunks; ++j) {
    const int64_t r = round_up(ceil_div(n * j, kRowChunks), 64);
    out->chunk_row[j] = j == kRowChunks || r > n ? n : r;
  }
  GCN_HIP(hipMemcpyAsync(chunk_bound.p, out->chunk_row, sizeof(int64_t) * (kRowChunks + 1), hipMemcpyHostToDevice, s));
  k_chunk_bounds<<<(unsigned)ceil_div((kRowChunks + 1) * 34, 256), 256, 0, s>>>(
      wave_rows.as<int32_t>(), class_begin.as<int64_t>(), hub_rows.as<int32_t>(), n_hub, hub_chunk_ptr.as<int64_t>(),
      chunk_bound.as<int64_t>(), kRowChunks + 1, chunk_cb.as<int64_t>());
  GCN_CHECK_LAUNCH();
  GCN_HIP(hipMemcpyAsync(chunk_table, chunk_cb.p, sizeof(chunk_table), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));   // temporaries are freed on return
  for (int j = 0; j <= kRowChunks; ++j) {
    for (int c = 0; c < 33; ++c) out->chunk_class_begin[j][c] = chunk_table[j * 35 + c];
    out->chunk_hub_begin[j] = chunk_table[j * 35 + 33];
    out->chunk_hubchunk_begin[j] = chunk_table[j * 35 + 34];
  }
  out->wave_rows = (int32_t*)wave_rows.release();
  out->n_wave_rows = n_wave;
  out->hub_rows = (int32_t*)hub_rows.release();
  out->n_hub_rows = n_hub;
  out->hub_chunk_ptr = (int64_t*)hub_chunk_ptr.release();
  out->chunk_hub = (int32_t*)chunk_hub.release();
  out->n_chunks = n_chunks;
  return GCN_OK;
}

static int bits_for(int64_t max_value_exclusive) {   // smallest b with 2^b - 1 > max_value_exclusive - 1 ... i.e. 2^b > max_value_exclusive
  int b = 1;
  while ((1LL << b) <= max_value_exclusive) ++b;
  return b;
}

static int build_impl(const int32_t* d_src, const int32_t* d_dst, int64_t n_edges, int64_t n_global,
                      int64_t row_lo, int64_t row_hi, const int32_t* d_deg_global, int flags,
                      hipStream_t s, gcn_csr* A) {
  const int64_t nr = row_hi - row_lo;
  const bool whole = (row_lo == 0 && row_hi == n_global);
  const int64_t m = n_edges + nr;          // candidate entries: edges + diagonal

  // -- validation and halo bitmap
  const int64_t words = ceil_div(n_global, 32);
  DevBuf bad, bitmap, wcnt, wprefix, tmp;
  GCN_TRY(bad.alloc(sizeof(int)));
  GCN_TRY(bitmap.alloc(sizeof(uint32_t) * (size_t)words));
  GCN_TRY(wcnt.alloc(sizeof(uint32_t) * (size_t)words));
  GCN_TRY(wprefix.alloc(sizeof(int64_t) * (size_t)(words + 1)));
  size_t tb = sort_tmp_bytes(m);
  if (scan_tmp_bytes(m) > tb) tb = scan_tmp_bytes(m);
  if (scan_tmp_bytes(words) > tb) tb = scan_tmp_bytes(words);
  GCN_TRY(tmp.alloc(tb));
  GCN_HIP(hipMemsetAsync(bad.p, 0, sizeof(int), s));
  GCN_HIP(hipMemsetAsync(bitmap.p, 0, sizeof(uint32_t) * (size_t)words, s));
  if (n_edges > 0) {
    k_validate<<<grid_for(n_edges), kThreads, 0, s>>>(d_src, d_dst, n_edges, n_global, bad.as<int>());
    GCN_CHECK_LAUNCH();
  }
  if (d_deg_global) k_validate_deg<<<grid_for(n_global), kThreads, 0, s>>>(d_deg_global, n_global, bad.as<int>());
  int h_bad = 0;
  GCN_HIP(hipMemcpyAsync(&h_bad, bad.p, sizeof(int), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  if (h_bad & 1) return fail(GCN_EINVAL, "gcn_csr_build: a vertex id lies outside [0, n_global)");
  if (h_bad & 2) return fail(GCN_EINVAL, "gcn_csr_build: d_deg_global holds a degree < 1");

  if (n_edges > 0) k_mark_halo<<<grid_for(n_edges), kThreads, 0, s>>>(d_src, d_dst, n_edges, row_lo, row_hi, bitmap.as<uint32_t>());
  k_popc<<<grid_for(words), kThreads, 0, s>>>(bitmap.as<uint32_t>(), words, wcnt.as<uint32_t>());
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(wcnt.as<uint32_t>(), wprefix.as<int64_t>(), words, tmp.p, s));
  int64_t nh = 0;
  GCN_HIP(hipMemcpyAsync(&nh, wprefix.as<int64_t>() + words, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  const int64_t nc = nr + nh;
  if (nc >= 0x7fffffffLL) return fail(GCN_EINVAL, "gcn_csr_build: more than 2^31-1 local columns");
  DevBuf halo_gid;
  GCN_TRY(halo_gid.alloc(sizeof(int32_t) * (size_t)(nh > 0 ? nh : 1)));
  if (nh > 0) k_halo_list<<<grid_for(words), kThreads, 0, s>>>(bitmap.as<uint32_t>(), wprefix.as<int64_t>(), words, halo_gid.as<int32_t>());
  GCN_CHECK_LAUNCH();

  // -- keys, sort, unique
  const int colbits = bits_for(nc);
  const int rowbits = bits_for(nr);
  if (colbits + rowbits > 62) return fail(GCN_EINVAL, "gcn_csr_build: block too large for 64-bit sort keys");
  DevBuf keys_a, keys_b, flag, pos;
  GCN_TRY(keys_a.alloc(sizeof(uint64_t) * (size_t)m));
  GCN_TRY(keys_b.alloc(sizeof(uint64_t) * (size_t)m));
  k_make_keys<<<grid_for(m), kThreads, 0, s>>>(d_src, d_dst, n_edges, row_lo, row_hi, nr, colbits,
                                                bitmap.as<uint32_t>(), wprefix.as<int64_t>(), keys_a.as<uint64_t>());
  GCN_CHECK_LAUNCH();
  uint64_t* sorted = nullptr;
  GCN_TRY(radix_sort_u64(keys_a.as<uint64_t>(), keys_b.as<uint64_t>(), nullptr, nullptr, m, 0, colbits + rowbits,
                         tmp.p, s, &sorted, nullptr));
  uint64_t* other = (sorted == keys_a.as<uint64_t>()) ? keys_b.as<uint64_t>() : keys_a.as<uint64_t>();
  GCN_TRY(flag.alloc(sizeof(uint32_t) * (size_t)m));
  GCN_TRY(pos.alloc(sizeof(int64_t) * (size_t)(m + 1)));
  k_flag_unique<<<grid_for(m), kThreads, 0, s>>>(sorted, m, flag.as<uint32_t>());
  GCN_CHECK_LAUNCH();
  GCN_TRY(exclusive_scan_u32(flag.as<uint32_t>(), pos.as<int64_t>(), m, tmp.p, s));
  int64_t nnz = 0;
  GCN_HIP(hipMemcpyAsync(&nnz, pos.as<int64_t>() + m, sizeof(int64_t), hipMemcpyDeviceToHost, s));
  GCN_HIP(hipStreamSynchronize(s));
  if (nnz < nr) return fail(GCN_EHIP, "gcn_csr_build: internal error (nnz %lld < rows %lld)", (long long)nnz, (long long)nr);
  if (nnz >= 0xffffffffLL) return fail(GCN_EINVAL, "gcn_csr_build: more than 2^32-2 stored entries in one block");

  DevBuf rowptr, col, val, deg;
  GCN_TRY(rowptr.alloc(sizeof(int64_t) * (size_t)(nr + 1)));
  GCN_TRY(col.alloc(sizeof(int32_t) * (size_t)nnz));
  GCN_TRY(val.alloc(sizeof(float) * (size_t)nnz));
  GCN_TRY(deg.alloc(sizeof(int32_t) * (size_t)nr));
  uint64_t* ukeys = other;                  // unique keys, row-major order
  k_compact<<<grid_for(m), kThreads, 0, s>>>(sorted, flag.as<uint32_t>(), pos.as<int64_t>(), m, colbits, ukeys, col.as<int32_t>());
  k_boundaries<<<grid_for(nnz), kThreads, 0, s>>>(ukeys, nnz, colbits, nr, rowptr.as<int64_t>());
  k_row_lengths<<<grid_for(nr), kThreads, 0, s>>>(rowptr.as<int64_t>(), nr, deg.as<int32_t>());
  k_values<<<grid_for(nnz), kThreads, 0, s>>>(ukeys, nnz, colbits, nr, row_lo, deg.as<int32_t>(),
                                               whole && !d_deg_global ? nullptr : d_deg_global,
                                               halo_gid.as<int32_t>(), val.as<float>());
  GCN_CHECK_LAUNCH();

  DevBuf mid;
  if (nh > 0) {
    GCN_TRY(mid.alloc(sizeof(int64_t) * (size_t)nr));
    k_row_mid<<<grid_for(nr), kThreads, 0, s>>>(rowptr.as<int64_t>(), col.as<int32_t>(), nr, mid.as<int64_t>());
    GCN_CHECK_LAUNCH();
  }

  // -- column-major copy
  DevBuf colptr, rowidx, val_t;
  if (flags & GCN_BUILD_CSC) {
    DevBuf pay_a, pay_b;
    GCN_TRY(pay_a.alloc(sizeof(uint32_t) * (size_t)nnz));
    GCN_TRY(pay_b.alloc(sizeof(uint32_t) * (size_t)nnz));
    GCN_TRY(colptr.alloc(sizeof(int64_t) * (size_t)(nc + 1)));
    GCN_TRY(rowidx.alloc(sizeof(int32_t) * (size_t)nnz));
    GCN_TRY(val_t.alloc(sizeof(float) * (size_t)nnz));
    uint64_t* tk_a = sorted;               // the sorted-with-duplicates buffer is free again
    k_make_tkeys<<<grid_for(nnz), kThreads, 0, s>>>(ukeys, nnz, colbits, tk_a, pay_a.as<uint32_t>());
    GCN_CHECK_LAUNCH();
    // ukeys lives in `other`; the sort ping-pongs between tk_a and a third buffer
    DevBuf tk_b;
    GCN_TRY(tk_b.alloc(sizeof(uint64_t) * (size_t)nnz));
    uint64_t* tsorted = nullptr; uint32_t* psorted = nullptr;
    GCN_TRY(radix_sort_u64(tk_a, tk_b.as<uint64_t>(), pay_a.as<uint32_t>(), pay_b.as<uint32_t>(), nnz, 32,
                           32 + colbits, tmp.p, s, &tsorted, &psorted));
    k_boundaries<<<grid_for(nnz), kThreads, 0, s>>>(tsorted, nnz, 32, nc, colptr.as<int64_t>());
    k_finish_csc<<<grid_for(nnz), kThreads, 0, s>>>(tsorted, psorted, val.as<float>(), nnz, rowidx.as<int32_t>(), val_t.as<float>());
    GCN_CHECK_LAUNCH();
    GCN_HIP(hipStreamSynchronize(s));
  }
  GCN_HIP(hipStreamSynchronize(s));

  A->n_global = n_global; A->row_lo = row_lo;
  A->nr = nr; A->nh = nh; A->nc = nc; A->nnz = nnz;
  GCN_TRY(build_schedule(rowptr.as<int64_t>(), nr, s, &A->sched));
  if (flags & GCN_BUILD_CSC) GCN_TRY(build_schedule(colptr.as<int64_t>(), nc, s, &A->sched_t));
  A->rowptr = (int64_t*)rowptr.release(); A->col = (int32_t*)col.release();
  A->val = (float*)val.release(); A->deg = (int32_t*)deg.release();
  A->halo_gid = (int32_t*)halo_gid.release();
  A->colptr = (int64_t*)colptr.release(); A->rowidx = (int32_t*)rowidx.release();
  A->val_t = (float*)val_t.release();
  A->mid = nh > 0 ? (int64_t*)mid.release() : nullptr;
  return GCN_OK;
}

int segment_boundaries(const uint64_t* keys, int64_t n, int shift, int64_t n_seg, int64_t* ptr, hipStream_t s) {
  if (n < 1) return fail(GCN_EINVAL, "segment_boundaries: empty input");
  k_boundaries<<<grid_for(n), kThreads, 0, s>>>(keys, n, shift, n_seg, ptr);
  GCN_CHECK_LAUNCH();
  return GCN_OK;
}

int ensure_workspace(gcn_csr* A, size_t bytes) {
  if (bytes <= A->ws_bytes) return GCN_OK;
  if (A->ws) {
    GCN_HIP(hipDeviceSynchronize());
    (void)hipFree(A->ws);
    A->ws = nullptr; A->ws_bytes = 0;
  }
  size_t want = (size_t)round_up((int64_t)bytes, 1 << 20);
  hipError_t e = hipMalloc(&A->ws, want);
  if (e != hipSuccess) { A->ws = nullptr; return fail(GCN_ENOMEM, "workspace of %zu bytes: %s", want, hipGetErrorString(e)); }
  A->ws_bytes = want;
  return GCN_OK;
}

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_csr_build(const int32_t* d_src, const int32_t* d_dst, int64_t n_edges, int64_t n_global,
                             int64_t row_lo, int64_t row_hi, const int32_t* d_deg_global, int flags,
                             void* stream, gcn_csr_t** out) {
  clear_error();
  if (!out) return fail(GCN_EINVAL, "gcn_csr_build: out is NULL");
  *out = nullptr;
  if (n_edges < 0 || (n_edges > 0 && (!d_src || !d_dst))) return fail(GCN_EINVAL, "gcn_csr_build: bad edge list");
  if (n_global < 1 || n_global > 0x7fffffffLL) return fail(GCN_EINVAL, "gcn_csr_build: n_global must be in [1, 2^31)");
  // entry positions travel through the sorts as 32-bit payloads
  if (n_edges + n_global >= 0xffffffffLL) return fail(GCN_EINVAL, "gcn_csr_build: more than 2^32 - 1 edges and rows");
  if (row_lo < 0 || row_hi <= row_lo || row_hi > n_global) return fail(GCN_EINVAL, "gcn_csr_build: need 0 <= row_lo < row_hi <= n_global");
  if (!(row_lo == 0 && row_hi == n_global) && !d_deg_global)
    return fail(GCN_EINVAL, "gcn_csr_build: a block that is not the whole graph needs d_deg_global");
  if (flags & ~GCN_BUILD_CSC) return fail(GCN_EINVAL, "gcn_csr_build: unknown flag");
  gcn_csr* A = new (std::nothrow) gcn_csr();
  if (!A) return fail(GCN_ENOMEM, "gcn_csr_build: host allocation failed");
  if (hipGetDevice(&A->device) != hipSuccess) { delete A; return fail(GCN_EHIP, "hipGetDevice failed"); }
  int rc = build_impl(d_src, d_dst, n_edges, n_global, row_lo, row_hi, d_deg_global, flags, (hipStream_t)stream, A);
  if (rc != GCN_OK) { gcn_csr_free(A); return rc; }
  *out = A;
  return GCN_OK;
}

extern "C" int gcn_csr_info(const gcn_csr_t* A, int64_t* nr, int64_t* nh, int64_t* nnz) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_csr_info: NULL handle");
  if (nr) *nr = A->nr;
  if (nh) *nh = A->nh;
  if (nnz) *nnz = A->nnz;
  return GCN_OK;
}

extern "C" int gcn_csr_arrays(const gcn_csr_t* A, const int64_t** rowptr, const int32_t** col, const float** val,
                              const int32_t** deg, const int32_t** halo_gid, const int64_t** colptr,
                              const int32_t** rowidx, const float** val_t) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_csr_arrays: NULL handle");
  if (rowptr) *rowptr = A->rowptr;
  if (col) *col = A->col;
  if (val) *val = A->val;
  if (deg) *deg = A->deg;
  if (halo_gid) *halo_gid = A->halo_gid;
  if (colptr) *colptr = A->colptr;
  if (rowidx) *rowidx = A->rowidx;
  if (val_t) *val_t = A->val_t;
  return GCN_OK;
}

extern "C" int gcn_csr_free(gcn_csr_t* A) {
  if (!A) return GCN_OK;
  (void)hipDeviceSynchronize();
  void* ptrs[] = {A->rowptr, A->col, A->val, A->deg, A->halo_gid, A->colptr, A->rowidx, A->val_t, A->mid, A->ws};
  for (void* p : ptrs) if (p) (void)hipFree(p);
  free_schedule(&A->sched);
  free_schedule(&A->sched_t);
  free_panel_plans(A);
  for (hipEvent_t e : A->side_events) if (e) (void)hipEventDestroy(e);
  if (A->side_stream) (void)hipStreamDestroy(A->side_stream);
  delete A;
  return GCN_OK;
}
