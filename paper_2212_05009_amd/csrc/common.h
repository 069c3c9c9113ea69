// Shared host-side declarations of the gfx950 GCN library (internal; the public ABI is gcn.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/gcn.h"

namespace gcn {

// ---- error reporting -------------------------------------------------------------------
int fail(int code, const char* fmt, ...);   // records the thread-local message, returns code
void clear_error();

#define GCN_HIP(expr)                                                                      \
  do {                                                                                     \
    hipError_t e__ = (expr);                                                               \
    if (e__ != hipSuccess)                                                                 \
      return ::gcn::fail(e__ == hipErrorOutOfMemory ? GCN_ENOMEM : GCN_EHIP, "%s: %s",     \
                         #expr, hipGetErrorString(e__));                                   \
  } while (0)

#define GCN_TRY(expr)            \
  do {                           \
    int rc__ = (expr);           \
    if (rc__ != GCN_OK) return rc__; \
  } while (0)

#define GCN_CHECK_LAUNCH() GCN_HIP(hipGetLastError())

// ---- overrides for experiments and tests ---------------------------------------------------------
// Each field starts from the environment variable of the same name in upper case with the prefix GCN_ (read
// once, when the library first needs any of them); gcn_debug_set_tuning() changes a field afterwards.  None
// changes what is computed, only which kernel or launch shape computes it.
struct Tuning {
  int spmm_panel = -1;          // column sweep: -1 by heuristic, 0 never, 1 wherever its plan can be built
  int panel_narrow = 0;         // column sweep: 8-lane groups even where half-wavefront groups apply
  int panel_nosync = 0;         // column sweep: drop the per-column-block waits
  int panel_verbose = 0;        // column sweep: print the plan chosen
  int spmm_slices = 0;          // feature slices of the row kernel (0: by rule)
  int spmm_epg = 0;             // entries per lane group before a row is shared by more groups (0: default)
  int spmm_wide = 0;            // 64-bit gather addresses even where 32 bits suffice
  int gemm_direct = 1, gemm_fast = 1, gemm_tn_wide = 1, gemm_bf16 = 1, gemm_regw = 1;   // 0 switches a dense kernel family off
  int gemm_tn_lds = 1;          // A^T B with both operands streamed through LDS: 0 off, 1 for wide fp32 outputs, 2 wherever it fits
  int gemm_regw_blocks = 0;     // workgroups of the register-resident-W kernel; 0 = one per compute unit
  int gemm_tn_lds_blocks = 0;   // workgroups of the LDS-streamed A^T B kernel; 0 = one per compute unit
  int overlap = 1;              // the weight gradient beside the sparse product of the same layer call: 0 never, 1 on large blocks, 2 wherever possible
  int overlap_cus = 64;         // compute units the dense kernels take while the sparse product runs
  int pause_rounds = 4;         // rounds of about 3.7 us that stream_pause sleeps (measured: 1 is too short, 2 is enough)
  int overlap_chunks = 4;       // row chunks of a sparse product that a dense product follows: 2, 4 or 8; 0: no such pipeline
  int gemm_tn_blocks = 512;     // blocks the A^T B kernel aims for
  int gather_host_blocks = 32;  // workgroups of the host-table gather
};
const Tuning& tune();

// ---- optional per-kernel timing (profile.hip) ------------------------------------------------
// Put one on the stack around a kernel launch: records a start event now and a stop event when it
// goes out of scope, both on `s`, if profiling is enabled; otherwise costs one relaxed load.
struct ProfScope {
  ProfScope(int kind, hipStream_t s, int d, int dtype, int64_t rows, int64_t inner, double alg_bytes,
            double touched_bytes, double flops);
  ~ProfScope();
  ProfScope(const ProfScope&) = delete;
  ProfScope& operator=(const ProfScope&) = delete;
 private:
  int64_t slot_ = -1;
  hipStream_t s_;
};

// While one of these is alive on a host thread, ProfScope records nothing on that thread (recording creates
// events on first use; the entry point that allocates nothing must not).
struct ProfSuppress {
  ProfSuppress();
  ~ProfSuppress();
  ProfSuppress(const ProfSuppress&) = delete;
  ProfSuppress& operator=(const ProfSuppress&) = delete;
};

// RAII device buffer so that every error path frees what it allocated.
struct DevBuf {
  void* p = nullptr;
  DevBuf() = default;
  DevBuf(const DevBuf&) = delete;
  DevBuf& operator=(const DevBuf&) = delete;
  ~DevBuf() { if (p) (void)hipFree(p); }
  int alloc(size_t bytes) {
    if (p) { (void)hipFree(p); p = nullptr; }
    hipError_t e = hipMalloc(&p, bytes ? bytes : 256);
    if (e != hipSuccess) { p = nullptr; return fail(GCN_ENOMEM, "hipMalloc(%zu bytes): %s", bytes, hipGetErrorString(e)); }
    return GCN_OK;
  }
  template <class T> T* as() const { return (T*)p; }
  void* release() { void* q = p; p = nullptr; return q; }
};

static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline int64_t round_up(int64_t a, int64_t b) { return ceil_div(a, b) * b; }

// Launch geometry.  The runtime does not refuse a launch whose x extent (blocks x threads per block) reaches 2^32
// threads: it runs that count modulo 2^32 and reports success (measured on gfx950: 2^24 + 1 blocks of 256 threads ran
// one block), while a grid of two dimensions runs completely (65536 x 65535 blocks measured).  Grids that grow with
// the problem are therefore folded: at most max_grid_x() blocks in x, the rest in y; the kernel takes its number from
// block_id() and checks it against the count it was given.  gcn_debug_max_grid_x() lowers the bound so that tests
// exercise the folding on small inputs.
int64_t max_grid_x();
static inline dim3 fold_grid(int64_t blocks) {
  const int64_t mx = max_grid_x();
  if (blocks < 1) blocks = 1;
  if (blocks <= mx) return dim3((unsigned)blocks);
  return dim3((unsigned)mx, (unsigned)ceil_div(blocks, mx));
}
// blocks the runtime can take in one folded launch (y is kept within 16 bits)
static inline bool grid_fits(int64_t blocks) { return blocks <= max_grid_x() * 65535; }
#ifdef __HIPCC__
__device__ __forceinline__ int64_t block_id() { return (int64_t)blockIdx.y * gridDim.x + blockIdx.x; }

// bf16 features: a value is the upper half of the fp32 pattern.  Stores round to nearest even; NaN stays NaN.
typedef uint16_t bf16_t;
__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
// one element of a feature buffer of type T (float or bf16_t), widened to / rounded from fp32
template <typename T> __device__ __forceinline__ float load_one(const T* p) {
  if constexpr (sizeof(T) == 4) return (float)*p;
  else return bf16_to_f32((bf16_t)*p);
}
template <typename T> __device__ __forceinline__ void store_one(T* p, float v) {
  if constexpr (sizeof(T) == 4) *p = v;
  else *p = f32_to_bf16(v);
}
#endif

// ---- execution schedule of a compressed sparse matrix (row binning) ----------------------
// Rows are split by length.  Rows longer than kHubRowNnz ("hub" rows of a power-law graph)
// are cut into chunks of kHubChunkNnz entries, one 256-thread block per chunk; their partial
// sums are combined by a finalisation kernel.  All other rows get one wavefront each, in an
// order that starts the longest rows first.  The schedule only fixes the order of execution
// and the chunking; the matrix arrays stay in row order.
constexpr int kHubRowNnz = 2048;
constexpr int kHubChunkNnz = 1024;

constexpr int kRowChunks = 8;      // row ranges a sparse product can be launched on separately (or on runs of them)

struct Schedule {
  int32_t* wave_rows = nullptr;   // [n_wave_rows] rows handled one wavefront each
  int64_t n_wave_rows = 0;
  int32_t* hub_rows = nullptr;    // [n_hub_rows] rows handled by chunks
  int64_t n_hub_rows = 0;
  int64_t* hub_chunk_ptr = nullptr;  // [n_hub_rows+1] first chunk of each hub row
  int32_t* chunk_hub = nullptr;      // [n_chunks] index into hub_rows of each chunk
  int64_t n_chunks = 0;
  // host copy: rows of length class c (lengths in [2^(31-c), 2^(32-c)); class 32 = empty rows) are
  // wave_rows[class_begin[c] .. class_begin[c+1]); classes are stored longest first.
  int64_t class_begin[34] = {0};
  // host copy: the same lists cut at kRowChunks row boundaries chunk_row[j] (multiples of 64 rows; within a class the
  // rows ascend): rows of class c in [chunk_row[j], chunk_row[j+1]) are wave_rows[chunk_class_begin[j][c] ..
  // chunk_class_begin[j+1][c]); the hub rows (ascending too) of that range are hub_rows[chunk_hub_begin[j] ..
  // chunk_hub_begin[j+1]), their chunks of entries chunk_hubchunk_begin[j] .. chunk_hubchunk_begin[j+1].  A product
  // launched on one range of rows can be followed by dense work on those rows while the next range is multiplied.
  int64_t chunk_row[kRowChunks + 1] = {0};
  int64_t chunk_class_begin[kRowChunks + 1][33] = {{0}};
  int64_t chunk_hub_begin[kRowChunks + 1] = {0};
  int64_t chunk_hubchunk_begin[kRowChunks + 1] = {0};
};

// ---- panel plan: the column-sweep execution layout of a sparse matrix (spmm_panel.hip) -------
// Rows are cut into "virtual rows" of at most part_len entries (entry k of a row with P parts
// belongs to part k % P); consecutive rows are packed into panels of at most nv_max virtual rows
// whose accumulators fit in one workgroup's LDS.  A workgroup has kPanelWaves wavefronts of
// 64 / lpg lane groups; every lane group owns some virtual rows of the panel (dealt out so that all
// groups get about the same number of entries) and reads its own stream of entries, sorted by
// (column block, virtual row, column).  The streams of the groups of one wavefront are stored
// interleaved in batches of 8 entries per group (32 for half-wavefront groups), padded with kNoEntry
// where a stream has ended.
constexpr int kPanelWaves = 16;
constexpr int kPanelLists = 8;      // one work list per XCD
struct PanelPlan {
  bool unusable = false;   // a record that the matrix does not fit the format for this shape (no arrays)
  bool transposed = false;
  int ns = 1;              // feature slices (32 wide) the panel size was chosen for
  int sw = 32;             // accumulator floats per virtual row: 32, or 16 for products of width <= 16
  int lpg = 8;             // lanes per group
  int cb_shift = 14;       // log2(columns per column block)
  int part_len = 512;
  int nv_max = 0;          // most virtual rows in one panel
  int n_panels = 0;
  int64_t n_rows = 0, total_vrows = 0, n_batches = 0;
  uint2* ent = nullptr;           // [n_batches * epb * (64 / lpg)] {index in owner << 24 | column, value bits}; epb = 8, or 32 for lpg 32
  int64_t* wb = nullptr;          // [n_panels * kPanelWaves + 1] first batch of each wavefront
  int32_t* nfull = nullptr;       // [n_panels * kPanelWaves] leading batches without padding
  int n_cb = 1;                   // column blocks
  int32_t* cbend = nullptr;       // [n_panels * kPanelWaves * n_cb] batches of a wavefront up to the end of a column block
  int32_t* obase = nullptr;       // [n_panels * kPanelWaves * (64 / lpg)] first accumulator row of each group
  int32_t* panel_row0 = nullptr;  // [n_panels + 1] first row of each panel
  int32_t* row_v = nullptr;       // [n_rows + 1] index of the first virtual row of each row
  int32_t* vlds = nullptr;        // [total_vrows] accumulator row of each virtual row inside its panel
  int32_t* order = nullptr;       // [n_panels] panels by falling entry count
  uint32_t* ctr = nullptr;        // [2 * kPanelLists] per-launch work counters
};

}  // namespace gcn

// ---- the opaque handle -------------------------------------------------------------------
struct gcn_csr {
  int device = 0;
  int64_t n_global = 0, row_lo = 0;
  int64_t nr = 0, nh = 0, nc = 0, nnz = 0;
  int64_t* rowptr = nullptr;
  int32_t* col = nullptr;
  float* val = nullptr;
  int32_t* deg = nullptr;
  int32_t* halo_gid = nullptr;
  int64_t* colptr = nullptr;
  int32_t* rowidx = nullptr;
  float* val_t = nullptr;
  int64_t* mid = nullptr;  // [nr] first entry of each row whose column is a halo column (null when nh == 0)
  gcn::Schedule sched;     // for A   (rows = owned rows)
  gcn::Schedule sched_t;   // for A^T (rows = local columns)
  void* ws = nullptr;      // scratch workspace, grown on demand
  size_t ws_bytes = 0;
  std::vector<gcn::PanelPlan*> plans;   // column-sweep layouts, built on first use (spmm_panel.hip)
  // A second stream of the library's own (default priority, created on first use) for dense work that runs beside
  // a sparse product of the same layer call, and the two events that order it against the caller's stream (one per
  // hand-over to the side stream, one for the way back).
  hipStream_t side_stream = nullptr;
  hipEvent_t side_events[gcn::kRowChunks + 2] = {};
};

namespace gcn {

// Makes sure the handle's workspace holds at least `bytes`; may synchronise the device when it
// has to grow (the old buffer could still be in use by enqueued work).
int ensure_workspace(gcn_csr* A, size_t bytes);

// ---- device primitives (scan_sort.hip) ----------------------------------------------------
// out[i] = sum_{k<i} in[k] for i in [0, n]; out has n+1 entries (out[n] = total).
// tmp must hold scan_tmp_bytes(n).
size_t scan_tmp_bytes(int64_t n);
int exclusive_scan_u32(const uint32_t* in, int64_t* out, int64_t n, void* tmp, hipStream_t s);

// Stable least-significant-digit radix sort of 64-bit keys on bits [bit_lo, bit_hi), with an
// optional 32-bit payload.  Result ends in (keys_out, pay_out); both key buffers and both
// payload buffers are clobbered.  tmp must hold sort_tmp_bytes(n).
size_t sort_tmp_bytes(int64_t n);
int radix_sort_u64(uint64_t* keys_a, uint64_t* keys_b, uint32_t* pay_a, uint32_t* pay_b, int64_t n,
                   int bit_lo, int bit_hi, void* tmp, hipStream_t s, uint64_t** keys_out,
                   uint32_t** pay_out);

// ---- schedule construction (csr_build.hip) -------------------------------------------------
int build_schedule(const int64_t* ptr, int64_t n_rows, hipStream_t s, Schedule* out);
void free_schedule(Schedule* sc);

// ---- kernels behind the public entry points -------------------------------------------------
struct SpmmArgs {
  const int64_t* ptr; const int32_t* idx; const float* val; const Schedule* sched;
  int64_t n_rows;            // rows of the sparse matrix (= rows of Y)
  int64_t n_cols;            // columns of the sparse matrix (= rows of X)
  int64_t nnz;               // stored entries
  bool transposed;           // the arrays are the column-major copy (only labels the profile record)
  int64_t n_mask_rows;       // rows covered by bias / relu / mask epilogues that need Zprev
  const void* X; int64_t ldx;
  void* Y; int64_t ldy;      // epilogue result
  void* Y2; int64_t ldy2;    // optional second output: the value before ReLU (may be null)
  int d; int dtype; int epilogue; const float* bias; const void* Zprev; int64_t ldz;
  // true when every row of X, the last one included, is backed by ldx readable elements (library
  // buffers with a padded leading dimension): vector loads may then run past column d
  bool x_rows_padded = false;
  // a product split by column range (Sec. 4.1, the block form: local part first, then the received rows):
  // 0 whole rows; 1 entries [ptr[r], mid[r]) and plain store; 2 entries [mid[r], ptr[r+1]) added to Y
  int part = 0;
  const int64_t* mid = nullptr;
  gcn_csr* owner = nullptr;  // handle the arrays belong to (lets the launch cache a panel plan); may be null
  bool no_alloc = false;     // the launch must not allocate: no column-sweep plan is built
  // row_chunk >= 0: only the rows [sched->chunk_row[row_chunk], sched->chunk_row[row_chunk + row_chunk_n)) (never
  // through the column sweep)
  int row_chunk = -1, row_chunk_n = 1;
};
// ws: workspace for hub partial sums, at least spmm_ws_bytes(sched, d)
size_t spmm_ws_bytes(const Schedule* sc, int d);
int spmm_launch(const SpmmArgs& a, void* ws, hipStream_t s);
// column-sweep variant (spmm_panel.hip): *used = false when the product does not qualify and
// nothing was enqueued
int spmm_panel_try(const SpmmArgs& a, hipStream_t s, bool* used);
// whether spmm_panel_try would take this product (a.X only matters for its alignment)
bool spmm_panel_wanted(const SpmmArgs& a);
void free_panel_plans(gcn_csr* A);
// ptr[q] = first position whose key >> shift is >= q, q in [0, n_seg]; keys sorted, n >= 1
int segment_boundaries(const uint64_t* keys, int64_t n, int shift, int64_t n_seg, int64_t* ptr, hipStream_t s);

struct GemmEpilogue {
  const float* bias = nullptr;   // [N] added to every row
  int relu = 0;                  // C = max(.,0)
  const void* mask = nullptr;    // [mask_rows x N] (ld = ldmask): C *= [mask > 0] for rows < mask_rows
  int64_t ldmask = 0, mask_rows = 0;
  void* C2 = nullptr;            // optional second output: value before ReLU
  int64_t ldc2 = 0;
  int max_blocks = 0;            // > 0: a kernel with one workgroup per compute unit launches at most this many
};
// true when gemm_nn runs this product on the kernel that occupies whole compute units, one workgroup each, and
// therefore honours GemmEpilogue::max_blocks (the rest of the chip is left to a kernel on another stream)
bool gemm_nn_limits_blocks(const void* A, int64_t lda, int64_t M, int N, int K, int dtype);
// C[M x N] = A[M x K] * B[K x N];  A, C (and C2, mask) have element type dtype, B is f32.
int gemm_nn(const void* A, int64_t lda, const float* B, int64_t ldb, void* C, int64_t ldc,
            int64_t M, int N, int K, int dtype, const GemmEpilogue& epi, hipStream_t s);
// C[M x N] (f32) = A[Kdim x M]^T * B[Kdim x N], Kdim huge: split over blocks, partial tiles in ws
// (gemm_tn_ws_bytes), then summed in a fixed order.  A, B element type dtype.
size_t gemm_tn_ws_bytes(int64_t Kdim, int M, int N);
// max_blocks > 0: as GemmEpilogue::max_blocks, honoured when gemm_tn_limits_blocks says so
bool gemm_tn_limits_blocks(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kdim, int M, int N, int dtype);
int gemm_tn(const void* A, int64_t lda, const void* B, int64_t ldb, float* C, int64_t ldc,
            int64_t Kdim, int M, int N, int dtype, void* ws, hipStream_t s, int max_blocks = 0);
// streaming variants (gemm_direct.hip): the long operand goes from global memory straight into the
// MFMA operand registers; nn_direct needs W to fit in LDS (gemm_nn_direct_ok)
bool gemm_nn_direct_ok(int N, int K);
// W held in registers as MFMA operands, A streamed past it (gemm_regw.hip): fp32, K <= 256, N a multiple of 64 up to 256
bool gemm_nn_regw_ok(const void* A, int64_t lda, int64_t M, int N, int K, int dtype);
int gemm_nn_regw(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N, int K,
                 const GemmEpilogue& epi, hipStream_t s);
// bf16 features on the bf16 matrix pipe (gemm_bf16.hip): W rounded to bf16 in LDS, fp32 accumulation
bool gemm_nn_bf16_ok(const void* A, int64_t lda, void* C, int64_t ldc, int64_t M, int N, int K, const GemmEpilogue& epi);
// A^T B for bf16 operands on the bf16 matrix pipe: partial tiles per row split, as gemm_tn_direct_partials
bool gemm_tn_bf16_ok(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N);
int gemm_tn_bf16_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, float* partial,
                          int* nsplit_out, hipStream_t s);
// launch shape shared by the vector-request A^T B kernels: column tiles of B per block, number of row splits
int tn_wide_wn(int N);
int tn_wide_splits(int64_t Kd, int M, int N);
int gemm_nn_bf16(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N, int K,
                 const GemmEpilogue& epi, hipStream_t s);
int gemm_nn_direct(const void* A, int64_t lda, const float* W, int64_t ldw, void* C, int64_t ldc, int64_t M, int N,
                   int K, int dtype, const GemmEpilogue& epi, hipStream_t s);
// A^T B partial tiles with the output in registers and both operands streamed through LDS (wide fp32 operands)
bool gemm_tn_lds_ok(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, int dtype);
size_t gemm_tn_lds_ws_bytes(int64_t Kd, int M, int N);
int gemm_tn_lds_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, float* partial,
                         int* nsplit_out, hipStream_t s, int max_blocks = 0);
size_t gemm_tn_direct_ws_bytes(int64_t Kd, int M, int N);
int gemm_tn_direct_partials(const void* A, int64_t lda, const void* B, int64_t ldb, int64_t Kd, int M, int N, int dtype,
                            float* partial, int* nsplit_out, hipStream_t s, int max_blocks = 0);
// Holds the stream back for about 15 us (one sleeping wavefront): gives a kernel that was just released on another
// stream, and that needs whole compute units, time to be placed before this stream's next kernel fills the chip.
int stream_pause(hipStream_t s);
// dst[rows x ld_dst] = src[rows x d] (leading dimension ld_src), zero in the padding columns
int pad_rows(const void* src, int64_t ld_src, void* dst, int64_t ld_dst, int64_t rows, int d, int dtype, hipStream_t s);
// Wt[N x K] = W[K x N]^T (f32, small)
int transpose_f32(const float* W, int K, int N, float* Wt, hipStream_t s);
// out[c] = sum_i G[i, c]  (deterministic), ws at least colsum_ws_bytes
size_t colsum_ws_bytes(int64_t rows, int N);
int colsum(const void* G, int64_t ldg, int64_t rows, int N, int dtype, float* out, void* ws,
           hipStream_t s);

}  // namespace gcn
