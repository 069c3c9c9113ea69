// Y = epilogue(A X): sparse (CSR or CSC arrays) times dense row-major features, gfx950.
//
// Sec. 4.1 defines the per-row task  sum_{j in cols(A(i,:))} A(i,j) X(j,:)  and Sec. 4.3 notes
// that its cost is proportional to the row's entry count, so rows are binned by length:
//   * ordinary rows: the 64 lanes of a wavefront form G = 64 / LPR groups of LPR lanes; a group
//     covers (a slice of) the feature dimension with V-wide vector loads, so one gathered feature
//     row is one coalesced request.  Rows of a length class of about 32*g entries are shared by g
//     groups (g = 1 .. G), so a wavefront takes G / g rows at once: short rows do not idle lanes,
//     long rows get all groups; a butterfly over the g groups finishes a row.
//   * hub rows (more than kHubRowNnz entries): cut into chunks of kHubChunkNnz entries, one
//     4-wave block per chunk; the waves' partial rows meet in LDS and the chunk's partial row
//     goes to a workspace, which a finishing kernel adds up in chunk order.
//   * the feature dimension is cut into S slices and block b works on slice b % S: blocks go to
//     the 8 XCDs round-robin, so each XCD's private L2 only ever holds 1/S of every feature row.
// Every sum has a fixed association, so results are bitwise reproducible.
#include <stdlib.h>

#include <atomic>

#include "spmm_kernel.h"

namespace gcn {

size_t spmm_ws_bytes(const Schedule* sc, int d) {
  return sizeof(float) * (size_t)(sc->n_chunks > 0 ? sc->n_chunks : 1) * (size_t)d;
}

static bool aligned(const void* p, size_t a) { return p == nullptr || ((uintptr_t)p % a) == 0; }

// Feature slices.  Blocks are handed to the 8 XCDs round-robin, so with S slices and slice = block % S every XCD
// only ever touches 1/S of each feature row and its 4 MB L2 holds S times as many distinct rows; the price is that
// the sparse arrays are streamed S times and that a lane group gets narrower.
//
// Slices are whole 128-byte lines (two XCDs that each want half a line both fetch all of it), so slicing needs rows
// that start on a line: pitch a multiple of 128 bytes, base aligned.  What decides how far to go is the pitch counted
// in lines, P: slice s of row j is line j * P + s, and an XCD that only asks for lines = s (mod P) uses the few L2
// channels (and memory channels) those addresses select when P is a power of two.  Measured on a 2.45 M x 256 fp32
// operand (R-MAT, 126 M entries): pitch 8 lines 17.6 / 15.4 / 15.5 / 17.2 ms for S = 1 / 2 / 4 / 8, pitch 9 lines
// 16.5 / 14.7 / 13.9 ms for S = 2 / 4 / 8 (L2 hits 19 % -> 33 %).  With an odd pitch every slice gets one line
// (up to 8 slices); otherwise the earlier rule stands: two slices for operands above 100 MB whose halves are whole lines.
// Returns S and sets *vps (vectors of V elements per slice; 0: split evenly).
static int pick_slices(const SpmmArgs& a, size_t es, int V, int* vps) {
  *vps = 0;
  const int forced = tune().spmm_slices;                 // override for experiments
  const int64_t row_bytes = (int64_t)a.d * (int64_t)es, pitch = a.ldx * (int64_t)es;
  const double xbytes = (double)a.n_cols * (double)row_bytes;
  const bool on_lines = pitch % 128 == 0 && aligned(a.X, 128) && (int64_t)V * (int64_t)es == 16;
  const int64_t nl = ceil_div(row_bytes, 128);
  if (on_lines && nl >= 2 && ((pitch / 128) & 1) && (forced > 0 || xbytes > 16e6)) {
    int S = 2;
    while (S < nl && S < 8) S <<= 1;
    if (forced > 0 && forced < S) S = forced;
    if (S != 1 && S != 2 && S != 4 && S != 8) S = 1;
    *vps = (int)(ceil_div(nl, S) * 8);                   // 8 vectors of 16 bytes per line
    return S;
  }
  int S = 1;
  if (forced > 0) S = forced;
  else if (xbytes > 100e6) S = 2;
  while (S > 1 && (double)row_bytes / S < 128.0) S >>= 1;
  // a slice that does not consist of whole 128-byte lines makes every gathered row touch more lines in all than
  // the undivided row does: 400-byte rows (width 100) in two slices took 11.7 ms where one slice takes 8.0 ms
  if (forced <= 0 && S > 1 && row_bytes % (128 * S) != 0) S = 1;
  if (S != 1 && S != 2 && S != 4 && S != 8) S = 1;
  return S;
}

int spmm_launch(const SpmmArgs& a, void* ws, hipStream_t s) {
  SpmmK k{};
  k.ptr = a.ptr; k.idx = a.idx; k.val = a.val;
  k.lo = a.part == 2 ? a.mid : a.ptr;
  k.hi = a.part == 1 ? a.mid : a.ptr + 1;
  k.accumulate = a.part == 2 ? 1 : 0;
  k.wave_rows = a.sched->wave_rows;
  k.hub_rows = a.sched->hub_rows; k.hub_chunk_ptr = a.sched->hub_chunk_ptr;
  k.chunk_hub = a.sched->chunk_hub; k.n_chunks = a.sched->n_chunks; k.n_hub_rows = a.sched->n_hub_rows;
  k.X = a.X; k.ldx = a.ldx; k.Y = a.Y; k.ldy = a.ldy; k.Y2 = a.Y2; k.ldy2 = a.ldy2;
  k.bias = a.bias; k.Zprev = a.Zprev; k.ldz = a.ldz; k.n_mask_rows = a.n_mask_rows;
  k.partial = (float*)ws; k.d = a.d; k.epilogue = a.epilogue;
  if (a.n_rows == 0) return GCN_OK;
  if (a.row_chunk >= 0 && (a.row_chunk_n < 1 || a.row_chunk + a.row_chunk_n > kRowChunks)) return fail(GCN_EINVAL, "spmm: no such row chunks");
  const int rc1 = a.row_chunk + a.row_chunk_n;
  if (a.row_chunk >= 0) {          // the long rows of this row range, and their chunks of entries
    const Schedule* sc = a.sched;
    k.chunk_lo = sc->chunk_hubchunk_begin[a.row_chunk]; k.n_chunks = sc->chunk_hubchunk_begin[rc1] - k.chunk_lo;
    k.hub_lo = sc->chunk_hub_begin[a.row_chunk]; k.n_hub_rows = sc->chunk_hub_begin[rc1] - k.hub_lo;
  }
  bool swept = false;
  // the column-sweep plan covers whole rows of the whole matrix only
  if (a.part == 0 && !a.no_alloc && a.row_chunk < 0) GCN_TRY(spmm_panel_try(a, s, &swept));
  if (swept) return GCN_OK;
  const size_t es = a.dtype == GCN_BF16 ? 2 : 4;
  // widest vector such that every feature-row load stays aligned (and inside the row's storage)
  int V = a.dtype == GCN_BF16 ? 8 : 4;
  while (V > 1 && !((a.ldx % V) == 0 && aligned(a.X, V * es) && ((a.d % V) == 0 || a.x_rows_padded))) V >>= 1;
  k.y_vec = (a.ldy % V) == 0 && aligned(a.Y, V * es) && (!a.Y2 || ((a.ldy2 % V) == 0 && aligned(a.Y2, V * es)));
  k.S = pick_slices(a, es, V, &k.vps);
  SpmmProf pf;
  pf.kind = a.transposed ? GCN_K_SPMM_T : GCN_K_SPMM; pf.dtype = a.dtype; pf.rows = a.n_rows; pf.nnz = a.nnz;
  const double csr = 8.0 * (double)a.nnz + 8.0 * (double)(a.n_rows + 1), fe = (double)es * a.d;
  pf.alg = csr + fe * (double)(a.n_cols + a.n_rows);
  pf.touched = csr + fe * (double)(a.nnz + a.n_rows);
  pf.flops = 2.0 * (double)a.nnz * a.d;
  if (a.row_chunk >= 0) {            // a range of rows is charged its share of the rows (the host does not know its entry count)
    const int64_t rows = a.sched->chunk_row[rc1] - a.sched->chunk_row[a.row_chunk];
    const double share = (double)rows / (double)a.n_rows;
    pf.alg *= share; pf.touched *= share; pf.flops *= share;
    pf.rows = rows;
    pf.nnz = (int64_t)((double)a.nnz * share);
    pf.row_chunk = a.row_chunk; pf.row_chunk_n = a.row_chunk_n;
  }
  // 32-bit addressing of X: row index and row pitch below 2^24, whole matrix below 4 GiB
  const double xspan = (double)a.n_cols * (double)a.ldx * (double)es;
  const bool narrow = a.n_cols < (1 << 24) && (double)a.ldx * (double)es < (double)(1 << 24) && xspan < 4294967296.0 &&
                      !tune().spmm_wide;
  k.row_bytes = narrow ? (uint32_t)(a.ldx * (int64_t)es) : 0u;
  if (a.dtype == GCN_BF16) return spmm_dispatch_bf16(k, a.sched, pf, V, narrow, s);
  return spmm_dispatch_f32(k, a.sched, pf, V, narrow, s);
}

// ---- scratch of the entry point that allocates nothing ------------------------------------------------------
// The partial rows of long-row chunks (n_chunks x d floats) of gcn_spmm_noalloc live in this fixed array instead
// of the handle's workspace.  Every GPU the library runs on holds its own copy until the process ends.  The
// array's name is a host-side stand-in: its device address is asked for once per device and kept.
constexpr size_t kNoAllocScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];
constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_addr[kMaxDevices];

static int noalloc_scratch(void** out) {
  int dev = -1;
  GCN_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(GCN_EINVAL, "gcn_spmm_noalloc: device ordinal %d is not supported", dev);
  void* p = g_scratch_addr[dev].load(std::memory_order_acquire);
  if (!p) {
    GCN_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));      // this device's copy (the current device)
    if (!p) return fail(GCN_EHIP, "gcn_spmm_noalloc: no device address for the scratch array");
    g_scratch_addr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return GCN_OK;
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
  a.owner = Am;
  return spmm_launch(a, Am->ws, (hipStream_t)stream);
}

extern "C" int gcn_spmm_noalloc(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y, int64_t ldy,
                                int epilogue, const float* bias, const void* Zprev, int64_t ldz, void* stream) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_spmm_noalloc: NULL handle");
  GCN_TRY(check_dense("gcn_spmm_noalloc", X, ldx, Y, ldy, d, dtype));
  if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_EINVAL, "gcn_spmm_noalloc: unknown epilogue");
  if (epilogue == GCN_EPI_MASK && (!Zprev || ldz < d)) return fail(GCN_EINVAL, "gcn_spmm_noalloc: mask epilogue needs Zprev with ldz >= d");
  const size_t need = spmm_ws_bytes(&A->sched, d);
  if (need > kNoAllocScratchBytes)
    return fail(GCN_EINVAL, "gcn_spmm_noalloc: %lld long-row chunks x %d features need %zu bytes of scratch, the fixed buffer holds %zu",
                (long long)A->sched.n_chunks, d, need, kNoAllocScratchBytes);
  void* ws = nullptr;
  GCN_TRY(noalloc_scratch(&ws));
  SpmmArgs a{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, X, ldx, Y, ldy, nullptr, 0,
             d, dtype, epilogue, bias, Zprev, ldz};
  a.no_alloc = true;
  ProfSuppress quiet;
  return spmm_launch(a, ws, (hipStream_t)stream);
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
  a.owner = Am;
  return spmm_launch(a, Am->ws, (hipStream_t)stream);
}

extern "C" int gcn_spmm_part(const gcn_csr_t* A, int part, const void* X, int64_t ldx, int d, int dtype, void* Y,
                             int64_t ldy, int epilogue, const float* bias, const void* Zprev, int64_t ldz, void* stream) {
  clear_error();
  if (!A) return fail(GCN_EINVAL, "gcn_spmm_part: NULL handle");
  if (part != GCN_PART_LOCAL && part != GCN_PART_HALO) return fail(GCN_EINVAL, "gcn_spmm_part: part must be GCN_PART_LOCAL or GCN_PART_HALO");
  GCN_TRY(check_dense("gcn_spmm_part", X, ldx, Y, ldy, d, dtype));
  if (epilogue < GCN_EPI_NONE || epilogue > GCN_EPI_MASK) return fail(GCN_EINVAL, "gcn_spmm_part: unknown epilogue");
  if (part == GCN_PART_LOCAL && (epilogue != GCN_EPI_NONE || bias))
    return fail(GCN_EINVAL, "gcn_spmm_part: the local part stores plain sums; bias and epilogue belong to the halo part");
  if (epilogue == GCN_EPI_MASK && (!Zprev || ldz < d)) return fail(GCN_EINVAL, "gcn_spmm_part: mask epilogue needs Zprev with ldz >= d");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  GCN_TRY(ensure_workspace(Am, spmm_ws_bytes(&A->sched, d)));
  SpmmArgs a{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, X, ldx, Y, ldy, nullptr, 0,
             d, dtype, epilogue, bias, Zprev, ldz};
  a.owner = Am;
  if (A->mid) { a.part = part; a.mid = A->mid; }
  else if (part == GCN_PART_HALO) {
    // no halo columns: the local part was the whole product; only the epilogue is left to apply
    a.part = 2; a.mid = A->rowptr + 1;            // empty ranges [ptr[r+1], ptr[r+1])
  }
  return spmm_launch(a, Am->ws, (hipStream_t)stream);
}
