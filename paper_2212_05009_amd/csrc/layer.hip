// gcn_layer_fwd / gcn_layer_bwd: one GCN layer on a row block, composed from the sparse and
// dense kernels (Sec. 3.1 equations for Z, S and dW; Sec. 4.1 / 4.2 for the block form).
//
// The three-matrix products are associative, so the order is chosen by cost; every choice is
// the same real-number sum:
//   forward   (A H) W   sparse product at width d_in  (also what Sec. 4.1 writes), or
//             A (H W)   sparse product at width d_out, dense product over all nc rows;
//   backward  T = A^T G at width d_out, then dH = T W^T and dW = H^T T  (Sec. 4.2 notes that the
//             sparse product with G is shared between S and dW), or
//             Q = G W^T, dH = A^T Q at width d_in, and dW = (A H)^T G.
#include "common.h"

namespace gcn {

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
static size_t es_of(int dtype) { return dtype == GCN_BF16 ? 2 : 4; }

// Leading dimension of an internal buffer whose rows a sparse product gathers.  A row that starts at a multiple
// of s bytes and is s bytes long touches (s + 128 - gcd(s, 128)) / 128 lines of 128 bytes on average.  The row is
// rounded up to 16 bytes, or to 64 or 128 bytes where that saves at least 8 % of the lines for at most half as
// many bytes again (fp32 width 41: 176 -> 192 bytes, 2.25 -> 2 lines; bf16 width 47: 96 -> 128 bytes, 1.5 -> 1).
static int64_t gather_ld(int d, size_t es) {
  auto lines = [](int64_t sb) {
    int64_t g = 128;
    while (sb % g) g >>= 1;
    return (double)(sb + 128 - g) / 128.0;
  };
  const int64_t base = round_up((int64_t)d * (int64_t)es, 16);
  int64_t best = base;
  for (int64_t unit : {64, 128}) {
    const int64_t cand = round_up((int64_t)d * (int64_t)es, unit);
    if (cand * 2 <= base * 3 && lines(cand) <= 0.92 * lines(best)) best = cand;
  }
  return best / (int64_t)es;
}

// The pitch of a library-owned operand of the sparse product with the n_rows x n_cols matrix of the handle (the
// transposed copy where `transposed`).  The column sweep asks for a row in slices of 128 bytes, one request per
// slice: a slice that straddles two lines costs two line reads, so rows longer than a line then start on a line
// (measured, fp32 width 41 over 233 k rows with 490 entries each: pitch 192 bytes 2.29 ms, 256 bytes 1.91 ms).
//
// Operands large enough for the row kernel to work in feature slices (spmm.hip: one 128-byte line per slice and
// group of compute units) get gcn_feature_ld's pitch: rows on lines, an odd number of lines apart.
static int64_t gather_ld_for(const gcn_csr* A, bool transposed, int d, int dtype) {
  const int64_t es = (int64_t)es_of(dtype);
  const int64_t ld = gather_ld(d, (size_t)es), ld_line = round_up((int64_t)d * es, 128) / es;
  if ((int64_t)d * es <= 128) return ld;
  const int64_t n_cols = transposed ? A->nr : A->nc;
  if ((double)n_cols * (double)d * (double)es > 16e6 && tune().spmm_panel != 1) {
    SpmmArgs probe0{};
    probe0.owner = const_cast<gcn_csr*>(A);
    probe0.transposed = transposed;
    probe0.n_rows = transposed ? A->nc : A->nr;
    probe0.n_cols = n_cols;
    probe0.nnz = A->nnz; probe0.d = d; probe0.dtype = dtype;
    probe0.X = reinterpret_cast<const void*>((uintptr_t)256); probe0.ldx = ld_line; probe0.x_rows_padded = true;
    if (!spmm_panel_wanted(probe0)) return gcn_feature_ld(d, dtype);
  }
  if (ld_line == ld) return ld;
  SpmmArgs probe{};
  probe.owner = const_cast<gcn_csr*>(A);
  probe.transposed = transposed;
  probe.n_rows = transposed ? A->nc : A->nr;
  probe.n_cols = transposed ? A->nr : A->nc;
  probe.nnz = A->nnz; probe.d = d; probe.dtype = dtype;
  probe.X = reinterpret_cast<const void*>((uintptr_t)256); probe.ldx = ld_line; probe.x_rows_padded = true;
  return spmm_panel_wanted(probe) ? ld_line : ld;
}

// Average number of 128-byte lines that a row of `len` bytes touches when rows start at multiples of `pitch` bytes.
static double lines_touched(int64_t pitch, int64_t len) {
  int64_t g = 128;
  while (pitch % g) g >>= 1;
  double sum = 0.0;
  for (int64_t o = 0; o < 128; o += g) sum += (double)((o + len + 127) / 128);
  return sum / (double)(128 / g);
}

// A caller's operand [n_cols x d] with pitch ldx that a sparse product is about to gather: the pitch of a padded
// copy worth making first, or ldx.  The copy moves every row once, the product reads a row per stored entry, so
// it pays when there are several entries per column and the padded rows touch clearly fewer lines (bf16 width
// 100: 200-byte rows at a pitch of 200 bytes touch 2.5 lines and admit 8-byte requests only; at 256 bytes 2 lines
// and 16-byte requests).
static int64_t padded_operand_ld(const gcn_csr* A, bool transposed, int d, int dtype, int64_t ldx) {
  const int64_t es = (int64_t)es_of(dtype);
  const int64_t ldp = gather_ld_for(A, transposed, d, dtype);
  if (ldp == ldx) return ldx;
  const int64_t n_cols = transposed ? A->nr : A->nc;
  if (A->nnz < 8 * n_cols) return ldx;
  return lines_touched(ldp * es, (int64_t)d * es) <= 0.85 * lines_touched(ldx * es, (int64_t)d * es) ? ldp : ldx;
}

// Dense work beside a sparse product.  The sparse product of a large block is bound by its gathers and leaves the
// matrix pipes idle; the weight gradient dW = (A^ H)^T G from a saved A^ H needs nothing of the backward pass's
// sparse product, is bound by the matrix pipes, and on a quarter of the compute units, on a second stream, costs the
// sparse product next to nothing.  Measured on 2.45 M rows, 126 M entries, width 256: sparse product alone 14.3 ms,
// the 256 x 256 gradient alone 2.6 ms (9.5 ms on 64 compute units), both at once 14.7 ms.  A dense product that
// needs the sparse product's result follows it row chunk by row chunk (Schedule::chunk_row), one chunk behind.
struct SideStream {
  gcn_csr* A = nullptr; hipStream_t main = nullptr; hipStream_t side = nullptr;
  bool open = false;       // forked and not yet joined
  SideStream() = default;
  SideStream(const SideStream&) = delete;
  SideStream& operator=(const SideStream&) = delete;
  // a call that fails between fork and join still leaves the caller's stream behind the side stream's work
  ~SideStream() {
    if (open && hipEventRecord(A->side_events[1], side) == hipSuccess) (void)hipStreamWaitEvent(main, A->side_events[1], 0);
  }
  // what the caller's stream holds so far is done before anything enqueued on the side stream from here on
  int fork(gcn_csr* A_, hipStream_t main_) {
    A = A_; main = main_;
    if (!A->side_stream) GCN_HIP(hipStreamCreateWithFlags(&A->side_stream, hipStreamNonBlocking));
    for (hipEvent_t& e : A->side_events)
      if (!e) GCN_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    side = A->side_stream;
    GCN_HIP(hipEventRecord(A->side_events[0], main));
    GCN_HIP(hipStreamWaitEvent(side, A->side_events[0], 0));
    open = true;
    return GCN_OK;
  }
  // hand-over number `slot` (2 .. kRowChunks + 1): what the caller's stream holds so far is done before what the side
  // stream gets next; then the caller's stream pauses, so that a side kernel that needs whole compute units is placed
  // before the caller's next kernel fills the chip (a kernel of small workgroups that is already running takes every
  // slot that frees up: a 256 x 256 product on 96 compute units that arrives 3 ms into a sparse product takes 18 ms
  // instead of 7)
  int hand_over(int slot) {
    GCN_HIP(hipEventRecord(A->side_events[slot], main));
    GCN_HIP(hipStreamWaitEvent(side, A->side_events[slot], 0));
    return stream_pause(main);
  }
  // the caller's stream goes on only when the side stream's work is done
  int join() {
    open = false;
    GCN_HIP(hipEventRecord(A->side_events[1], side));
    GCN_HIP(hipStreamWaitEvent(main, A->side_events[1], 0));
    return GCN_OK;
  }
};

// row chunks of a sparse product that a dense product follows one chunk behind: a power of two up to kRowChunks, 0 = none
static int side_chunks() { const int c = tune().overlap_chunks; return c >= 8 ? 8 : c >= 4 ? 4 : c >= 2 ? 2 : 0; }

// Is a sparse product over this many rows and entries at this width long enough to put the weight gradient beside it?
static bool overlap_worthwhile(int64_t rows, int64_t nnz, int d) {
  if (tune().overlap == 2) return true;
  return tune().overlap == 1 && rows >= (1 << 17) && (double)nnz * (double)d >= 4e9;
}

struct Carver {              // hands out 256-byte aligned pieces of the workspace
  char* base; size_t used = 0;
  void* take(size_t bytes) { void* p = base ? base + used : nullptr; used += align256(bytes); return p; }
};

}  // namespace gcn

using namespace gcn;

extern "C" int gcn_layer_fwd(const gcn_csr_t* A, const void* H, int64_t ldh, const float* W, const float* bias,
                             int d_in, int d_out, int act, int dtype, void* Z, void* Hout, void* AH_save,
                             void* stream) {
  return gcn_layer_fwd_ld(A, H, ldh, W, bias, d_in, d_out, act, dtype, Z, d_out, Hout, d_out, AH_save, d_in, stream);
}

extern "C" int gcn_layer_fwd_ld(const gcn_csr_t* A, const void* H, int64_t ldh, const float* W, const float* bias,
                                int d_in, int d_out, int act, int dtype, void* Z, int64_t ldz, void* Hout, int64_t ldo,
                                void* AH_save, int64_t ldah, void* stream) {
  clear_error();
  if (!A || !H || !W || !Hout) return fail(GCN_EINVAL, "gcn_layer_fwd: NULL argument");
  if (d_in < 1 || d_out < 1 || ldh < d_in) return fail(GCN_EINVAL, "gcn_layer_fwd: bad dimensions");
  if (ldo < d_out || (Z && ldz < d_out) || (AH_save && ldah < d_in))
    return fail(GCN_EINVAL, "gcn_layer_fwd: leading dimension smaller than the row");
  if (act != GCN_ACT_NONE && act != GCN_ACT_RELU) return fail(GCN_EINVAL, "gcn_layer_fwd: unknown activation");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_layer_fwd: unknown dtype");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  hipStream_t s = (hipStream_t)stream;
  const size_t es = es_of(dtype);
  // sparse-first costs nnz*d_in gathers and a dense product over nr rows; dense-first costs
  // nnz*d_out gathers and a dense product over nc rows
  const bool sparse_first = AH_save != nullptr || d_in <= d_out;
  const int relu = act == GCN_ACT_RELU;

  for (int pass = 0; pass < 2; ++pass) {      // pass 0 sizes the workspace, pass 1 runs
    Carver ws{pass ? (char*)Am->ws : nullptr};
    void* hub = ws.take(spmm_ws_bytes(&A->sched, sparse_first ? d_in : d_out));
    if (sparse_first) {
      void* AH = AH_save ? AH_save : ws.take((size_t)A->nr * d_in * es);
      const int64_t ldAH = AH_save ? ldah : (int64_t)d_in;
      const int64_t ldhp = padded_operand_ld(A, false, d_in, dtype, ldh);
      void* Hp = ldhp != ldh ? ws.take((size_t)A->nc * ldhp * es) : nullptr;
      if (pass) {
        if (Hp) GCN_TRY(pad_rows(H, ldh, Hp, ldhp, A->nc, d_in, dtype, s));
        SpmmArgs sp{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, Hp ? Hp : H, Hp ? ldhp : ldh, AH, ldAH,
                    nullptr, 0, d_in, dtype, GCN_EPI_NONE, nullptr, nullptr, 0};
        sp.owner = Am;
        sp.x_rows_padded = Hp != nullptr;
        GemmEpilogue epi;
        epi.bias = bias; epi.relu = relu; epi.C2 = Z; epi.ldc2 = ldz;
        const bool pipelined = side_chunks() > 0 && overlap_worthwhile(A->nr, A->nnz, d_in) && !spmm_panel_wanted(sp) &&
                               gemm_nn_limits_blocks(AH, ldAH, A->nr, d_out, d_in, dtype);
        if (!pipelined) {
          GCN_TRY(spmm_launch(sp, hub, s));
          GCN_TRY(gemm_nn(AH, ldAH, W, d_out, Hout, ldo, A->nr, d_out, d_in, dtype, epi, s));
        } else {
          // the dense product of a row chunk runs beside the sparse product of the next chunk
          SideStream side;
          GCN_TRY(side.fork(Am, s));
          const int step = kRowChunks / side_chunks();
          int last = 0;
          for (int c = 0; c < kRowChunks; c += step)
            if (A->sched.chunk_row[c + step] > A->sched.chunk_row[c]) last = c;
          for (int c = 0; c < kRowChunks; c += step) {
            const int64_t r0 = A->sched.chunk_row[c], r1 = A->sched.chunk_row[c + step];
            if (r1 <= r0) continue;
            sp.row_chunk = c; sp.row_chunk_n = step;
            GCN_TRY(spmm_launch(sp, hub, s));
            GCN_TRY(side.hand_over(2 + c));
            GemmEpilogue e = epi;
            if (Z) e.C2 = (char*)Z + (size_t)r0 * ldz * es;
            e.max_blocks = c == last ? 0 : tune().overlap_cus;
            GCN_TRY(gemm_nn((const char*)AH + (size_t)r0 * ldAH * es, ldAH, W, d_out, (char*)Hout + (size_t)r0 * ldo * es, ldo,
                            r1 - r0, d_out, d_in, dtype, e, side.side));
          }
          GCN_TRY(side.join());
        }
      }
    } else {
      const int64_t ldp = gather_ld_for(A, false, d_out, dtype);
      void* P = ws.take((size_t)A->nc * ldp * es);
      if (pass) {
        GemmEpilogue epi;
        GCN_TRY(gemm_nn(H, ldh, W, d_out, P, ldp, A->nc, d_out, d_in, dtype, epi, s));
        SpmmArgs sp{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, P, ldp, Hout, ldo, Z, ldz,
                    d_out, dtype, relu ? GCN_EPI_RELU : GCN_EPI_NONE, bias, nullptr, 0};
        sp.owner = Am;
        sp.x_rows_padded = true;
        GCN_TRY(spmm_launch(sp, hub, s));
      }
    }
    if (!pass) GCN_TRY(ensure_workspace(Am, ws.used));
  }
  return GCN_OK;
}

extern "C" int gcn_layer_bwd(const gcn_csr_t* A, const void* H, int64_t ldh, const void* AH_saved, const float* W,
                             int d_in, int d_out, int dtype, const void* G, const void* Zprev, float* dW,
                             float* dbias, void* dH, void* stream) {
  return gcn_layer_bwd_ld(A, H, ldh, AH_saved, d_in, W, d_in, d_out, dtype, G, d_out, Zprev, d_in, dW, dbias, dH, d_in, stream);
}

extern "C" int gcn_layer_bwd_ld(const gcn_csr_t* A, const void* H, int64_t ldh, const void* AH_saved, int64_t ldah,
                                const float* W, int d_in, int d_out, int dtype, const void* G, int64_t ldg,
                                const void* Zprev, int64_t ldzp, float* dW, float* dbias, void* dH, int64_t lddh,
                                void* stream) {
  clear_error();
  if (!A || !H || !W || !G || !dW) return fail(GCN_EINVAL, "gcn_layer_bwd: NULL argument");
  if (d_in < 1 || d_out < 1 || ldh < d_in) return fail(GCN_EINVAL, "gcn_layer_bwd: bad dimensions");
  if (ldg < d_out || (AH_saved && ldah < d_in) || (Zprev && ldzp < d_in) || (dH && lddh < d_in))
    return fail(GCN_EINVAL, "gcn_layer_bwd: leading dimension smaller than the row");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_layer_bwd: unknown dtype");
  if (dH && !A->colptr) return fail(GCN_EINVAL, "gcn_layer_bwd: dH needs a handle built with GCN_BUILD_CSC");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  hipStream_t s = (hipStream_t)stream;
  const size_t es = es_of(dtype);
  const bool have_csc = A->colptr != nullptr;
  // share one transposed sparse product of width d_out between dH and dW when that is narrower
  const bool via_T = have_csc && d_out < d_in && (dH != nullptr || AH_saved == nullptr);

  for (int pass = 0; pass < 2; ++pass) {
    Carver ws{pass ? (char*)Am->ws : nullptr};
    const int dmax = d_in > d_out ? d_in : d_out;
    size_t hub_bytes = spmm_ws_bytes(&A->sched, dmax);
    if (have_csc && spmm_ws_bytes(&A->sched_t, dmax) > hub_bytes) hub_bytes = spmm_ws_bytes(&A->sched_t, dmax);
    void* hub = ws.take(hub_bytes);
    float* Wt = (float*)ws.take(sizeof(float) * (size_t)d_in * d_out);
    void* cs = dbias ? ws.take(colsum_ws_bytes(A->nr, d_out)) : nullptr;
    if (pass && dbias) GCN_TRY(colsum(G, ldg, A->nr, d_out, dtype, dbias, cs, s));

    if (via_T) {
      const int64_t ldt = round_up(d_out, 4);
      void* T = ws.take((size_t)A->nc * ldt * es);
      const int64_t kd = AH_saved ? A->nr : A->nc;
      void* tn = ws.take(gemm_tn_ws_bytes(kd, d_in, d_out));
      // rows of G whose pitch is not a multiple of 16 bytes are first copied to a padded buffer: the
      // sparse product then gathers with vector loads
      // a caller's G that the sparse product cannot gather with 16-byte requests, or only across more lines than
      // need be, is first copied to a padded buffer
      // (a pitched G is backed to the end of every row, the last included: the contract of the _ld entry points; so a
      // row that is no whole number of 16-byte vectors can still be gathered with them when the pitch leaves room)
      const bool g_rows_backed = ldg >= round_up(d_out, 16 / (int64_t)es);
      const bool g_unaligned = (ldg * (int64_t)es) % 16 != 0 || ((uintptr_t)G % 16) != 0 ||
                               ((d_out * (int64_t)es) % 16 != 0 && !g_rows_backed);
      const int64_t ldgp = g_unaligned ? gather_ld_for(A, true, d_out, dtype) : padded_operand_ld(A, true, d_out, dtype, ldg);
      const bool pad_g = g_unaligned || ldgp != ldg;
      void* Gp = pad_g ? ws.take((size_t)A->nr * ldgp * es) : nullptr;
      if (pass) {
        if (pad_g) GCN_TRY(pad_rows(G, ldg, Gp, ldgp, A->nr, d_out, dtype, s));
        SpmmArgs sp{A->colptr, A->rowidx, A->val_t, &A->sched_t, A->nc, A->nr, A->nnz, true, A->nr, pad_g ? Gp : G,
                    pad_g ? ldgp : ldg, T, ldt, nullptr, 0, d_out, dtype, GCN_EPI_NONE, nullptr, nullptr, 0};
        sp.x_rows_padded = pad_g || g_rows_backed;
        sp.owner = Am;
        // dW from a saved A^ H needs nothing of this product: it runs beside it
        SideStream side;
        const bool beside = AH_saved && overlap_worthwhile(A->nc, A->nnz, d_out) &&
                            gemm_tn_limits_blocks(AH_saved, ldah, G, ldg, A->nr, d_in, d_out, dtype);
        if (beside) {
          GCN_TRY(side.fork(Am, s));
          GCN_TRY(gemm_tn(AH_saved, ldah, G, ldg, dW, d_out, A->nr, d_in, d_out, dtype, tn, side.side, tune().overlap_cus));
        }
        GCN_TRY(spmm_launch(sp, hub, s));
        if (dH) {
          GCN_TRY(transpose_f32(W, d_in, d_out, Wt, s));
          // owned rows carry the ReLU mask, halo rows do not: two calls, so that each is uniform in its epilogue
          GemmEpilogue epi;
          epi.mask = Zprev; epi.ldmask = ldzp; epi.mask_rows = Zprev ? A->nr : 0;
          GCN_TRY(gemm_nn(T, ldt, Wt, d_in, dH, lddh, A->nr, d_in, d_out, dtype, epi, s));
          if (A->nh > 0)
            GCN_TRY(gemm_nn((const char*)T + (size_t)A->nr * ldt * es, ldt, Wt, d_in, (char*)dH + (size_t)A->nr * lddh * es, lddh,
                            A->nh, d_in, d_out, dtype, GemmEpilogue(), s));
        }
        if (beside) GCN_TRY(side.join());
        else if (AH_saved) GCN_TRY(gemm_tn(AH_saved, ldah, G, ldg, dW, d_out, A->nr, d_in, d_out, dtype, tn, s));
        else GCN_TRY(gemm_tn(H, ldh, T, ldt, dW, d_out, A->nc, d_in, d_out, dtype, tn, s));
      }
    } else {
      const int64_t ldq = gather_ld_for(A, true, d_in, dtype);
      void* Q = dH ? ws.take((size_t)A->nr * ldq * es) : nullptr;
      void* AH = AH_saved ? nullptr : ws.take((size_t)A->nr * ldq * es);
      // the product A^ H gathers the caller's H: from a padded copy where that saves line reads, as in the forward pass
      const int64_t ldhp = AH_saved ? ldh : padded_operand_ld(A, false, d_in, dtype, ldh);
      void* Hp = ldhp != ldh ? ws.take((size_t)A->nc * ldhp * es) : nullptr;
      void* tn = ws.take(gemm_tn_ws_bytes(A->nr, d_in, d_out));
      if (pass) {
        SideStream side;
        const bool beside = dH && AH_saved && overlap_worthwhile(A->nc, A->nnz, d_in) &&
                            gemm_tn_limits_blocks(AH_saved, ldah, G, ldg, A->nr, d_in, d_out, dtype);
        if (dH) {
          GCN_TRY(transpose_f32(W, d_in, d_out, Wt, s));
          GemmEpilogue epi;
          GCN_TRY(gemm_nn(G, ldg, Wt, d_in, Q, ldq, A->nr, d_in, d_out, dtype, epi, s));
          if (beside) {        // after Q = G W^T, which wants the matrix pipes of every compute unit itself
            GCN_TRY(side.fork(Am, s));
            GCN_TRY(gemm_tn(AH_saved, ldah, G, ldg, dW, d_out, A->nr, d_in, d_out, dtype, tn, side.side, tune().overlap_cus));
          }
          SpmmArgs sp{A->colptr, A->rowidx, A->val_t, &A->sched_t, A->nc, A->nr, A->nnz, true, A->nr, Q, ldq, dH, lddh, nullptr, 0,
                      d_in, dtype, Zprev ? GCN_EPI_MASK : GCN_EPI_NONE, nullptr, Zprev, ldzp};
          sp.owner = Am;
          sp.x_rows_padded = true;
          GCN_TRY(spmm_launch(sp, hub, s));
        }
        const void* ah = AH_saved; int64_t ld_ah = ldah;
        if (!AH_saved) {
          if (Hp) GCN_TRY(pad_rows(H, ldh, Hp, ldhp, A->nc, d_in, dtype, s));
          SpmmArgs sp{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, Hp ? Hp : H, Hp ? ldhp : ldh, AH, ldq,
                      nullptr, 0, d_in, dtype, GCN_EPI_NONE, nullptr, nullptr, 0};
          sp.owner = Am;
          sp.x_rows_padded = Hp != nullptr;
          GCN_TRY(spmm_launch(sp, hub, s));
          ah = AH; ld_ah = ldq;
        }
        if (beside) GCN_TRY(side.join());
        else GCN_TRY(gemm_tn(ah, ld_ah, G, ldg, dW, d_out, A->nr, d_in, d_out, dtype, tn, s));
      }
    }
    if (!pass) GCN_TRY(ensure_workspace(Am, ws.used));
  }
  return GCN_OK;
}

extern "C" int gcn_dense_fwd(const void* X, int64_t ldx, int64_t rows, const float* W, const float* bias, int d_in,
                             int d_out, int act, int dtype, void* Z, void* Out, int64_t ldo, void* stream) {
  clear_error();
  if (rows < 0) return fail(GCN_EINVAL, "gcn_dense_fwd: negative row count");
  if (rows == 0) return GCN_OK;
  if (!X || !W || !Out) return fail(GCN_EINVAL, "gcn_dense_fwd: NULL argument");
  if (d_in < 1 || d_out < 1 || ldx < d_in || ldo < d_out) return fail(GCN_EINVAL, "gcn_dense_fwd: bad dimensions");
  if (act != GCN_ACT_NONE && act != GCN_ACT_RELU) return fail(GCN_EINVAL, "gcn_dense_fwd: unknown activation");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_dense_fwd: unknown dtype");
  GemmEpilogue epi;
  epi.bias = bias; epi.relu = act == GCN_ACT_RELU; epi.C2 = Z; epi.ldc2 = d_out;
  return gemm_nn(X, ldx, W, d_out, Out, ldo, rows, d_out, d_in, dtype, epi, (hipStream_t)stream);
}

extern "C" int gcn_layer_bwd_pull(const gcn_csr_t* A, int phase, const void* H, int64_t ldh, const float* W, int d_in,
                                  int d_out, int dtype, const void* G, int64_t ldg, const void* Zprev, void* T,
                                  float* dW, float* dbias, void* dH, void* stream) {
  clear_error();
  if (!A || !G || !T) return fail(GCN_EINVAL, "gcn_layer_bwd_pull: NULL argument");
  if (phase != 0 && phase != GCN_PART_LOCAL && phase != GCN_PART_HALO)
    return fail(GCN_EINVAL, "gcn_layer_bwd_pull: phase must be 0, GCN_PART_LOCAL or GCN_PART_HALO");
  if (d_in < 1 || d_out < 1 || ldg < d_out) return fail(GCN_EINVAL, "gcn_layer_bwd_pull: bad dimensions");
  if (dtype != GCN_F32 && dtype != GCN_BF16) return fail(GCN_EINVAL, "gcn_layer_bwd_pull: unknown dtype");
  const bool finish = phase != GCN_PART_LOCAL;
  if (finish && (!H || !W || !dW || ldh < d_in)) return fail(GCN_EINVAL, "gcn_layer_bwd_pull: H, W and dW are needed to finish");
  gcn_csr* Am = const_cast<gcn_csr*>(A);
  hipStream_t s = (hipStream_t)stream;

  for (int pass = 0; pass < 2; ++pass) {
    Carver ws{pass ? (char*)Am->ws : nullptr};
    void* hub = ws.take(spmm_ws_bytes(&A->sched, d_out));
    float* Wt = finish && dH ? (float*)ws.take(sizeof(float) * (size_t)d_in * d_out) : nullptr;
    void* cs = finish && dbias ? ws.take(colsum_ws_bytes(A->nr, d_out)) : nullptr;
    void* tn = finish ? ws.take(gemm_tn_ws_bytes(A->nr, d_in, d_out)) : nullptr;
    if (pass) {
      // T = A^_m [G_m; G_halo]: the product that serves both S and dW (Sec. 4.2)
      SpmmArgs sp{A->rowptr, A->col, A->val, &A->sched, A->nr, A->nc, A->nnz, false, A->nr, G, ldg, T, d_out, nullptr, 0,
                  d_out, dtype, GCN_EPI_NONE, nullptr, nullptr, 0};
      sp.owner = Am;
      if (phase != 0) {
        if (A->mid) { sp.part = phase; sp.mid = A->mid; }
        else if (phase == GCN_PART_HALO) { sp.part = 2; sp.mid = A->rowptr + 1; }
      }
      GCN_TRY(spmm_launch(sp, hub, s));
      if (finish) {
        if (dbias) GCN_TRY(colsum(G, ldg, A->nr, d_out, dtype, dbias, cs, s));
        if (dH) {
          GCN_TRY(transpose_f32(W, d_in, d_out, Wt, s));
          GemmEpilogue epi;
          epi.mask = Zprev; epi.ldmask = d_in; epi.mask_rows = Zprev ? A->nr : 0;
          GCN_TRY(gemm_nn(T, d_out, Wt, d_in, dH, d_in, A->nr, d_in, d_out, dtype, epi, s));
        }
        GCN_TRY(gemm_tn(H, ldh, T, d_out, dW, d_out, A->nr, d_in, d_out, dtype, tn, s));
      }
    }
    if (!pass) GCN_TRY(ensure_workspace(Am, ws.used));
  }
  return GCN_OK;
}
