/*
 * gcn.h -- C ABI of the MI355X (gfx950) GCN layer library.
 *
 * One full-batch GCN layer on one GPU's row block of a 1D row-partitioned graph
 * ("Scalable Graph Convolutional Network Training on Distributed-Memory Systems",
 * Sec. 3.1 graph convolution, Sec. 4.1 feedforward, Sec. 4.2 backpropagation):
 *
 *     forward   Z = A^ H W,  Hout = act(Z)                       (Sec. 3.1, first equation)
 *     backward  dW = (A^ H)^T G,  dH = (A^T G W^T) (.) [Zprev>0] (Sec. 3.1, 2nd/3rd equations;
 *                                                                 A^T for directed graphs)
 *
 * with A^ = D^-1/2 (A + I) D^-1/2 stored in CSR (and CSC for the transpose).  A block owns
 * nr consecutive global rows [row_lo, row_hi); the nh distinct non-owned columns it touches
 * ("halo", Sec. 4.1: the rows received from other processors, each one once) are numbered
 * nr .. nr+nh-1 in ascending global id.  Dense operands of a block therefore have
 * nc = nr + nh rows: owned rows first, then halo rows in halo-list order.
 *
 * General conventions
 *  - Every function returns 0 (GCN_OK) or a negative error code; gcn_last_error() gives a
 *    thread-local message for the last failure.  Nothing aborts, throws or prints.
 *  - All dense buffers are caller-owned DEVICE pointers (gcn_halo_gather's table may also be
 *    pinned host memory), row-major, with the leading dimension given in elements.  The
 *    library never frees or keeps them.
 *  - gcn_csr_t is an opaque, library-owned handle (device arrays + a scratch workspace that
 *    grows on demand and is reused by later calls).  Calls that use the same handle must not
 *    overlap in time.
 *  - `stream` is a hipStream_t passed as void* (NULL = default stream).  Calls only enqueue
 *    work; they do not synchronise, except gcn_csr_build (it must learn nnz and nh), a
 *    call that has to grow the handle's workspace, and the first sparse product of a new
 *    width class on a handle whose matrix qualifies for the column-sweep kernel: that call
 *    builds an execution plan (a re-sorted copy of the matrix, 8 bytes per stored entry plus
 *    padding, kept in the handle until gcn_csr_free), which allocates and waits for the
 *    stream.  Later calls of that width class reuse the plan.
 *  - Sizes: vertex ids and n_global lie below 2^31, edges + rows of a build below 2^32; dense buffers may
 *    run past 2^32 bytes and 2^31 elements (row offsets are 64-bit).  A size that a kernel cannot take is
 *    an error (GCN_EINVAL), never a truncated result.
 *  - Indices are int32, row/column pointers int64, matrix values and all accumulators fp32.
 *    dtype selects the element type of *feature* buffers: GCN_F32, or GCN_BF16 (bf16 storage,
 *    fp32 accumulation, round-to-nearest-even on store).
 */
#ifndef GCN_H_
#define GCN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GCN_OK 0
#define GCN_EINVAL (-1) /* bad argument: null pointer, negative size, ld < d, id out of range ... */
#define GCN_ENOMEM (-2) /* device allocation failed */
#define GCN_EHIP (-3)   /* HIP runtime error */

#define GCN_F32 0
#define GCN_BF16 1

#define GCN_BUILD_CSC 1 /* also build the column-major copy needed by gcn_spmm_t / gcn_layer_bwd */

#define GCN_EPI_NONE 0 /* Y = A X (+ bias) */
#define GCN_EPI_RELU 1 /* Y = max(A X (+ bias), 0) */
#define GCN_EPI_MASK 2 /* Y = (A X) * [Zprev > 0]   (ReLU derivative: 1 for z > 0, else 0) */

#define GCN_ACT_NONE 0
#define GCN_ACT_RELU 1

typedef struct gcn_csr gcn_csr_t;

/* Message of the last error raised on the calling thread ("" if none). */
const char* gcn_last_error(void);

/*
 * Build the normalised adjacency block (Sec. 3.1: A^ = D^-1/2 (A+I) D^-1/2, D(i,i) = row sum
 * of A+I; Sec. 4.1: halo rows = cols(A_m) not owned by m, each listed once).
 *
 *   d_src, d_dst  device int32[n_edges]: directed edges (row = src, column = dst) in GLOBAL
 *                 ids.  Duplicates and self-loops are allowed (A is a 0/1 pattern: duplicates
 *                 collapse, input self-loops are replaced by the single diagonal entry of I).
 *                 Edges whose src is outside [row_lo, row_hi) are ignored.
 *   n_global      number of vertices of the whole graph; every id must lie in [0, n_global).
 *   row_lo,row_hi owned rows; (0, n_global) means the whole graph.
 *   d_deg_global  device int32[n_global] or NULL: degrees INCLUDING the self-loop of every
 *                 global vertex, every entry >= 1.  Required when the block is not the whole graph:
 *                 the degrees of halo vertices cannot be derived from the block's own rows.  Only
 *                 those are read from it; an owned vertex's degree is always the entry count of its
 *                 row, which the block holds whole (Sec. 4.1).
 *   flags         GCN_BUILD_CSC or 0.
 *
 * Result: CSR with columns in local numbering (owned j -> j - row_lo, halo -> nr + rank),
 * strictly ascending inside each row; val(i,j) = fl(1/sqrt(d_i)) * fl(1/sqrt(d_j)) in fp32;
 * deg[i] = number of entries of row i.  Synchronises `stream`.  On error *out is NULL.
 */
int gcn_csr_build(const int32_t* d_src, const int32_t* d_dst, int64_t n_edges, int64_t n_global,
                  int64_t row_lo, int64_t row_hi, const int32_t* d_deg_global, int flags,
                  void* stream, gcn_csr_t** out);

/* Sizes of a block: owned rows, halo rows, stored entries.  Any output pointer may be NULL. */
int gcn_csr_info(const gcn_csr_t* A, int64_t* nr, int64_t* nh, int64_t* nnz);

/*
 * Device pointers to the handle's arrays (for inspection / parity checks; owned by the
 * handle, valid until gcn_csr_free).  Any output pointer may be NULL.  colptr/rowidx/val_t
 * are NULL if the handle was built without GCN_BUILD_CSC.
 *   rowptr int64[nr+1], col int32[nnz], val f32[nnz], deg int32[nr], halo_gid int32[nh],
 *   colptr int64[nc+1], rowidx int32[nnz] (ascending inside each column), val_t f32[nnz].
 */
int gcn_csr_arrays(const gcn_csr_t* A, const int64_t** rowptr, const int32_t** col,
                   const float** val, const int32_t** deg, const int32_t** halo_gid,
                   const int64_t** colptr, const int32_t** rowidx, const float** val_t);

/* Free the handle, its device arrays and its workspace.  NULL is accepted. */
int gcn_csr_free(gcn_csr_t* A);

/*
 * Y[nr x d] = epilogue( A^_m X[nc x d] + bias )          (Sec. 4.1, the sum of the per-row task:
 *                                                         sum_{j in cols(A(i,:))} A(i,j) X(j,:))
 *   X, Y      device, element type `dtype`, leading dimensions ldx >= d, ldy >= d.
 *   epilogue  GCN_EPI_NONE | GCN_EPI_RELU | GCN_EPI_MASK.
 *   bias      device f32[d] or NULL (added before the activation; not part of the paper's layer).
 *   Zprev     device [nr x d] (ldz), only read for GCN_EPI_MASK.
 * X and Y must not alias.  Rows are reduced in a fixed order: results are run-to-run identical.
 */
int gcn_spmm(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y,
             int64_t ldy, int epilogue, const float* bias, const void* Zprev, int64_t ldz,
             void* stream);

/*
 * gcn_spmm for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, same kernels and the same result as gcn_spmm's row kernel; the partial rows
 * of long-row chunks go to a fixed 64 MiB device array of the library (held by every GPU the library runs on
 * until the process ends) instead of the handle's workspace, the column-sweep variant (whose plan would have to
 * be built) is never taken, and the launches are not recorded by the profiling hooks.  The call allocates and
 * frees nothing and does not synchronise.
 *   Limit: (chunks of 1024 entries of rows longer than 2048 entries) x d x 4 bytes <= 64 MiB; beyond it the
 *   call returns GCN_EINVAL and enqueues nothing.
 *   All calls on one GPU share that array: nothing in it has to start at zero (every partial row is written
 *   before it is read), but two calls that overlap in time on one GPU (different streams) race on it.
 */
int gcn_spmm_noalloc(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y,
                     int64_t ldy, int epilogue, const float* bias, const void* Zprev, int64_t ldz,
                     void* stream);

/*
 * Y[nc x d] = epilogue( A^_m^T X[nr x d] )   (Sec. 3.1: for a directed graph backpropagation
 * uses the transpose).  Needs GCN_BUILD_CSC.  Rows nr..nc-1 of Y are the contributions of
 * this block to rows owned elsewhere.  GCN_EPI_MASK applies to the owned rows 0..nr-1 only
 * (Zprev is [nr x d]); halo rows are written unmasked.
 */
int gcn_spmm_t(const gcn_csr_t* A, const void* X, int64_t ldx, int d, int dtype, void* Y,
               int64_t ldy, int epilogue, const void* Zprev, int64_t ldz, void* stream);

/*
 * recv[s, :] = table[idx[s], :] for s < n_idx   (Sec. 4.1: selecting the rows of H named by an
 * index set -- the selector-matrix product that copies instead of multiplying -- and filling
 * the receive buffer of non-local rows).
 *   table   [n_table_rows x d] (ld), DEVICE memory or PINNED HOST memory mapped into the device.
 *   d_idx   device int32[n_idx]; every index must lie in [0, n_table_rows).  An out-of-range
 *           index is never dereferenced: that output row is zero-filled instead.
 *   recv    device [n_idx x d] (ldr).  Element type `dtype` for both table and recv.
 */
int gcn_halo_gather(const void* table, int64_t ld, int64_t n_table_rows, int d, int dtype,
                    const int32_t* d_idx, int64_t n_idx, void* recv, int64_t ldr, void* stream);

/*
 * Forward pass of one layer on the block (Sec. 3.1 first equation, Sec. 4.1):
 *   Z = A^_m H W (+ bias),  Hout = act(Z).
 *   H        device [nc x d_in] (ldh): owned rows, then halo rows.
 *   W        device f32 [d_in x d_out], dense (ld = d_out).   bias: device f32[d_out] or NULL.
 *   Z        device [nr x d_out] (ld = d_out) or NULL: pre-activation values.
 *   Hout     device [nr x d_out] (ld = d_out), required.
 *   AH_save  device [nr x d_in] (ld = d_in) or NULL.  When given, the layer is evaluated as
 *            (A^ H) W and A^ H is stored here for the backward pass; otherwise the library
 *            picks the cheaper of (A^ H) W and A^ (H W).  Both are the same sum; only the
 *            rounding order differs.
 * Streams: the result is ordered on `stream` like that of any other call.  On large blocks (fp32, from about 10^5
 * rows) the call may run its dense product on a second stream that the handle owns (default priority, created on
 * first use, destroyed by gcn_csr_free), beside the sparse product of the same call, which is then launched on ranges
 * of rows with the dense product one range behind (Sec. 4.1's row-wise tasks are independent; Sec. 4.1 overlaps
 * communication with the local product in the same way).  Events tie that stream to `stream` at both ends: nothing of
 * the call is pending on it when work enqueued on `stream` after the call starts.  The results do not depend on it
 * (gcn_debug_set_tuning "GCN_OVERLAP" 0 keeps everything on `stream`).  Capture: once a first call has sized the
 * workspace and created the second stream, the layer calls only enqueue kernels and event waits, and can be captured
 * into a HIP graph through `stream` (the second stream joins the capture through its events).
 */
int gcn_layer_fwd(const gcn_csr_t* A, const void* H, int64_t ldh, const float* W,
                  const float* bias, int d_in, int d_out, int act, int dtype, void* Z, void* Hout,
                  void* AH_save, void* stream);
/* The same layer (Sec. 3.1 first equation, Sec. 4.1) with a leading dimension for every feature buffer, so that a
 * layer's output can be written straight into a buffer with the pitch the next layer's sparse product gathers
 * best from (gcn_feature_ld): Z (ldz), Hout (ldo), AH_save (ldah), each >= its row width.  For this call and
 * gcn_layer_bwd_ld a buffer whose leading dimension exceeds its row width must be backed by memory to the end of
 * EVERY row's pitch, the last row included (rows x ld elements, as gcn_feature_ld's users allocate): the kernels may
 * read the padding of an input row (whatever it holds, NaN included, reaches no result) and may write the padding of
 * an output row up to the next multiple of 16 bytes of the row width (content unspecified). */
int gcn_layer_fwd_ld(const gcn_csr_t* A, const void* H, int64_t ldh, const float* W, const float* bias, int d_in,
                     int d_out, int act, int dtype, void* Z, int64_t ldz, void* Hout, int64_t ldo, void* AH_save,
                     int64_t ldah, void* stream);

/*
 * Backward pass of one layer on the block (Sec. 3.1 second and third equations, Sec. 4.2):
 *   dW    = (A^_m H)^T G                 f32 [d_in x d_out]  (this block's partial sum)
 *   dbias = column sums of G             f32 [d_out] or NULL
 *   dH    = (A^_m^T G W^T) (.) [Zprev>0] [nc x d_in] (ld = d_in) or NULL (first layer: skipped).
 *           The mask covers the owned rows (Zprev is [nr x d_in], ld = d_in; NULL = no mask);
 *           halo rows nr..nc-1 are this block's unmasked contributions to rows owned elsewhere.
 *   H        device [nc x d_in] (ldh), the layer's input.
 *   AH_saved device [nr x d_in] from gcn_layer_fwd or NULL.
 *   G        device [nr x d_out] (ld = d_out): gradient w.r.t. this layer's Z.
 * Needs GCN_BUILD_CSC when dH is requested.
 * Streams: as gcn_layer_fwd; here it is dW from AH_saved, which needs nothing of the call's sparse product, that
 * runs beside it on the handle's second stream.
 */
int gcn_layer_bwd(const gcn_csr_t* A, const void* H, int64_t ldh, const void* AH_saved,
                  const float* W, int d_in, int d_out, int dtype, const void* G,
                  const void* Zprev, float* dW, float* dbias, void* dH, void* stream);
/* The same backward pass (Sec. 3.1 second and third equations, Sec. 4.2) with a leading dimension for every
 * feature buffer: AH_saved (ldah), G (ldg), Zprev (ldzp), dH (lddh), each >= its row width and, where larger, backed
 * to the end of every row as stated for gcn_layer_fwd_ld. */
int gcn_layer_bwd_ld(const gcn_csr_t* A, const void* H, int64_t ldh, const void* AH_saved, int64_t ldah,
                     const float* W, int d_in, int d_out, int dtype, const void* G, int64_t ldg, const void* Zprev,
                     int64_t ldzp, float* dW, float* dbias, void* dH, int64_t lddh, void* stream);

/*
 * Output-layer loss and gradient (Sec. 3.1: G^L = grad J (.) act'(Z^L), identity activation on
 * the last layer, J = softmax cross-entropy):
 *   loss = -scale * sum_i log softmax(Z_i)[y_i],   G = scale * (softmax(Z) - onehot(y)).
 *   Z     device [nr x C] (ldz), element type dtype.   y: device int32[nr]; y[i] < 0 means
 *         "no label": no loss term, zero gradient row; y[i] >= C is treated the same way.
 *   loss  device f32 scalar (accumulated in fp64 in a fixed order: run-to-run identical).
 *   G     device [nr x C] (ldg), element type dtype.
 * The per-block partial sums live in a fixed device buffer of the library with 64 rows; every
 * call takes the next row, so calls may overlap in time on different streams as long as fewer
 * than 64 of them are in flight on one GPU.
 */
int gcn_softmax_xent(const void* Z, int64_t ldz, int64_t nr, int C, int dtype, const int32_t* y,
                     float scale, float* loss, void* G, int64_t ldg, void* stream);

/*
 * The product of gcn_spmm in two steps (Sec. 4.1, block form Z_m = A_m H_m + sum_n A_m H_nm, and
 * Algorithm 1: the local product does not wait for the rows of other processors):
 *   GCN_PART_LOCAL  Y = A^[:, 0..nr) X[0..nr)        plain sums; reads only the owned rows of X, so it can run
 *                                                    while the halo rows are still on their way.  epilogue must
 *                                                    be GCN_EPI_NONE and bias NULL.
 *   GCN_PART_HALO   Y = epilogue(Y + A^[:, nr..nc) X[nr..nc) + bias)    adds the halo columns to what the local
 *                                                    step left in Y and finishes the product.
 * Arguments as gcn_spmm.  The two steps in this order give gcn_spmm's result up to the order of the additions
 * (same tolerance); a handle without halo columns takes the second step as "apply the epilogue".
 */
#define GCN_PART_LOCAL 1
#define GCN_PART_HALO 2
int gcn_spmm_part(const gcn_csr_t* A, int part, const void* X, int64_t ldx, int d, int dtype, void* Y,
                  int64_t ldy, int epilogue, const float* bias, const void* Zprev, int64_t ldz, void* stream);

/*
 * The dense half of a layer on `rows` rows (Sec. 3.1: the product with W^k and the activation), for callers
 * that drive the sparse half themselves (gcn_spmm_part):
 *   Out = act(X W + bias),  Z (nullable) = X W + bias.   X: device [rows x d_in] (ldx), W: device f32
 *   [d_in x d_out], Out / Z: device [rows x d_out] (ldo / contiguous), element type dtype.
 */
int gcn_dense_fwd(const void* X, int64_t ldx, int64_t rows, const float* W, const float* bias, int d_in, int d_out,
                  int act, int dtype, void* Z, void* Out, int64_t ldo, void* stream);

/*
 * Backward pass of one layer in the form of Algorithm 2 (Sec. 4.2), for a symmetric A^: every block pulls the
 * gradient rows it needs instead of pushing contributions.
 *   T     = A^_m [G_m; G_halo]               [nr x d_out] (ld = d_out), element type dtype: the product that serves
 *                                            both results below; written to the caller's buffer T.
 *   dH    = (T W^T) (.) [Zprev > 0]          [nr x d_in] (ld = d_in) or NULL: the owned rows of G^(k-1), complete
 *                                            (nothing to send back).  Zprev [nr x d_in] (ld = d_in); NULL = no mask.
 *   dW    = H_m^T T                          f32 [d_in x d_out]: this block's partial sum; only the nr owned rows
 *                                            of H (ldh) are read.
 *   dbias = column sums of the owned rows of G, f32 [d_out] or NULL.
 *   G     device [nc x d_out] (ldg): owned rows, then the halo rows in halo-list order (fetched by the caller, e.g.
 *         with gcn_halo_gather, as the rows of H are in the forward pass).
 *   phase 0: everything.  GCN_PART_LOCAL: only T = A^[:, 0..nr) G_m, which reads no halo row of G and can run while
 *         those arrive (H, W, dW may be NULL).  GCN_PART_HALO: adds the halo columns to T, then dH, dW, dbias.
 * On a directed graph this is not the gradient (the algorithm relies on A^ = A^T); gcn_layer_bwd is.
 */
int gcn_layer_bwd_pull(const gcn_csr_t* A, int phase, const void* H, int64_t ldh, const float* W, int d_in, int d_out,
                       int dtype, const void* G, int64_t ldg, const void* Zprev, void* T, float* dW, float* dbias,
                       void* dH, void* stream);

/*
 * The subgraph induced by a vertex list, as a graph of its own (Sec. 4.3.3: a mini-batch is a subgraph
 * G' = (V', E') of the input graph on which the convolutions run as in full-batch training).
 *   A           handle of a whole graph (all rows, no halo columns).
 *   d_vertices  device int32 [n_sub]: distinct vertex ids of A, in any order; vertex k of the result is d_vertices[k].
 *   flags       GCN_BUILD_CSC or 0.
 * Result: a new whole-graph handle on n_sub vertices whose stored entries are (a, b) for every stored entry
 * (d_vertices[a], d_vertices[b]) of A, with degrees, diagonal and normalisation taken within the subgraph
 * (A^' = D'^-1/2 (A' + I) D'^-1/2); arrays laid out as gcn_csr_build's.  Features and labels of the subgraph are
 * the rows d_vertices of the parent's (gcn_halo_gather with d_vertices as the index list).  Integer arrays and
 * values are bit-identical to building the relabelled edge list of G' with gcn_csr_build.
 * Errors: an id outside the graph or listed twice gives GCN_EINVAL.  Allocates temporaries, synchronises the
 * stream; free the result with gcn_csr_free.
 */
int gcn_csr_induced(const gcn_csr_t* A, const int32_t* d_vertices, int64_t n_sub, int flags, void* stream,
                    gcn_csr_t** out);

/*
 * Communication figures of a 1D row partition, counted on the device (Sec. 4.3.2, the column-net hypergraph model
 * and its total-volume formula; Sec. 5, the per-processor volume and message counts of the communication table).
 * Net n_j joins the rows with a stored entry in column j; the part that owns vertex j sends row j once to every
 * other part of the net's connectivity set.
 *   A        handle of a whole graph (all rows, no halo columns).
 *   d_part   device int32 [n]: part of every vertex, in [0, p);  1 <= p <= 32768.
 * Results, device int64, each nullable:
 *   d_load [p]       stored entries in the part's rows (sum of the vertex weights w(v_i) = |cols(A(i,:))|)
 *   d_send_rows [p]  rows the part sends per sparse product;  d_recv_rows [p]  rows it receives (its halo size)
 *   d_send_msgs [p]  parts it sends to;                       d_recv_msgs [p]  parts it receives from
 *   d_totals [2]     { sum_j (lambda(n_j) - 1): all rows moved per product (the paper's total without the constant
 *                      factors 2 and cost(n_j));  stored entries whose ends lie in different parts (what the graph
 *                      model charges instead) }
 * Integer work: exact.  Allocates temporaries (about 30 bytes per stored entry) and synchronises the stream.
 */
int gcn_partition_stats(const gcn_csr_t* A, const int32_t* d_part, int p, int64_t* d_load, int64_t* d_send_rows,
                        int64_t* d_recv_rows, int64_t* d_send_msgs, int64_t* d_recv_msgs, int64_t* d_totals,
                        void* stream);

/*
 * Weight update of gradient descent (Sec. 3.1, last equation; last line of Algorithm 2):
 *   W <- W - lr * dW,   elementwise on n fp32 values (W and dW: device, contiguous, may not overlap).
 * One fused multiply-add per element.  Not part of the timed forward+backward epoch.
 */
int gcn_sgd_update(float* W, const float* dW, int64_t n, float lr, void* stream);

/*
 * Per-kernel timing, for benchmarks (instrumentation; no part of the paper's method).
 * While enabled, every kernel launch of the library is bracketed by a pair of HIP events recorded
 * on the stream the kernel is launched on, and described by one record.  Records are kept in
 * launch order up to a fixed capacity (65536); later launches run untimed and are counted as
 * dropped.  gcn_profile_enable(1) clears the records and starts recording, gcn_profile_enable(0)
 * stops.  gcn_profile_get synchronises with the record's stop event.
 *
 *   kind       GCN_K_* below.
 *   d          feature width of the launch (N of a dense product, C of the loss).
 *   rows       output rows (sparse products, gather, loss) or M of a dense product.
 *   inner      stored entries of the sparse matrix, or the reduction length K of a dense product.
 *   alg_bytes  bytes the operation has to move at least once: every operand and result once
 *              (sparse products: 8 bytes per stored entry + 8 per row pointer + each feature row
 *              of the input and of the output once).
 *   touched_bytes  sparse products only: as alg_bytes, but a gathered feature row is counted every
 *              time it is read (what caches and HBM together serve); else equal to alg_bytes.
 *   flops      2 * multiply-adds.
 *   ms         elapsed time between the two events.
 */
#define GCN_K_SPMM 0          /* A X, main kernel */
#define GCN_K_SPMM_T 1        /* A^T X, main kernel */
#define GCN_K_SPMM_FINISH 2   /* sum of the partial rows of long rows + epilogue */
#define GCN_K_GEMM_NN 3
#define GCN_K_GEMM_TN 4       /* partial tiles of A^T B */
#define GCN_K_GEMM_TN_SUM 5   /* sum of the partial tiles */
#define GCN_K_SOFTMAX_XENT 6
#define GCN_K_GATHER 7
#define GCN_K_OTHER 8         /* small helpers: weight transpose, column sums, loss finish */

typedef struct {
  int32_t kind, d, dtype, reserved;
  int64_t rows, inner;
  double alg_bytes, touched_bytes, flops, ms;
} gcn_profile_rec;

int gcn_profile_enable(int on);
/* Restricts recording to launches whose kind k has bit k set in kind_mask (-1: all kinds) and, if d >= 0,
 * whose feature width equals d.  Lets a benchmark time one kernel inside its timed region at the cost of two
 * events per launch of that kernel only.  Stays in force until changed. */
int gcn_profile_filter(int kind_mask, int d);
/* number of records held; *dropped (may be NULL) = launches not recorded for lack of capacity */
int64_t gcn_profile_count(int64_t* dropped);
int gcn_profile_get(int64_t i, gcn_profile_rec* out);

/* ---- row pitch the sparse products gather best from -----------------------------------------------
 * Every dense argument carries its own leading dimension, and any pitch >= d works.  What the gathers of
 * gcn_spmm / gcn_spmm_t (and the layer calls built on them) run fastest from is rows that start on a 128-byte
 * line with a pitch of an ODD number of lines: the feature dimension is then worked on in slices of one line per
 * group of compute units (Sec. 4.1's per-row task, split over the feature dimension), and an odd pitch spreads the
 * lines of one slice over all cache and memory channels.  Returns that pitch in elements for rows of d elements of
 * dtype (d itself for rows of at most one line), or -1 for a bad argument.  Pure host arithmetic. */
int64_t gcn_feature_ld(int d, int dtype);

/* ---- launch geometry (a test hook) -------------------------------------------------------------
 * Kernels whose grid grows with the problem size are launched with at most 2^22 blocks in the grid's x
 * dimension and the rest in y, because a launch whose x extent reaches 2^32 threads is not refused by the
 * runtime but run with the count taken modulo 2^32.  This call lowers that bound (1 .. 2^22; 0 restores the
 * default) for the whole process, so that tests reach the two-dimensional form on small inputs.  Results do
 * not depend on it.  With a bound b, a call whose kernel would need more than 65535 b blocks returns
 * GCN_EINVAL.  Not thread-safe against launches in flight on other host threads. */
int gcn_debug_max_grid_x(int64_t blocks);

/* ---- kernel-selection overrides (a test and experiment hook) -----------------------------------
 * The library picks kernels and launch shapes by rules of its own.  Each rule can be overridden through an
 * environment variable, read ONCE per process when the library first consults any of them, or afterwards through
 * this call (name = the variable's name, e.g. "GCN_SPMM_PANEL"; value = what the variable would hold;
 * GCN_TUNE_DEFAULT restores the built-in default).  Names: GCN_SPMM_PANEL (0 never / 1 always use the column
 * sweep; default by heuristic, -1), GCN_PANEL_NARROW, GCN_PANEL_NOSYNC, GCN_PANEL_VERBOSE, GCN_SPMM_SLICES
 * (1, 2, 4, 8; 0 = by rule), GCN_SPMM_EPG, GCN_SPMM_WIDE, GCN_GEMM_DIRECT, GCN_GEMM_FAST, GCN_GEMM_TN_WIDE,
 * GCN_GEMM_BF16, GCN_GEMM_REGW, GCN_GEMM_TN_LDS (0 = that kernel family off), GCN_GEMM_TN_BLOCKS, GCN_GEMM_REGW_BLOCKS,
 * GCN_GEMM_TN_LDS_BLOCKS (workgroups of the kernels that take whole compute units), GCN_GATHER_HOST_BLOCKS, GCN_OVERLAP
 * (dense products beside sparse ones on a second stream: 0 never, 1 on large inputs, 2 wherever possible),
 * GCN_OVERLAP_CUS (compute units those dense kernels take), GCN_OVERLAP_CHUNKS (row ranges of the sparse product that
 * a dense product follows: 0, 2, 4, 8), GCN_PAUSE_ROUNDS (how long the caller's stream sleeps at a hand-over).  No override changes
 * what is computed.  Returns GCN_EINVAL for an unknown name or a value out of range.  Process-wide and not
 * thread-safe against calls in flight on other host threads. */
#define GCN_TUNE_DEFAULT (-2147483647 - 1)
int gcn_debug_set_tuning(const char* name, int value);

#ifdef __cplusplus
}
#endif
#endif /* GCN_H_ */
