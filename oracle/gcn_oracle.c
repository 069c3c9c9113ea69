/*
 * gcn_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow CPU statement of what one full-batch GCN layer computes, written from the
 * paper's definitions (Sec. 3.1 graph convolution, Sec. 4.1 feedforward, Sec. 4.2
 * backpropagation).  It exists only so that the GPU library can be checked against it and
 * timed beside it; it shares no code with the GPU path.  Every sum is accumulated in fp64
 * from the fp32 inputs, in the order the formula is written; the only "parallelism" is an
 * OpenMP loop over independent output rows.
 *
 * Conventions: dense matrices are row-major with a leading dimension in elements.
 * "Bound" outputs hold the same sum with every factor replaced by its absolute value; the
 * parity tolerance is a multiple of that bound.
 *
 * Readings of points the paper leaves open are listed next to each function.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* ------------------------------------------------------------------------------------
 * Normalised adjacency of a row block (Sec. 3.1: A^ = D^-1/2 (A + I) D^-1/2 with
 * D(i,i) = sum_j (A+I)(i,j); Sec. 4.1: processor m stores the rows A_m and needs the
 * feature rows cols(A_m) that it does not own, each one once).
 *
 * Readings: A is a 0/1 pattern (duplicate edges collapse); self-loops in the input are
 * dropped before I is added, so (A+I)(i,i) = 1; the degree is the row sum (out-degree + 1)
 * on both sides of the product; halo ids are listed in ascending global order; local column
 * numbering is "owned columns (global id - row_lo) first, then halo slot nr + rank", and the
 * entries of a row are ascending in that local numbering.
 * ---------------------------------------------------------------------------------- */
typedef struct {
  int64_t nr, nh, nnz;
  int64_t* rowptr;   /* [nr+1] */
  int32_t* col;      /* [nnz] local column ids */
  float* val;        /* [nnz] fp32: (1/sqrtf(d_i)) * (1/sqrtf(d_j)), each op rounded to fp32 */
  double* val64;     /* [nnz] fp64: 1/sqrt(d_i d_j) */
  int32_t* deg;      /* [nr] = entries in row i = row sum of A+I */
  int32_t* halo_gid; /* [nh] ascending global ids of non-owned columns */
  int64_t* colptr;   /* [nr+nh+1] */
  int32_t* rowidx;   /* [nnz] ascending inside each column */
  float* val_t;      /* [nnz] */
} orc_graph;

static int cmp_u64(const void* a, const void* b) {
  uint64_t x = *(const uint64_t*)a, y = *(const uint64_t*)b;
  return (x > y) - (x < y);
}

void orc_graph_free(orc_graph* g) {
  if (!g) return;
  free(g->rowptr); free(g->col); free(g->val); free(g->val64); free(g->deg);
  free(g->halo_gid); free(g->colptr); free(g->rowidx); free(g->val_t);
  memset(g, 0, sizeof(*g));
}

/* returns 0, or -1 for an id outside [0, n_global) / a block that is not the whole graph
 * without global degrees. Edges whose source row is not owned are ignored. */
int orc_graph_build(const int32_t* src, const int32_t* dst, int64_t n_edges, int64_t n_global,
                    int64_t row_lo, int64_t row_hi, const int32_t* deg_global, orc_graph* g) {
  memset(g, 0, sizeof(*g));
  if (row_lo < 0 || row_hi < row_lo || row_hi > n_global) return -1;
  int whole = (row_lo == 0 && row_hi == n_global);
  if (!whole && !deg_global) return -1;
  int64_t nr = row_hi - row_lo;
  for (int64_t e = 0; e < n_edges; ++e)
    if (src[e] < 0 || src[e] >= n_global || dst[e] < 0 || dst[e] >= n_global) return -1;

  /* halo list: non-owned global ids that occur as a column of an owned row */
  unsigned char* needed = (unsigned char*)calloc((size_t)n_global + 1, 1);
  for (int64_t e = 0; e < n_edges; ++e)
    if (src[e] >= row_lo && src[e] < row_hi && (dst[e] < row_lo || dst[e] >= row_hi)) needed[dst[e]] = 1;
  int64_t nh = 0;
  for (int64_t j = 0; j < n_global; ++j) nh += needed[j];
  int32_t* halo = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nh + 1));
  int32_t* slot = (int32_t*)malloc(sizeof(int32_t) * (size_t)(n_global + 1));
  nh = 0;
  for (int64_t j = 0; j < n_global; ++j) {
    slot[j] = -1;
    if (needed[j]) { slot[j] = (int32_t)nh; halo[nh++] = (int32_t)j; }
  }
  free(needed);

  /* (row, local col) pairs: every off-diagonal owned-row edge, plus the diagonal of I */
  uint64_t* key = (uint64_t*)malloc(sizeof(uint64_t) * (size_t)(n_edges + nr + 1));
  int64_t m = 0;
  for (int64_t e = 0; e < n_edges; ++e) {
    int64_t s = src[e], t = dst[e];
    if (s < row_lo || s >= row_hi || s == t) continue;
    int64_t lc = (t >= row_lo && t < row_hi) ? t - row_lo : nr + slot[t];
    key[m++] = ((uint64_t)(s - row_lo) << 32) | (uint64_t)lc;
  }
  for (int64_t i = 0; i < nr; ++i) key[m++] = ((uint64_t)i << 32) | (uint64_t)i;
  qsort(key, (size_t)m, sizeof(uint64_t), cmp_u64);
  int64_t nnz = 0;
  for (int64_t k = 0; k < m; ++k)
    if (k == 0 || key[k] != key[k - 1]) key[nnz++] = key[k];

  g->nr = nr; g->nh = nh; g->nnz = nnz;
  g->rowptr = (int64_t*)calloc((size_t)nr + 1, sizeof(int64_t));
  g->col = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz + 1));
  g->val = (float*)malloc(sizeof(float) * (size_t)(nnz + 1));
  g->val64 = (double*)malloc(sizeof(double) * (size_t)(nnz + 1));
  g->deg = (int32_t*)calloc((size_t)nr + 1, sizeof(int32_t));
  g->halo_gid = halo;
  for (int64_t k = 0; k < nnz; ++k) {
    int64_t i = (int64_t)(key[k] >> 32);
    g->col[k] = (int32_t)(key[k] & 0xffffffffu);
    g->rowptr[i + 1]++;
    g->deg[i]++;
  }
  for (int64_t i = 0; i < nr; ++i) g->rowptr[i + 1] += g->rowptr[i];
  free(key);

  /* values.  D(i,i) is the row sum of A + I (Sec. 3.1).  A row block holds its rows whole (Sec. 4.1), so for an
   * owned vertex that sum is the entry count of its row, counted above; only a halo vertex, whose row lives on
   * another processor, takes its degree from deg_global. */
  for (int64_t i = 0; i < nr; ++i) {
    int64_t di = g->deg[i];
    for (int64_t k = g->rowptr[i]; k < g->rowptr[i + 1]; ++k) {
      int64_t c = g->col[k];
      int64_t dj = c < nr ? g->deg[c] : deg_global[halo[c - nr]];
      float inv_i = 1.0f / sqrtf((float)di);
      float inv_j = 1.0f / sqrtf((float)dj);
      g->val[k] = inv_i * inv_j;
      g->val64[k] = 1.0 / sqrt((double)di * (double)dj);
    }
  }
  free(slot);

  /* transpose (column-major copy): for a directed graph backpropagation uses A^T (Sec. 3.1) */
  int64_t nc = nr + nh;
  g->colptr = (int64_t*)calloc((size_t)nc + 1, sizeof(int64_t));
  g->rowidx = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz + 1));
  g->val_t = (float*)malloc(sizeof(float) * (size_t)(nnz + 1));
  for (int64_t k = 0; k < nnz; ++k) g->colptr[g->col[k] + 1]++;
  for (int64_t c = 0; c < nc; ++c) g->colptr[c + 1] += g->colptr[c];
  int64_t* fill = (int64_t*)malloc(sizeof(int64_t) * (size_t)(nc + 1));
  memcpy(fill, g->colptr, sizeof(int64_t) * (size_t)nc);
  for (int64_t i = 0; i < nr; ++i)
    for (int64_t k = g->rowptr[i]; k < g->rowptr[i + 1]; ++k) {
      int64_t p = fill[g->col[k]]++;
      g->rowidx[p] = (int32_t)i;
      g->val_t[p] = g->val[k];
    }
  free(fill);
  return 0;
}

/* ------------------------------------------------------------------------------------
 * Y = A X for a sparse A in compressed-row form (Sec. 4.1, the sum inside the per-row
 * task: sum over j in cols(A(i,:)) of A(i,j) X(j,:)).   Y, B are [n_rows x d] fp64.
 * The same routine serves A^T when handed the column-major arrays.
 * If rows != NULL only the listed rows are computed (output row r <- matrix row rows[r]).
 * ---------------------------------------------------------------------------------- */
void orc_spmm(const int64_t* ptr, const int32_t* idx, const float* val, int64_t n_rows,
              const int64_t* rows, const float* X, int64_t ldx, int64_t d, double* Y, double* B) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t r = 0; r < n_rows; ++r) {
    int64_t i = rows ? rows[r] : r;
    double* y = Y + r * d;
    double* b = B ? B + r * d : NULL;
    for (int64_t c = 0; c < d; ++c) { y[c] = 0.0; if (b) b[c] = 0.0; }
    for (int64_t k = ptr[i]; k < ptr[i + 1]; ++k) {
      double a = (double)val[k];
      const float* x = X + (int64_t)idx[k] * ldx;
      for (int64_t c = 0; c < d; ++c) {
        y[c] += a * (double)x[c];
        if (b) b[c] += fabs(a) * fabs((double)x[c]);
      }
    }
  }
}

/* same with fp64 right-hand side (used inside the layer formulas, where the product of
 * three matrices is accumulated without rounding the intermediate to fp32) */
static void spmm_dd(const int64_t* ptr, const int32_t* idx, const float* val, int64_t n_rows,
                    const double* X, int64_t d, double* Y, int take_abs) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < n_rows; ++i) {
    double* y = Y + i * d;
    for (int64_t c = 0; c < d; ++c) y[c] = 0.0;
    for (int64_t k = ptr[i]; k < ptr[i + 1]; ++k) {
      double a = take_abs ? fabs((double)val[k]) : (double)val[k];
      const double* x = X + (int64_t)idx[k] * d;
      for (int64_t c = 0; c < d; ++c) y[c] += a * x[c];
    }
  }
}

/* ------------------------------------------------------------------------------------
 * Dense products, the textbook triple loops.  op selects which operand is transposed:
 *   0: C[M x N] = A[M x K]   B[K x N]
 *   1: C[M x N] = A[M x K]   B[N x K]^T
 *   2: C[M x N] = A[K x M]^T B[K x N]
 * ---------------------------------------------------------------------------------- */
void orc_gemm(int op, int64_t M, int64_t N, int64_t K, const float* A, int64_t lda,
              const float* Bm, int64_t ldb, double* C, double* Bnd) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = 0; j < N; ++j) {
      double s = 0.0, t = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double a = (op == 2) ? (double)A[k * lda + i] : (double)A[i * lda + k];
        double b = (op == 1) ? (double)Bm[j * ldb + k] : (double)Bm[k * ldb + j];
        s += a * b;
        t += fabs(a) * fabs(b);
      }
      C[i * N + j] = s;
      if (Bnd) Bnd[i * N + j] = t;
    }
}

/* The same three products for operands that are already fp64 (a product whose factor is itself
 * an fp64 result, e.g. S = T W^T with T = A G in Sec. 4.2): C only, no bound. */
void orc_gemm_dd(int op, int64_t M, int64_t N, int64_t K, const double* A, int64_t lda,
                 const double* Bm, int64_t ldb, double* C) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < M; ++i)
    for (int64_t j = 0; j < N; ++j) {
      double s = 0.0;
      for (int64_t k = 0; k < K; ++k) {
        double a = (op == 2) ? A[k * lda + i] : A[i * lda + k];
        double b = (op == 1) ? Bm[j * ldb + k] : Bm[k * ldb + j];
        s += a * b;
      }
      C[i * N + j] = s;
    }
}

/* ------------------------------------------------------------------------------------
 * Feedforward of one layer on a row block (Sec. 3.1 first equation; Sec. 4.1 per-row task
 * and block form):  Z(i,:) = ( sum_j A(i,j) H(j,:) ) W  (+ bias),  Hout = act(Z).
 * H holds the owned rows followed by the halo rows, [nc x d_in].
 * Outputs (fp64): AH [nr x d_in], Z, Hout, Bz [nr x d_out] (bound of Z).
 * bias is not part of the paper's layer; it is an optional extra (may be NULL).
 * act: 0 identity, 1 ReLU.
 * ---------------------------------------------------------------------------------- */
void orc_layer_fwd(const int64_t* rowptr, const int32_t* col, const float* val, int64_t nr, int64_t nc,
                   const float* H, int64_t ldh, const float* W, const float* bias, int64_t d_in,
                   int64_t d_out, int act, double* AH, double* Z, double* Hout, double* Bz) {
  double* Hd = (double*)malloc(sizeof(double) * (size_t)(nc * d_in + 1));
  double* Ha = (double*)malloc(sizeof(double) * (size_t)(nc * d_in + 1));
  double* AHa = (double*)malloc(sizeof(double) * (size_t)(nr * d_in + 1));
  for (int64_t j = 0; j < nc; ++j)
    for (int64_t k = 0; k < d_in; ++k) {
      Hd[j * d_in + k] = (double)H[j * ldh + k];
      Ha[j * d_in + k] = fabs((double)H[j * ldh + k]);
    }
  spmm_dd(rowptr, col, val, nr, Hd, d_in, AH, 0);
  spmm_dd(rowptr, col, val, nr, Ha, d_in, AHa, 1);
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < nr; ++i)
    for (int64_t c = 0; c < d_out; ++c) {
      double s = 0.0, t = 0.0;
      for (int64_t k = 0; k < d_in; ++k) {
        s += AH[i * d_in + k] * (double)W[k * d_out + c];
        t += AHa[i * d_in + k] * fabs((double)W[k * d_out + c]);
      }
      if (bias) { s += (double)bias[c]; t += fabs((double)bias[c]); }
      Z[i * d_out + c] = s;
      Hout[i * d_out + c] = (act == 1 && !(s > 0.0)) ? 0.0 : s;
      Bz[i * d_out + c] = t;
    }
  free(Hd); free(Ha); free(AHa);
}

/* ------------------------------------------------------------------------------------
 * Backpropagation through one layer on a row block (Sec. 3.1 second and third equations,
 * Sec. 4.2).  G [nr x d_out] is the gradient w.r.t. Z of this layer (already multiplied by
 * the activation derivative).  With Z = A H W:
 *   dW(k,c)  = sum_i sum_j A(i,j) H(j,k) G(i,c)                (= (A H)^T G)
 *   S(j,k)   = sum_i sum_c A(i,j) G(i,c) W(k,c)                (= A^T G W^T; A^T = A when symmetric)
 *   dH(j,k)  = S(j,k) * [Zprev(j,k) > 0]  for owned rows j < nr when Zprev is given
 *              (ReLU derivative taken as 1 for z > 0, else 0);
 *              halo rows j >= nr stay unmasked: they are partial sums owed to their owner.
 *   dbias(c) = sum_i G(i,c)                                     (extra, not in the paper)
 * Outputs fp64 with bounds: dW,BdW [d_in x d_out]; dH,BdH [nc x d_in]; dbias,Bdb [d_out].
 * colptr/rowidx/val_t is the column-major copy of the block.
 * ---------------------------------------------------------------------------------- */
void orc_layer_bwd(const int64_t* rowptr, const int32_t* col, const float* val,
                   const int64_t* colptr, const int32_t* rowidx, const float* val_t,
                   int64_t nr, int64_t nc, const float* H, int64_t ldh, const float* W,
                   const float* G, int64_t ldg, const float* Zprev, int64_t ldz,
                   int64_t d_in, int64_t d_out,
                   double* dW, double* BdW, double* dH, double* BdH, double* dbias, double* Bdb) {
  /* dW */
  double* Hd = (double*)malloc(sizeof(double) * (size_t)(nc * d_in + 1));
  double* Ha = (double*)malloc(sizeof(double) * (size_t)(nc * d_in + 1));
  double* AH = (double*)malloc(sizeof(double) * (size_t)(nr * d_in + 1));
  double* AHa = (double*)malloc(sizeof(double) * (size_t)(nr * d_in + 1));
  for (int64_t j = 0; j < nc; ++j)
    for (int64_t k = 0; k < d_in; ++k) {
      Hd[j * d_in + k] = (double)H[j * ldh + k];
      Ha[j * d_in + k] = fabs((double)H[j * ldh + k]);
    }
  spmm_dd(rowptr, col, val, nr, Hd, d_in, AH, 0);
  spmm_dd(rowptr, col, val, nr, Ha, d_in, AHa, 1);
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < d_in; ++k)
    for (int64_t c = 0; c < d_out; ++c) {
      double s = 0.0, t = 0.0;
      for (int64_t i = 0; i < nr; ++i) {
        s += AH[i * d_in + k] * (double)G[i * ldg + c];
        t += AHa[i * d_in + k] * fabs((double)G[i * ldg + c]);
      }
      dW[k * d_out + c] = s;
      BdW[k * d_out + c] = t;
    }
  free(Hd); free(Ha); free(AH); free(AHa);

  if (dbias)
    for (int64_t c = 0; c < d_out; ++c) {
      double s = 0.0, t = 0.0;
      for (int64_t i = 0; i < nr; ++i) { s += (double)G[i * ldg + c]; t += fabs((double)G[i * ldg + c]); }
      dbias[c] = s; Bdb[c] = t;
    }

  if (dH) {
    double* Gd = (double*)malloc(sizeof(double) * (size_t)(nr * d_out + 1));
    double* Ga = (double*)malloc(sizeof(double) * (size_t)(nr * d_out + 1));
    double* T = (double*)malloc(sizeof(double) * (size_t)(nc * d_out + 1));
    double* Ta = (double*)malloc(sizeof(double) * (size_t)(nc * d_out + 1));
    for (int64_t i = 0; i < nr; ++i)
      for (int64_t c = 0; c < d_out; ++c) {
        Gd[i * d_out + c] = (double)G[i * ldg + c];
        Ga[i * d_out + c] = fabs((double)G[i * ldg + c]);
      }
    spmm_dd(colptr, rowidx, val_t, nc, Gd, d_out, T, 0);
    spmm_dd(colptr, rowidx, val_t, nc, Ga, d_out, Ta, 1);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < nc; ++j)
      for (int64_t k = 0; k < d_in; ++k) {
        double s = 0.0, t = 0.0;
        for (int64_t c = 0; c < d_out; ++c) {
          s += T[j * d_out + c] * (double)W[k * d_out + c];
          t += Ta[j * d_out + c] * fabs((double)W[k * d_out + c]);
        }
        if (Zprev && j < nr && !(Zprev[j * ldz + k] > 0.0f)) s = 0.0;
        dH[j * d_in + k] = s;
        BdH[j * d_in + k] = t;
      }
    free(Gd); free(Ga); free(T); free(Ta);
  }
}

/* ------------------------------------------------------------------------------------
 * Output-layer gradient (Sec. 3.1: G^L = grad_{H^L} J (.) act'(Z^L); Sec. 4.2 leaves J open).
 * Reading: the last layer has identity activation and J is the softmax cross-entropy
 *   J = -scale * sum_i log softmax(Z_i)[y_i],   G = scale * (softmax(Z) - onehot(y)),
 * rows with y_i < 0 carry no label (no loss, zero gradient).
 * Outputs fp64: *loss, G [nr x C]; *labs = scale * sum_i |log-probability| (bound of the loss sum).
 * ---------------------------------------------------------------------------------- */
void orc_softmax_xent(const float* Z, int64_t ldz, int64_t nr, int64_t C, const int32_t* y,
                      double scale, double* loss, double* labs, double* G) {
  double total = 0.0, tabs = 0.0;
  for (int64_t i = 0; i < nr; ++i) {
    const float* z = Z + i * ldz;
    double* g = G + i * C;
    if (y[i] < 0) { for (int64_t c = 0; c < C; ++c) g[c] = 0.0; continue; }
    double mx = (double)z[0];
    for (int64_t c = 1; c < C; ++c) if ((double)z[c] > mx) mx = (double)z[c];
    double se = 0.0;
    for (int64_t c = 0; c < C; ++c) se += exp((double)z[c] - mx);
    double logp = (double)z[y[i]] - mx - log(se);
    total += -logp;
    tabs += fabs(logp);
    for (int64_t c = 0; c < C; ++c) {
      double p = exp((double)z[c] - mx) / se;
      g[c] = scale * (p - (c == y[i] ? 1.0 : 0.0));
    }
  }
  *loss = scale * total;
  *labs = fabs(scale) * tabs;
}

/* ------------------------------------------------------------------------------------
 * Row selection by an index list (Sec. 4.1: the rows of H named by the non-zero diagonal
 * entries of the selector matrix are copied, not multiplied): recv[s,:] = table[idx[s],:].
 * Returns -1 if an index is outside [0, n_table_rows).
 * ---------------------------------------------------------------------------------- */
int orc_gather(const float* table, int64_t ld, int64_t n_table_rows, int64_t d,
               const int32_t* idx, int64_t n_idx, float* recv, int64_t ldr) {
  for (int64_t s = 0; s < n_idx; ++s) {
    if (idx[s] < 0 || idx[s] >= n_table_rows) return -1;
    for (int64_t c = 0; c < d; ++c) recv[s * ldr + c] = table[(int64_t)idx[s] * ld + c];
  }
  return 0;
}
