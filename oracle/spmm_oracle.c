/*
 * CPU oracle for the brick SpMM hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C.  It shares no code, header, table or
 * helper with the HIP library; only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it.  The product path never does.
 *
 * What each function follows in the paper (arxiv 2504.06443):
 *   oracle_spmm_f64        Section 3.1: C[MxN] = A[MxK] . B[KxN], B and C
 *                          row-major with leading dimension N (Algorithm 1
 *                          indexes B as B[b_row*N + j]).  Zero filling only
 *                          adds exact zeros, so the method's result is the
 *                          plain definition up to summation order; the oracle
 *                          is that definition, accumulated in fp64.
 *   oracle_bricks_*        Section 3.2: per 16-row panel, active columns are
 *                          packed to the left, grouped four at a time into
 *                          16x4 bricks; each brick carries a 64-bit pattern
 *                          (bit i <=> i-th element of the brick, elements
 *                          numbered row-major: i = 4*row + col) and its
 *                          non-zeros appended in row-major order.
 *   oracle_bricks_to_csr   the inverse walk of the same description.
 *   oracle_synergy         Section 4 (alpha, OI_shmem = 512*alpha, Eq. 4) and
 *                          Section 6.4 / Table 1 (Low / Medium / High ranges).
 *
 * Readings taken where the paper is silent (listed in full in the design
 * notes): active columns keep ascending original order; a panel's last brick
 * is padded with column id 0xFFFFFFFF; alpha = nnz / (64 * bricks); class
 * boundaries are the half-open ranges of Table 1.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define PANEL 16
#define BRICK_K 4
#define PAD_COL 0xFFFFFFFFu

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* C[i][j] = sum_e (double)vals[e] * (double)B[colind[e]][j], CSR order.
 * S (optional) = sum_e |vals[e] * B[colind[e]][j]|, the error normaliser. */
void oracle_spmm_f64(int64_t M, int64_t N, const int32_t *rowptr, const int32_t *colind,
                     const float *vals, const float *B, double *C, double *S) {
#pragma omp parallel for schedule(dynamic, 64)
  for (int64_t i = 0; i < M; ++i) {
    double *c = C + i * N;
    double *s = S ? S + i * N : NULL;
    for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
    if (s)
      for (int64_t j = 0; j < N; ++j) s[j] = 0.0;
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
      const double a = (double)vals[e];
      const float *b = B + (int64_t)colind[e] * N;
      for (int64_t j = 0; j < N; ++j) {
        const double p = a * (double)b[j];
        c[j] += p;
        if (s) s[j] += fabs(p);
      }
    }
  }
}

/* Same product for a chosen subset of rows (sampled checks at full size). */
void oracle_spmm_rows_f64(int64_t nrows, const int64_t *rows, int64_t N, const int32_t *rowptr,
                          const int32_t *colind, const float *vals, const float *B, double *C,
                          double *S) {
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t t = 0; t < nrows; ++t) {
    const int64_t i = rows[t];
    double *c = C + t * N;
    double *s = S + t * N;
    for (int64_t j = 0; j < N; ++j) c[j] = s[j] = 0.0;
    for (int64_t e = rowptr[i]; e < rowptr[i + 1]; ++e) {
      const double a = (double)vals[e];
      const float *b = B + (int64_t)colind[e] * N;
      for (int64_t j = 0; j < N; ++j) {
        const double p = a * (double)b[j];
        c[j] += p;
        s[j] += fabs(p);
      }
    }
  }
}

/* ---------------------------------------------------------------- bricks */

typedef struct {
  int32_t col;
  int32_t row; /* row inside the panel, 0..15 */
  float val;
} entry_t;

static int cmp_col_row(const void *a, const void *b) {
  const entry_t *x = (const entry_t *)a, *y = (const entry_t *)b;
  if (x->col != y->col) return x->col < y->col ? -1 : 1;
  return (x->row > y->row) - (x->row < y->row);
}

typedef struct {
  int32_t bit;
  float val;
} bitval_t;

static int cmp_bit(const void *a, const void *b) {
  const bitval_t *x = (const bitval_t *)a, *y = (const bitval_t *)b;
  return (x->bit > y->bit) - (x->bit < y->bit);
}

static int64_t panel_begin(int64_t M, const int32_t *rowptr, int64_t p) {
  int64_t r = p * PANEL;
  return rowptr[r < M ? r : M];
}

/* Gather the panel's stored entries, sorted by (column, row). Returns count. */
static int64_t collect_panel(int64_t M, const int32_t *rowptr, const int32_t *colind,
                             const float *vals, int64_t p, entry_t **out) {
  const int64_t r0 = p * PANEL, r1 = (r0 + PANEL < M) ? r0 + PANEL : M;
  const int64_t n = rowptr[r1] - rowptr[r0];
  entry_t *e = (entry_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(entry_t));
  int64_t k = 0;
  for (int64_t r = r0; r < r1; ++r)
    for (int64_t x = rowptr[r]; x < rowptr[r + 1]; ++x) {
      e[k].col = colind[x];
      e[k].row = (int32_t)(r - r0);
      e[k].val = vals ? vals[x] : 0.0f;
      ++k;
    }
  qsort(e, (size_t)n, sizeof(entry_t), cmp_col_row);
  *out = e;
  return n;
}

/* Number of active (distinct) columns of every panel. ncols has P entries. */
void oracle_panel_active_cols(int64_t M, const int32_t *rowptr, const int32_t *colind,
                              int64_t *ncols) {
  const int64_t P = (M + PANEL - 1) / PANEL;
#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t p = 0; p < P; ++p) {
    entry_t *e;
    const int64_t n = collect_panel(M, rowptr, colind, NULL, p, &e);
    int64_t d = 0;
    for (int64_t k = 0; k < n; ++k)
      if (k == 0 || e[k].col != e[k - 1].col) ++d;
    ncols[p] = d;
    free(e);
  }
}

/* Build the brick format.
 *   in : CSR; ncols[P] from oracle_panel_active_cols
 *   out: panel_ptr[P+1]   first brick of each panel (exclusive scan of ceil(ncols/4))
 *        brick_cols[4*nb] original column id of each brick column, pad 0xFFFFFFFF
 *        brick_mask[nb]   bit 4*r+c set <=> element (r,c) of the brick is stored
 *        brick_valptr[nb+1] start of each brick's values in packed[]
 *        packed[nnz]      values, bricks in order, row-major inside a brick
 * The caller sizes the outputs with nb = sum ceil(ncols/4). */
void oracle_bricks_build(int64_t M, const int32_t *rowptr, const int32_t *colind, const float *vals,
                         const int64_t *ncols, uint32_t *panel_ptr, uint32_t *brick_cols,
                         uint64_t *brick_mask, uint32_t *brick_valptr, float *packed) {
  const int64_t P = (M + PANEL - 1) / PANEL;
  int64_t nb = 0;
  for (int64_t p = 0; p < P; ++p) {
    panel_ptr[p] = (uint32_t)nb;
    nb += (ncols[p] + BRICK_K - 1) / BRICK_K;
  }
  panel_ptr[P] = (uint32_t)nb;
  brick_valptr[nb] = (uint32_t)rowptr[M];

#pragma omp parallel for schedule(dynamic, 16)
  for (int64_t p = 0; p < P; ++p) {
    entry_t *e;
    const int64_t n = collect_panel(M, rowptr, colind, vals, p, &e);
    const int64_t b0 = panel_ptr[p], nbp = panel_ptr[p + 1] - b0;
    for (int64_t b = 0; b < nbp; ++b) {
      brick_mask[b0 + b] = 0;
      for (int c = 0; c < BRICK_K; ++c) brick_cols[4 * (b0 + b) + c] = PAD_COL;
    }
    /* rank[k] = position of entry k's column in the panel's ascending active list */
    int64_t *rank = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
    for (int64_t k = 0; k < n; ++k)
      rank[k] = (k == 0) ? 0 : rank[k - 1] + (e[k].col != e[k - 1].col);
    /* entries of panels before p fill packed[0 .. panel_begin) */
    int64_t out = panel_begin(M, rowptr, p);
    bitval_t *bv = (bitval_t *)malloc(64 * sizeof(bitval_t));
    int64_t k = 0;
    for (int64_t b = 0; b < nbp; ++b) { /* brick b holds active columns 4b .. 4b+3 */
      int64_t nbv = 0;
      for (; k < n && rank[k] / BRICK_K == b; ++k) {
        const int c = (int)(rank[k] % BRICK_K);
        const int bit = 4 * e[k].row + c;
        brick_cols[4 * (b0 + b) + c] = (uint32_t)e[k].col;
        brick_mask[b0 + b] |= (uint64_t)1 << bit;
        bv[nbv].bit = bit;
        bv[nbv].val = e[k].val;
        ++nbv;
      }
      qsort(bv, (size_t)nbv, sizeof(bitval_t), cmp_bit); /* row-major inside the brick */
      brick_valptr[b0 + b] = (uint32_t)out;
      for (int64_t t = 0; t < nbv; ++t) packed[out++] = bv[t].val;
    }
    free(rank);
    free(bv);
    free(e);
  }
}

/* Inverse: decode the brick format back to CSR (rowptr[M+1], colind, vals). */
void oracle_bricks_to_csr(int64_t M, const uint32_t *panel_ptr, const uint32_t *brick_cols,
                          const uint64_t *brick_mask, const uint32_t *brick_valptr,
                          const float *packed, int32_t *rowptr, int32_t *colind, float *vals) {
  const int64_t P = (M + PANEL - 1) / PANEL;
  for (int64_t i = 0; i <= M; ++i) rowptr[i] = 0;
  for (int64_t p = 0; p < P; ++p)
    for (int64_t b = panel_ptr[p]; b < panel_ptr[p + 1]; ++b)
      for (int bit = 0; bit < 64; ++bit)
        if ((brick_mask[b] >> bit) & 1) {
          const int64_t row = p * PANEL + bit / 4;
          if (row < M) rowptr[row + 1] += 1;
        }
  for (int64_t i = 0; i < M; ++i) rowptr[i + 1] += rowptr[i];
  int32_t *fill = (int32_t *)malloc((size_t)(M + 1) * sizeof(int32_t));
  memcpy(fill, rowptr, (size_t)(M + 1) * sizeof(int32_t));
  for (int64_t p = 0; p < P; ++p)
    for (int64_t b = panel_ptr[p]; b < panel_ptr[p + 1]; ++b) {
      int64_t idx = 0;
      for (int bit = 0; bit < 64; ++bit)
        if ((brick_mask[b] >> bit) & 1) {
          const int64_t row = p * PANEL + bit / 4;
          const int c = bit % 4;
          if (row < M) {
            const int64_t dst = fill[row]++;
            colind[dst] = (int32_t)brick_cols[4 * b + c];
            vals[dst] = packed[brick_valptr[b] + idx];
          }
          ++idx;
        }
    }
  free(fill);
}

/* ---------------------------------------------------------------- synergy */

enum { SYN_LOW = 0, SYN_MEDIUM = 1, SYN_HIGH = 2 };

/* Table 1: Low [0,12.5%), Medium [12.5%,25%), High [25%,100%] of alpha =
 * nnz/(64*nb); decided in integers so the boundaries are exact. */
static int classify(int64_t nnz, int64_t nb) {
  if (nnz < 8 * nb) return SYN_LOW;
  if (nnz < 16 * nb) return SYN_MEDIUM;
  return SYN_HIGH;
}

/* Integer counts (icnt, 82 entries) and model values (fval, 10 entries).
 * icnt layout: 0 M, 1 K, 2 nnz, 3 n_panels, 4 n_nonempty_panels, 5 n_bricks,
 *   6 n_active_cols (sum over panels), 7 n_distinct_cols (whole matrix),
 *   8..10 panels_by_class, 11..13 bricks_by_class, 14..16 nnz_by_class,
 *   17..81 brick_pop_hist[0..64], and the matrix class is returned.
 * fval layout: 0 alpha_brick, 1 alpha_col, 2 beta, 3 oi_shmem, 4 bytes_min,
 *   5 bytes_noreuse, 6 oi_hbm_min, 7 oi_hbm_noreuse, 8 roof_gflops_hbm,
 *   9 roof_gflops_mfma.
 * Bytes model: A = 4 nnz + (8+16+4) nb + 4 + 4 (P+1); B rows once each (min) or
 * once per panel that uses them (noreuse); C written once. */
int oracle_synergy(int64_t M, int64_t K, int64_t N, const int32_t *rowptr, const int32_t *colind,
                   const uint32_t *panel_ptr, const uint64_t *brick_mask, const int64_t *ncols,
                   double hbm_bytes_per_s, double mfma_flops_per_s, int64_t *icnt, double *fval) {
  const int64_t P = (M + PANEL - 1) / PANEL;
  const int64_t nnz = rowptr[M];
  const int64_t nb = panel_ptr[P];
  for (int i = 0; i < 82; ++i) icnt[i] = 0;
  icnt[0] = M; icnt[1] = K; icnt[2] = nnz; icnt[3] = P; icnt[5] = nb;
  unsigned char *seen = (unsigned char *)calloc((size_t)(K > 0 ? K : 1), 1);
  for (int64_t e = 0; e < nnz; ++e) seen[colind[e]] = 1;
  for (int64_t k = 0; k < K; ++k) icnt[7] += seen[k];
  free(seen);
  for (int64_t p = 0; p < P; ++p) {
    const int64_t nbp = panel_ptr[p + 1] - panel_ptr[p];
    const int64_t nnzp = panel_begin(M, rowptr, p + 1) - panel_begin(M, rowptr, p);
    icnt[6] += ncols[p];
    if (nbp == 0) continue;
    icnt[4] += 1;
    const int c = classify(nnzp, nbp);
    icnt[8 + c] += 1;
    icnt[11 + c] += nbp;
    icnt[14 + c] += nnzp;
  }
  for (int64_t b = 0; b < nb; ++b) icnt[17 + __builtin_popcountll(brick_mask[b])] += 1;

  const double alpha = nb ? (double)nnz / (64.0 * (double)nb) : 0.0;
  const double alpha_col = icnt[6] ? (double)nnz / (16.0 * (double)icnt[6]) : 0.0;
  const double a_bytes = 4.0 * nnz + 28.0 * nb + 4.0 + 4.0 * (P + 1);
  const double bytes_min = a_bytes + 4.0 * N * (double)icnt[7] + 4.0 * N * (double)M;
  const double bytes_noreuse = a_bytes + 4.0 * N * (double)icnt[6] + 4.0 * N * (double)M;
  const double flops = 2.0 * (double)nnz * (double)N;
  fval[0] = alpha;
  fval[1] = alpha_col;
  fval[2] = 1.0;
  fval[3] = 512.0 * alpha * fval[2];
  fval[4] = bytes_min;
  fval[5] = bytes_noreuse;
  fval[6] = flops / bytes_min;
  fval[7] = flops / bytes_noreuse;
  fval[8] = fval[6] * hbm_bytes_per_s * 1e-9;
  fval[9] = alpha * mfma_flops_per_s * 1e-9;
  return nb ? classify(nnz, nb) : -1;
}
