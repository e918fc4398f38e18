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
 *   oracle_tm32_*          Section 4, Eq. 5: row panels of 32 rows, up to two
 *                          bricks per brick column sharing one B operand
 *                          (see the comment above those functions).
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

/* ------------------------------------------------- 32-row panels (Section 4, Eq. 5) */
/*
 * Row panels of TM = 32 rows hold up to TM / brick_m = 2 bricks per brick column (the
 * paper's Block keeps, per block, the brick-row id of every active brick in `rows` and the
 * start of every brick column in `colPtr`).  A B operand loaded for a brick column is reused
 * by all its active bricks: beta = active bricks per brick column (Eq. 5).
 *
 * The paper always ran TM = 16 and gives no rule for when 32 pays; Section 4 only describes
 * the two extremes (both halves share their active columns / have disjoint ones).  Reading
 * taken here: the two 16-row halves of a 32-row super-panel are packed together only where
 * their active columns nearly coincide,
 *     |cols(top) U cols(bottom)| * den < num * max(|cols(top)|, |cols(bottom)|)
 * (num/den = 6/5 by default); otherwise each half keeps its own left-packed column list and
 * the super-panel simply holds the brick columns of the top half followed by those of the
 * bottom half, one brick each, i.e. exactly the bricks of the 16-row format.
 *
 * Layout (Q = ceil(M/32) super-panels, nbc brick columns, nbr bricks):
 *   sp_ptr    u32[Q+1]    first brick column of each super-panel
 *   sp_merged u8 [Q]      1 if the halves were packed together
 *   bc_cols   u32[4 nbc]  original column ids, ascending inside a packed list, pad 0xFFFFFFFF
 *   bc_brick  u32[nbc+1]  first brick of each brick column (1 or 2 bricks each)
 *   br_row    u8 [nbr]    brick-row id: 0 = rows 0..15 of the super-panel, 1 = rows 16..31
 *   br_mask   u64[nbr]    bit 4 r + c, r = row inside the half
 *   br_valptr u32[nbr+1]  start of each brick's values
 *   vals      f32[nnz]    bricks in order, row-major inside a brick
 */
#define SUPER 32

typedef struct {
  int32_t col;
  int32_t row; /* 0..31 inside the super-panel */
  float val;
} sentry_t;

static int cmp_scol_row(const void *a, const void *b) {
  const sentry_t *x = (const sentry_t *)a, *y = (const sentry_t *)b;
  if (x->col != y->col) return x->col < y->col ? -1 : 1;
  return (x->row > y->row) - (x->row < y->row);
}

/* entries of super-panel q sorted by (column, row); returns the count */
static int64_t collect_super(int64_t M, const int32_t *rowptr, const int32_t *colind,
                             const float *vals, int64_t q, sentry_t **out) {
  const int64_t r0 = q * SUPER, r1 = (r0 + SUPER < M) ? r0 + SUPER : M;
  const int64_t n = rowptr[r1] - rowptr[r0];
  sentry_t *e = (sentry_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(sentry_t));
  int64_t k = 0;
  for (int64_t r = r0; r < r1; ++r)
    for (int64_t x = rowptr[r]; x < rowptr[r + 1]; ++x) {
      e[k].col = colind[x];
      e[k].row = (int32_t)(r - r0);
      e[k].val = vals ? vals[x] : 0.0f;
      ++k;
    }
  qsort(e, (size_t)n, sizeof(sentry_t), cmp_scol_row);
  *out = e;
  return n;
}

/* distinct columns of each half and of their union */
static void super_counts(const sentry_t *e, int64_t n, int64_t *n_top, int64_t *n_bot,
                         int64_t *n_union) {
  int64_t t = 0, b = 0, u = 0;
  for (int64_t k = 0; k < n;) {
    int has_t = 0, has_b = 0;
    int64_t x = k;
    for (; x < n && e[x].col == e[k].col; ++x) {
      if (e[x].row < PANEL) has_t = 1; else has_b = 1;
    }
    t += has_t; b += has_b; u += 1;
    k = x;
  }
  *n_top = t; *n_bot = b; *n_union = u;
}

static int super_is_merged(int64_t n_top, int64_t n_bot, int64_t n_union, int64_t num,
                           int64_t den) {
  const int64_t mx = n_top > n_bot ? n_top : n_bot;
  return n_top > 0 && n_bot > 0 && n_union * den < num * mx;
}

/* Sizes of the 32-row format: out[0] = Q, out[1] = nbc, out[2] = nbr, out[3] = merged
 * super-panels. */
void oracle_tm32_sizes(int64_t M, const int32_t *rowptr, const int32_t *colind, int64_t num,
                       int64_t den, int64_t *out) {
  const int64_t Q = (M + SUPER - 1) / SUPER;
  int64_t nbc = 0, nbr = 0, merged = 0;
  for (int64_t q = 0; q < Q; ++q) {
    sentry_t *e;
    const int64_t n = collect_super(M, rowptr, colind, NULL, q, &e);
    int64_t nt, nb, nu;
    super_counts(e, n, &nt, &nb, &nu);
    if (super_is_merged(nt, nb, nu, num, den)) {
      merged += 1;
      const int64_t bcs = (nu + BRICK_K - 1) / BRICK_K;
      nbc += bcs;
      /* a brick exists where a half has an entry in the brick column */
      int64_t rank = -1;
      int32_t prev = -1;
      unsigned char *seen = (unsigned char *)calloc((size_t)(2 * bcs > 0 ? 2 * bcs : 1), 1);
      for (int64_t k = 0; k < n; ++k) {
        if (k == 0 || e[k].col != prev) { ++rank; prev = e[k].col; }
        seen[2 * (rank / BRICK_K) + (e[k].row >= PANEL)] = 1;
      }
      for (int64_t i = 0; i < 2 * bcs; ++i) nbr += seen[i];
      free(seen);
    } else {
      const int64_t bcs = (nt + BRICK_K - 1) / BRICK_K + (nb + BRICK_K - 1) / BRICK_K;
      nbc += bcs;
      nbr += bcs;
    }
    free(e);
  }
  out[0] = Q; out[1] = nbc; out[2] = nbr; out[3] = merged;
}

void oracle_tm32_build(int64_t M, const int32_t *rowptr, const int32_t *colind, const float *vals,
                       int64_t num, int64_t den, uint32_t *sp_ptr, uint8_t *sp_merged,
                       uint32_t *bc_cols, uint32_t *bc_brick, uint8_t *br_row, uint64_t *br_mask,
                       uint32_t *br_valptr, float *packed) {
  const int64_t Q = (M + SUPER - 1) / SUPER;
  int64_t bc = 0, br = 0, out = 0;
  bitval_t *bv = (bitval_t *)malloc(64 * sizeof(bitval_t));
  for (int64_t q = 0; q < Q; ++q) {
    sp_ptr[q] = (uint32_t)bc;
    sentry_t *e;
    const int64_t n = collect_super(M, rowptr, colind, vals, q, &e);
    int64_t nt, nb, nu;
    super_counts(e, n, &nt, &nb, &nu);
    const int merged = super_is_merged(nt, nb, nu, num, den);
    sp_merged[q] = (uint8_t)merged;
    /* pass h over the column lists: merged -> one list (both halves); else top list, then bottom */
    for (int list = 0; list < (merged ? 1 : 2); ++list) {
      /* rank of every entry's column inside this list (-1: entry not in this list) */
      int64_t *rank = (int64_t *)malloc((size_t)(n > 0 ? n : 1) * sizeof(int64_t));
      int64_t r = -1;
      int32_t prev = -1;
      int have_prev = 0;
      for (int64_t k = 0; k < n; ++k) {
        const int half = e[k].row >= PANEL;
        if (!merged && half != list) { rank[k] = -1; continue; }
        if (!have_prev || e[k].col != prev) { ++r; prev = e[k].col; have_prev = 1; }
        rank[k] = r;
      }
      const int64_t ncols = r + 1;
      const int64_t bcs = (ncols + BRICK_K - 1) / BRICK_K;
      for (int64_t k = 0; k < bcs; ++k) {
        for (int c = 0; c < BRICK_K; ++c) bc_cols[4 * (bc + k) + c] = PAD_COL;
      }
      for (int64_t k = 0; k < n; ++k)
        if (rank[k] >= 0) bc_cols[4 * bc + rank[k]] = (uint32_t)e[k].col;
      for (int64_t k = 0; k < bcs; ++k) {
        bc_brick[bc + k] = (uint32_t)br;
        for (int half = 0; half < 2; ++half) {
          if (!merged && half != list) continue;
          uint64_t mask = 0;
          int64_t nbv = 0;
          for (int64_t x = 0; x < n; ++x) {
            if (rank[x] < 0 || rank[x] / BRICK_K != k || (e[x].row >= PANEL) != half) continue;
            const int bit = 4 * (e[x].row % PANEL) + (int)(rank[x] % BRICK_K);
            mask |= (uint64_t)1 << bit;
            bv[nbv].bit = bit;
            bv[nbv].val = e[x].val;
            ++nbv;
          }
          if (!mask) continue;
          qsort(bv, (size_t)nbv, sizeof(bitval_t), cmp_bit);
          br_row[br] = (uint8_t)half;
          br_mask[br] = mask;
          br_valptr[br] = (uint32_t)out;
          for (int64_t t = 0; t < nbv; ++t) packed[out++] = bv[t].val;
          ++br;
        }
      }
      bc += bcs;
      free(rank);
    }
    free(e);
  }
  sp_ptr[Q] = (uint32_t)bc;
  bc_brick[bc] = (uint32_t)br;
  br_valptr[br] = (uint32_t)out;
  free(bv);
}

/* Inverse of the 32-row format: back to CSR. */
void oracle_tm32_to_csr(int64_t M, const uint32_t *sp_ptr, const uint32_t *bc_cols,
                        const uint32_t *bc_brick, const uint8_t *br_row, const uint64_t *br_mask,
                        const uint32_t *br_valptr, const float *packed, int32_t *rowptr,
                        int32_t *colind, float *vals) {
  const int64_t Q = (M + SUPER - 1) / SUPER;
  for (int64_t i = 0; i <= M; ++i) rowptr[i] = 0;
  for (int pass = 0; pass < 2; ++pass) {
    int32_t *fill = NULL;
    if (pass == 1) {
      for (int64_t i = 0; i < M; ++i) rowptr[i + 1] += rowptr[i];
      fill = (int32_t *)malloc((size_t)(M + 1) * sizeof(int32_t));
      memcpy(fill, rowptr, (size_t)(M + 1) * sizeof(int32_t));
    }
    /* entries of a row must come out in ascending column order: inside a super-panel walk
     * the brick columns in order; in an unmerged super-panel a row only occurs in one list */
    for (int64_t q = 0; q < Q; ++q)
      for (int64_t k = sp_ptr[q]; k < sp_ptr[q + 1]; ++k)
        for (int64_t b = bc_brick[k]; b < bc_brick[k + 1]; ++b) {
          int64_t idx = 0;
          for (int bit = 0; bit < 64; ++bit)
            if ((br_mask[b] >> bit) & 1) {
              const int64_t row = q * SUPER + PANEL * br_row[b] + bit / 4;
              if (pass == 0) {
                if (row < M) rowptr[row + 1] += 1;
              } else if (row < M) {
                const int64_t dst = fill[row]++;
                colind[dst] = (int32_t)bc_cols[4 * k + bit % 4];
                vals[dst] = packed[br_valptr[b] + idx];
              }
              ++idx;
            }
        }
    if (pass == 1) free(fill);
  }
}
