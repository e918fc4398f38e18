/*
 * Brick SpMM for MI355X (gfx950): C = A . B with A sparse (CSR in, 16-row panels
 * of column-compacted 16x4 bricks inside), B and C dense row-major fp32.
 *
 * C ABI.  Every function returns an spmm_status (0 = success, negative = error),
 * never throws, aborts or prints; spmm_last_error() gives a thread-local message.
 * "dev" pointers are HIP device pointers on the current device, "host" pointers
 * are ordinary host memory.  The library never takes ownership of caller memory.
 *
 * Paper: arxiv 2504.06443.  Section 3.1 defines the operation and the layouts,
 * Section 3.2 the panel/brick format, Section 3.3 / Algorithm 1 the kernel,
 * Section 4 the operational-intensity model, Section 5 the load balancer,
 * Section 6.4 / Table 1 the synergy classes.
 */
#ifndef SPMM_H_
#define SPMM_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spmm_plan spmm_plan_t; /* opaque; owns every device/host buffer it creates */

enum spmm_status {
  SPMM_OK = 0,
  SPMM_EINVAL = -1,  /* null pointer, negative size, bad enum value                          */
  SPMM_EFORMAT = -2, /* CSR not valid: rowptr not monotone / wrong ends, column out of range,
                        columns of a row not strictly ascending                              */
  SPMM_ENOMEM = -3,  /* host or device allocation failed                                     */
  SPMM_EHIP = -4,    /* a HIP call failed; text in spmm_last_error()                         */
  SPMM_ELIMIT = -5   /* nnz >= 2^31, 4*bricks >= 2^32 or M >= 2^31                           */
};

enum spmm_route {
  SPMM_ROUTE_AUTO = 0,  /* the measured policy for MI355X: the MFMA brick kernel for every
                           panel (it loads each B row of a panel once, CSR loads it once per
                           entry; over the benchmark's sweep of brick fill 0.05..0.8 and
                           N = 16..512 the CSR kernel is nowhere ahead by more than a few
                           percent)                                                          */
  SPMM_ROUTE_MFMA = 1,  /* every panel through the MFMA brick kernel (an empty panel is a work
                           item without bricks that stores zeros)                            */
  SPMM_ROUTE_VALU = 2,  /* every panel through the vector-ALU CSR kernel                      */
  SPMM_ROUTE_CLASS = 3  /* the paper's rule per panel: Low synergy (Table 1) -> CSR kernel,
                           Medium/High -> MFMA brick kernel                                   */
};

enum spmm_class { SPMM_NONE = -1, SPMM_LOW = 0, SPMM_MEDIUM = 1, SPMM_HIGH = 2 };

/* ---------------------------------------------------------------------------
 * spmm_plan -- CSR -> brick format (Section 3.2), built by HIP kernels.
 *
 *   M, K     rows / columns of A (>= 0, M < 2^31)
 *   nnz      stored entries (0 <= nnz < 2^31); must equal rowptr[M]
 *   rowptr   dev int32[M+1], rowptr[0] = 0, non-decreasing
 *   colind   dev int32[nnz], inside each row strictly ascending, 0 <= col < K
 *   vals     dev float[nnz]; explicitly stored zeros are kept as entries
 *   stream   hipStream_t (NULL = default stream); all work is enqueued there
 *   out      receives the plan; destroy with spmm_plan_destroy
 *
 * The CSR arrays are only read during the call (the plan keeps its own copies of
 * what it needs later) and may be freed after it returns.  The call synchronises
 * `stream` several times (it reads back sizes to allocate).  The input is
 * validated on the device first; an invalid CSR gives SPMM_EFORMAT and no plan.
 *
 * Format (panel p = rows 16p..16p+15; P = ceil(M/16) panels; nb bricks):
 *   panel_ptr    u32[P+1]  first brick of each panel
 *   brick_cols   u32[4 nb] original column of each brick column; a panel's active
 *                          columns in ascending order, four per brick, the last
 *                          brick padded with 0xFFFFFFFF
 *   brick_mask   u64[nb]   bit 4*r+c set <=> element (row r, brick column c) stored
 *   brick_valptr u32[nb+1] start of each brick's values
 *   vals         f32[nnz]  values of each brick in ascending bit order (row-major)
 */
int spmm_plan(int64_t M, int64_t K, int64_t nnz, const int32_t *rowptr, const int32_t *colind,
              const float *vals, void *stream, spmm_plan_t **out);

/* ---------------------------------------------------------------------------
 * spmm_plan_update_values -- new values for the same sparsity pattern (the use
 * cases of Section 6, "Pre-processing Overheads": many products with one pattern,
 * e.g. a matrix re-assembled every time step).  One gather/scatter kernel instead
 * of a new plan.
 *
 *   vals    dev float[nnz], in the order of the colind array the plan was built
 *           from; read by a kernel enqueued on `stream`, so it must stay valid
 *           until that kernel has run
 *
 * Replaces the packed brick values and the plan's CSR copy; pattern, masks,
 * offsets, synergy counts and work lists are unchanged (an entry whose new value
 * is 0 stays a stored entry).  Enqueues only; allocates nothing.  Must not run
 * concurrently with spmm_exec on the same plan.
 */
int spmm_plan_update_values(spmm_plan_t *plan, const float *vals, void *stream);

/* ---------------------------------------------------------------------------
 * spmm_exec -- C = A . B (Section 3.1; Algorithm 1 re-designed for MFMA).
 *
 *   B   dev float[K*N], row-major, leading dimension N; must be finite (zero
 *       filling multiplies every B row of an active column by explicit zeros)
 *   N   columns of B and C, >= 0
 *   C   dev float[M*N], row-major, leading dimension N; fully overwritten (rows
 *       of A without entries become zero); must not overlap B
 *   stream  hipStream_t; the call only enqueues kernels and returns
 *
 * By default fp32 multiply and fp32 accumulate, no reduced-precision rounding of inputs
 * (spmm_plan_set_precision offers split-bf16 arithmetic with its own stated bounds).  The
 * result is deterministic for a given plan, N and device.  The first call for a
 * new N builds and caches that N's work list (a host computation plus one small
 * upload, which synchronises the stream once); later calls allocate nothing.
 * A plan must not be used by two spmm_exec calls at the same time.  The device the plan
 * was made on must be the current device (SPMM_EINVAL otherwise).
 */
int spmm_exec(spmm_plan_t *plan, const float *B, int64_t N, float *C, void *stream);

/* ---------------------------------------------------------------------------
 * spmm_exec_noalloc -- the same product for callers that cannot allocate device
 * memory: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Arguments, result and kernels are those of spmm_exec (bit-identical C),
 * but the call makes no hipMalloc / hipFree, not even on its first use for a new N:
 * the work list of the MFMA kernel and the partial tiles of split panels live in one
 * static device array of 32 MiB per GPU (held until the process ends) instead of
 * plan-owned allocations.
 *
 *   - Work list plus partial tiles (16 x N floats per part of a split panel) must fit
 *     the 32 MiB; otherwise SPMM_ELIMIT with the sizes in spmm_last_error(), and
 *     nothing is enqueued.
 *   - The array keeps the work list of the last (plan, N) that used it on this GPU;
 *     a call with another plan or N first copies its list in with hipMemcpyAsync on
 *     `stream` (from host memory the plan owns), a repeat call copies nothing and
 *     only enqueues kernels.  Partial tiles are fully overwritten before they are
 *     read, so nothing needs clearing.
 *   - All calls on one GPU share the array: two calls that overlap in time on one
 *     GPU (different streams, different plans) race.  Order them.
 *   - Uses the current device; the array's address is looked up once per device.
 */
int spmm_exec_noalloc(spmm_plan_t *plan, const float *B, int64_t N, float *C, void *stream);

/* ---------------------------------------------------------------------------
 * spmm_synergy -- brick density, modeled operational intensity and synergy class
 * (Section 4, Eq. 4; Section 6.4, Table 1), plus an HBM / MFMA roofline model
 * for MI355X.  Pure host arithmetic on counts gathered at plan time.
 */
typedef struct spmm_synergy {
  /* integer counts: reproducible bit for bit */
  int64_t M, K, nnz;
  int64_t n_panels;          /* P = ceil(M/16)                                   */
  int64_t n_nonempty_panels; /* panels with at least one brick                   */
  int64_t n_bricks;          /* nb                                               */
  int64_t n_active_cols;     /* sum over panels of distinct columns              */
  int64_t n_distinct_cols;   /* distinct columns of the whole matrix             */
  int64_t panels_by_class[3]; /* per-panel class, Low/Medium/High (empty: none)  */
  int64_t bricks_by_class[3];
  int64_t nnz_by_class[3];
  int64_t brick_pop_hist[65]; /* bricks by number of stored elements             */
  int32_t synergy_class;      /* spmm_class of the whole matrix from alpha_brick */
  int32_t reserved_;
  /* model */
  double alpha_brick;      /* nnz / (64 nb): brick density (Section 4)           */
  double alpha_col;        /* nnz / (16 n_active_cols): density of active columns */
  double beta;             /* bricks per brick column; 1 for 16-row panels       */
  double oi_shmem;         /* 512 alpha beta (Eq. 4, Eq. 5)                      */
  double bytes_min;        /* 4 nnz + 28 nb + 4 + 4 (P+1) + 4 N n_distinct_cols + 4 N M */
  double bytes_noreuse;    /* same with n_active_cols in place of n_distinct_cols */
  double oi_hbm_min;       /* 2 nnz N / bytes_min   (flop per HBM byte)          */
  double oi_hbm_noreuse;   /* 2 nnz N / bytes_noreuse                            */
  double roof_gflops_hbm;  /* oi_hbm_min * 8e12 B/s, in GFLOP/s                  */
  double roof_gflops_mfma; /* alpha_brick * 157.3e12 flop/s, in GFLOP/s          */
} spmm_synergy_t;

int spmm_synergy(const spmm_plan_t *plan, int64_t N, spmm_synergy_t *out /* host */);

/* ---------------------------------------------------------------------------
 * Format export (tests, debugging).  spmm_plan_sizes fills counts; then
 * spmm_plan_export copies each array into host buffers of those sizes
 * (any pointer may be NULL to skip that array).  Synchronises the device.
 */
typedef struct spmm_sizes {
  int64_t M, K, nnz, n_panels, n_bricks;
} spmm_sizes_t;

int spmm_plan_sizes(const spmm_plan_t *plan, spmm_sizes_t *out /* host */);
int spmm_plan_export(const spmm_plan_t *plan, uint32_t *panel_ptr /* host [P+1] */,
                     uint32_t *brick_cols /* host [4 nb] */, uint64_t *brick_mask /* host [nb] */,
                     uint32_t *brick_valptr /* host [nb+1] */, float *vals /* host [nnz] */);

/* ---------------------------------------------------------------------------
 * Routing and load balancing (Section 5).  Both setters drop cached work lists.
 *
 * spmm_plan_set_route: which kernel handles which panel (enum spmm_route).
 * spmm_plan_set_split: how heavy panels are split along K into virtual panels
 *   (Eq. 6-7: ratio_p = blocks_p / avg_blocks / num_waves, with
 *   num_waves = ceil(work items / (CUs * resident waves per CU)); the paper gives no
 *   rounding rule beyond "no partition if the ratio is 1"):
 *   SPMM_SPLIT_EQ7_FROM2 (0)    parts_p = 1 while ratio_p < 2, else round-half-up(ratio_p);
 *                               the default, chosen by measurement on MI355X
 *   SPMM_SPLIT_EQ7_NEAREST (-1) parts_p = max(1, round-half-up(ratio_p)): the literal reading,
 *                               a panel is split from ratio 1.5
 *   Under both Eq. 7 policies a part keeps at least 4 blocks (16 bricks): parts_p is capped
 *   at blocks_p / 4, because splitting a smaller panel saves less than its merge costs.
 *   1                           never split
 *   parts > 1                   split every panel that has at least `parts` blocks into
 *                               `parts` (for tests of the merge path)
 * Partial tiles of a split panel go to a plan-owned workspace and are summed in
 * part order by a merge kernel, so results stay deterministic (the paper merges
 * with atomics).
 */
enum spmm_split_policy { SPMM_SPLIT_EQ7_NEAREST = -1, SPMM_SPLIT_EQ7_FROM2 = 0, SPMM_SPLIT_NEVER = 1 };
int spmm_plan_set_route(spmm_plan_t *plan, int route);
int spmm_plan_set_split(spmm_plan_t *plan, int parts);

/* Order in which the work items of the MFMA kernel are handed to the wavefronts.  Section 5
 * considers and rejects sorting panels by weight, because consecutive panels share B rows;
 * SPMM_ORDER_HEAVY_FIRST is that rejected schedule, kept to measure the argument
 * (heaviest work item first, ties in panel order).  Drops cached work lists. */
enum spmm_order { SPMM_ORDER_PANEL = 0, SPMM_ORDER_HEAVY_FIRST = 1 };
int spmm_plan_set_order(spmm_plan_t *plan, int order);

/* Arithmetic of the MFMA brick kernel.  The paper rounds its FP32 inputs to TF32 (10-bit
 * mantissa) and accumulates in FP32 (Section 2, "Background"); that buys its tensor cores an
 * eightfold rate over the ordinary ALUs.  gfx950's FP32 MFMA has no such advantage, so
 * matrices of Medium synergy are bound by zero-filled FP32 MFMA work.  The opt-in modes below
 * move that work to the bf16 matrix cores while keeping more mantissa than TF32: each FP32
 * input is split into a sum of bf16 numbers and the leading partial products are accumulated
 * in FP32.
 *   SPMM_PRECISION_FP32    v_mfma_f32_16x16x4_f32 on the unrounded inputs (default);
 *                          |C - C_exact| <= 1e-5 * sum|a.b| for the sizes tested
 *   SPMM_PRECISION_BF16X3  two bf16 terms per input (8 significant bits each, so what they
 *                          leave of a number is at most 2^-16 of it), three products
 *                          (a1 b1 + a1 b2 + a2 b1); the three dropped terms are at most
 *                          2^-16 |a.b| each: |C - C_exact| <= 5e-5 * sum|a.b|
 *                          (TF32 rounding of both inputs: about 1e-3)
 *   SPMM_PRECISION_BF16X6  three bf16 terms per input, six products; dropped terms are at
 *                          most 2^-24 |a.b| each: the same 1e-5 bound as FP32
 * The modes apply to the MFMA kernel when N is a multiple of 4 (of N itself below 64:
 * of the vector width), B and C are 16-byte aligned, B is smaller than 4 GiB and K <= 2^24;
 * other shapes, and the CSR kernel, compute in FP32.  Inputs must be finite and their
 * products within FP32 range.  Drops cached work lists. */
enum spmm_precision { SPMM_PRECISION_FP32 = 0, SPMM_PRECISION_BF16X3 = 1, SPMM_PRECISION_BF16X6 = 2 };
int spmm_plan_set_precision(spmm_plan_t *plan, int precision);

/* Large N (Section 3.3: several thread blocks work on one row panel and share its decoded
 * bricks).  By default every 128-column tile of a panel is an independent wavefront that
 * fetches and decodes the panel's bricks itself.  SPMM_SHARE_WORKGROUP instead gives a panel
 * to one workgroup of two or four wavefronts, one per tile, which decode each brick once into
 * LDS and all read their A operands from there.  Applies to the FP32 MFMA kernel with 16-row
 * panels when N >= 256 is a multiple of 4 whose number of 128-column tiles is even, B and C
 * are 16-byte aligned and B is below 4 GiB; other calls are unaffected.  C is bit-identical
 * in both modes. */
enum spmm_tile_sharing { SPMM_SHARE_NONE = 0, SPMM_SHARE_WORKGROUP = 1 };
int spmm_plan_set_tile_sharing(spmm_plan_t *plan, int mode);

/* ---------------------------------------------------------------------------
 * Row panels of 32 rows (Section 4, Eq. 5).  With TM = 32 a brick column holds up to two
 * 16x4 bricks (rows 0..15 and rows 16..31 of the super-panel) and the B rows loaded for it
 * serve both: beta = bricks per brick column.  The paper always ran TM = 16 and gives no rule
 * for when 32 pays; here the two halves of a super-panel share one left-packed column list
 * only where |cols(top) U cols(bottom)| * merge_den < merge_num * max(|cols(top)|,
 * |cols(bottom)|) (6/5 is a sensible choice; 0/1 never merges), and keep their own lists
 * elsewhere, so that unrelated halves do not dilute each other's bricks.
 *
 * spmm_plan_set_panel_height(plan, 32, num, den, stream) builds that format on the GPU from
 * the 16-row one (synchronises `stream`, allocates) and makes spmm_exec use the 32-row kernel
 * whenever every panel is routed to the MFMA kernel (SPMM_ROUTE_AUTO / _MFMA), the arithmetic
 * is FP32, N is a multiple of 4 (of the vector width below 64), B and C are 16-byte aligned
 * and B is below 4 GiB; other calls use the 16-row path.  Heavy panels are not split along K
 * in this mode.  Height 16 switches back (the 32-row arrays are kept).
 *
 * 32-row format (Q = ceil(P/2) super-panels, nbc brick columns, nbr bricks):
 *   sp_ptr u32[Q+1]     first brick column of each super-panel
 *   sp_merged u8[Q]     1 where the halves share a column list
 *   bc_cols u32[4 nbc]  column ids (ascending per list, pad 0xFFFFFFFF)
 *   bc_brick u32[nbc+1] first brick of each brick column (one or two bricks: top first)
 *   br_row u8[nbr]      0 = rows 0..15, 1 = rows 16..31 of the super-panel
 *   br_mask u64[nbr], br_valptr u32[nbr+1], vals f32[nnz]  as in the 16-row format
 */
typedef struct spmm_tm32_sizes {
  int64_t n_super_panels, n_brick_cols, n_bricks, n_merged;
} spmm_tm32_sizes_t;
int spmm_plan_set_panel_height(spmm_plan_t *plan, int rows, uint32_t merge_num, uint32_t merge_den,
                               void *stream);
int spmm_plan_tm32_sizes(const spmm_plan_t *plan, spmm_tm32_sizes_t *out /* host */);
int spmm_plan_tm32_export(const spmm_plan_t *plan, uint32_t *sp_ptr, uint8_t *sp_merged,
                          uint32_t *bc_cols, uint32_t *bc_brick, uint8_t *br_row, uint64_t *br_mask,
                          uint32_t *br_valptr, float *vals /* all host, sized by the above */);

/* Host-only arithmetic of Eq. 6-7; needs no GPU.
 *   n_panels, nbricks[n_panels]  bricks per panel (a block is 4 bricks)
 *   work_items   thread-block count before splitting ("Total_thread_blocks")
 *   num_cus, resident_per_cu     device capacity for one wave of work
 *   policy                       SPMM_SPLIT_EQ7_FROM2 or SPMM_SPLIT_EQ7_NEAREST
 *   parts_out[n_panels]          virtual panels per panel (>= 1)
 *   waves_out                    num_waves (may be NULL)
 */
int spmm_partition_counts(int64_t n_panels, const uint32_t *nbricks /* host */, int64_t work_items,
                          int32_t num_cus, int32_t resident_per_cu, int32_t policy,
                          uint32_t *parts_out /* host */, int64_t *waves_out /* host */);

/* Work list that spmm_exec would use for N (builds and caches it).
 * Items are (panel, brick_begin, brick_end, part, nparts); brick indices are
 * global (into brick_mask).  Call with items = NULL to get the counts only. */
typedef struct spmm_work_item {
  uint32_t panel, brick_begin, brick_end, part, nparts;
} spmm_work_item_t;

typedef struct spmm_worklist_info {
  int64_t n_mfma_items;   /* work items of the MFMA kernel                   */
  int64_t n_valu_panels;  /* panels handled by the vector-ALU kernel          */
  int64_t n_split_panels; /* panels split into more than one part             */
  int64_t num_waves;      /* Eq. 7 denominator actually used                  */
  int32_t n_tile;         /* columns of C per wavefront (16, 32, 64 or 128)   */
  int32_t n_tiles;        /* ceil(N / n_tile)                                 */
  int32_t num_cus;        /* compute units of the plan's device               */
  int32_t resident_waves_per_cu; /* wavefronts of the MFMA kernel variant for
                             this N that fit on one CU at a time; num_waves =
                             max(1, ceil(panels * n_tiles / (num_cus * this))) */
} spmm_worklist_info_t;

int spmm_plan_worklist(spmm_plan_t *plan, int64_t N, spmm_worklist_info_t *info /* host */,
                       spmm_work_item_t *items /* host [n_mfma_items] or NULL */,
                       uint32_t *valu_panels /* host [n_valu_panels] or NULL */);

/* Measurement aid (used by bench.py to calibrate the memory roofline of the brick kernel):
 * enqueues one kernel in which each of n_waves wavefronts reads loads_per_wave x 1 KiB from
 * `buf` the way the brick kernel reads B at N = 128 -- four rows of 512 bytes picked at
 * random per pair of load instructions, 16 lanes x 16 contiguous bytes per half row, 8 loads
 * in flight.  The caller times it; bytes moved = n_waves * loads_per_wave * 1024.
 *   buf     dev, n_rows * 512 bytes, finite values; n_rows a power of two
 *   loads_per_wave  multiple of 8;  n_waves  multiple of 4
 *   sink    dev float[256], never written for finite inputs (keeps the loads alive)
 * SPMM_EINVAL for sizes outside these rules. */
int spmm_calibrate_gather(const float *buf, int64_t n_rows, int64_t loads_per_wave,
                          int64_t n_waves, float *sink, void *stream);

void spmm_plan_destroy(spmm_plan_t *plan); /* NULL is allowed */

const char *spmm_last_error(void); /* thread-local, valid until the next failing call */

#ifdef __cplusplus
}
#endif
#endif /* SPMM_H_ */
