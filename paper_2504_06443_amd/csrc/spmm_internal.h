// Internal declarations shared by the HIP translation units of libspmm_brick.
// Host-callable launchers only; every launcher enqueues on `s` and returns the
// launch status.  All pointers are device pointers unless named h_*.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace spmm {

constexpr int kPanel = 16;            // TM: rows per row panel (Section 3.2)
constexpr int kBrickK = 4;            // brick_k: columns per brick
constexpr uint32_t kPadCol = 0xFFFFFFFFu;

// error bits written by the validation kernels
enum : uint32_t {
  kErrRowptrEnds = 1u,      // rowptr[0] != 0 or rowptr[M] != nnz
  kErrRowptrOrder = 2u,     // rowptr decreases or leaves [0, nnz]
  kErrColRange = 4u,        // column outside [0, K)
  kErrColOrder = 8u         // columns of a row not strictly ascending
};

// counters gathered at plan time (device array of kNumCounters u64)
enum : int {
  kCntPanelsByClass = 0,    // 3
  kCntBricksByClass = 3,    // 3
  kCntNnzByClass = 6,       // 3
  kCntNonEmptyPanels = 9,
  kCntDistinctCols = 10,
  kCntPopHist = 11,         // 65
  kCntLongRows = 76,        // rows with more entries than the CSR kernel handles side by side
  kNumCounters = 77
};

struct WorkItem {           // one wavefront's share of the MFMA kernel
  uint32_t panel;
  uint32_t brick_begin;     // global brick index
  uint32_t brick_end;
  uint32_t slot;            // kNoSlot: store to C; else index of a 16 x N partial tile
};
constexpr uint32_t kNoSlot = 0xFFFFFFFFu;

struct MergeItem {          // one split panel
  uint32_t panel;
  uint32_t slot_begin;      // its partial tiles are slot_begin .. slot_begin+nparts-1
  uint32_t nparts;
};

// ---- plan (a1..a5) -------------------------------------------------------
hipError_t launch_validate_rowptr(const int32_t* rowptr, int64_t M, int64_t nnz, uint32_t* err,
                                  hipStream_t s);
hipError_t launch_validate_cols(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t K,
                                int64_t nnz, uint32_t* ent_row, uint32_t* err, hipStream_t s);
hipError_t launch_first_in_panel(const int32_t* rowptr, const int32_t* colind,
                                 const uint32_t* ent_row, int64_t nnz, uint8_t* first,
                                 uint32_t* link, hipStream_t s);
hipError_t launch_compact_first(const uint8_t* first, const uint32_t* first_scan, int64_t nnz,
                                uint32_t* first_list, hipStream_t s);
hipError_t launch_panel_counts(const int32_t* rowptr, const uint32_t* first_scan, int64_t M,
                               int64_t P, uint32_t* nbricks_p, uint32_t* panel_nnzptr,
                               hipStream_t s);
hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s);
hipError_t launch_fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s);
hipError_t launch_rank_first(const int32_t* rowptr, const int32_t* colind, const uint32_t* ent_row,
                             const uint32_t* first_list, const uint32_t* first_scan,
                             const uint32_t* panel_ptr, int64_t M, int64_t n_active,
                             uint32_t* ent_rank, uint32_t* brick_cols, hipStream_t s);
hipError_t launch_scatter_bits(const int32_t* colind, const uint32_t* ent_row, const uint32_t* link,
                               const uint32_t* ent_rank, const uint32_t* panel_ptr, int64_t nnz,
                               uint64_t* brick_mask, uint32_t* ent_brick, uint8_t* ent_bit,
                               uint8_t* col_seen, hipStream_t s);
hipError_t launch_pack_values(const float* vals, const uint32_t* ent_brick, const uint8_t* ent_bit,
                              const uint64_t* brick_mask, const uint32_t* brick_valptr,
                              int64_t nnz, float* packed, uint32_t* ent_pos, hipStream_t s);
hipError_t launch_update_values(const float* vals, const uint32_t* ent_pos, int64_t nnz,
                                float* packed, float* csr_vals, hipStream_t s);
hipError_t launch_panel_classes(const uint32_t* panel_ptr, const uint32_t* panel_nnzptr, int64_t P,
                                uint8_t* panel_class, unsigned long long* counters, hipStream_t s);
hipError_t launch_brick_hist(const uint64_t* brick_mask, int64_t nb, unsigned long long* counters,
                             hipStream_t s);
hipError_t launch_count_flags(const uint8_t* flags, int64_t n, unsigned long long* counter,
                              hipStream_t s);
// rows with more than `threshold` entries -> list (any order), count added to *counter
hipError_t launch_find_long_rows(const int32_t* rowptr, int64_t M, int threshold,
                                 uint32_t* list, unsigned long long* counter, hipStream_t s);

// per-panel path (LDS bitmap over the panel's column span)
// out[0] = widest column span of a panel, out[1] = most entries of a panel
// (also flags a panel whose column span is inverted: unsorted rows or negative columns)
hipError_t launch_panel_span(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t P,
                             uint32_t* err, uint32_t* span_and_nnz, hipStream_t s);
// per-panel path by sorting (any column span, panels of limited size)
uint32_t panel_sort_keys(uint32_t max_nnz);   // 0: a panel has too many entries
bool panel_sort_build_fits(uint32_t n_cap, uint32_t nb_cap);
hipError_t launch_panel_sort_census(const int32_t* rowptr, const int32_t* colind, int64_t M,
                                    int64_t K, int64_t P, uint32_t n_cap, uint32_t* err,
                                    uint32_t* nbricks_p, uint32_t* panel_nnzptr, uint32_t* ncols_p,
                                    uint32_t* order /* [nnz]; read back by the build as ent_pos */,
                                    unsigned long long* n_active, uint32_t* max_cols,
                                    hipStream_t s);
hipError_t launch_panel_sort_build(const int32_t* rowptr, const int32_t* colind, const float* vals,
                                   int64_t M, int64_t K, int64_t P, uint32_t n_cap, uint32_t nb_cap,
                                   const uint32_t* panel_ptr, uint32_t* brick_cols,
                                   uint64_t* brick_mask, uint32_t* brick_valptr, float* packed,
                                   uint32_t* ent_pos, uint8_t* col_seen, hipStream_t s);
uint32_t panel_bitmap_words(uint32_t span);   // 0: span too wide for the per-panel path
hipError_t launch_panel_census(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t K,
                               int64_t P, uint32_t words_cap, uint32_t* err, uint32_t* nbricks_p,
                               uint32_t* panel_nnzptr, uint32_t* ncols_p,
                               unsigned long long* n_active, uint32_t* max_cols, hipStream_t s);
bool panel_build_fits(uint32_t words_cap, uint32_t nb_cap);   // LDS of launch_panel_build
hipError_t launch_panel_build(const int32_t* rowptr, const int32_t* colind, const float* vals,
                              int64_t M, int64_t K, int64_t P, uint32_t words_cap, uint32_t nb_cap,
                              const uint32_t* panel_ptr, uint32_t* brick_cols, uint64_t* brick_mask,
                              uint32_t* brick_valptr, float* packed, uint32_t* ent_pos,
                              uint8_t* col_seen, hipStream_t s);

// exclusive scans; out has n+1 entries (out[n] = total); tmp holds block sums
size_t scan_tmp_elems(int64_t n);
hipError_t launch_scan_u8(const uint8_t* in, int64_t n, uint32_t* out, uint32_t* tmp, hipStream_t s);
hipError_t launch_scan_u32(const uint32_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                           hipStream_t s);
hipError_t launch_scan_popc64(const uint64_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                              hipStream_t s);
hipError_t launch_scan_nonzero64(const uint64_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                                 hipStream_t s);

// ---- exec (a6..a8) -------------------------------------------------------
// Device arrays of the brick format.  Each carries spare entries past its end
// (kFormatPad bricks' worth: zero columns and patterns, value offsets equal to
// nnz, zero values) so that kernels may fetch metadata a few bricks past a work
// item's last brick without clamping.
constexpr int kFormatPad = 32;
struct BrickFormat {
  const uint32_t* brick_cols;    // 4 * (nb + kFormatPad)
  const uint64_t* brick_mask;    // nb + kFormatPad
  const uint32_t* brick_valptr;  // nb + 1 + kFormatPad
  const float* vals;             // nnz + 64
};

int mfma_tile_for(int64_t N);   // columns of C per wavefront: 16, 32, 64 or 128
int mfma_resident_waves_per_cu(int64_t N, int64_t K);
// shapes the fast FP32 kernel serves when B and C are 16-byte aligned: N a multiple of the
// vector width, B below 4 GiB
bool mfma_fast_shape(int64_t N, int64_t K);
hipError_t launch_spmm_mfma(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                            const float* B, float* C, float* partial, int64_t M, int64_t N,
                            int64_t K, int64_t nnz, hipStream_t s);
// wide-N variant (exec_wide.hip): one workgroup per work item whose wavefronts take different
// 128-column tiles and share the decoded bricks through LDS.  mfma_wide_waves: wavefronts per
// workgroup it would use for (N, K), 0 when the shape is not served
int mfma_wide_waves(int64_t N, int64_t K);
hipError_t launch_spmm_mfma_wide(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                                 const float* B, float* C, float* partial, int64_t M, int64_t N,
                                 int64_t K, hipStream_t s);
// split-bf16 variant (exec_bf16.hip): planes = 2 or 3 bf16 terms per FP32 input
bool bf16_path_shape(int64_t N, int64_t K);
int bf16_resident_waves_per_cu(int64_t N, int planes);
hipError_t launch_spmm_bf16(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                            const float* B, float* C, float* partial, int64_t M, int64_t N,
                            int64_t K, int planes, int64_t nnz, hipStream_t s);
// `panels` is sorted ascending; `long_rows` lists the rows of the whole matrix with more than
// long_row_threshold() entries (any order)
int long_row_threshold();
hipError_t launch_spmm_valu(const int32_t* rowptr, const int32_t* colind, const float* vals,
                            const uint32_t* panels, int64_t n_panels, const uint32_t* long_rows,
                            int64_t n_long_rows, const float* B, float* C, int64_t M, int64_t N,
                            hipStream_t s);
hipError_t launch_merge(const MergeItem* items, int64_t n_items, const float* partial, float* C,
                        int64_t M, int64_t N, hipStream_t s);

// ---- 32-row panels (tm32_kernels.hip; Section 4, Eq. 5) ------------------------------------
struct Tm32Meta {           // per brick column, for the kernel: its top and bottom brick
  uint64_t mask_top, mask_bot;   // zero where the half has no brick in this brick column
  uint32_t off_top, off_bot;     // start of the brick's values
};
hipError_t launch_tm32_count(const uint32_t* panel_ptr, const uint32_t* brick_cols, int64_t P,
                             int64_t Q, uint32_t num, uint32_t den, uint32_t* cpre,
                             uint8_t* sp_merged, uint32_t* nbc_q, hipStream_t s);
hipError_t launch_tm32_cols_masks(const uint32_t* panel_ptr, const uint32_t* brick_cols,
                                  const uint64_t* brick_mask, int64_t P, int64_t Q, int64_t nb,
                                  const uint32_t* cpre, const uint8_t* sp_merged,
                                  const uint32_t* sp_ptr, uint32_t* bc_cols, uint32_t* new_slot,
                                  uint8_t* brick_half, unsigned long long* tmask, hipStream_t s);
hipError_t launch_tm32_compact(const unsigned long long* tmask, const uint32_t* pos, int64_t nbc,
                               uint32_t* bc_brick, uint8_t* br_row, uint64_t* br_mask,
                               hipStream_t s);
hipError_t launch_tm32_values(const uint64_t* brick_mask, const uint32_t* brick_valptr,
                              const float* vals, const uint32_t* new_slot,
                              const uint8_t* brick_half, const uint32_t* pos,
                              const uint64_t* br_mask, const uint32_t* br_valptr, int64_t nb,
                              float* out, hipStream_t s);
hipError_t launch_tm32_meta(const uint32_t* bc_brick, const uint8_t* br_row, const uint64_t* br_mask,
                            const uint32_t* br_valptr, int64_t nbc, int64_t nnz, Tm32Meta* meta,
                            int64_t n_meta, hipStream_t s);
hipError_t launch_spmm_tm32(const uint32_t* sp_ptr, const uint32_t* bc_cols, const Tm32Meta* meta,
                            const float* vals, int64_t Q, const float* B, float* C, int64_t M,
                            int64_t N, int64_t K, hipStream_t s);

}  // namespace spmm
