// C ABI of libspmm_brick: plan construction (drives the kernels of
// plan_kernels.hip), work-list building with the load balancer of paper
// Section 5 (Eq. 6-7), kernel dispatch, the synergy model of Section 4 /
// Table 1, and export accessors.
#include "../../include/spmm.h"
#include "spmm_internal.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <atomic>
#include <map>
#include <mutex>
#include <new>
#include <vector>

using namespace spmm;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define HIP_TRY(expr)                                                                   \
  do {                                                                                  \
    hipError_t e_ = (expr);                                                             \
    if (e_ != hipSuccess) {                                                             \
      status = fail(e_ == hipErrorOutOfMemory ? SPMM_ENOMEM : SPMM_EHIP, "%s: %s", #expr, \
                    hipGetErrorString(e_));                                             \
      goto done;                                                                        \
    }                                                                                   \
  } while (0)

constexpr double kHbmBytesPerS = 8.0e12;    // MI355X published HBM3E bandwidth
constexpr double kMfmaFp32Flops = 157.3e12; // MI355X published dense fp32 matrix peak

// Host half of a work list: what the routing and Eq. 6-7 decide for one N.
struct HostList {
  uint64_t id = 0;                          // unique per list (tags the contents of the static scratch)
  int64_t N = 0;
  spmm_worklist_info_t info{};
  std::vector<spmm_work_item_t> h_items;   // exported form
  std::vector<WorkItem> items;             // device form
  std::vector<MergeItem> merges;
  std::vector<uint32_t> valu_panels;
  int64_t n_slots = 0;                      // partial 16 x N tiles of split panels
};

// Device half: plan-owned copies of a HostList plus the partial-tile workspace.
struct WorkList {
  const HostList* host = nullptr;
  WorkItem* d_items = nullptr;
  uint32_t* d_valu_panels = nullptr;
  MergeItem* d_merge = nullptr;
  float* d_partial = nullptr;               // n_slots tiles of 16 x N
  ~WorkList() {
    if (d_items) (void)hipFree(d_items);
    if (d_valu_panels) (void)hipFree(d_valu_panels);
    if (d_merge) (void)hipFree(d_merge);
    if (d_partial) (void)hipFree(d_partial);
  }
};

std::atomic<uint64_t> g_next_list_id{1};

}  // namespace

struct spmm_plan {
  int64_t M = 0, K = 0, nnz = 0, P = 0, nb = 0;
  int device = 0;
  int num_cus = 1;
  // brick format (device)
  uint32_t* panel_ptr = nullptr;
  uint32_t* brick_cols = nullptr;
  uint64_t* brick_mask = nullptr;
  uint32_t* brick_valptr = nullptr;
  float* vals = nullptr;          // nnz + 1
  // plan-owned CSR copy for the vector-ALU kernel (device)
  int32_t* rowptr = nullptr;
  int32_t* colind = nullptr;
  float* csr_vals = nullptr;
  uint32_t* ent_pos = nullptr;    // packed position of each CSR entry (value-only updates)
  uint32_t* long_rows = nullptr;  // rows with more than long_row_threshold() entries
  int64_t n_long_rows = 0;
  // host copies used by the work-list builder and the synergy model
  std::vector<uint32_t> h_panel_ptr;
  std::vector<uint32_t> h_panel_nnzptr;   // first CSR entry of each panel
  std::vector<uint8_t> h_panel_class;
  unsigned long long h_counters[kNumCounters] = {};
  int64_t n_active_cols = 0;
  int route = SPMM_ROUTE_AUTO;
  int split = 0;
  int order = SPMM_ORDER_PANEL;
  int precision = SPMM_PRECISION_FP32;
  int tile_sharing = SPMM_SHARE_NONE;
  // 32-row panel format (built on request; Section 4, Eq. 5)
  int panel_height = 16;
  struct Tm32 {
    int64_t Q = 0, nbc = 0, nbr = 0, n_merged = 0;
    char* arena = nullptr;        // everything below, one allocation
    uint32_t* sp_ptr = nullptr;
    uint8_t* sp_merged = nullptr;
    uint32_t* bc_cols = nullptr;
    uint32_t* bc_brick = nullptr;
    uint8_t* br_row = nullptr;
    uint64_t* br_mask = nullptr;
    uint32_t* br_valptr = nullptr;
    float* vals = nullptr;
    Tm32Meta* meta = nullptr;
    // kept for value-only updates: where the entries of the 16-row format went
    uint32_t* new_slot = nullptr;
    uint8_t* brick_half = nullptr;
    uint32_t* pos = nullptr;
  } tm32;
  std::map<int64_t, HostList*> host_lists;
  std::map<int64_t, WorkList*> lists;

  void drop_lists() {
    for (auto& kv : lists) delete kv.second;
    lists.clear();
    for (auto& kv : host_lists) delete kv.second;
    host_lists.clear();
  }
  // the arrays above are carved out of two device allocations
  char* fixed_arena = nullptr;   // panel_ptr, rowptr, colind, csr_vals, ent_pos
  char* brick_arena = nullptr;   // brick_cols, brick_mask, brick_valptr, vals
  ~spmm_plan() {
    drop_lists();
    if (fixed_arena) (void)hipFree(fixed_arena);
    if (brick_arena) (void)hipFree(brick_arena);
    if (tm32.arena) (void)hipFree(tm32.arena);
  }
};

namespace {

// Bump allocator over one device allocation; sub-arrays are 256-byte aligned.
struct Arena {
  char* base = nullptr;
  size_t used = 0, cap = 0;
  static size_t pad(size_t bytes) { return (bytes + 255) & ~size_t(255); }
  template <typename T> T* take(int64_t n) {
    T* p = reinterpret_cast<T*>(base + used);
    used += pad((size_t)std::max<int64_t>(n, 1) * sizeof(T));
    return used <= cap ? p : nullptr;
  }
};

template <typename T>
hipError_t dev_alloc(T** p, int64_t n) {
  return hipMalloc((void**)p, (size_t)std::max<int64_t>(n, 1) * sizeof(T));
}

int classify(int64_t nnz, int64_t nb) {
  if (nb == 0) return SPMM_NONE;
  if (nnz < 8 * nb) return SPMM_LOW;
  if (nnz < 16 * nb) return SPMM_MEDIUM;
  return SPMM_HIGH;
}

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

constexpr int64_t kMinBlocksPerPart = 4;   // Eq. 6-7 splits never go below this (16 bricks)

// Eq. 6-7 in integers: partition_ratio_p = blocks_p * P / (total_blocks * waves).
// SPMM_SPLIT_EQ7_FROM2 (the default): one part while the ratio is below 2, else the ratio
// rounded to the nearest integer, halves up.  SPMM_SPLIT_EQ7_NEAREST: the ratio rounded to
// the nearest integer from the start (a panel is split from ratio 1.5), at least one part.
void partition_counts(int64_t P, const uint32_t* nbricks, int64_t work_items, int64_t capacity,
                      int policy, uint32_t* parts, int64_t* waves_out) {
  int64_t total = 0;
  for (int64_t p = 0; p < P; ++p) total += ceil_div(nbricks[p], kBrickK);
  const int64_t waves = std::max<int64_t>(1, ceil_div(work_items, std::max<int64_t>(1, capacity)));
  for (int64_t p = 0; p < P; ++p) {
    const int64_t blocks = ceil_div(nbricks[p], kBrickK);
    int64_t q = 1;
    if (total > 0 && blocks > 0) {
      // blocks * P can exceed 2^63 only for absurd sizes; use 128-bit to be safe
      const __int128 num = (__int128)blocks * P;
      const __int128 den = (__int128)total * waves;
      const int64_t nearest = (int64_t)((2 * num + den) / (2 * den));
      q = (policy == SPMM_SPLIT_EQ7_FROM2 && num < 2 * den) ? 1 : nearest;
    }
    parts[p] = (uint32_t)std::max<int64_t>(1, q);
  }
  if (waves_out) *waves_out = waves;
}

// Routing and load balancing for N (host only, no device memory).  Cached in the plan.
int build_host_list(spmm_plan_t* pl, int64_t N, const HostList** out) {
  auto found = pl->host_lists.find(N);
  if (found != pl->host_lists.end()) {
    *out = found->second;
    return SPMM_OK;
  }
  HostList* hl = nullptr;
  try {
    hl = new HostList();
    hl->id = g_next_list_id.fetch_add(1);
    hl->N = N;
    const int tile = mfma_tile_for(std::max<int64_t>(N, 1));
    hl->info.n_tile = tile;
    hl->info.n_tiles = (int32_t)ceil_div(std::max<int64_t>(N, 1), tile);
    hl->info.num_cus = pl->num_cus;

    // routing: which panels go to the MFMA kernel
    std::vector<uint32_t> mfma_panels;
    std::vector<uint32_t> nbricks;
    for (int64_t p = 0; p < pl->P; ++p) {
      const uint8_t cls = pl->h_panel_class[p];
      bool to_mfma;
      // AUTO is the measured policy for MI355X: the brick kernel loads each B row of a panel
      // once where CSR loads it once per entry, and on the benchmark's sweep of brick fill
      // (0.05..0.8) and width (16..512) the CSR kernel is nowhere faster by more than a few
      // percent (a tie at fill 0.05, N = 16), so every panel goes to the brick kernel.  SPMM_ROUTE_CLASS is the
      // paper's per-class rule.
      // An empty panel (class 255) only needs its rows of C zeroed; either kernel does that, so
      // under CLASS it goes to the CSR kernel, whose launch the Low panels cause anyway.
      if (pl->route == SPMM_ROUTE_AUTO || pl->route == SPMM_ROUTE_MFMA) to_mfma = true;
      else if (pl->route == SPMM_ROUTE_VALU) to_mfma = false;
      else to_mfma = cls != SPMM_LOW && cls != 255;
      if (to_mfma) {
        mfma_panels.push_back((uint32_t)p);
        nbricks.push_back(pl->h_panel_ptr[p + 1] - pl->h_panel_ptr[p]);
      } else {
        hl->valu_panels.push_back((uint32_t)p);
      }
    }

    // load balancing over the MFMA panels
    const int64_t nm = (int64_t)mfma_panels.size();
    std::vector<uint32_t> parts((size_t)nm, 1u);
    int64_t waves = 1;
    const bool bf16 = pl->precision != SPMM_PRECISION_FP32 &&
                      bf16_path_shape(std::max<int64_t>(N, 1), pl->K);
    const int resident =
        bf16 ? bf16_resident_waves_per_cu(std::max<int64_t>(N, 1),
                                          pl->precision == SPMM_PRECISION_BF16X3 ? 2 : 3)
             : mfma_resident_waves_per_cu(std::max<int64_t>(N, 1), pl->K);
    hl->info.resident_waves_per_cu = resident;
    if (nm > 0) {
      if (pl->split == SPMM_SPLIT_EQ7_FROM2 || pl->split == SPMM_SPLIT_EQ7_NEAREST) {
        partition_counts(nm, nbricks.data(), nm * hl->info.n_tiles,
                         (int64_t)pl->num_cus * resident, pl->split, parts.data(), &waves);
        // A part keeps at least kMinBlocksPerPart blocks: splitting a panel of a few blocks saves
        // less than the merge launch it causes (measured on the 65,536-row sweep, fill 0.8: three panels of
        // about 20 bricks split in two, 24.8 us against 20.9 us unsplit).
        for (int64_t i = 0; i < nm; ++i) {
          const int64_t blocks = ceil_div(nbricks[i], kBrickK);
          parts[i] = (uint32_t)std::min<int64_t>(parts[i], std::max<int64_t>(1, blocks / kMinBlocksPerPart));
        }
      } else if (pl->split > 1) {
        for (int64_t i = 0; i < nm; ++i)
          if (ceil_div(nbricks[i], kBrickK) >= pl->split) parts[i] = (uint32_t)pl->split;
      }
    }
    hl->info.num_waves = waves;

    int64_t slots = 0;
    for (int64_t i = 0; i < nm; ++i) {
      const uint32_t p = mfma_panels[i];
      const uint32_t b0 = pl->h_panel_ptr[p];
      const int64_t nbp = nbricks[i];
      const int64_t blocks = ceil_div(nbp, kBrickK);
      const int64_t want = std::max<int64_t>(1, std::min<int64_t>(parts[i], blocks));
      const int64_t per = std::max<int64_t>(1, ceil_div(blocks, want));   // blocks per part
      const int64_t nparts = ceil_div(blocks, per);        // parts that are not empty
      if (nparts <= 1) {   // also an empty panel: one work item without bricks
        hl->items.push_back(WorkItem{p, b0, b0 + (uint32_t)nbp, kNoSlot});
        hl->h_items.push_back(spmm_work_item_t{p, b0, b0 + (uint32_t)nbp, 0, 1});
        continue;
      }
      hl->merges.push_back(MergeItem{p, (uint32_t)slots, (uint32_t)nparts});
      for (int64_t q = 0; q < nparts; ++q) {
        const int64_t lo = std::min<int64_t>(nbp, q * per * kBrickK);
        const int64_t hi = std::min<int64_t>(nbp, (q + 1) * per * kBrickK);
        hl->items.push_back(
            WorkItem{p, b0 + (uint32_t)lo, b0 + (uint32_t)hi, (uint32_t)(slots + q)});
        hl->h_items.push_back(
            spmm_work_item_t{p, b0 + (uint32_t)lo, b0 + (uint32_t)hi, (uint32_t)q, (uint32_t)nparts});
      }
      slots += nparts;
    }
    if (pl->order == SPMM_ORDER_HEAVY_FIRST) {
      // the schedule Section 5 argues against (it gives up the locality of consecutive panels);
      // kept as an experiment
      std::vector<size_t> perm(hl->items.size());
      for (size_t i = 0; i < perm.size(); ++i) perm[i] = i;
      std::stable_sort(perm.begin(), perm.end(), [&](size_t l, size_t r) {
        return hl->items[l].brick_end - hl->items[l].brick_begin >
               hl->items[r].brick_end - hl->items[r].brick_begin;
      });
      std::vector<WorkItem> sorted_items(hl->items.size());
      std::vector<spmm_work_item_t> sorted_h(hl->items.size());
      for (size_t i = 0; i < perm.size(); ++i) {
        sorted_items[i] = hl->items[perm[i]];
        sorted_h[i] = hl->h_items[perm[i]];
      }
      hl->items.swap(sorted_items);
      hl->h_items.swap(sorted_h);
    }
    hl->info.n_mfma_items = (int64_t)hl->items.size();
    hl->info.n_valu_panels = (int64_t)hl->valu_panels.size();
    hl->info.n_split_panels = (int64_t)hl->merges.size();
    hl->n_slots = slots;
    pl->host_lists[N] = hl;
  } catch (const std::bad_alloc&) {
    delete hl;
    return fail(SPMM_ENOMEM, "host allocation failed while building the work list");
  }
  *out = hl;
  return SPMM_OK;
}

// Device copy of the work list for N (allocates; synchronises the stream once).
int build_worklist(spmm_plan_t* pl, int64_t N, hipStream_t stream, WorkList** out) {
  auto found = pl->lists.find(N);
  if (found != pl->lists.end()) {
    *out = found->second;
    return SPMM_OK;
  }
  const HostList* hl = nullptr;
  int status = build_host_list(pl, N, &hl);
  if (status != SPMM_OK) return status;
  WorkList* wl = new (std::nothrow) WorkList();
  if (!wl) return fail(SPMM_ENOMEM, "host allocation failed");
  wl->host = hl;
  HIP_TRY(dev_alloc(&wl->d_items, (int64_t)hl->items.size()));
  HIP_TRY(dev_alloc(&wl->d_valu_panels, (int64_t)hl->valu_panels.size()));
  HIP_TRY(dev_alloc(&wl->d_merge, (int64_t)hl->merges.size()));
  if (hl->n_slots > 0)
    HIP_TRY(dev_alloc(&wl->d_partial, hl->n_slots * kPanel * std::max<int64_t>(N, 1)));
  if (!hl->items.empty())
    HIP_TRY(hipMemcpyAsync(wl->d_items, hl->items.data(), hl->items.size() * sizeof(WorkItem),
                           hipMemcpyHostToDevice, stream));
  if (!hl->valu_panels.empty())
    HIP_TRY(hipMemcpyAsync(wl->d_valu_panels, hl->valu_panels.data(),
                           hl->valu_panels.size() * sizeof(uint32_t), hipMemcpyHostToDevice,
                           stream));
  if (!hl->merges.empty())
    HIP_TRY(hipMemcpyAsync(wl->d_merge, hl->merges.data(), hl->merges.size() * sizeof(MergeItem),
                           hipMemcpyHostToDevice, stream));
  HIP_TRY(hipStreamSynchronize(stream));
  try {
    pl->lists[N] = wl;
  } catch (const std::bad_alloc&) {
    status = fail(SPMM_ENOMEM, "host allocation failed");
  }
done:
  if (status != SPMM_OK) {
    delete wl;
    return status;
  }
  *out = wl;
  return SPMM_OK;
}

// Builds the 32-row panel format from the 16-row one (device kernels; two size read-backs).
int build_tm32(spmm_plan_t* pl, uint32_t num, uint32_t den, hipStream_t s) {
  int status = SPMM_OK;
  auto need = [](int64_t n, size_t elem) { return Arena::pad((size_t)std::max<int64_t>(n, 1) * elem); };
  const int64_t P = pl->P, Q = (P + 1) / 2, nb = pl->nb, nnz = pl->nnz;
  Arena t1, t2, keep;
  uint32_t *cpre, *nbc_q, *sp_ptr_tmp, *scan_tmp, *pos_tmp, *new_slot_tmp, *bc_cols_tmp;
  uint8_t *merged_tmp, *half_tmp;
  unsigned long long* tmask;
  uint32_t h_nbc = 0, h_nbr = 0;
  int64_t nbc = 0, nbr = 0, n_meta = 0;
  spmm_plan::Tm32 f;
  std::vector<uint8_t> h_merged;

  t1.cap = need(4 * nb + P + 1, 4) + need(Q, 4) + need(Q + 1, 4) + need(Q, 1) + need(4 * nb, 4) +
           need(nb, 1) + need((int64_t)scan_tmp_elems(std::max<int64_t>(2 * 4 * nb + 2, Q + 1)), 4);
  HIP_TRY(hipMalloc((void**)&t1.base, t1.cap));
  cpre = t1.take<uint32_t>(4 * nb + P + 1);
  nbc_q = t1.take<uint32_t>(Q);
  sp_ptr_tmp = t1.take<uint32_t>(Q + 1);
  merged_tmp = t1.take<uint8_t>(Q);
  new_slot_tmp = t1.take<uint32_t>(4 * nb);
  half_tmp = t1.take<uint8_t>(nb);
  scan_tmp = t1.take<uint32_t>((int64_t)scan_tmp_elems(std::max<int64_t>(2 * 4 * nb + 2, Q + 1)));

  HIP_TRY(launch_tm32_count(pl->panel_ptr, pl->brick_cols, P, Q, num, den, cpre, merged_tmp, nbc_q, s));
  HIP_TRY(launch_scan_u32(nbc_q, Q, sp_ptr_tmp, scan_tmp, s));
  HIP_TRY(hipMemcpyAsync(&h_nbc, sp_ptr_tmp + Q, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  nbc = h_nbc;   // at most the bricks of the 16-row format

  t2.cap = need((nbc + kFormatPad) * kBrickK, 4) + need(2 * nbc, 8) + need(2 * nbc + 1, 4);
  HIP_TRY(hipMalloc((void**)&t2.base, t2.cap));
  bc_cols_tmp = t2.take<uint32_t>((nbc + kFormatPad) * kBrickK);
  tmask = t2.take<unsigned long long>(2 * nbc);
  pos_tmp = t2.take<uint32_t>(2 * nbc + 1);
  HIP_TRY(hipMemsetAsync(tmask, 0, (size_t)std::max<int64_t>(2 * nbc, 1) * 8, s));
  HIP_TRY(hipMemsetAsync(bc_cols_tmp + nbc * kBrickK, 0, kFormatPad * kBrickK * 4, s));
  HIP_TRY(launch_tm32_cols_masks(pl->panel_ptr, pl->brick_cols, pl->brick_mask, P, Q, nb, cpre,
                                 merged_tmp, sp_ptr_tmp, bc_cols_tmp, new_slot_tmp, half_tmp, tmask,
                                 s));
  HIP_TRY(launch_scan_nonzero64(reinterpret_cast<const uint64_t*>(tmask), 2 * nbc, pos_tmp, scan_tmp, s));
  HIP_TRY(hipMemcpyAsync(&h_nbr, pos_tmp + 2 * nbc, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  try { h_merged.resize((size_t)std::max<int64_t>(Q, 1)); }
  catch (const std::bad_alloc&) { status = fail(SPMM_ENOMEM, "host allocation failed"); goto done; }
  if (Q > 0)
    HIP_TRY(hipMemcpyAsync(h_merged.data(), merged_tmp, (size_t)Q, hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  nbr = h_nbr;
  n_meta = nbc + kFormatPad;

  keep.cap = need(Q + 1, 4) + need(Q, 1) + need((nbc + kFormatPad) * kBrickK, 4) + need(nbc + 1, 4) +
             need(nbr, 1) + need(nbr, 8) + need(nbr + 1, 4) + need(nnz + 64, 4) +
             need(n_meta, sizeof(Tm32Meta)) + need(4 * nb, 4) + need(nb, 1) + need(2 * nbc + 1, 4);
  HIP_TRY(hipMalloc((void**)&keep.base, keep.cap));
  f.arena = keep.base;
  f.Q = Q; f.nbc = nbc; f.nbr = nbr;
  for (int64_t q = 0; q < Q; ++q) f.n_merged += h_merged[q];
  f.sp_ptr = keep.take<uint32_t>(Q + 1);
  f.sp_merged = keep.take<uint8_t>(Q);
  f.bc_cols = keep.take<uint32_t>((nbc + kFormatPad) * kBrickK);
  f.bc_brick = keep.take<uint32_t>(nbc + 1);
  f.br_row = keep.take<uint8_t>(nbr);
  f.br_mask = keep.take<uint64_t>(nbr);
  f.br_valptr = keep.take<uint32_t>(nbr + 1);
  f.vals = keep.take<float>(nnz + 64);
  f.meta = keep.take<Tm32Meta>(n_meta);
  f.new_slot = keep.take<uint32_t>(4 * nb);
  f.brick_half = keep.take<uint8_t>(nb);
  f.pos = keep.take<uint32_t>(2 * nbc + 1);
  HIP_TRY(hipMemcpyAsync(f.sp_ptr, sp_ptr_tmp, (size_t)(Q + 1) * 4, hipMemcpyDeviceToDevice, s));
  if (Q > 0) HIP_TRY(hipMemcpyAsync(f.sp_merged, merged_tmp, (size_t)Q, hipMemcpyDeviceToDevice, s));
  HIP_TRY(hipMemcpyAsync(f.bc_cols, bc_cols_tmp, (size_t)(nbc + kFormatPad) * kBrickK * 4,
                         hipMemcpyDeviceToDevice, s));
  if (nb > 0) {
    HIP_TRY(hipMemcpyAsync(f.new_slot, new_slot_tmp, (size_t)nb * kBrickK * 4, hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipMemcpyAsync(f.brick_half, half_tmp, (size_t)nb, hipMemcpyDeviceToDevice, s));
  }
  HIP_TRY(hipMemcpyAsync(f.pos, pos_tmp, (size_t)(2 * nbc + 1) * 4, hipMemcpyDeviceToDevice, s));
  HIP_TRY(launch_tm32_compact(tmask, f.pos, nbc, f.bc_brick, f.br_row, f.br_mask, s));
  HIP_TRY(launch_scan_popc64(f.br_mask, nbr, f.br_valptr, scan_tmp, s));
  HIP_TRY(hipMemsetAsync(f.vals + nnz, 0, 64 * sizeof(float), s));
  HIP_TRY(launch_tm32_values(pl->brick_mask, pl->brick_valptr, pl->vals, f.new_slot, f.brick_half,
                             f.pos, f.br_mask, f.br_valptr, nb, f.vals, s));
  HIP_TRY(launch_tm32_meta(f.bc_brick, f.br_row, f.br_mask, f.br_valptr, nbc, nnz, f.meta, n_meta, s));
  HIP_TRY(hipStreamSynchronize(s));
done:
  if (status != SPMM_OK) (void)hipStreamSynchronize(s);
  if (t1.base) (void)hipFree(t1.base);
  if (t2.base) (void)hipFree(t2.base);
  if (status != SPMM_OK) {
    if (keep.base) (void)hipFree(keep.base);
    return status;
  }
  if (pl->tm32.arena) (void)hipFree(pl->tm32.arena);
  pl->tm32 = f;
  return SPMM_OK;
}

// ---- static scratch of spmm_exec_noalloc ------------------------------------------------
// One array per GPU, held until the process ends.  It carries what spmm_exec keeps in
// plan-owned allocations: the work list of the last (plan, N) that used it and the partial
// tiles of split panels.  In host code `scratch` is only a handle for hipGetSymbolAddress;
// the device address is looked up once per device and used everywhere else.
constexpr size_t kScratchBytes = size_t(32) << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
struct ScratchState {
  unsigned char* ptr = nullptr;   // device address of this GPU's copy of `scratch`
  uint64_t list_id = 0;           // HostList whose items the array currently holds (0: none)
};
ScratchState g_scratch[kMaxDevices];
std::mutex g_scratch_mutex;

size_t pad256(size_t b) { return (b + 255) & ~size_t(255); }

// Device address of the current device's copy of `scratch`, looked up on first use per device
// (the runtime materialises the array then; spmm_plan does this so that spmm_exec_noalloc
// itself never changes the amount of free device memory).  Caller holds g_scratch_mutex.
int scratch_state(ScratchState** out) {
  int status = SPMM_OK;
  int dev = 0;
  HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(SPMM_ELIMIT, "device index %d not supported", dev);
  if (!g_scratch[dev].ptr) {
    void* p = nullptr;
    HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    g_scratch[dev].ptr = static_cast<unsigned char*>(p);
  }
  *out = &g_scratch[dev];
done:
  return status;
}

}  // namespace

extern "C" {

const char* spmm_last_error(void) { return g_err; }

int spmm_plan(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
              const float* vals, void* stream_, spmm_plan_t** out) {
  if (!out) return fail(SPMM_EINVAL, "out is NULL");
  *out = nullptr;
  if (M < 0 || K < 0 || nnz < 0) return fail(SPMM_EINVAL, "negative size");
  if (!rowptr) return fail(SPMM_EINVAL, "rowptr is NULL");
  if (nnz > 0 && (!colind || !vals)) return fail(SPMM_EINVAL, "colind/vals is NULL with nnz > 0");
  if (nnz >= (int64_t(1) << 31) || M >= (int64_t(1) << 31) || K >= (int64_t(1) << 31))
    return fail(SPMM_ELIMIT, "M, K and nnz must be below 2^31");

  hipStream_t s = (hipStream_t)stream_;
  int status = SPMM_OK;
  spmm_plan_t* pl = new (std::nothrow) spmm_plan_t();
  if (!pl) return fail(SPMM_ENOMEM, "host allocation failed");
  const int64_t P = (M + kPanel - 1) / kPanel;
  pl->M = M; pl->K = K; pl->nnz = nnz; pl->P = P;

  // Device memory comes from three allocations (four on the search-based path): working
  // arrays (`work`, freed before returning), the plan's fixed-size arrays, and the brick arrays once their
  // count is known.  Sub-arrays are 256-byte aligned.
  auto need = [](int64_t n, size_t elem) { return Arena::pad((size_t)std::max<int64_t>(n, 1) * elem); };
  Arena work, wide, fixed, bricks;
  uint32_t *d_err, *d_span, *d_maxnb, *scan_tmp, *nbricks_p, *panel_nnzptr, *ncols_p;
  enum { kPathSearch, kPathBitmap, kPathSort } path = kPathSearch;
  uint32_t sort_cap = 0;
  uint32_t h_maxnb = 0;
  uint8_t *col_seen, *panel_class;
  unsigned long long *counters, *d_active;
  uint32_t h_small[3] = {0, 0, 0};   // error bits, widest panel span, most entries of a panel
  uint32_t h_err = 0, h_nb = 0, words_cap = 0;
  unsigned long long h_active = 0;
  const int64_t scan_elems = (int64_t)scan_tmp_elems(std::max(nnz, P + 1));  // bricks <= nnz

  // a1 of the search-based path: row of every entry (with the column check), first occurrences,
  // their scan and compacted list, bricks per panel
  auto wide_a1 = [&]() -> int {
    int status = SPMM_OK;
    uint32_t *ent_row, *first_scan, *link, *first_list;
    uint8_t* first;
    wide.cap = need(nnz, 4) + need(nnz, 1) + need(nnz + 1, 4) + need(nnz, 4) + need(nnz, 1) +
               3 * need(nnz, 4);
    HIP_TRY(hipMalloc((void**)&wide.base, wide.cap));
    ent_row = wide.take<uint32_t>(nnz);
    first = wide.take<uint8_t>(nnz);
    first_scan = wide.take<uint32_t>(nnz + 1);
    link = wide.take<uint32_t>(nnz);
    first_list = wide.take<uint32_t>(nnz);
    HIP_TRY(launch_validate_cols(rowptr, colind, M, K, nnz, ent_row, d_err, s));
    HIP_TRY(launch_first_in_panel(rowptr, colind, ent_row, nnz, first, link, s));
    HIP_TRY(launch_scan_u8(first, nnz, first_scan, scan_tmp, s));
    HIP_TRY(launch_compact_first(first, first_scan, nnz, first_list, s));
    HIP_TRY(launch_panel_counts(rowptr, first_scan, M, P, nbricks_p, panel_nnzptr, s));
    HIP_TRY(hipMemsetAsync(d_active, 0, sizeof(unsigned long long), s));
    HIP_TRY(hipMemcpyAsync(d_active, first_scan + nnz, sizeof(uint32_t), hipMemcpyDeviceToDevice, s));
  done:
    return status;
  };

  HIP_TRY(hipGetDevice(&pl->device));
  {   // set-up of the allocation-free entry point: resolve this device's static scratch once
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ScratchState* st = nullptr;
    status = scratch_state(&st);
    if (status != SPMM_OK) goto done;
  }
  HIP_TRY(hipDeviceGetAttribute(&pl->num_cus, hipDeviceAttributeMultiprocessorCount, pl->device));
  pl->num_cus = std::max(1, pl->num_cus);

  work.cap = need(4, 4) + need(scan_elems, 4) + 2 * need(P, 4) + need(P + 1, 4) + need(K, 1) +
                need(P, 1) + need(kNumCounters, 8) + need(1, 8);
  HIP_TRY(hipMalloc((void**)&work.base, work.cap));
  d_err = work.take<uint32_t>(4);   // error bits, widest span, most entries, most columns
  d_span = d_err + 1;
  d_maxnb = d_err + 3;
  scan_tmp = work.take<uint32_t>(scan_elems);
  nbricks_p = work.take<uint32_t>(P);
  ncols_p = work.take<uint32_t>(P);
  panel_nnzptr = work.take<uint32_t>(P + 1);
  col_seen = work.take<uint8_t>(K);
  panel_class = work.take<uint8_t>(P);
  counters = work.take<unsigned long long>(kNumCounters);
  d_active = work.take<unsigned long long>(1);

  fixed.cap = need(P + 1, 4) + need(M + 1, 4) + 3 * need(nnz, 4) +
              need(nnz / long_row_threshold() + 1, 4);
  HIP_TRY(hipMalloc((void**)&fixed.base, fixed.cap));
  pl->fixed_arena = fixed.base;
  pl->panel_ptr = fixed.take<uint32_t>(P + 1);
  pl->rowptr = fixed.take<int32_t>(M + 1);
  pl->colind = fixed.take<int32_t>(nnz);
  pl->csr_vals = fixed.take<float>(nnz);
  pl->ent_pos = fixed.take<uint32_t>(nnz);
  pl->long_rows = fixed.take<uint32_t>(nnz / long_row_threshold() + 1);

  // ---- rowptr validation and the widest panel span (device), before anything trusts rowptr
  HIP_TRY(hipMemsetAsync(d_err, 0, 4 * sizeof(uint32_t), s));
  HIP_TRY(hipMemsetAsync(d_active, 0, sizeof(unsigned long long), s));
  HIP_TRY(launch_validate_rowptr(rowptr, M, nnz, d_err, s));
  HIP_TRY(launch_panel_span(rowptr, colind, M, P, d_err, d_span, s));
  HIP_TRY(hipMemcpyAsync(h_small, d_err, 3 * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  h_err = h_small[0];
  if (h_err & (kErrRowptrEnds | kErrRowptrOrder)) {
    status = fail(SPMM_EFORMAT, "invalid rowptr (%s)",
                  (h_err & kErrRowptrEnds) ? "rowptr[0] != 0 or rowptr[M] != nnz" : "not monotone");
    goto done;
  }
  if (h_err & (kErrColRange | kErrColOrder)) {   // a panel whose column span is inverted
    status = fail(SPMM_EFORMAT, "invalid colind (columns of a row not strictly ascending)");
    goto done;
  }
  words_cap = panel_bitmap_words(h_small[1]);

  // Three ways to the same format.  The bitmap kernels walk a bitmap over the panel's column
  // span; that pays while the bitmaps are not much longer than the entry lists (band-like
  // matrices).  Scattered matrices (power-law graphs, random bricks: spans near K) sort each
  // panel's entries in LDS instead when panels are well filled and none is large (the sort
  // costs a fixed network per panel and LDS per wavefront); everything else takes the
  // search-based kernels.  Measured: config 5 (bitmap words x panels = 4 x nnz) 0.6 vs 1.0 ms
  // (search) in favour of the bitmap, config 3 (360 x) 4.0 vs 0.9 ms and the 1M-row sweep
  // (67 x) 31 vs 3.8 ms against it; sort against search: 1M-row sweep f = 0.4 (488 entries
  // per panel) 2.4 vs 4.5 ms, f = 0.8 3.8 vs 3.8 ms, config 3 (46 per panel, largest 3000+)
  // 1.45 vs 0.99 ms.
  sort_cap = panel_sort_keys(h_small[2]);
  if (words_cap != 0 && (int64_t)words_cap * P <= 8 * nnz) path = kPathBitmap;
  else if (sort_cap != 0 && sort_cap <= 2048 && nnz >= 128 * P) path = kPathSort;
  if (path == kPathBitmap) {
    // ---- a1/a2: census (also validates colind) -> bricks per panel
    HIP_TRY(launch_panel_census(rowptr, colind, M, K, P, words_cap, d_err, nbricks_p, panel_nnzptr,
                                ncols_p, d_active, d_maxnb, s));
  } else if (path == kPathSort) {
    HIP_TRY(launch_panel_sort_census(rowptr, colind, M, K, P, sort_cap, d_err, nbricks_p,
                                     panel_nnzptr, ncols_p, pl->ent_pos, d_active, d_maxnb, s));
  } else {
    // ---- search-based path for every other matrix.  Its a1
    // kernels only compare columns, so they may run before the host has seen the verdict of
    // the column check; everything that indexes by column or rank runs after it.
    status = wide_a1();
    if (status != SPMM_OK) goto done;
  }
  HIP_TRY(launch_scan_u32(nbricks_p, P, pl->panel_ptr, scan_tmp, s));
  HIP_TRY(hipMemcpyAsync(&h_nb, pl->panel_ptr + P, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync(&h_active, d_active, sizeof(unsigned long long), hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync(&h_err, d_err, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  if (path != kPathSearch)
    HIP_TRY(hipMemcpyAsync(&h_maxnb, d_maxnb, sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  // plan-owned CSR copy for the vector-ALU kernel, while the host waits for the counts
  HIP_TRY(hipMemcpyAsync(pl->rowptr, rowptr, (size_t)(M + 1) * sizeof(int32_t),
                         hipMemcpyDeviceToDevice, s));
  if (nnz > 0) {
    HIP_TRY(hipMemcpyAsync(pl->colind, colind, (size_t)nnz * sizeof(int32_t),
                           hipMemcpyDeviceToDevice, s));
    HIP_TRY(hipMemcpyAsync(pl->csr_vals, vals, (size_t)nnz * sizeof(float),
                           hipMemcpyDeviceToDevice, s));
  }
  HIP_TRY(hipStreamSynchronize(s));
  if (h_err) {
    status = fail(SPMM_EFORMAT, "invalid colind (%s)",
                  (h_err & kErrColRange) ? "column out of range"
                                         : "columns of a row not strictly ascending");
    goto done;
  }
  pl->nb = h_nb;
  pl->n_active_cols = (int64_t)h_active;
  if ((int64_t)h_nb * kBrickK >= (int64_t(1) << 32)) {
    status = fail(SPMM_ELIMIT, "4 * bricks must be below 2^32");
    goto done;
  }

  h_maxnb = (h_maxnb + kBrickK - 1) / kBrickK;   // read back as the largest column count of a panel
  if ((path == kPathBitmap && !panel_build_fits(words_cap, std::max<uint32_t>(h_maxnb, 1))) ||
      (path == kPathSort && !panel_sort_build_fits(sort_cap, std::max<uint32_t>(h_maxnb, 1)))) {
    path = kPathSearch;   // a panel with more bricks than fit in LDS: finish on the search-based path
    status = wide_a1();
    if (status != SPMM_OK) goto done;
  }

  // ---- brick arrays (they carry spare entries, see BrickFormat)
  bricks.cap = need((pl->nb + kFormatPad) * kBrickK, 4) + need(pl->nb + kFormatPad, 8) +
               need(pl->nb + 1 + kFormatPad, 4) + need(nnz + 64, 4);
  HIP_TRY(hipMalloc((void**)&bricks.base, bricks.cap));
  pl->brick_arena = bricks.base;
  pl->brick_cols = bricks.take<uint32_t>((pl->nb + kFormatPad) * kBrickK);
  pl->brick_mask = bricks.take<uint64_t>(pl->nb + kFormatPad);
  pl->brick_valptr = bricks.take<uint32_t>(pl->nb + 1 + kFormatPad);
  pl->vals = bricks.take<float>(nnz + 64);
  HIP_TRY(hipMemsetAsync(pl->brick_cols + pl->nb * kBrickK, 0, kFormatPad * kBrickK * 4, s));
  HIP_TRY(hipMemsetAsync(pl->brick_mask, 0, (size_t)(pl->nb + kFormatPad) * 8, s));
  HIP_TRY(launch_fill_u32(pl->brick_valptr + pl->nb, kFormatPad + 1, (uint32_t)nnz, s));
  HIP_TRY(hipMemsetAsync(pl->vals + nnz, 0, 64 * sizeof(float), s));
  HIP_TRY(hipMemsetAsync(col_seen, 0, (size_t)std::max<int64_t>(K, 1), s));
  HIP_TRY(hipMemsetAsync(counters, 0, kNumCounters * sizeof(unsigned long long), s));

  if (path == kPathSort) {
    HIP_TRY(launch_panel_sort_build(rowptr, colind, vals, M, K, P, sort_cap,
                                    std::max<uint32_t>(h_maxnb, 1), pl->panel_ptr, pl->brick_cols,
                                    pl->brick_mask, pl->brick_valptr, pl->vals, pl->ent_pos,
                                    col_seen, s));
  } else if (path == kPathBitmap) {
    // ---- a2 (placing), a3, a4, one wavefront per panel
    HIP_TRY(launch_panel_build(rowptr, colind, vals, M, K, P, words_cap,
                               std::max<uint32_t>(h_maxnb, 1), pl->panel_ptr,
                               pl->brick_cols, pl->brick_mask, pl->brick_valptr, pl->vals,
                               pl->ent_pos, col_seen, s));
  } else {
    // the arrays of the search-based path, in the order they were carved above
    Arena again = wide;
    again.used = 0;
    uint32_t* ent_row = again.take<uint32_t>(nnz);
    (void)again.take<uint8_t>(nnz);
    uint32_t* first_scan = again.take<uint32_t>(nnz + 1);
    uint32_t* link = again.take<uint32_t>(nnz);
    uint32_t* first_list = again.take<uint32_t>(nnz);
    uint32_t* ent_brick = again.take<uint32_t>(nnz);
    uint8_t* ent_bit = again.take<uint8_t>(nnz);
    uint32_t* ent_rank = again.take<uint32_t>(nnz);
    HIP_TRY(launch_fill_u32(pl->brick_cols, pl->nb * kBrickK, kPadCol, s));
    HIP_TRY(launch_rank_first(rowptr, colind, ent_row, first_list, first_scan, pl->panel_ptr, M,
                              pl->n_active_cols, ent_rank, pl->brick_cols, s));
    HIP_TRY(launch_scatter_bits(colind, ent_row, link, ent_rank, pl->panel_ptr, nnz,
                                pl->brick_mask, ent_brick, ent_bit, col_seen, s));
    HIP_TRY(launch_scan_popc64(pl->brick_mask, pl->nb, pl->brick_valptr, scan_tmp, s));
    HIP_TRY(launch_pack_values(vals, ent_brick, ent_bit, pl->brick_mask, pl->brick_valptr, nnz,
                               pl->vals, pl->ent_pos, s));
  }
  // ---- a5: per-panel classes and the synergy counts
  HIP_TRY(launch_panel_classes(pl->panel_ptr, panel_nnzptr, P, panel_class, counters, s));
  HIP_TRY(launch_brick_hist(pl->brick_mask, pl->nb, counters, s));
  HIP_TRY(launch_count_flags(col_seen, K, counters + kCntDistinctCols, s));
  HIP_TRY(launch_find_long_rows(rowptr, M, long_row_threshold(), pl->long_rows,
                                counters + kCntLongRows, s));

  // ---- host copies for the work-list builder and the model
  try {
    pl->h_panel_ptr.resize((size_t)P + 1);
    pl->h_panel_nnzptr.resize((size_t)P + 1);
    pl->h_panel_class.resize((size_t)std::max<int64_t>(P, 1));
  } catch (const std::bad_alloc&) {
    status = fail(SPMM_ENOMEM, "host allocation failed");
    goto done;
  }
  HIP_TRY(hipMemcpyAsync(pl->h_panel_ptr.data(), pl->panel_ptr, (size_t)(P + 1) * sizeof(uint32_t),
                         hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync(pl->h_panel_nnzptr.data(), panel_nnzptr, (size_t)(P + 1) * sizeof(uint32_t),
                         hipMemcpyDeviceToHost, s));
  if (P > 0)
    HIP_TRY(hipMemcpyAsync(pl->h_panel_class.data(), panel_class, (size_t)P,
                           hipMemcpyDeviceToHost, s));
  HIP_TRY(hipMemcpyAsync(pl->h_counters, counters, kNumCounters * sizeof(unsigned long long),
                         hipMemcpyDeviceToHost, s));
  HIP_TRY(hipStreamSynchronize(s));
  pl->n_long_rows = (int64_t)pl->h_counters[kCntLongRows];

done:
  if (status != SPMM_OK) (void)hipStreamSynchronize(s);
  if (work.base) (void)hipFree(work.base);
  if (wide.base) (void)hipFree(wide.base);
  if (status != SPMM_OK) {
    delete pl;
    return status;
  }
  *out = pl;
  return SPMM_OK;
}

int spmm_plan_update_values(spmm_plan_t* pl, const float* vals, void* stream_) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (pl->nnz > 0 && !vals) return fail(SPMM_EINVAL, "vals is NULL with nnz > 0");
  int status = SPMM_OK;
  HIP_TRY(launch_update_values(vals, pl->ent_pos, pl->nnz, pl->vals, pl->csr_vals,
                               (hipStream_t)stream_));
  if (pl->tm32.arena)   // the 32-row format holds its own copy of the packed values
    HIP_TRY(launch_tm32_values(pl->brick_mask, pl->brick_valptr, pl->vals, pl->tm32.new_slot,
                               pl->tm32.brick_half, pl->tm32.pos, pl->tm32.br_mask,
                               pl->tm32.br_valptr, pl->nb, pl->tm32.vals, (hipStream_t)stream_));
done:
  return status;
}

namespace {

bool ptr_is_aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int check_exec_args(const spmm_plan_t* pl, const float* B, int64_t N, const float* C) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (N < 0) return fail(SPMM_EINVAL, "N is negative");
  if (N == 0 || pl->M == 0) return 1;   // nothing to do
  if (!C) return fail(SPMM_EINVAL, "C is NULL");
  if (!B && pl->K > 0) return fail(SPMM_EINVAL, "B is NULL");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != pl->device)
    return fail(SPMM_EINVAL, "the plan was made on device %d, the current device is %d",
                pl->device, dev);
  return SPMM_OK;
}

// The 32-row kernel serves the whole matrix when the plan has that format, every panel is routed
// to the MFMA kernel, the arithmetic is FP32 and the shape is the fast kernel's.
bool uses_tm32(const spmm_plan_t* pl, const float* B, int64_t N, const float* C) {
  if (pl->panel_height != 32 || !pl->tm32.arena) return false;
  if (pl->route != SPMM_ROUTE_AUTO && pl->route != SPMM_ROUTE_MFMA) return false;
  if (pl->precision != SPMM_PRECISION_FP32) return false;
  if (pl->nnz + 64 >= (int64_t(1) << 30)) return false;   // the kernel's 32-bit value offsets
  return mfma_fast_shape(N, pl->K) && ptr_is_aligned16(B) && ptr_is_aligned16(C);
}

// the three launches of one product; every pointer is a device pointer
int launch_product(const spmm_plan_t* pl, const HostList* hl, const WorkItem* d_items,
                   const uint32_t* d_valu_panels, const MergeItem* d_merge, float* d_partial,
                   const float* B, int64_t N, float* C, hipStream_t s) {
  int status = SPMM_OK;
  const BrickFormat f{pl->brick_cols, pl->brick_mask, pl->brick_valptr, pl->vals};
  if (uses_tm32(pl, B, N, C)) {
    // 32-row panels: one wavefront per super-panel and column tile, no work list
    HIP_TRY(launch_spmm_tm32(pl->tm32.sp_ptr, pl->tm32.bc_cols, pl->tm32.meta, pl->tm32.vals,
                             pl->tm32.Q, B, C, pl->M, N, pl->K, s));
    return SPMM_OK;
  }
  {
    const int tile = mfma_tile_for(N);
    const int V = tile >= 64 ? 4 : tile / 16;
    const bool aligned = N % V == 0 && ptr_is_aligned16(B) && ptr_is_aligned16(C) &&
                         (d_partial == nullptr || ptr_is_aligned16(d_partial));
    if (pl->precision != SPMM_PRECISION_FP32 && aligned && bf16_path_shape(N, pl->K))
      HIP_TRY(launch_spmm_bf16(f, d_items, hl->info.n_mfma_items, B, C, d_partial, pl->M, N, pl->K,
                               pl->precision == SPMM_PRECISION_BF16X3 ? 2 : 3, pl->nnz, s));
    else if (pl->tile_sharing == SPMM_SHARE_WORKGROUP && aligned && mfma_wide_waves(N, pl->K) > 0)
      HIP_TRY(launch_spmm_mfma_wide(f, d_items, hl->info.n_mfma_items, B, C, d_partial, pl->M, N,
                                    pl->K, s));
    else
      HIP_TRY(launch_spmm_mfma(f, d_items, hl->info.n_mfma_items, B, C, d_partial, pl->M, N, pl->K,
                               pl->nnz, s));
  }
  HIP_TRY(launch_spmm_valu(pl->rowptr, pl->colind, pl->csr_vals, d_valu_panels,
                           hl->info.n_valu_panels, pl->long_rows, pl->n_long_rows, B, C, pl->M, N,
                           s));
  HIP_TRY(launch_merge(d_merge, (int64_t)hl->merges.size(), d_partial, C, pl->M, N, s));
done:
  return status;
}

}  // namespace

int spmm_exec(spmm_plan_t* pl, const float* B, int64_t N, float* C, void* stream_) {
  int status = check_exec_args(pl, B, N, C);
  if (status != SPMM_OK) return status > 0 ? SPMM_OK : status;
  hipStream_t s = (hipStream_t)stream_;
  WorkList* wl = nullptr;
  status = build_worklist(pl, N, s, &wl);
  if (status != SPMM_OK) return status;
  return launch_product(pl, wl->host, wl->d_items, wl->d_valu_panels, wl->d_merge, wl->d_partial,
                        B, N, C, s);
}

int spmm_exec_noalloc(spmm_plan_t* pl, const float* B, int64_t N, float* C, void* stream_) {
  int status = check_exec_args(pl, B, N, C);
  if (status != SPMM_OK) return status > 0 ? SPMM_OK : status;
  hipStream_t s = (hipStream_t)stream_;
  const HostList* hl = nullptr;
  status = build_host_list(pl, N, &hl);   // host arithmetic only; cached per N
  if (status != SPMM_OK) return status;

  const size_t items_b = pad256(hl->items.size() * sizeof(WorkItem));
  const size_t valu_b = pad256(hl->valu_panels.size() * sizeof(uint32_t));
  const size_t merge_b = pad256(hl->merges.size() * sizeof(MergeItem));
  const size_t partial_b = (size_t)hl->n_slots * kPanel * (size_t)N * sizeof(float);
  if (items_b + valu_b + merge_b + partial_b > kScratchBytes)
    return fail(SPMM_ELIMIT,
                "spmm_exec_noalloc: work list (%zu B) and partial tiles of split panels (%zu B) "
                "exceed the static scratch of %zu B; use spmm_exec",
                items_b + valu_b + merge_b, partial_b, kScratchBytes);

  {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    ScratchState* stp = nullptr;
    status = scratch_state(&stp);
    if (status != SPMM_OK) return status;
    ScratchState& st = *stp;
    unsigned char* base = st.ptr;
    WorkItem* d_items = reinterpret_cast<WorkItem*>(base);
    uint32_t* d_valu = reinterpret_cast<uint32_t*>(base + items_b);
    MergeItem* d_merge = reinterpret_cast<MergeItem*>(base + items_b + valu_b);
    float* d_partial = reinterpret_cast<float*>(base + items_b + valu_b + merge_b);
    if (st.list_id != hl->id) {
      // the array holds another list: bring this one in (copies from plan-owned host memory
      // that lives as long as the list; ordered on `s` before the kernels below)
      st.list_id = 0;
      if (!hl->items.empty())
        HIP_TRY(hipMemcpyAsync(d_items, hl->items.data(), hl->items.size() * sizeof(WorkItem),
                               hipMemcpyHostToDevice, s));
      if (!hl->valu_panels.empty())
        HIP_TRY(hipMemcpyAsync(d_valu, hl->valu_panels.data(),
                               hl->valu_panels.size() * sizeof(uint32_t), hipMemcpyHostToDevice, s));
      if (!hl->merges.empty())
        HIP_TRY(hipMemcpyAsync(d_merge, hl->merges.data(), hl->merges.size() * sizeof(MergeItem),
                               hipMemcpyHostToDevice, s));
      st.list_id = hl->id;
    }
    // Partial tiles need no clearing: every part of a split panel overwrites its whole tile
    // before the merge kernel reads it.
    status = launch_product(pl, hl, d_items, d_valu, d_merge, hl->n_slots ? d_partial : nullptr,
                            B, N, C, s);
    if (status != SPMM_OK) st.list_id = 0;
  }
done:
  return status;
}

int spmm_synergy(const spmm_plan_t* pl, int64_t N, spmm_synergy_t* o) {
  if (!pl || !o) return fail(SPMM_EINVAL, "NULL argument");
  if (N < 0) return fail(SPMM_EINVAL, "N is negative");
  memset(o, 0, sizeof(*o));
  o->M = pl->M; o->K = pl->K; o->nnz = pl->nnz;
  o->n_panels = pl->P;
  o->n_nonempty_panels = (int64_t)pl->h_counters[kCntNonEmptyPanels];
  o->n_bricks = pl->nb;
  o->n_active_cols = pl->n_active_cols;
  o->n_distinct_cols = (int64_t)pl->h_counters[kCntDistinctCols];
  for (int c = 0; c < 3; ++c) {
    o->panels_by_class[c] = (int64_t)pl->h_counters[kCntPanelsByClass + c];
    o->bricks_by_class[c] = (int64_t)pl->h_counters[kCntBricksByClass + c];
    o->nnz_by_class[c] = (int64_t)pl->h_counters[kCntNnzByClass + c];
  }
  for (int k = 0; k < 65; ++k) o->brick_pop_hist[k] = (int64_t)pl->h_counters[kCntPopHist + k];
  o->synergy_class = classify(pl->nnz, pl->nb);
  const double nnz = (double)pl->nnz, nb = (double)pl->nb, n = (double)N;
  o->alpha_brick = pl->nb ? nnz / (64.0 * nb) : 0.0;
  o->alpha_col = pl->n_active_cols ? nnz / (16.0 * (double)pl->n_active_cols) : 0.0;
  o->beta = 1.0;
  o->oi_shmem = 512.0 * o->alpha_brick * o->beta;
  const double a_bytes = 4.0 * nnz + 28.0 * nb + 4.0 + 4.0 * (double)(pl->P + 1);
  o->bytes_min = a_bytes + 4.0 * n * (double)o->n_distinct_cols + 4.0 * n * (double)pl->M;
  o->bytes_noreuse = a_bytes + 4.0 * n * (double)o->n_active_cols + 4.0 * n * (double)pl->M;
  const double flops = 2.0 * nnz * n;
  o->oi_hbm_min = flops / o->bytes_min;
  o->oi_hbm_noreuse = flops / o->bytes_noreuse;
  o->roof_gflops_hbm = o->oi_hbm_min * kHbmBytesPerS * 1e-9;
  o->roof_gflops_mfma = o->alpha_brick * kMfmaFp32Flops * 1e-9;
  return SPMM_OK;
}

int spmm_plan_sizes(const spmm_plan_t* pl, spmm_sizes_t* o) {
  if (!pl || !o) return fail(SPMM_EINVAL, "NULL argument");
  o->M = pl->M; o->K = pl->K; o->nnz = pl->nnz; o->n_panels = pl->P; o->n_bricks = pl->nb;
  return SPMM_OK;
}

int spmm_plan_export(const spmm_plan_t* pl, uint32_t* panel_ptr, uint32_t* brick_cols,
                     uint64_t* brick_mask, uint32_t* brick_valptr, float* vals) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  int status = SPMM_OK;
  HIP_TRY(hipDeviceSynchronize());
  if (panel_ptr)
    HIP_TRY(hipMemcpy(panel_ptr, pl->panel_ptr, (size_t)(pl->P + 1) * 4, hipMemcpyDeviceToHost));
  if (brick_cols && pl->nb)
    HIP_TRY(hipMemcpy(brick_cols, pl->brick_cols, (size_t)pl->nb * 16, hipMemcpyDeviceToHost));
  if (brick_mask && pl->nb)
    HIP_TRY(hipMemcpy(brick_mask, pl->brick_mask, (size_t)pl->nb * 8, hipMemcpyDeviceToHost));
  if (brick_valptr)
    HIP_TRY(hipMemcpy(brick_valptr, pl->brick_valptr, (size_t)(pl->nb + 1) * 4,
                      hipMemcpyDeviceToHost));
  if (vals && pl->nnz)
    HIP_TRY(hipMemcpy(vals, pl->vals, (size_t)pl->nnz * 4, hipMemcpyDeviceToHost));
done:
  return status;
}

int spmm_plan_set_route(spmm_plan_t* pl, int route) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (route < SPMM_ROUTE_AUTO || route > SPMM_ROUTE_CLASS) return fail(SPMM_EINVAL, "bad route");
  if (hipDeviceSynchronize() != hipSuccess) return fail(SPMM_EHIP, "hipDeviceSynchronize failed");
  pl->route = route;
  pl->drop_lists();
  return SPMM_OK;
}

int spmm_plan_set_split(spmm_plan_t* pl, int parts) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (parts < SPMM_SPLIT_EQ7_NEAREST) return fail(SPMM_EINVAL, "unknown split policy");
  if (hipDeviceSynchronize() != hipSuccess) return fail(SPMM_EHIP, "hipDeviceSynchronize failed");
  pl->split = parts;
  pl->drop_lists();
  return SPMM_OK;
}

int spmm_plan_set_precision(spmm_plan_t* pl, int precision) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (precision < SPMM_PRECISION_FP32 || precision > SPMM_PRECISION_BF16X6)
    return fail(SPMM_EINVAL, "unknown precision");
  if (hipDeviceSynchronize() != hipSuccess) return fail(SPMM_EHIP, "hipDeviceSynchronize failed");
  pl->precision = precision;
  pl->drop_lists();   // the kernels differ in occupancy, which Eq. 7 uses
  return SPMM_OK;
}

int spmm_plan_set_tile_sharing(spmm_plan_t* pl, int mode) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (mode != SPMM_SHARE_NONE && mode != SPMM_SHARE_WORKGROUP)
    return fail(SPMM_EINVAL, "unknown tile-sharing mode");
  pl->tile_sharing = mode;   // work lists do not depend on it
  return SPMM_OK;
}

int spmm_plan_set_panel_height(spmm_plan_t* pl, int rows, uint32_t merge_num, uint32_t merge_den,
                               void* stream_) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (rows != 16 && rows != 32) return fail(SPMM_EINVAL, "panel height must be 16 or 32");
  if (rows == 32 && merge_den == 0) return fail(SPMM_EINVAL, "merge_den is zero");
  if (hipDeviceSynchronize() != hipSuccess) return fail(SPMM_EHIP, "hipDeviceSynchronize failed");
  if (rows == 32) {
    const int status = build_tm32(pl, merge_num, merge_den, (hipStream_t)stream_);
    if (status != SPMM_OK) return status;
  }
  pl->panel_height = rows;
  return SPMM_OK;
}

int spmm_plan_tm32_sizes(const spmm_plan_t* pl, spmm_tm32_sizes_t* o) {
  if (!pl || !o) return fail(SPMM_EINVAL, "NULL argument");
  if (!pl->tm32.arena) return fail(SPMM_EINVAL, "the plan has no 32-row format");
  o->n_super_panels = pl->tm32.Q;
  o->n_brick_cols = pl->tm32.nbc;
  o->n_bricks = pl->tm32.nbr;
  o->n_merged = pl->tm32.n_merged;
  return SPMM_OK;
}

int spmm_plan_tm32_export(const spmm_plan_t* pl, uint32_t* sp_ptr, uint8_t* sp_merged,
                          uint32_t* bc_cols, uint32_t* bc_brick, uint8_t* br_row, uint64_t* br_mask,
                          uint32_t* br_valptr, float* vals) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (!pl->tm32.arena) return fail(SPMM_EINVAL, "the plan has no 32-row format");
  int status = SPMM_OK;
  const auto& f = pl->tm32;
  HIP_TRY(hipDeviceSynchronize());
  if (sp_ptr) HIP_TRY(hipMemcpy(sp_ptr, f.sp_ptr, (size_t)(f.Q + 1) * 4, hipMemcpyDeviceToHost));
  if (sp_merged && f.Q) HIP_TRY(hipMemcpy(sp_merged, f.sp_merged, (size_t)f.Q, hipMemcpyDeviceToHost));
  if (bc_cols && f.nbc) HIP_TRY(hipMemcpy(bc_cols, f.bc_cols, (size_t)f.nbc * 16, hipMemcpyDeviceToHost));
  if (bc_brick) HIP_TRY(hipMemcpy(bc_brick, f.bc_brick, (size_t)(f.nbc + 1) * 4, hipMemcpyDeviceToHost));
  if (br_row && f.nbr) HIP_TRY(hipMemcpy(br_row, f.br_row, (size_t)f.nbr, hipMemcpyDeviceToHost));
  if (br_mask && f.nbr) HIP_TRY(hipMemcpy(br_mask, f.br_mask, (size_t)f.nbr * 8, hipMemcpyDeviceToHost));
  if (br_valptr) HIP_TRY(hipMemcpy(br_valptr, f.br_valptr, (size_t)(f.nbr + 1) * 4, hipMemcpyDeviceToHost));
  if (vals && pl->nnz) HIP_TRY(hipMemcpy(vals, f.vals, (size_t)pl->nnz * 4, hipMemcpyDeviceToHost));
done:
  return status;
}

int spmm_plan_set_order(spmm_plan_t* pl, int order) {
  if (!pl) return fail(SPMM_EINVAL, "plan is NULL");
  if (order != SPMM_ORDER_PANEL && order != SPMM_ORDER_HEAVY_FIRST)
    return fail(SPMM_EINVAL, "unknown order");
  if (hipDeviceSynchronize() != hipSuccess) return fail(SPMM_EHIP, "hipDeviceSynchronize failed");
  pl->order = order;
  pl->drop_lists();
  return SPMM_OK;
}

int spmm_partition_counts(int64_t n_panels, const uint32_t* nbricks, int64_t work_items,
                          int32_t num_cus, int32_t resident_per_cu, int32_t policy,
                          uint32_t* parts_out, int64_t* waves_out) {
  if (n_panels < 0 || work_items < 0 || num_cus < 1 || resident_per_cu < 1 ||
      (policy != SPMM_SPLIT_EQ7_FROM2 && policy != SPMM_SPLIT_EQ7_NEAREST))
    return fail(SPMM_EINVAL, "bad argument");
  if (n_panels > 0 && (!nbricks || !parts_out)) return fail(SPMM_EINVAL, "NULL argument");
  partition_counts(n_panels, nbricks, work_items, (int64_t)num_cus * resident_per_cu, policy,
                   parts_out, waves_out);
  return SPMM_OK;
}

int spmm_plan_worklist(spmm_plan_t* pl, int64_t N, spmm_worklist_info_t* info,
                       spmm_work_item_t* items, uint32_t* valu_panels) {
  if (!pl || !info) return fail(SPMM_EINVAL, "NULL argument");
  if (N < 1) return fail(SPMM_EINVAL, "N must be positive");
  const HostList* hl = nullptr;
  const int status = build_host_list(pl, N, &hl);
  if (status != SPMM_OK) return status;
  *info = hl->info;
  if (items && !hl->h_items.empty())
    memcpy(items, hl->h_items.data(), hl->h_items.size() * sizeof(spmm_work_item_t));
  if (valu_panels && !hl->valu_panels.empty())
    memcpy(valu_panels, hl->valu_panels.data(), hl->valu_panels.size() * sizeof(uint32_t));
  return SPMM_OK;
}

void spmm_plan_destroy(spmm_plan_t* pl) {
  if (!pl) return;
  (void)hipDeviceSynchronize();
  delete pl;
}

}  // extern "C"
