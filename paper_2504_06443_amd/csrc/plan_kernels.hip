// CSR -> brick format on the GPU (paper Section 3.2: active-column compaction,
// bricks of 4 columns, 64-bit pattern per brick, values packed row-major).
//
// No kernel waits on another workgroup; the only atomics are integer OR / ADD / MAX,
// so every output is reproducible bit for bit.
//
// Two ways to find a panel's active columns and their ranks, neither of which sorts:
//  * search-based (any matrix): the rows of a panel are already sorted, so "is this the
//    first row of the panel that holds column j" and "how many distinct columns of the
//    panel are smaller than j" are answered by binary searches in the (at most 16) rows of
//    the panel plus one exclusive scan of the first-occurrence flags over the whole entry
//    array.  The second question is only asked once per active column (the
//    first-occurrence entries, compacted into a list); the other entries of that column
//    follow a link to it.  One thread per entry (or per row / panel / brick).
//  * per-panel (matrices whose panels span few columns compared with their entries): one
//    wavefront per panel keeps a bitmap of the panel's column span in LDS; see the section
//    "per-panel path" below.
#include "spmm_internal.h"

#include <algorithm>

namespace spmm {

namespace {

constexpr int kThreads = 256;

inline unsigned grid_for(int64_t n, int threads = kThreads) {
  int64_t g = (n + threads - 1) / threads;
  return (unsigned)(g > 0 ? g : 1);
}

// first index in [lo, hi) whose column is >= j
__device__ inline int64_t lower_bound_col(const int32_t* __restrict__ colind, int64_t lo,
                                          int64_t hi, int32_t j) {
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if (colind[mid] < j) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// ---------------------------------------------------------------- validation
__global__ void k_validate_rowptr(const int32_t* __restrict__ rowptr, int64_t M, int64_t nnz,
                                  uint32_t* err) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i > M) return;
  uint32_t e = 0;
  const int64_t a = rowptr[i];
  if (i == 0 && a != 0) e |= kErrRowptrEnds;
  if (i == M && a != nnz) e |= kErrRowptrEnds;
  if (a < 0 || a > nnz) e |= kErrRowptrOrder;
  if (i < M) {
    const int64_t b = rowptr[i + 1];
    if (b < a) e |= kErrRowptrOrder;
  }
  if (e) atomicOr(err, e);
}

// Requires a valid rowptr.  Also records the row of every entry.
__global__ void k_validate_cols(const int32_t* __restrict__ rowptr,
                                const int32_t* __restrict__ colind, int64_t M, int64_t K,
                                int64_t nnz, uint32_t* __restrict__ ent_row, uint32_t* err) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  int64_t lo = 0, hi = M;  // rowptr[lo] <= e < rowptr[hi]
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (rowptr[mid] <= e) lo = mid; else hi = mid;
  }
  ent_row[e] = (uint32_t)lo;
  const int64_t j = colind[e];
  uint32_t bad = 0;
  if (j < 0 || j >= K) bad |= kErrColRange;
  if (e > rowptr[lo] && colind[e - 1] >= j) bad |= kErrColOrder;
  if (bad) atomicOr(err, bad);
}

// ---------------------------------------------------------------- a1 census
// first[e] = 1 iff no earlier row of the same panel stores column colind[e].
// link[e] = the entry of that first row that stores the same column (e itself if first).
__global__ void k_first_in_panel(const int32_t* __restrict__ rowptr,
                                 const int32_t* __restrict__ colind,
                                 const uint32_t* __restrict__ ent_row, int64_t nnz,
                                 uint8_t* __restrict__ first, uint32_t* __restrict__ link) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const int64_t i = ent_row[e];
  const int32_t j = colind[e];
  const int64_t r0 = i & ~(int64_t)(kPanel - 1);
  uint8_t f = 1;
  int64_t where = e;
  for (int64_t r = r0; r < i; ++r) {  // rows in ascending order: the first hit is the first occurrence
    const int64_t s = rowptr[r], t = rowptr[r + 1];
    const int64_t pos = lower_bound_col(colind, s, t, j);
    if (pos < t && colind[pos] == j) { f = 0; where = pos; break; }
  }
  first[e] = f;
  link[e] = (uint32_t)where;
}

// first_list[k] = the k-th first-occurrence entry (k = exclusive scan of the flags)
__global__ void k_compact_first(const uint8_t* __restrict__ first,
                                const uint32_t* __restrict__ first_scan, int64_t nnz,
                                uint32_t* __restrict__ first_list) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < nnz && first[e]) first_list[first_scan[e]] = (uint32_t)e;
}

// a2: bricks per panel and the entry offset of each panel.
__global__ void k_panel_counts(const int32_t* __restrict__ rowptr,
                               const uint32_t* __restrict__ first_scan, int64_t M, int64_t P,
                               uint32_t* __restrict__ nbricks_p,
                               uint32_t* __restrict__ panel_nnzptr) {
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p > P) return;
  const int64_t r0 = min(p * kPanel, M);
  const int64_t e0 = rowptr[r0];
  panel_nnzptr[p] = (uint32_t)e0;
  if (p < P) {
    const int64_t r1 = min(r0 + kPanel, M);
    const uint32_t ncols = first_scan[rowptr[r1]] - first_scan[e0];
    nbricks_p[p] = (ncols + kBrickK - 1) / kBrickK;
  }
}

template <typename T>
__global__ void k_fill(T* __restrict__ p, int64_t n, T v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// a2: one thread per active column (= per first-occurrence entry): its rank among the
// panel's active columns = number of first-occurrence entries of the panel with a smaller
// column, counted row by row with one binary search and two reads of the scanned flags.
__global__ void k_rank_first(const int32_t* __restrict__ rowptr,
                             const int32_t* __restrict__ colind,
                             const uint32_t* __restrict__ ent_row,
                             const uint32_t* __restrict__ first_list,
                             const uint32_t* __restrict__ first_scan,
                             const uint32_t* __restrict__ panel_ptr, int64_t M, int64_t n_active,
                             uint32_t* __restrict__ ent_rank, uint32_t* __restrict__ brick_cols) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_active) return;
  const int64_t e = first_list[k];
  const int64_t i = ent_row[e];
  const int32_t j = colind[e];
  const int64_t p = i / kPanel;
  const int64_t r0 = p * kPanel, r1 = min(r0 + kPanel, M);
  uint32_t rank = 0;
  for (int64_t r = r0; r < r1; ++r) {
    const int64_t s = rowptr[r], t = rowptr[r + 1];
    const int64_t pos = (r == i) ? e : lower_bound_col(colind, s, t, j);
    rank += first_scan[pos] - first_scan[s];
  }
  ent_rank[e] = rank;
  brick_cols[(int64_t)panel_ptr[p] * kBrickK + rank] = (uint32_t)j;
}

// a3: every entry takes the rank of its column's first occurrence, which gives its brick,
// its brick column and its pattern bit 4*row + column.
__global__ void k_scatter_bits(const int32_t* __restrict__ colind,
                               const uint32_t* __restrict__ ent_row,
                               const uint32_t* __restrict__ link,
                               const uint32_t* __restrict__ ent_rank,
                               const uint32_t* __restrict__ panel_ptr, int64_t nnz,
                               uint64_t* brick_mask, uint32_t* __restrict__ ent_brick,
                               uint8_t* __restrict__ ent_bit, uint8_t* __restrict__ col_seen) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const int64_t i = ent_row[e];
  const uint32_t rank = ent_rank[link[e]];
  const uint32_t b = panel_ptr[i / kPanel] + rank / kBrickK;
  const uint32_t c = rank % kBrickK;
  const uint32_t bit = (uint32_t)(i % kPanel) * kBrickK + c;
  atomicOr((unsigned long long*)&brick_mask[b], 1ull << bit);
  ent_brick[e] = b;
  ent_bit[e] = (uint8_t)bit;
  col_seen[colind[e]] = 1;
}

// a4: position of a value = start of its brick + set bits below its own bit.
__global__ void k_pack_values(const float* __restrict__ vals,
                              const uint32_t* __restrict__ ent_brick,
                              const uint8_t* __restrict__ ent_bit,
                              const uint64_t* __restrict__ brick_mask,
                              const uint32_t* __restrict__ brick_valptr, int64_t nnz,
                              float* __restrict__ packed, uint32_t* __restrict__ ent_pos) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const uint32_t b = ent_brick[e];
  const uint64_t below = brick_mask[b] & ((1ull << ent_bit[e]) - 1ull);
  const uint32_t pos = brick_valptr[b] + (uint32_t)__popcll(below);
  packed[pos] = vals[e];
  ent_pos[e] = pos;
}

// New values for an unchanged pattern: entry e of the CSR goes to the packed position
// recorded when the plan was built, and into the plan's CSR copy.
__global__ void k_update_values(const float* __restrict__ vals,
                                const uint32_t* __restrict__ ent_pos, int64_t nnz,
                                float* __restrict__ packed, float* __restrict__ csr_vals) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= nnz) return;
  const float v = vals[e];
  packed[ent_pos[e]] = v;
  csr_vals[e] = v;
}

// a5: per-panel class (Table 1, integer compare) and class totals.
__global__ void k_panel_classes(const uint32_t* __restrict__ panel_ptr,
                                const uint32_t* __restrict__ panel_nnzptr, int64_t P,
                                uint8_t* __restrict__ panel_class, unsigned long long* counters) {
  __shared__ unsigned long long acc[10];
  if (threadIdx.x < 10) acc[threadIdx.x] = 0;
  __syncthreads();
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p < P) {
    const unsigned long long nb = panel_ptr[p + 1] - panel_ptr[p];
    const unsigned long long nz = panel_nnzptr[p + 1] - panel_nnzptr[p];
    uint8_t cls = 255;
    if (nb) {
      cls = nz < 8 * nb ? 0 : (nz < 16 * nb ? 1 : 2);
      atomicAdd(&acc[kCntPanelsByClass + cls], 1ull);
      atomicAdd(&acc[kCntBricksByClass + cls], nb);
      atomicAdd(&acc[kCntNnzByClass + cls], nz);
      atomicAdd(&acc[kCntNonEmptyPanels], 1ull);
    }
    panel_class[p] = cls;
  }
  __syncthreads();
  if (threadIdx.x < 10 && acc[threadIdx.x]) atomicAdd(&counters[threadIdx.x], acc[threadIdx.x]);
}

__global__ void k_brick_hist(const uint64_t* __restrict__ brick_mask, int64_t nb,
                             unsigned long long* counters) {
  __shared__ unsigned int h[65];
  for (int t = threadIdx.x; t < 65; t += blockDim.x) h[t] = 0;
  __syncthreads();
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t b = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; b < nb; b += stride)
    atomicAdd(&h[__popcll(brick_mask[b])], 1u);
  __syncthreads();
  for (int t = threadIdx.x; t < 65; t += blockDim.x)
    if (h[t]) atomicAdd(&counters[kCntPopHist + t], (unsigned long long)h[t]);
}

__global__ void k_count_flags(const uint8_t* __restrict__ flags, int64_t n,
                              unsigned long long* counter) {
  __shared__ unsigned int total;
  if (threadIdx.x == 0) total = 0;
  __syncthreads();
  unsigned int mine = 0;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    mine += flags[i];
  if (mine) atomicAdd(&total, mine);
  __syncthreads();
  if (threadIdx.x == 0 && total) atomicAdd(counter, (unsigned long long)total);
}

// Rows with more than `threshold` entries, compacted in any order (the CSR kernel gives each of
// them a workgroup of its own).  The list has room for nnz / threshold + 1 rows.
__global__ void k_find_long_rows(const int32_t* __restrict__ rowptr, int64_t M, int threshold,
                                 uint32_t* __restrict__ list, unsigned long long* counter) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= M) return;
  if (rowptr[i + 1] - rowptr[i] > threshold) list[atomicAdd(counter, 1ull)] = (uint32_t)i;
}

// ---------------------------------------------------------------- scan
// Three-pass exclusive scan (block sums, scan of block sums, rescan + offset).
constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanTile = kScanThreads * kScanItems;

struct LoadU8 { const uint8_t* p; __device__ uint32_t operator()(int64_t i) const { return p[i]; } };
struct LoadU32 { const uint32_t* p; __device__ uint32_t operator()(int64_t i) const { return p[i]; } };
struct LoadPopc { const uint64_t* p; __device__ uint32_t operator()(int64_t i) const { return __popcll(p[i]); } };
struct LoadNonZero { const uint64_t* p; __device__ uint32_t operator()(int64_t i) const { return p[i] != 0 ? 1u : 0u; } };

// exclusive scan of one value per thread across the block; returns the block total
__device__ inline uint32_t block_exclusive(uint32_t v, uint32_t* total_out) {
  __shared__ uint32_t wave_sum[kScanThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  __syncthreads();  // protect wave_sum from the previous use
  if (lane == 63) wave_sum[wave] = incl;
  __syncthreads();
  uint32_t base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / 64; ++w) {
    if (w < wave) base += wave_sum[w];
    total += wave_sum[w];
  }
  *total_out = total;
  return base + incl - v;
}

template <typename Load>
__global__ void k_scan_block_sums(Load load, int64_t n, uint32_t* __restrict__ block_sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k)
    if (base + k < n) s += load(base + k);
  uint32_t total;
  block_exclusive(s, &total);
  if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// single block: in-place exclusive scan of block_sums[0..nblocks), total to *grand
__global__ void k_scan_of_sums(uint32_t* __restrict__ block_sums, int64_t nblocks,
                               uint32_t* __restrict__ grand) {
  uint32_t carry = 0;
  for (int64_t base = 0; base < nblocks; base += kScanThreads) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = i < nblocks ? block_sums[i] : 0;
    uint32_t total;
    const uint32_t ex = block_exclusive(v, &total);
    if (i < nblocks) block_sums[i] = carry + ex;
    carry += total;
  }
  if (threadIdx.x == 0) *grand = carry;
}

template <typename Load>
__global__ void k_scan_final(Load load, int64_t n, const uint32_t* __restrict__ block_offsets,
                             uint32_t* __restrict__ out) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  uint32_t v[kScanItems];
  uint32_t s = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    v[k] = base + k < n ? load(base + k) : 0;
    s += v[k];
  }
  uint32_t total;
  uint32_t run = block_offsets[blockIdx.x] + block_exclusive(s, &total);
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (base + k < n) out[base + k] = run;
    run += v[k];
  }
}

template <typename Load>
hipError_t scan_impl(Load load, int64_t n, uint32_t* out, uint32_t* tmp, hipStream_t s) {
  // out[n] receives the total even when n == 0
  const int64_t nblocks = (n + kScanTile - 1) / kScanTile;
  if (nblocks > 0)
    hipLaunchKernelGGL(k_scan_block_sums<Load>, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s,
                       load, n, tmp);
  hipLaunchKernelGGL(k_scan_of_sums, dim3(1), dim3(kScanThreads), 0, s, tmp, nblocks, out + n);
  if (nblocks > 0)
    hipLaunchKernelGGL(k_scan_final<Load>, dim3((unsigned)nblocks), dim3(kScanThreads), 0, s, load,
                       n, tmp, out);
  return hipGetLastError();
}

// ---------------------------------------------------------------- per-panel path
// One wavefront (a 64-thread workgroup) per panel, the panel's active columns as a bitmap in
// LDS over the panel's column span [cmin, cmax]: setting a bit per entry is the census (a1),
// the number of set bits below a column is its rank (a2), and from the rank follow brick,
// brick column and pattern bit (a3, patterns accumulated in LDS) and, after a scan of the
// panel's pattern popcounts, the value positions (a4; a panel's values are contiguous, so
// brick_valptr needs no scan across panels).  Used when the widest panel span and the largest
// brick count of a panel fit in LDS; other matrices take the search-based kernels above.
constexpr int kPanelThreads = 64;
constexpr int kGroupWords = 8;   // bitmap words per entry of the coarse rank table
constexpr uint32_t kPanelMaxWords = 32768;          // 1 Mi columns of span
constexpr size_t kPanelMaxLds = 150 * 1024;         // of the 160 KiB of a CU
constexpr uint32_t kPanelMaxSortKeys = 8192;        // entries of a panel on the sort-based path

struct PanelExtent {
  int64_t e0, e1;        // entries of the panel
  int32_t cmin, cmax;    // column span (valid if e0 < e1)
};

// exclusive scan of one value per lane across the wavefront; returns the total in *total_out
__device__ inline uint32_t wave_exclusive(uint32_t v, uint32_t* total_out) {
  const int lane = threadIdx.x & 63;
  uint32_t incl = v;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  *total_out = __shfl(incl, 63, 64);
  return incl - v;
}

// rows of panel p -> rp[0..16] (entry offsets, repeated past the last row), span of columns
__device__ inline PanelExtent panel_extent(const int32_t* __restrict__ rowptr,
                                           const int32_t* __restrict__ colind, int64_t M,
                                           int64_t p, int32_t* rp /* LDS [17] */) {
  const int64_t r0 = p * kPanel;
  if (threadIdx.x <= kPanel) rp[threadIdx.x] = rowptr[min(r0 + (int64_t)threadIdx.x, M)];
  __syncthreads();
  int32_t lo = 0x7FFFFFFF, hi = -1;
  if (threadIdx.x < kPanel) {
    const int32_t s = rp[threadIdx.x], t = rp[threadIdx.x + 1];
    if (s < t) {   // sorted rows: first and last entry bound the row's columns
      lo = colind[s];
      hi = colind[t - 1];
    }
  }
#pragma unroll
  for (int d = 8; d > 0; d >>= 1) {   // rows sit in lanes 0..15
    lo = min(lo, __shfl_xor(lo, d, 64));
    hi = max(hi, __shfl_xor(hi, d, 64));
  }
  lo = __shfl(lo, 0, 64);
  hi = __shfl(hi, 0, 64);
  return PanelExtent{rp[0], rp[kPanel], lo, hi};
}

// row (0..15) of entry e inside the panel whose row offsets are rp[0..16]
__device__ inline int row_in_panel(const int32_t* rp, int64_t e) {
  int r = 0;
#pragma unroll
  for (int d = 8; d > 0; d >>= 1)
    if (rp[r + d] <= e) r += d;
  return r;
}

// widest column span and largest entry count of any panel (0 for an empty matrix); requires
// a valid rowptr.  out[0] = span, out[1] = entries.
__global__ void k_panel_span(const int32_t* __restrict__ rowptr,
                             const int32_t* __restrict__ colind, int64_t M, int64_t P,
                             uint32_t* err, uint32_t* out) {
  __shared__ uint32_t s_span, s_nnz, s_bad;
  if (*err & (kErrRowptrEnds | kErrRowptrOrder)) return;
  if (threadIdx.x == 0) { s_span = 0; s_nnz = 0; s_bad = 0; }
  __syncthreads();
  const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (p < P) {
    int32_t lo = 0x7FFFFFFF, hi = -1;
    const int64_t r0 = p * kPanel, r1 = min((p + 1) * kPanel, M);
    for (int64_t r = r0; r < r1; ++r) {
      const int32_t s = rowptr[r], t = rowptr[r + 1];
      if (s < t) { lo = min(lo, colind[s]); hi = max(hi, colind[t - 1]); }
    }
    if (hi >= lo) atomicMax(&s_span, (uint32_t)((int64_t)hi - lo + 1));
    else if (rowptr[r1] > rowptr[r0]) atomicOr(&s_bad, 1u);   // entries, but an inverted span
    atomicMax(&s_nnz, (uint32_t)(rowptr[r1] - rowptr[r0]));
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    if (s_span) atomicMax(&out[0], s_span);
    if (s_nnz) atomicMax(&out[1], s_nnz);
    // a panel whose rows end below where they start is not sorted (or has a negative column)
    if (s_bad) atomicOr(err, (uint32_t)kErrColOrder);
  }
}

// sets the panel's bitmap; checks the columns on the way (range, order, inside the span)
__device__ inline void panel_bitmap(const int32_t* __restrict__ colind, const PanelExtent& x,
                                    const int32_t* rp, int64_t K, uint32_t words, uint32_t* bm,
                                    uint32_t* err) {
  for (uint32_t w = threadIdx.x; w < words; w += kPanelThreads) bm[w] = 0;
  __syncthreads();
  uint32_t bad = 0;
  for (int64_t e = x.e0 + threadIdx.x; e < x.e1; e += kPanelThreads) {
    const int32_t j = colind[e];
    if (err) {
      if (j < 0 || j >= K) bad |= kErrColRange;
      if (e > rp[row_in_panel(rp, e)] && colind[e - 1] >= j) bad |= kErrColOrder;
    }
    if (j >= x.cmin && j <= x.cmax) {
      const uint32_t d = (uint32_t)(j - x.cmin);
      atomicOr(&bm[d >> 5], 1u << (d & 31));
    } else {
      bad |= kErrColOrder;   // outside the span its sorted row promised
    }
  }
  if (err && bad) atomicOr(err, bad);
  __syncthreads();
}

// a1/a2 (counting half): bricks of each panel, entry offset of each panel, total of active
// columns, largest brick count of a panel; validates colind.  Dynamic LDS: the bitmap.
__global__ __launch_bounds__(kPanelThreads) void k_panel_census(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind, int64_t M, int64_t K,
    int64_t P, uint32_t words_cap, uint32_t* err, uint32_t* __restrict__ nbricks_p,
    uint32_t* __restrict__ panel_nnzptr, uint32_t* __restrict__ ncols_p) {
  extern __shared__ uint32_t lds[];
  __shared__ int32_t rp[kPanel + 1];
  if (*err & (kErrRowptrEnds | kErrRowptrOrder)) return;   // uniform: nothing below is safe
  const int64_t p = blockIdx.x;
  const PanelExtent x = panel_extent(rowptr, colind, M, p, rp);
  if (threadIdx.x == 0) {
    panel_nnzptr[p] = (uint32_t)x.e0;
    if (p == P - 1) panel_nnzptr[P] = (uint32_t)x.e1;
  }
  if (x.e0 >= x.e1 || x.cmax < x.cmin) {
    // Entries but an inverted span (the last column of every row lies below the first column
    // of some row): a row is stored in descending order, or a column is negative.  No bitmap
    // can hold that, so the per-entry checks below would never see it.
    if (threadIdx.x == 0) {
      if (x.e0 < x.e1) atomicOr(err, (uint32_t)kErrColOrder);
      nbricks_p[p] = 0;
      ncols_p[p] = 0;
    }
    return;
  }
  const uint32_t words = (uint32_t)(x.cmax - x.cmin) / 32u + 1u;
  if (words > words_cap) {   // cannot happen for sorted rows (the cap comes from k_panel_span)
    if (threadIdx.x == 0) { atomicOr(err, (uint32_t)kErrColOrder); nbricks_p[p] = 0; ncols_p[p] = 0; }
    return;
  }
  panel_bitmap(colind, x, rp, K, words, lds, err);
  uint32_t cnt = 0;
  for (uint32_t w = threadIdx.x; w < words; w += kPanelThreads) cnt += __popc(lds[w]);
  uint32_t total;
  wave_exclusive(cnt, &total);
  if (threadIdx.x == 0) {
    nbricks_p[p] = (total + kBrickK - 1) / kBrickK;
    ncols_p[p] = total;
  }
}

// ---- per-panel path for scattered matrices: sort instead of a bitmap
// One wavefront per panel sorts the panel's entries by (column, entry) in LDS (bitonic network
// on 64-bit keys: column in the high half, entry index inside the panel in the low half).
// Equal columns end up next to each other: flags + a scan give the rank of every column, with
// no dependence on the width of the panel's column span.
// Loads the keys (padded with all-ones to n_sort, a power of two >= 64), checks the columns,
// sorts ascending.  KT = uint32_t packs (column << 11 | index) for matrices with fewer than
// 2^21 columns and panels of at most 2048 entries: half the LDS traffic of 64-bit keys.
template <typename KT> struct SortKey;
template <> struct SortKey<unsigned long long> {
  static __device__ unsigned long long make(uint32_t col, uint32_t idx) { return ((unsigned long long)col << 32) | idx; }
  static __device__ uint32_t col(unsigned long long k) { return (uint32_t)(k >> 32); }
  static __device__ uint32_t idx(unsigned long long k) { return (uint32_t)k; }
};
template <> struct SortKey<uint32_t> {
  static __device__ uint32_t make(uint32_t col, uint32_t idx) { return (col << 11) | idx; }
  static __device__ uint32_t col(uint32_t k) { return k >> 11; }
  static __device__ uint32_t idx(uint32_t k) { return k & 2047u; }
};

template <typename KT>
__device__ inline void panel_sort(const int32_t* __restrict__ colind, const PanelExtent& x,
                                  const int32_t* rp, int64_t K, uint32_t n_sort, KT* keys,
                                  uint32_t* err) {
  const uint32_t n = (uint32_t)(x.e1 - x.e0);
  uint32_t bad = 0;
  for (uint32_t i = threadIdx.x; i < n_sort; i += kPanelThreads) {
    KT key = (KT)~(KT)0;
    if (i < n) {
      const int64_t e = x.e0 + i;
      const int32_t j = colind[e];
      if (j < 0 || j >= K) bad |= kErrColRange;
      if (e > rp[row_in_panel(rp, e)] && colind[e - 1] >= j) bad |= kErrColOrder;
      key = SortKey<KT>::make((uint32_t)j, i);
    }
    keys[i] = key;
  }
  if (bad) atomicOr(err, bad);
  __syncthreads();
  for (uint32_t k = 2; k <= n_sort; k <<= 1) {
    for (uint32_t j = k >> 1; j > 0; j >>= 1) {
      for (uint32_t i = threadIdx.x; i < n_sort / 2; i += kPanelThreads) {
        const uint32_t a = ((i & ~(j - 1)) << 1) | (i & (j - 1));
        const uint32_t b = a | j;
        const KT ka = keys[a], kb = keys[b];
        const bool ascending = (a & k) == 0;
        if ((ka > kb) == ascending) { keys[a] = kb; keys[b] = ka; }
      }
      __syncthreads();
    }
  }
}

__device__ inline uint32_t sort_size(uint32_t n) {
  uint32_t m = 64;
  while (m < n) m <<= 1;
  return m;
}

// census by sorting: distinct columns of each panel; validates colind; leaves the sorted order
// of each panel's entries (indices inside the panel) in `order`.  Dynamic LDS: keys.
template <typename KT>
__global__ __launch_bounds__(kPanelThreads) void k_panel_sort_census(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind, int64_t M, int64_t K,
    int64_t P, uint32_t n_cap, uint32_t* err, uint32_t* __restrict__ nbricks_p,
    uint32_t* __restrict__ panel_nnzptr, uint32_t* __restrict__ ncols_p,
    uint32_t* __restrict__ order) {
  extern __shared__ unsigned long long lds64[];
  KT* keys = reinterpret_cast<KT*>(lds64);
  __shared__ int32_t rp[kPanel + 1];
  if (*err & (kErrRowptrEnds | kErrRowptrOrder)) return;   // uniform: nothing below is safe
  const int64_t p = blockIdx.x;
  const PanelExtent x = panel_extent(rowptr, colind, M, p, rp);
  if (threadIdx.x == 0) {
    panel_nnzptr[p] = (uint32_t)x.e0;
    if (p == P - 1) panel_nnzptr[P] = (uint32_t)x.e1;
  }
  const uint32_t n = (uint32_t)(x.e1 - x.e0);
  if (n == 0 || n > n_cap) {   // (n > n_cap cannot happen: the cap comes from k_panel_span)
    if (threadIdx.x == 0) { nbricks_p[p] = 0; ncols_p[p] = 0; }
    return;
  }
  panel_sort<KT>(colind, x, rp, K, sort_size(n), keys, err);
  uint32_t cnt = 0;
  for (uint32_t i = threadIdx.x; i < n; i += kPanelThreads) {
    cnt += (i == 0 || SortKey<KT>::col(keys[i]) != SortKey<KT>::col(keys[i - 1])) ? 1u : 0u;
    order[x.e0 + i] = SortKey<KT>::idx(keys[i]);   // sorted order of the panel's entries
  }
  uint32_t total;
  wave_exclusive(cnt, &total);
  if (threadIdx.x == 0) {
    nbricks_p[p] = (total + kBrickK - 1) / kBrickK;
    ncols_p[p] = total;
  }
}

// a2 (placing half), a3 and a4 for one panel from the sorted order left by the census in
// `ent_pos` (which this kernel then overwrites with the value positions).  Dynamic LDS: keys
// (n_cap x u64), patterns (nb_cap x u64), value offsets (nb_cap words).
__global__ __launch_bounds__(kPanelThreads) void k_panel_sort_build(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
    const float* __restrict__ vals, int64_t M, int64_t K, uint32_t n_cap, uint32_t nb_cap,
    const uint32_t* __restrict__ panel_ptr, uint32_t* __restrict__ brick_cols,
    uint64_t* __restrict__ brick_mask, uint32_t* __restrict__ brick_valptr,
    float* __restrict__ packed, uint32_t* ent_pos, uint8_t* __restrict__ col_seen) {
  extern __shared__ unsigned long long lds64[];
  __shared__ int32_t rp[kPanel + 1];
  unsigned long long* keys = lds64;                                  // [n_cap]
  unsigned long long* pat = lds64 + n_cap;                           // [nb_cap]
  uint32_t* vptr = reinterpret_cast<uint32_t*>(pat + nb_cap);        // [nb_cap]
  const int64_t p = blockIdx.x;
  const uint32_t pp = panel_ptr[p];
  const uint32_t nb = panel_ptr[p + 1] - pp;
  const PanelExtent x = panel_extent(rowptr, colind, M, p, rp);
  if (nb == 0) return;
  const uint32_t n = (uint32_t)(x.e1 - x.e0);
  if (n > n_cap || nb > nb_cap) return;   // (cannot happen: both caps are maxima over the panels)
  for (uint32_t k = threadIdx.x; k < nb; k += kPanelThreads) pat[k] = 0;
  for (uint32_t i = threadIdx.x; i < n; i += kPanelThreads) {
    const uint32_t idx = min(ent_pos[x.e0 + i], n - 1);   // (always below n)
    keys[i] = ((unsigned long long)(uint32_t)colind[x.e0 + idx] << 32) | idx;
  }
  __syncthreads();

  // rank of each sorted entry's column = number of column changes before it; first
  // occurrences write brick_cols; then the key's column is replaced by the rank.  The column
  // before a batch of 64 is carried in a register: its key has been rewritten by then.
  uint32_t carry = 0;
  uint32_t col_before = 0xFFFFFFFFu;   // never a column (columns are below 2^31)
  for (uint32_t base = 0; base < n; base += kPanelThreads) {
    const uint32_t i = base + threadIdx.x;
    uint32_t col = 0xFFFFFFFFu, first = 0;
    if (i < n) col = (uint32_t)(keys[i] >> 32);
    uint32_t prev = __shfl_up(col, 1, 64);
    if (threadIdx.x == 0) prev = col_before;
    if (i < n) first = (col != prev) ? 1u : 0u;
    uint32_t total;
    const uint32_t ex = wave_exclusive(first, &total);
    if (i < n) {
      const uint32_t rank = carry + ex + first - 1u;   // inclusive count of firsts, minus one
      if (first && rank < nb * kBrickK) {
        brick_cols[(int64_t)pp * kBrickK + rank] = col;
        col_seen[col] = 1;
      }
      keys[i] = ((unsigned long long)rank << 32) | (uint32_t)keys[i];
    }
    col_before = __shfl(col, 63, 64);
    carry += total;
  }
  __syncthreads();
  for (uint32_t k = carry + threadIdx.x; k < nb * kBrickK; k += kPanelThreads)
    brick_cols[(int64_t)pp * kBrickK + k] = kPadCol;

  // a3: pattern bits, accumulated in LDS
  for (uint32_t i = threadIdx.x; i < n; i += kPanelThreads) {
    const uint32_t rank = (uint32_t)(keys[i] >> 32);
    const int64_t e = x.e0 + (uint32_t)keys[i];
    const uint32_t bit = (uint32_t)row_in_panel(rp, e) * kBrickK + rank % kBrickK;
    if (rank / kBrickK < nb) atomicOr(&pat[rank / kBrickK], 1ull << bit);
  }
  __syncthreads();

  // a4: value offsets = entries before the panel + popcounts of the panel's earlier bricks
  uint32_t off = (uint32_t)x.e0;
  for (uint32_t base = 0; base < nb; base += kPanelThreads) {
    const uint32_t k = base + threadIdx.x;
    uint32_t c = 0;
    if (k < nb) {
      const unsigned long long m = pat[k];
      brick_mask[pp + k] = m;
      c = (uint32_t)__popcll(m);
    }
    uint32_t total;
    const uint32_t ex = wave_exclusive(c, &total);
    if (k < nb) {
      vptr[k] = off + ex;
      brick_valptr[pp + k] = off + ex;
    }
    off += total;
  }
  __syncthreads();
  for (uint32_t i = threadIdx.x; i < n; i += kPanelThreads) {
    const uint32_t rank = (uint32_t)(keys[i] >> 32);
    const int64_t e = x.e0 + (uint32_t)keys[i];
    const uint32_t bit = (uint32_t)row_in_panel(rp, e) * kBrickK + rank % kBrickK;
    const uint32_t k = min(rank / kBrickK, nb - 1);
    const uint32_t pos = vptr[k] + (uint32_t)__popcll(pat[k] & ((1ull << bit) - 1ull));
    if (pos < (uint32_t)x.e1) {   // (always, for a census and a build that agree)
      packed[pos] = vals[e];
      ent_pos[e] = pos;
    }
  }
}

// sum and maximum of ncols_p (one atomic pair per workgroup: per-panel atomics on one address
// serialise at more than 100 ns each)
__global__ void k_cols_sum_max(const uint32_t* __restrict__ ncols_p, int64_t P,
                               unsigned long long* sum, uint32_t* max_cols) {
  __shared__ unsigned long long s_sum;
  __shared__ uint32_t s_max;
  if (threadIdx.x == 0) { s_sum = 0; s_max = 0; }
  __syncthreads();
  unsigned long long mine = 0;
  uint32_t mx = 0;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; p < P; p += stride) {
    mine += ncols_p[p];
    mx = max(mx, ncols_p[p]);
  }
  if (mine) atomicAdd(&s_sum, mine);
  if (mx) atomicMax(&s_max, mx);
  __syncthreads();
  if (threadIdx.x == 0) {
    if (s_sum) atomicAdd(sum, s_sum);
    if (s_max) atomicMax(max_cols, s_max);
  }
}

// a2 (placing half), a3 and a4 for one panel.  Dynamic LDS: patterns of the
// panel's bricks (nb_cap x u64), the bitmap (words_cap words), the coarse rank table
// (words_cap / 8 + 1 words), value offsets of the panel's bricks (nb_cap words).
__global__ __launch_bounds__(kPanelThreads) void k_panel_build(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
    const float* __restrict__ vals, int64_t M, int64_t K, uint32_t words_cap, uint32_t nb_cap,
    const uint32_t* __restrict__ panel_ptr, uint32_t* __restrict__ brick_cols,
    uint64_t* __restrict__ brick_mask, uint32_t* __restrict__ brick_valptr,
    float* __restrict__ packed, uint32_t* __restrict__ ent_pos, uint8_t* __restrict__ col_seen) {
  extern __shared__ unsigned long long lds64[];
  __shared__ int32_t rp[kPanel + 1];
  unsigned long long* pat = lds64;                                   // [nb_cap]
  uint32_t* bm = reinterpret_cast<uint32_t*>(lds64 + nb_cap);        // [words_cap]
  uint32_t* pre = bm + words_cap;     // [words_cap / 8 + 1]; pre[g] = set bits in words [0, 8g)
  uint32_t* vptr = pre + words_cap / kGroupWords + 1;                // [nb_cap]
  const int64_t p = blockIdx.x;
  const uint32_t pp = panel_ptr[p];
  const uint32_t nb = panel_ptr[p + 1] - pp;
  const PanelExtent x = panel_extent(rowptr, colind, M, p, rp);
  if (nb == 0) return;
  const uint32_t words = (uint32_t)(x.cmax - x.cmin) / 32u + 1u;
  if (words > words_cap || nb > nb_cap) return;   // (cannot happen: both caps are maxima)
  for (uint32_t k = threadIdx.x; k < nb; k += kPanelThreads) pat[k] = 0;
  panel_bitmap(colind, x, rp, K, words, bm, nullptr);

  // coarse rank table: exclusive scan over groups of 8 words, a contiguous run per lane
  const uint32_t ngroups = (words + kGroupWords - 1) / kGroupWords;
  const uint32_t per = (ngroups + kPanelThreads - 1) / kPanelThreads;
  const uint32_t g0 = min(threadIdx.x * per, ngroups), g1 = min(g0 + per, ngroups);
  uint32_t mine = 0;
  for (uint32_t g = g0; g < g1; ++g) {
    uint32_t s = 0;
    for (uint32_t w = g * kGroupWords; w < min((g + 1) * kGroupWords, words); ++w) s += __popc(bm[w]);
    pre[g] = s;
    mine += s;
  }
  uint32_t ncols;
  uint32_t run = wave_exclusive(mine, &ncols);
  for (uint32_t g = g0; g < g1; ++g) {
    const uint32_t s = pre[g];
    pre[g] = run;
    run += s;
  }
  __syncthreads();
  auto bits_before_word = [&](uint32_t w) {
    uint32_t r = pre[w / kGroupWords];
    for (uint32_t v = w & ~(uint32_t)(kGroupWords - 1); v < w; ++v) r += __popc(bm[v]);
    return r;
  };

  // a2: active columns in ascending order, four per brick, the tail padded
  for (uint32_t w = threadIdx.x; w < words; w += kPanelThreads) {
    uint32_t bits = bm[w];
    if (!bits) continue;
    uint32_t r = bits_before_word(w);
    while (bits) {
      const uint32_t col = (uint32_t)x.cmin + 32u * w + (uint32_t)__builtin_ctz(bits);
      brick_cols[(int64_t)pp * kBrickK + r++] = col;
      col_seen[col] = 1;
      bits &= bits - 1;
    }
  }
  for (uint32_t k = ncols + threadIdx.x; k < nb * kBrickK; k += kPanelThreads)
    brick_cols[(int64_t)pp * kBrickK + k] = kPadCol;

  // a3: pattern bits, accumulated in LDS
  for (int64_t e = x.e0 + threadIdx.x; e < x.e1; e += kPanelThreads) {
    const uint32_t d = (uint32_t)(colind[e] - x.cmin);
    const uint32_t rank = bits_before_word(d >> 5) + __popc(bm[d >> 5] & ((1u << (d & 31)) - 1u));
    const uint32_t bit = (uint32_t)row_in_panel(rp, e) * kBrickK + rank % kBrickK;
    if (rank / kBrickK < nb) atomicOr(&pat[rank / kBrickK], 1ull << bit);
  }
  __syncthreads();

  // a4: value offsets = entries before the panel + popcounts of the panel's earlier bricks
  uint32_t carry = (uint32_t)x.e0;
  for (uint32_t base = 0; base < nb; base += kPanelThreads) {
    const uint32_t k = base + threadIdx.x;
    uint32_t c = 0;
    if (k < nb) {
      const unsigned long long m = pat[k];
      brick_mask[pp + k] = m;
      c = (uint32_t)__popcll(m);
    }
    uint32_t total;
    const uint32_t ex = wave_exclusive(c, &total);
    if (k < nb) {
      vptr[k] = carry + ex;
      brick_valptr[pp + k] = carry + ex;
    }
    carry += total;
  }
  __syncthreads();
  for (int64_t e = x.e0 + threadIdx.x; e < x.e1; e += kPanelThreads) {
    const uint32_t d = (uint32_t)(colind[e] - x.cmin);
    const uint32_t rank = bits_before_word(d >> 5) + __popc(bm[d >> 5] & ((1u << (d & 31)) - 1u));
    const uint32_t bit = (uint32_t)row_in_panel(rp, e) * kBrickK + rank % kBrickK;
    const uint32_t k = min(rank / kBrickK, nb - 1);
    const uint32_t pos = vptr[k] + (uint32_t)__popcll(pat[k] & ((1ull << bit) - 1ull));
    if (pos < (uint32_t)x.e1) {   // (always, for a census and a build that agree)
      packed[pos] = vals[e];
      ent_pos[e] = pos;
    }
  }
}

}  // namespace

size_t scan_tmp_elems(int64_t n) { return (size_t)((n + kScanTile - 1) / kScanTile) + 1; }

hipError_t launch_scan_u8(const uint8_t* in, int64_t n, uint32_t* out, uint32_t* tmp, hipStream_t s) {
  return scan_impl(LoadU8{in}, n, out, tmp, s);
}
hipError_t launch_scan_u32(const uint32_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                           hipStream_t s) {
  return scan_impl(LoadU32{in}, n, out, tmp, s);
}
hipError_t launch_scan_popc64(const uint64_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                              hipStream_t s) {
  return scan_impl(LoadPopc{in}, n, out, tmp, s);
}

hipError_t launch_scan_nonzero64(const uint64_t* in, int64_t n, uint32_t* out, uint32_t* tmp,
                                 hipStream_t s) {
  return scan_impl(LoadNonZero{in}, n, out, tmp, s);
}

hipError_t launch_validate_rowptr(const int32_t* rowptr, int64_t M, int64_t nnz, uint32_t* err,
                                  hipStream_t s) {
  hipLaunchKernelGGL(k_validate_rowptr, dim3(grid_for(M + 1)), dim3(kThreads), 0, s, rowptr, M, nnz,
                     err);
  return hipGetLastError();
}

hipError_t launch_validate_cols(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t K,
                                int64_t nnz, uint32_t* ent_row, uint32_t* err, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_validate_cols, dim3(grid_for(nnz)), dim3(kThreads), 0, s, rowptr, colind, M,
                     K, nnz, ent_row, err);
  return hipGetLastError();
}

hipError_t launch_first_in_panel(const int32_t* rowptr, const int32_t* colind,
                                 const uint32_t* ent_row, int64_t nnz, uint8_t* first,
                                 uint32_t* link, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_first_in_panel, dim3(grid_for(nnz)), dim3(kThreads), 0, s, rowptr, colind,
                     ent_row, nnz, first, link);
  return hipGetLastError();
}

hipError_t launch_compact_first(const uint8_t* first, const uint32_t* first_scan, int64_t nnz,
                                uint32_t* first_list, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_compact_first, dim3(grid_for(nnz)), dim3(kThreads), 0, s, first, first_scan,
                     nnz, first_list);
  return hipGetLastError();
}

hipError_t launch_panel_counts(const int32_t* rowptr, const uint32_t* first_scan, int64_t M,
                               int64_t P, uint32_t* nbricks_p, uint32_t* panel_nnzptr,
                               hipStream_t s) {
  hipLaunchKernelGGL(k_panel_counts, dim3(grid_for(P + 1)), dim3(kThreads), 0, s, rowptr,
                     first_scan, M, P, nbricks_p, panel_nnzptr);
  return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* p, int64_t n, uint32_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill<uint32_t>, dim3(grid_for(n)), dim3(kThreads), 0, s, p, n, v);
  return hipGetLastError();
}

hipError_t launch_fill_u64(uint64_t* p, int64_t n, uint64_t v, hipStream_t s) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill<uint64_t>, dim3(grid_for(n)), dim3(kThreads), 0, s, p, n, v);
  return hipGetLastError();
}

hipError_t launch_rank_first(const int32_t* rowptr, const int32_t* colind, const uint32_t* ent_row,
                             const uint32_t* first_list, const uint32_t* first_scan,
                             const uint32_t* panel_ptr, int64_t M, int64_t n_active,
                             uint32_t* ent_rank, uint32_t* brick_cols, hipStream_t s) {
  if (n_active == 0) return hipSuccess;
  hipLaunchKernelGGL(k_rank_first, dim3(grid_for(n_active)), dim3(kThreads), 0, s, rowptr, colind,
                     ent_row, first_list, first_scan, panel_ptr, M, n_active, ent_rank, brick_cols);
  return hipGetLastError();
}

hipError_t launch_scatter_bits(const int32_t* colind, const uint32_t* ent_row, const uint32_t* link,
                               const uint32_t* ent_rank, const uint32_t* panel_ptr, int64_t nnz,
                               uint64_t* brick_mask, uint32_t* ent_brick, uint8_t* ent_bit,
                               uint8_t* col_seen, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_scatter_bits, dim3(grid_for(nnz)), dim3(kThreads), 0, s, colind, ent_row,
                     link, ent_rank, panel_ptr, nnz, brick_mask, ent_brick, ent_bit, col_seen);
  return hipGetLastError();
}

hipError_t launch_pack_values(const float* vals, const uint32_t* ent_brick, const uint8_t* ent_bit,
                              const uint64_t* brick_mask, const uint32_t* brick_valptr,
                              int64_t nnz, float* packed, uint32_t* ent_pos, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_pack_values, dim3(grid_for(nnz)), dim3(kThreads), 0, s, vals, ent_brick,
                     ent_bit, brick_mask, brick_valptr, nnz, packed, ent_pos);
  return hipGetLastError();
}

hipError_t launch_update_values(const float* vals, const uint32_t* ent_pos, int64_t nnz,
                                float* packed, float* csr_vals, hipStream_t s) {
  if (nnz == 0) return hipSuccess;
  hipLaunchKernelGGL(k_update_values, dim3(grid_for(nnz)), dim3(kThreads), 0, s, vals, ent_pos,
                     nnz, packed, csr_vals);
  return hipGetLastError();
}

hipError_t launch_panel_classes(const uint32_t* panel_ptr, const uint32_t* panel_nnzptr, int64_t P,
                                uint8_t* panel_class, unsigned long long* counters, hipStream_t s) {
  if (P == 0) return hipSuccess;
  hipLaunchKernelGGL(k_panel_classes, dim3(grid_for(P)), dim3(kThreads), 0, s, panel_ptr,
                     panel_nnzptr, P, panel_class, counters);
  return hipGetLastError();
}

hipError_t launch_brick_hist(const uint64_t* brick_mask, int64_t nb, unsigned long long* counters,
                             hipStream_t s) {
  if (nb == 0) return hipSuccess;
  const unsigned g = (unsigned)std::min<int64_t>(grid_for(nb), 2048);
  hipLaunchKernelGGL(k_brick_hist, dim3(g), dim3(kThreads), 0, s, brick_mask, nb, counters);
  return hipGetLastError();
}

hipError_t launch_count_flags(const uint8_t* flags, int64_t n, unsigned long long* counter,
                              hipStream_t s) {
  if (n == 0) return hipSuccess;
  const unsigned g = (unsigned)std::min<int64_t>(grid_for(n), 2048);
  hipLaunchKernelGGL(k_count_flags, dim3(g), dim3(kThreads), 0, s, flags, n, counter);
  return hipGetLastError();
}

hipError_t launch_find_long_rows(const int32_t* rowptr, int64_t M, int threshold, uint32_t* list,
                                 unsigned long long* counter, hipStream_t s) {
  if (M == 0) return hipSuccess;
  hipLaunchKernelGGL(k_find_long_rows, dim3(grid_for(M)), dim3(kThreads), 0, s, rowptr, M,
                     threshold, list, counter);
  return hipGetLastError();
}

// ---- per-panel path
hipError_t launch_panel_span(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t P,
                             uint32_t* err, uint32_t* span_and_nnz, hipStream_t s) {
  if (P == 0) return hipSuccess;
  hipLaunchKernelGGL(k_panel_span, dim3(grid_for(P)), dim3(kThreads), 0, s, rowptr, colind, M, P,
                     err, span_and_nnz);
  return hipGetLastError();
}

// ---- sort-based per-panel path
// keys of the sort for panels of up to max_nnz entries (a power of two), or 0 if too many
uint32_t panel_sort_keys(uint32_t max_nnz) {
  uint32_t n = 64;
  while (n < max_nnz && n < kPanelMaxSortKeys) n *= 2;
  return n >= max_nnz ? n : 0;
}
static size_t panel_sort_build_lds(uint32_t n_cap, uint32_t nb_cap) {
  return (size_t)n_cap * 8 + (size_t)nb_cap * 12;
}
bool panel_sort_build_fits(uint32_t n_cap, uint32_t nb_cap) {
  return n_cap != 0 && panel_sort_build_lds(n_cap, nb_cap) <= kPanelMaxLds;
}

hipError_t launch_panel_sort_census(const int32_t* rowptr, const int32_t* colind, int64_t M,
                                    int64_t K, int64_t P, uint32_t n_cap, uint32_t* err,
                                    uint32_t* nbricks_p, uint32_t* panel_nnzptr, uint32_t* ncols_p,
                                    uint32_t* order, unsigned long long* n_active,
                                    uint32_t* max_cols, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const bool narrow = K < (int64_t(1) << 21) && n_cap <= 2048;   // (column, index) fits 32 bits
  const size_t lds = (size_t)n_cap * (narrow ? 4 : 8);
  const void* fn = narrow ? reinterpret_cast<const void*>(k_panel_sort_census<uint32_t>)
                          : reinterpret_cast<const void*>(k_panel_sort_census<unsigned long long>);
  if (lds > 48 * 1024) {
    const hipError_t e =
        hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  if (narrow)
    hipLaunchKernelGGL(k_panel_sort_census<uint32_t>, dim3((unsigned)P), dim3(kPanelThreads), lds,
                       s, rowptr, colind, M, K, P, n_cap, err, nbricks_p, panel_nnzptr, ncols_p,
                       order);
  else
    hipLaunchKernelGGL(k_panel_sort_census<unsigned long long>, dim3((unsigned)P),
                       dim3(kPanelThreads), lds, s, rowptr, colind, M, K, P, n_cap, err, nbricks_p,
                       panel_nnzptr, ncols_p, order);
  hipLaunchKernelGGL(k_cols_sum_max, dim3((unsigned)std::min<int64_t>(grid_for(P), 1024)),
                     dim3(kThreads), 0, s, ncols_p, P, n_active, max_cols);
  return hipGetLastError();
}

hipError_t launch_panel_sort_build(const int32_t* rowptr, const int32_t* colind, const float* vals,
                                   int64_t M, int64_t K, int64_t P, uint32_t n_cap, uint32_t nb_cap,
                                   const uint32_t* panel_ptr, uint32_t* brick_cols,
                                   uint64_t* brick_mask, uint32_t* brick_valptr, float* packed,
                                   uint32_t* ent_pos, uint8_t* col_seen, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t lds = panel_sort_build_lds(n_cap, nb_cap);
  if (lds > 48 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_panel_sort_build),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_panel_sort_build, dim3((unsigned)P), dim3(kPanelThreads), lds, s, rowptr,
                     colind, vals, M, K, n_cap, nb_cap, panel_ptr, brick_cols, brick_mask,
                     brick_valptr, packed, ent_pos, col_seen);
  return hipGetLastError();
}

// bitmap words (a power of two, at least 64) for a widest panel span of `span` columns, or 0 if
// that does not fit the LDS bitmap
uint32_t panel_bitmap_words(uint32_t span) {
  uint32_t words = 64;
  while ((uint64_t)words * 32 < span && words < kPanelMaxWords) words *= 2;
  return (uint64_t)words * 32 >= span ? words : 0;
}

// LDS bytes of k_panel_build for a bitmap of words_cap words and panels of up to nb_cap bricks
static size_t panel_build_lds(uint32_t words_cap, uint32_t nb_cap) {
  return (size_t)nb_cap * 8 + ((size_t)words_cap + words_cap / kGroupWords + 1 + nb_cap) * 4;
}
bool panel_build_fits(uint32_t words_cap, uint32_t nb_cap) {
  return words_cap != 0 && panel_build_lds(words_cap, nb_cap) <= kPanelMaxLds;
}

hipError_t launch_panel_census(const int32_t* rowptr, const int32_t* colind, int64_t M, int64_t K,
                               int64_t P, uint32_t words_cap, uint32_t* err, uint32_t* nbricks_p,
                               uint32_t* panel_nnzptr, uint32_t* ncols_p,
                               unsigned long long* n_active, uint32_t* max_cols, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t lds = (size_t)words_cap * 4;
  if (lds > 48 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_panel_census),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_panel_census, dim3((unsigned)P), dim3(kPanelThreads), lds, s, rowptr, colind,
                     M, K, P, words_cap, err, nbricks_p, panel_nnzptr, ncols_p);
  hipLaunchKernelGGL(k_cols_sum_max, dim3((unsigned)std::min<int64_t>(grid_for(P), 1024)),
                     dim3(kThreads), 0, s, ncols_p, P, n_active, max_cols);
  return hipGetLastError();
}

hipError_t launch_panel_build(const int32_t* rowptr, const int32_t* colind, const float* vals,
                              int64_t M, int64_t K, int64_t P, uint32_t words_cap, uint32_t nb_cap,
                              const uint32_t* panel_ptr, uint32_t* brick_cols, uint64_t* brick_mask,
                              uint32_t* brick_valptr, float* packed, uint32_t* ent_pos,
                              uint8_t* col_seen, hipStream_t s) {
  if (P == 0) return hipSuccess;
  const size_t lds = panel_build_lds(words_cap, nb_cap);
  if (lds > 48 * 1024) {
    const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(k_panel_build),
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(k_panel_build, dim3((unsigned)P), dim3(kPanelThreads), lds, s, rowptr, colind,
                     vals, M, K, words_cap, nb_cap, panel_ptr, brick_cols, brick_mask, brick_valptr,
                     packed, ent_pos, col_seen);
  return hipGetLastError();
}

}  // namespace spmm
