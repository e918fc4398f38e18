// Row panels of 32 rows (paper Section 4, Eq. 5): a brick column of a 32-row panel holds up to
// two 16x4 bricks (rows 0..15 and 16..31), and the B operand loaded for the brick column is
// used by both (beta = bricks per brick column).  This file builds that format on the GPU from
// the 16-row brick format and multiplies with it.
//
// The two halves of a super-panel are packed into one left-compacted column list only where
// their active columns nearly coincide (|union| * den < num * max(|top|, |bottom|)); elsewhere
// each half keeps its own list and the super-panel holds the brick columns of the top half
// followed by those of the bottom half, which are exactly the bricks of the 16-row format.
// The paper gives no such rule (it always ran 16-row panels and only describes the two extreme
// cases); without one, packing unrelated halves together lowers the brick density.
//
// Layout (Q = ceil(P/2) super-panels, nbc brick columns, nbr bricks):
//   sp_ptr u32[Q+1], sp_merged u8[Q], bc_cols u32[4 nbc] (pad 0xFFFFFFFF), bc_brick u32[nbc+1]
//   (first brick of each brick column; the paper's colPtr), br_row u8[nbr] (brick-row id; the
//   paper's rows), br_mask u64[nbr], br_valptr u32[nbr+1], vals f32[nnz].
// For the kernel a second, derived array holds per brick column the patterns and value offsets
// of its top and bottom brick (zero pattern where a half has no brick).
#include "exec_common.h"

#include <type_traits>

namespace spmm {

namespace {

constexpr int kThreads = 256;

inline unsigned grid_for(int64_t n, int threads = kThreads) {
  const int64_t g = (n + threads - 1) / threads;
  return (unsigned)(g > 0 ? g : 1);
}

// active columns of 16-row panel p: a sorted list inside brick_cols, pads only at the end
__device__ inline void panel_cols(const uint32_t* __restrict__ panel_ptr,
                                  const uint32_t* __restrict__ brick_cols, int64_t P, int64_t p,
                                  const uint32_t** list, uint32_t* n, uint32_t* nb) {
  *list = nullptr; *n = 0; *nb = 0;
  if (p >= P) return;
  const uint32_t b0 = panel_ptr[p], b1 = panel_ptr[p + 1];
  if (b1 == b0) return;
  const uint32_t* l = brick_cols + (size_t)b0 * kBrickK;
  uint32_t cnt = (b1 - b0) * kBrickK;
  while (cnt > 0 && l[cnt - 1] == kPadCol) --cnt;   // at most three pads
  *list = l; *n = cnt; *nb = b1 - b0;
}

// number of entries of the sorted list that are smaller than x
__device__ inline uint32_t count_below(const uint32_t* __restrict__ l, uint32_t n, uint32_t x) {
  uint32_t lo = 0, hi = n;
  while (lo < hi) {
    const uint32_t mid = (lo + hi) >> 1;
    if (l[mid] < x) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// exclusive scan of one value per lane across the wavefront; returns the total in *total_out
__device__ inline uint32_t wave_excl(uint32_t v, uint32_t* total_out) {
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

// Pass 1: one wavefront per super-panel.  cpre[i] = number of columns among the first i of the
// bottom list that also occur in the top list (n1 + 1 entries per super-panel, stored at
// 4 * first brick of the bottom panel + its panel index); from it the size of the union, the
// merge decision and the number of brick columns.
__global__ __launch_bounds__(64) void k_tm32_count(const uint32_t* __restrict__ panel_ptr,
                                                  const uint32_t* __restrict__ brick_cols,
                                                  int64_t P, uint32_t num, uint32_t den,
                                                  uint32_t* __restrict__ cpre,
                                                  uint8_t* __restrict__ sp_merged,
                                                  uint32_t* __restrict__ nbc_q) {
  const int64_t q = blockIdx.x;
  const uint32_t *l0, *l1;
  uint32_t n0, n1, nb0, nb1;
  panel_cols(panel_ptr, brick_cols, P, 2 * q, &l0, &n0, &nb0);
  panel_cols(panel_ptr, brick_cols, P, 2 * q + 1, &l1, &n1, &nb1);
  uint32_t common = 0;
  if (2 * q + 1 < P) {
    uint32_t* pre = cpre + (size_t)panel_ptr[2 * q + 1] * kBrickK + (2 * q + 1);
    uint32_t carry = 0;
    for (uint32_t base = 0; base < n1; base += 64) {
      const uint32_t i = base + threadIdx.x;
      uint32_t f = 0;
      if (i < n1) {
        const uint32_t c = l1[i];
        const uint32_t pos = count_below(l0, n0, c);
        f = (pos < n0 && l0[pos] == c) ? 1u : 0u;
      }
      uint32_t total;
      const uint32_t ex = wave_excl(f, &total);
      if (i < n1) pre[i] = carry + ex;
      carry += total;
    }
    if (threadIdx.x == 0) pre[n1] = carry;
    common = carry;
  }
  if (threadIdx.x == 0) {
    const uint64_t nu = (uint64_t)n0 + n1 - common;
    const uint64_t mx = n0 > n1 ? n0 : n1;
    const bool merged = n0 > 0 && n1 > 0 && nu * den < (uint64_t)num * mx;
    sp_merged[q] = merged ? 1 : 0;
    nbc_q[q] = merged ? (uint32_t)((nu + kBrickK - 1) / kBrickK) : nb0 + nb1;
  }
}

// Pass 2: column ids of the brick columns, and for every column slot of the 16-row format
// (4 b + c) the slot it moves to (4 * brick column + column inside it).  In a merged
// super-panel the rank of a column c in the union is
//   (top columns below c) + (bottom columns below c) - (common columns below c),
// the last term being cpre at the number of bottom columns below c.
__global__ __launch_bounds__(64) void k_tm32_cols(const uint32_t* __restrict__ panel_ptr,
                                                 const uint32_t* __restrict__ brick_cols,
                                                 int64_t P, const uint32_t* __restrict__ cpre,
                                                 const uint8_t* __restrict__ sp_merged,
                                                 const uint32_t* __restrict__ sp_ptr,
                                                 uint32_t* __restrict__ bc_cols,
                                                 uint32_t* __restrict__ new_slot) {
  const int64_t q = blockIdx.x;
  const uint32_t *l0, *l1;
  uint32_t n0, n1, nb0, nb1;
  panel_cols(panel_ptr, brick_cols, P, 2 * q, &l0, &n0, &nb0);
  panel_cols(panel_ptr, brick_cols, P, 2 * q + 1, &l1, &n1, &nb1);
  const uint32_t k0 = sp_ptr[q], k1 = sp_ptr[q + 1];
  const uint32_t out0 = k0 * kBrickK;
  const uint32_t src0 = 2 * q < P ? panel_ptr[2 * q] * kBrickK : 0u;
  const uint32_t src1 = 2 * q + 1 < P ? panel_ptr[2 * q + 1] * kBrickK : 0u;
  if (!sp_merged[q]) {   // top list (with its pads), then bottom list
    for (uint32_t i = threadIdx.x; i < nb0 * kBrickK; i += 64) {
      bc_cols[out0 + i] = l0[i];
      new_slot[src0 + i] = out0 + i;
    }
    for (uint32_t i = threadIdx.x; i < nb1 * kBrickK; i += 64) {
      bc_cols[out0 + nb0 * kBrickK + i] = l1[i];
      new_slot[src1 + i] = out0 + nb0 * kBrickK + i;
    }
    return;
  }
  const uint32_t* pre = cpre + (size_t)src1 + (2 * q + 1);
  for (uint32_t i = threadIdx.x; i < n0; i += 64) {
    const uint32_t c = l0[i];
    const uint32_t pos1 = count_below(l1, n1, c);
    const uint32_t rank = i + pos1 - pre[pos1];
    new_slot[src0 + i] = out0 + rank;
    bc_cols[out0 + rank] = c;
  }
  for (uint32_t i = threadIdx.x; i < n1; i += 64) {
    const uint32_t c = l1[i];
    const uint32_t pos0 = count_below(l0, n0, c);
    const uint32_t rank = pos0 + i - pre[i];
    new_slot[src1 + i] = out0 + rank;
    bc_cols[out0 + rank] = c;   // (a common column is written twice, with the same value)
  }
  const uint32_t nu = n0 + n1 - pre[n1];
  for (uint32_t i = nu + threadIdx.x; i < (k1 - k0) * kBrickK; i += 64) bc_cols[out0 + i] = kPadCol;
}

// Pass 3: patterns.  One thread per column slot of the 16-row format: the 16 row bits of that
// column move to its new brick column (tmask[2 * brick column + half]).
__global__ void k_tm32_masks(const uint32_t* __restrict__ brick_cols,
                             const uint64_t* __restrict__ brick_mask,
                             const uint32_t* __restrict__ new_slot,
                             const uint8_t* __restrict__ brick_half, int64_t n_slots,
                             unsigned long long* tmask) {
  const int64_t sl = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (sl >= n_slots || brick_cols[sl] == kPadCol) return;
  const int64_t b = sl / kBrickK;
  const int c = (int)(sl % kBrickK);
  const uint64_t m = brick_mask[b] >> c;          // bits 4 r of m: column c of row r
  const uint32_t ns = new_slot[sl];
  const int c2 = (int)(ns % kBrickK);
  const uint64_t moved = (m & 0x1111111111111111ull) << c2;
  if (moved) atomicOr(&tmask[2 * (size_t)(ns / kBrickK) + brick_half[b]], moved);
}

// half (0 = top, 1 = bottom of its super-panel) of every brick of the 16-row format
__global__ void k_tm32_brick_half(const uint32_t* __restrict__ panel_ptr, int64_t P,
                                  uint8_t* __restrict__ brick_half) {
  const int64_t p = blockIdx.x;
  for (uint32_t b = panel_ptr[p] + threadIdx.x; b < panel_ptr[p + 1]; b += blockDim.x)
    brick_half[b] = (uint8_t)(p & 1);
}

struct LoadPresent {
  const unsigned long long* t;
  __device__ uint32_t operator()(int64_t i) const { return t[i] != 0 ? 1u : 0u; }
};

// Pass 4: compact the present bricks.  pos[s] = exclusive scan of (tmask[s] != 0), 2 nbc + 1
// entries.
__global__ void k_tm32_compact(const unsigned long long* __restrict__ tmask,
                               const uint32_t* __restrict__ pos, int64_t nbc,
                               uint32_t* __restrict__ bc_brick, uint8_t* __restrict__ br_row,
                               uint64_t* __restrict__ br_mask) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s > 2 * nbc) return;
  if ((s & 1) == 0) bc_brick[s / 2] = pos[s];     // also the closing entry at s = 2 nbc
  if (s < 2 * nbc && tmask[s]) {
    br_row[pos[s]] = (uint8_t)(s & 1);
    br_mask[pos[s]] = tmask[s];
  }
}

// Pass 5: values.  One lane per pattern bit of the 16-row format: old position -> new position.
__global__ __launch_bounds__(256) void k_tm32_values(
    const uint64_t* __restrict__ brick_mask, const uint32_t* __restrict__ brick_valptr,
    const float* __restrict__ vals, const uint32_t* __restrict__ new_slot,
    const uint8_t* __restrict__ brick_half, const uint32_t* __restrict__ pos,
    const uint64_t* __restrict__ br_mask, const uint32_t* __restrict__ br_valptr, int64_t nb,
    float* __restrict__ out) {
  const int64_t b = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (b >= nb) return;
  const int bit = threadIdx.x & 63;
  const uint64_t m = brick_mask[b];
  if (!((m >> bit) & 1)) return;
  const uint32_t src = brick_valptr[b] + (uint32_t)__popcll(m & ((1ull << bit) - 1ull));
  const uint32_t ns = new_slot[b * kBrickK + (bit & 3)];
  const uint32_t j = pos[2 * (size_t)(ns / kBrickK) + brick_half[b]];
  const int bit2 = (bit & ~3) | (int)(ns % kBrickK);
  out[br_valptr[j] + (uint32_t)__popcll(br_mask[j] & ((1ull << bit2) - 1ull))] = vals[src];
}

// Per brick column, for the kernel: patterns and value offsets of its top and bottom brick
// (zero pattern where there is none).
__global__ void k_tm32_meta(const uint32_t* __restrict__ bc_brick, const uint8_t* __restrict__ br_row,
                            const uint64_t* __restrict__ br_mask,
                            const uint32_t* __restrict__ br_valptr, int64_t nbc, uint32_t nnz,
                            Tm32Meta* __restrict__ meta, int64_t n_meta) {
  const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n_meta) return;
  Tm32Meta m{0ull, 0ull, nnz, nnz};
  if (k < nbc) {
    for (uint32_t j = bc_brick[k]; j < bc_brick[k + 1]; ++j) {
      if (br_row[j] == 0) { m.mask_top = br_mask[j]; m.off_top = br_valptr[j]; }
      else { m.mask_bot = br_mask[j]; m.off_bot = br_valptr[j]; }
    }
  }
  meta[k] = m;
}

// ------------------------------------------------------------------ SpMM on 32-row panels
// One wavefront owns a super-panel and 16 T columns of C: 32 x 16 T accumulators.  The loop
// runs over brick columns; the B rows of a brick column are loaded once and multiplied with its
// top brick and with its bottom brick (the reuse of Eq. 5).  Everything else follows the
// 16-row kernel: patterns and value offsets through the scalar cache (four brick columns per
// fetch), decode in pattern-bit order with v_mbcnt and one ds_bpermute into MFMA lane order,
// B-row byte offsets handed out across lanes, a ring of register stages for the loads.
constexpr int kTmChunk = 4;    // brick columns per metadata fetch
constexpr int kTmStages = 4;   // brick columns whose loads are in flight

template <int T>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_spmm_tm32(
    const uint32_t* __restrict__ sp_ptr, const uint32_t* __restrict__ bc_cols,
    const Tm32Meta* __restrict__ meta, const float* __restrict__ vals, int64_t Q,
    const float* __restrict__ B, float* __restrict__ C, int64_t M, int64_t N, uint32_t k_last) {
  constexpr int V = T < 4 ? T : 4;
  constexpr int NV = T / V;
  constexpr int R = kTmStages;
  constexpr int CH = kTmChunk;
  static_assert(CH % R == 0 && CH * kBrickK <= 64, "stage and lane mapping assume this");

  const int lane = threadIdx.x & 63;
  const uint32_t vblock = xcd_contiguous_block();
  // the wavefront's index as a scalar: its range comes through the scalar cache
  const int64_t q = (int64_t)vblock * kWavesPerBlock + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (q >= Q) return;  // whole wavefront leaves together
  const uint32_t k_begin = sp_ptr[q];
  const uint32_t k_end = sp_ptr[q + 1];

  const int j = lane & 15;
  const int kq = lane >> 4;
  const uint32_t perm_transpose = 4u * (uint32_t)(4 * j + kq);  // ds_bpermute: read lane 4j + kq
  const int64_t ncol0 = (int64_t)blockIdx.y * (16 * T) + V * j;
  const uint32_t row_bytes = (uint32_t)N * 4u;
  uint32_t lane_off[NV];
#pragma unroll
  for (int qv = 0; qv < NV; ++qv)
    lane_off[qv] = (uint32_t)min<int64_t>(ncol0 + qv * 16 * V, N - V) * 4u;
  const uint32_t perm_base = 4u * (uint32_t)kq;

  float4_t acc[2][T];
#pragma unroll
  for (int h = 0; h < 2; ++h)
#pragma unroll
    for (int u = 0; u < T; ++u) acc[h][u] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (k_begin < k_end) {
    const uint32_t ncols = k_end - k_begin;   // brick columns
    const char* Bbytes = reinterpret_cast<const char*>(B);

    struct Chunk { uint64_t mt[CH], mb[CH]; uint32_t ot[CH], ob[CH]; };
    auto load_meta = [&](uint32_t base) {   // uniform addresses: scalar loads
      const Tm32Meta* __restrict__ mp = meta + base;
      Chunk c;
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        c.mt[i] = mp[i].mask_top; c.mb[i] = mp[i].mask_bot;
        c.ot[i] = mp[i].off_top; c.ob[i] = mp[i].off_bot;
      }
      return c;
    };
    // lane 4*i + c: byte offset of B row bc_cols[4*(base+i) + c]; steps past the last brick
    // column re-read that column's rows (cache hits)
    auto load_col = [&](uint32_t base) {
      const uint32_t slot = (uint32_t)lane & (CH * kBrickK - 1);
      const uint32_t idx = min(base * kBrickK + slot, (k_end - 1) * kBrickK + (slot & (kBrickK - 1)));
      return bc_cols[idx];
    };
    auto row_offset = [&](uint32_t col) { return min(col, k_last) * row_bytes; };

    uint64_t st_mt[R], st_mb[R];
    float st_at[R], st_ab[R];
    float st_b[R][T];
    auto issue = [&](uint64_t mt, uint64_t mb, uint32_t ot, uint32_t ob, uint32_t ro, int s) {
      st_mt[s] = mt;
      st_mb[s] = mb;
      const uint32_t ct = __builtin_amdgcn_mbcnt_hi((uint32_t)(mt >> 32),
                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)mt, 0u));
      const uint32_t cb = __builtin_amdgcn_mbcnt_hi((uint32_t)(mb >> 32),
                                                    __builtin_amdgcn_mbcnt_lo((uint32_t)mb, 0u));
      // scalar base + 32-bit byte offset (the launcher's caller checks that the values fit)
      const char* vbytes = reinterpret_cast<const char*>(vals);
      st_at[s] = *reinterpret_cast<const float*>(vbytes + (ot * 4u + ct * 4u));
      st_ab[s] = *reinterpret_cast<const float*>(vbytes + (ob * 4u + cb * 4u));
#pragma unroll
      for (int qv = 0; qv < NV; ++qv) {
        float tmp[V];
        load_vec<V>(reinterpret_cast<const float*>(Bbytes + (ro + lane_off[qv])), tmp);
#pragma unroll
        for (int w = 0; w < V; ++w) st_b[s][qv * V + w] = tmp[w];
      }
    };
    // the A operand of a brick: zero fill by its pattern, then the transposition
    auto operand = [&](float v, uint64_t mask) {
      float in_bit_order;
      asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(in_bit_order) : "v"(v), "s"(mask));
      return __builtin_bit_cast(
          float, __builtin_amdgcn_ds_bpermute(perm_transpose, __builtin_bit_cast(int, in_bit_order)));
    };
    auto multiply = [&](float a, float4_t (&a_acc)[T], const float (&b)[T]) {
#pragma unroll
      for (int u = 0; u < T; ++u)
        a_acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b[u], a_acc[u], 0, 0, 0);
    };
    auto compute = [&](int s) {   // the B operands of the stage serve both bricks
      if (st_mt[s] != 0) multiply(operand(st_at[s], st_mt[s]), acc[0], st_b[s]);
      if (st_mb[s] != 0) multiply(operand(st_ab[s], st_mb[s]), acc[1], st_b[s]);
    };
    // steady chunks: both operands of the next brick column are made one step early, under the
    // current column's MFMAs (an empty half costs one wasted cross-lane move)
    float at_ahead = 0.f, ab_ahead = 0.f;

    Chunk cur = load_meta(k_begin);
    uint32_t ro_cur = row_offset(load_col(k_begin));
    asm volatile("" : "+v"(ro_cur));
#pragma unroll
    for (int i = 0; i < CH; ++i)
      asm volatile("" : "+s"(cur.mt[i]), "+s"(cur.mb[i]), "+s"(cur.ot[i]), "+s"(cur.ob[i]));

    // Step g computes brick column g-R from stage g%R and refills that stage with brick column
    // g.  Chunks that lie inside the super-panel and behind its first R steps ("steady") need
    // none of the per-step checks; scheduling barriers keep their steps in order (see the
    // 16-row kernel).  The next chunk's columns become row offsets in the chunk's last step.
    const uint32_t total = ncols + R;
    uint32_t ro_next = __builtin_amdgcn_ds_bpermute(perm_base, ro_cur);
    uint32_t ro_following = 0;
    auto step = [&](auto steady, int i, uint32_t g, const Chunk& m, uint32_t ro_this,
                    uint32_t col_following) {
      constexpr bool kSteady = decltype(steady)::value;
      if constexpr (kSteady) {
        const int s = i % R, sn = (i + 1) % R;
        const float at = at_ahead, ab = ab_ahead;
        at_ahead = operand(st_at[sn], st_mt[sn]);
        ab_ahead = operand(st_ab[sn], st_mb[sn]);
        if (st_mt[s] != 0) multiply(at, acc[0], st_b[s]);
        if (st_mb[s] != 0) multiply(ab, acc[1], st_b[s]);
      } else {
        if (g >= (uint32_t)R && g - R < ncols) compute(i % R);
      }
      const uint32_t ro = ro_next;
      if (i + 1 < CH) {
        ro_next = __builtin_amdgcn_ds_bpermute(perm_base + 16u * (i + 1), ro_this);
      } else {
        ro_following = row_offset(col_following);
        ro_next = __builtin_amdgcn_ds_bpermute(perm_base, ro_following);
      }
      const bool live = kSteady || g < ncols;   // uniform: scalar selects
      issue(live ? m.mt[i] : 0ull, live ? m.mb[i] : 0ull, m.ot[i], m.ob[i], ro, i % R);
      if constexpr (kSteady) __builtin_amdgcn_sched_barrier(0);
    };
    uint32_t c = 0;
    auto chunk = [&](auto steady) {
      const Chunk nxt = load_meta(k_begin + c + CH);
      const uint32_t col_nxt = load_col(k_begin + c + CH);
#pragma unroll
      for (int i = 0; i < CH; ++i) step(steady, i, c + i, cur, ro_cur, col_nxt);
      cur = nxt;
      ro_cur = ro_following;
    };
    if (c + CH <= total) {
      chunk(std::false_type{});
      c += CH;
    }
    if (c + CH <= ncols) {   // c is a multiple of CH = R here, so stage 0 is next
      at_ahead = operand(st_at[0], st_mt[0]);
      ab_ahead = operand(st_ab[0], st_mb[0]);
    }
    for (; c + CH <= ncols; c += CH) chunk(std::true_type{});
    for (; c + CH <= total; c += CH) chunk(std::false_type{});
    if (c < total) {
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        if (i % R == 0 && i > 0 && c + i >= total) break;
        step(std::false_type{}, i, c + i, cur, ro_cur, 0u);
      }
    }
  }

  // acc[h][qv*V + w][v] = C[row 32 q + 16 h + 4 kq + v][ncol0 + qv*16*V + w]
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t row0 = q * 32 + 16 * h + 4 * kq;
    float* out = C + row0 * N;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      if (row0 + v < M) {
#pragma unroll
        for (int qv = 0; qv < NV; ++qv) {
          const int64_t ncol = ncol0 + qv * 16 * V;
          if (ncol < N) {
            typedef typename Vec<V>::type vt;
            vt t;
            if constexpr (V == 1) t = acc[h][qv][v];
            else {
#pragma unroll
              for (int w = 0; w < V; ++w) t[w] = acc[h][qv * V + w][v];
            }
            __builtin_nontemporal_store(t, reinterpret_cast<vt*>(out + v * N + ncol));
          }
        }
      }
    }
  }
}

}  // namespace

// ---- host side: builder passes (enqueue only; the caller reads back the two totals) and launch
hipError_t launch_tm32_count(const uint32_t* panel_ptr, const uint32_t* brick_cols, int64_t P,
                             int64_t Q, uint32_t num, uint32_t den, uint32_t* cpre,
                             uint8_t* sp_merged, uint32_t* nbc_q, hipStream_t s) {
  if (Q == 0) return hipSuccess;
  hipLaunchKernelGGL(k_tm32_count, dim3((unsigned)Q), dim3(64), 0, s, panel_ptr, brick_cols, P, num,
                     den, cpre, sp_merged, nbc_q);
  return hipGetLastError();
}

hipError_t launch_tm32_cols_masks(const uint32_t* panel_ptr, const uint32_t* brick_cols,
                                  const uint64_t* brick_mask, int64_t P, int64_t Q, int64_t nb,
                                  const uint32_t* cpre, const uint8_t* sp_merged,
                                  const uint32_t* sp_ptr, uint32_t* bc_cols, uint32_t* new_slot,
                                  uint8_t* brick_half, unsigned long long* tmask, hipStream_t s) {
  if (Q == 0 || nb == 0) return hipSuccess;
  hipLaunchKernelGGL(k_tm32_cols, dim3((unsigned)Q), dim3(64), 0, s, panel_ptr, brick_cols, P, cpre,
                     sp_merged, sp_ptr, bc_cols, new_slot);
  hipLaunchKernelGGL(k_tm32_brick_half, dim3((unsigned)P), dim3(64), 0, s, panel_ptr, P, brick_half);
  hipLaunchKernelGGL(k_tm32_masks, dim3(grid_for(nb * kBrickK)), dim3(kThreads), 0, s, brick_cols,
                     brick_mask, new_slot, brick_half, nb * kBrickK, tmask);
  return hipGetLastError();
}

hipError_t launch_tm32_compact(const unsigned long long* tmask, const uint32_t* pos, int64_t nbc,
                               uint32_t* bc_brick, uint8_t* br_row, uint64_t* br_mask,
                               hipStream_t s) {
  hipLaunchKernelGGL(k_tm32_compact, dim3(grid_for(2 * nbc + 1)), dim3(kThreads), 0, s, tmask, pos,
                     nbc, bc_brick, br_row, br_mask);
  return hipGetLastError();
}

hipError_t launch_tm32_values(const uint64_t* brick_mask, const uint32_t* brick_valptr,
                              const float* vals, const uint32_t* new_slot,
                              const uint8_t* brick_half, const uint32_t* pos,
                              const uint64_t* br_mask, const uint32_t* br_valptr, int64_t nb,
                              float* out, hipStream_t s) {
  if (nb == 0) return hipSuccess;
  hipLaunchKernelGGL(k_tm32_values, dim3((unsigned)((nb + 3) / 4)), dim3(256), 0, s, brick_mask,
                     brick_valptr, vals, new_slot, brick_half, pos, br_mask, br_valptr, nb, out);
  return hipGetLastError();
}

hipError_t launch_tm32_meta(const uint32_t* bc_brick, const uint8_t* br_row, const uint64_t* br_mask,
                            const uint32_t* br_valptr, int64_t nbc, int64_t nnz, Tm32Meta* meta,
                            int64_t n_meta, hipStream_t s) {
  hipLaunchKernelGGL(k_tm32_meta, dim3(grid_for(n_meta)), dim3(kThreads), 0, s, bc_brick, br_row,
                     br_mask, br_valptr, nbc, (uint32_t)nnz, meta, n_meta);
  return hipGetLastError();
}

hipError_t launch_spmm_tm32(const uint32_t* sp_ptr, const uint32_t* bc_cols, const Tm32Meta* meta,
                            const float* vals, int64_t Q, const float* B, float* C, int64_t M,
                            int64_t N, int64_t K, hipStream_t s) {
  if (Q == 0 || N == 0) return hipSuccess;
  const int tile = mfma_tile_for(N);
  unsigned gx = (unsigned)((Q + kWavesPerBlock - 1) / kWavesPerBlock);
  gx = (gx + kXcds - 1) / kXcds * kXcds;  // whole rounds over the XCDs
  const dim3 grid(gx, (unsigned)((N + tile - 1) / tile)), block(64 * kWavesPerBlock);
  const uint32_t k_last = (uint32_t)(K - 1);
#define SPMM_LAUNCH_TM32(TT)                                                                    \
  hipLaunchKernelGGL((k_spmm_tm32<TT>), grid, block, 0, s, sp_ptr, bc_cols, meta, vals, Q, B, C, \
                     M, N, k_last)
  switch (tile) {
    case 16: SPMM_LAUNCH_TM32(1); break;
    case 32: SPMM_LAUNCH_TM32(2); break;
    case 64: SPMM_LAUNCH_TM32(4); break;
    default: SPMM_LAUNCH_TM32(8); break;
  }
#undef SPMM_LAUNCH_TM32
  return hipGetLastError();
}

}  // namespace spmm
