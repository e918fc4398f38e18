// SpMM kernels for gfx950 (paper Section 3.3 / Algorithm 1, re-designed for
// wave64 and v_mfma_f32_16x16x4_f32).
//
// MFMA brick kernel.  One wavefront owns one work item: the bricks
// [brick_begin, brick_end) of one 16-row panel and a tile of n_tile = 16*T
// columns of C.  A 16x4 brick is exactly the A operand of the 16x16x4 MFMA:
//   A operand (1 VGPR): lane l holds A[row l%16][k = l/16]
//   B operand (1 VGPR): lane l holds B[k = l/16][col l%16]
//   D (4 VGPRs):        lane l, register v holds D[row 4*(l/16)+v][col l%16]
// so lane l expands pattern bit 4*(l%16) + l/16 (the paper numbers brick
// elements row-major): value index = popcount of the pattern below that bit,
// which is the prefix-count decode of Algorithm 1 done per lane on a
// wave-uniform mask.  Which column of the C tile an MFMA "column" stands for is
// free, so lane l loads T consecutive floats of B row brick_cols[4b + l/16]
// (dwordx4 loads, 256 contiguous bytes per 16 lanes) and feeds element u to
// MFMA u; its accumulators then hold T consecutive columns of 4 rows of C and
// are stored as dwordx4.  B therefore goes HBM/L2 -> registers directly; no
// LDS staging is needed because a B row of a panel is used by exactly one
// brick when panels are 16 rows high.
//
// Loads are software-pipelined through a ring of register stages: while the
// MFMAs of brick b issue, the values and B rows of the next kStages bricks are
// in flight; brick metadata is fetched 16 bricks at a time with coalesced loads
// and distributed by cross-lane reads.
//
// Vector-ALU CSR kernels (the paper's "scalar core" path): one B-row load and one FMA per
// stored entry, no zero filling and no reuse of B rows inside a panel.  Rows are processed
// side by side in a wavefront (k_spmm_valu_rows), very long rows by a workgroup each
// (k_spmm_valu_long); k_spmm_valu (one wavefront per row) serves widths that are not a
// multiple of four.  Used for the panels that the routing sends to the CSR path.
#include "exec_common.h"

#include <type_traits>

namespace spmm {

int long_row_threshold() { return 256; }

int mfma_tile_for(int64_t N) { return N <= 16 ? 16 : (N <= 32 ? 32 : (N <= 64 ? 64 : 128)); }

namespace {

constexpr int kStages = 4;   // bricks whose loads are in flight per wavefront (MFMA kernel)
constexpr int kChunk = 16;   // bricks per coalesced metadata fetch
static_assert(kChunk % kStages == 0 && kChunk == 16, "stage and lane mapping assume this");

// T floats of one B row for this lane: NV vectors of V floats.
// ALIGNED: N % V == 0 and 16-byte aligned base, so a vector is entirely inside
// or entirely outside [0, N).  Columns at or beyond N are read from a clamped,
// valid address instead of being zeroed: column j of the product depends only
// on column j of B, and columns >= N of the tile are never stored.
template <int T, bool ALIGNED>
__device__ inline void load_b(const float* __restrict__ brow, int64_t N, int64_t ncol0,
                              float (&bv)[T]) {
  constexpr int V = T < 4 ? T : 4;
  constexpr int NV = T / V;
#pragma unroll
  for (int q = 0; q < NV; ++q) {
    const int64_t n = ncol0 + q * 16 * V;
    if constexpr (ALIGNED) {
      float tmp[V];
      load_vec<V>(brow + min(n, N - V), tmp);
#pragma unroll
      for (int w = 0; w < V; ++w) bv[q * V + w] = tmp[w];
    } else {
#pragma unroll
      for (int w = 0; w < V; ++w) bv[q * V + w] = brow[min(n + w, N - 1)];
    }
  }
}

template <int T, bool ALIGNED>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_spmm_mfma(
    BrickFormat f, const WorkItem* __restrict__ items, int64_t n_items,
    const float* __restrict__ B, float* __restrict__ C, float* __restrict__ partial, int64_t M,
    int64_t N) {
  constexpr int V = T < 4 ? T : 4;
  constexpr int NV = T / V;
  const int lane = threadIdx.x & 63;
  const uint32_t vblock = xcd_contiguous_block();   // contiguous range of work items per XCD
  const int64_t item_id = (int64_t)vblock * kWavesPerBlock + (threadIdx.x >> 6);
  if (item_id >= n_items) return;  // whole wavefront leaves together
  const WorkItem it = items[item_id];
  const uint32_t panel = __builtin_amdgcn_readfirstlane(it.panel);
  const uint32_t b_begin = __builtin_amdgcn_readfirstlane(it.brick_begin);
  const uint32_t b_end = __builtin_amdgcn_readfirstlane(it.brick_end);
  const uint32_t slot = __builtin_amdgcn_readfirstlane(it.slot);

  const int j = lane & 15;   // MFMA column / brick row
  const int kq = lane >> 4;  // MFMA k / brick column
  const int bit = 4 * j + kq;
  const uint64_t below = (1ull << bit) - 1ull;
  const int64_t ncol0 = (int64_t)blockIdx.y * (16 * T) + V * j;  // first C column of this lane

  float4_t acc[T];
#pragma unroll
  for (int u = 0; u < T; ++u) acc[u] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (b_begin < b_end) {
    const uint32_t last = b_end - 1;
    const uint32_t nbricks = b_end - b_begin;
    constexpr int R = kStages;   // bricks in flight per wavefront
    constexpr int CH = kChunk;   // bricks per metadata chunk

    // Metadata of CH consecutive bricks, fetched with three coalesced loads and
    // handed out per brick by cross-lane reads (no memory latency per brick):
    //   cols: lane l holds brick_cols[4*(base + l/4) + l%4]
    //   mask, off: lane l holds brick_mask / brick_valptr of brick base + l%16
    struct Chunk { uint32_t cols; uint32_t mask_lo, mask_hi; uint32_t off; };
    auto load_chunk = [&](uint32_t base) {
      const uint32_t bc = min(base + (uint32_t)(lane >> 2), last);
      const uint32_t bm = min(base + (uint32_t)(lane & (CH - 1)), last);
      const uint64_t m = f.brick_mask[bm];
      return Chunk{f.brick_cols[(int64_t)bc * kBrickK + (lane & 3)], (uint32_t)m,
                   (uint32_t)(m >> 32), f.brick_valptr[bm]};
    };

    // R register stages; stage s holds the loads of one brick in flight.
    uint64_t st_mask[R];
    float st_a[R];
    float st_b[R][T];

    // Issue the loads of brick i of the chunk into stage s.  The value index is
    // the number of pattern bits below this lane's bit; lanes whose bit is clear
    // read a neighbouring value (vals has one pad element) that is discarded.
    auto issue = [&](const Chunk& ch, uint32_t i, int s) {
      const uint32_t mlo = __builtin_amdgcn_readlane(ch.mask_lo, i);
      const uint32_t mhi = __builtin_amdgcn_readlane(ch.mask_hi, i);
      const uint32_t off = __builtin_amdgcn_readlane(ch.off, i);
      const uint64_t mask = ((uint64_t)mhi << 32) | mlo;
      const uint32_t col = __builtin_amdgcn_ds_bpermute(4 * (4 * i + kq), ch.cols);
      st_mask[s] = mask;
      st_a[s] = f.vals[(int64_t)off + __popcll(mask & below)];
      load_b<T, ALIGNED>(B + (int64_t)(col == kPadCol ? 0u : col) * N, N, ncol0, st_b[s]);
    };
    auto compute = [&](int s) {
      const float a = ((st_mask[s] >> bit) & 1ull) ? st_a[s] : 0.f;
#pragma unroll
      for (int u = 0; u < T; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, st_b[s][u], acc[u], 0, 0, 0);
    };

    // The first chunk passes through an empty asm statement so that it is not a
    // plain load: otherwise the compiler merges it with the in-loop chunk load
    // into one load at the top of the loop, serialising that latency.
    Chunk cur = load_chunk(b_begin);
    asm volatile("" : "+v"(cur.cols), "+v"(cur.mask_lo), "+v"(cur.mask_hi), "+v"(cur.off));

    // Step g computes brick g-R from stage g%R and then refills that stage with
    // brick g, so R bricks' loads are in flight while the MFMAs issue.  Refills
    // are unconditional (past the end they re-read the last brick, which is
    // harmless and keeps the compiler's count of outstanding loads exact); only
    // the MFMAs are skipped for steps that hold no brick.
    const uint32_t total = nbricks + R;
    for (uint32_t c = 0; c < total; c += CH) {
      const Chunk nxt = load_chunk(b_begin + c + CH);
#pragma unroll 1
      for (uint32_t i0 = 0; i0 < (uint32_t)CH; i0 += R) {
        if (c + i0 >= total) break;
#pragma unroll
        for (int s = 0; s < R; ++s) {
          const uint32_t g = c + i0 + s;
          if (g >= (uint32_t)R && g - R < nbricks) compute(s);
          issue(cur, i0 + s, s);
        }
      }
      cur = nxt;
    }
  }

  // acc[q*V + w][v] = C[row 4*kq + v][ncol0 + q*16*V + w]
  float* out;
  int64_t rows_left;
  if (slot == kNoSlot) {
    const int64_t row0 = (int64_t)panel * kPanel + 4 * kq;
    out = C + row0 * N;
    rows_left = M - row0;
  } else {
    out = partial + ((int64_t)slot * kPanel + 4 * kq) * N;
    rows_left = 4;
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    if (v < rows_left) {
#pragma unroll
      for (int q = 0; q < NV; ++q) {
        const int64_t n = ncol0 + q * 16 * V;
        float tmp[V];
#pragma unroll
        for (int w = 0; w < V; ++w) tmp[w] = acc[q * V + w][v];
        if constexpr (ALIGNED) {
          if (n < N) store_vec<V>(out + v * N + n, tmp);
        } else {
#pragma unroll
          for (int w = 0; w < V; ++w)
            if (n + w < N) out[v * N + n + w] = tmp[w];
        }
      }
    }
  }
}

// ------------------------------------------------------------------ MFMA, fast path
// Same lane mapping as above for the common case: N a multiple of the vector
// width, 16-byte aligned B and C, and B smaller than 4 GiB (32-bit byte offsets).
//
// Vector-ALU instructions overlap only partly with MFMAs on a SIMD (measured:
// about 2 cycles of MFMA time lost per extra VALU instruction), so the per-brick
// VALU work is kept small:
//   * pattern and value offset of each brick come through the scalar cache into
//     SGPRs (8 bricks per fetch), not through vector loads and cross-lane reads;
//   * the B-row byte offsets of 8 bricks are computed once per 8 bricks (one
//     lane per brick column) and handed out with ds_bpermute, which issues on
//     the LDS port;
//   * loads use a scalar base plus a 32-bit lane offset.
// The arrays behind BrickFormat carry kFormatPad spare bricks at the end, so
// patterns and value offsets are fetched 8 bricks at a time without clamping.
// The loads issued for the few steps past a work item's last brick repeat that
// brick's B rows and values (cache hits, data never used): with short panels (ten
// bricks, say) four steps of the next panel's rows would otherwise add 40 % to
// the traffic from memory.
constexpr int kFastChunk = 8;

template <int T, bool FULL>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_spmm_mfma_fast(
    const uint32_t* __restrict__ brick_cols, const uint64_t* __restrict__ brick_mask,
    const uint32_t* __restrict__ brick_valptr, const float* __restrict__ vals,
    const WorkItem* __restrict__ items, int64_t n_items, const float* __restrict__ B,
    float* __restrict__ C, float* __restrict__ partial, int64_t M, int64_t N, uint32_t k_last) {
  // (the format arrays are separate __restrict__ parameters, not a struct, so that
  // the compiler knows they are read-only here and may use the scalar cache)
  constexpr int V = T < 4 ? T : 4;
  constexpr int NV = T / V;
  constexpr int R = kStages;
  constexpr int CH = kFastChunk;
  static_assert(CH % R == 0 && CH * kBrickK <= 64, "stage and lane mapping assume this");

  const int lane = threadIdx.x & 63;
  const uint32_t vblock = xcd_contiguous_block();   // contiguous range of work items per XCD
  // the wavefront's index as a scalar, so that its work item comes through the scalar cache
  // (one round trip less through the vector-memory path before the first brick)
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t item_id = (int64_t)vblock * kWavesPerBlock + wave;
  if (item_id >= n_items) return;  // whole wavefront leaves together
  const WorkItem it = items[item_id];
  const uint32_t panel = it.panel;
  const uint32_t b_begin = it.brick_begin;
  const uint32_t b_end = it.brick_end;
  const uint32_t slot = it.slot;

  const int j = lane & 15;
  const int kq = lane >> 4;
  const uint32_t perm_transpose = 4u * (uint32_t)(4 * j + kq);  // ds_bpermute: read lane 4j + kq
  const int64_t ncol0 = (int64_t)blockIdx.y * (16 * T) + V * j;
  const uint32_t row_bytes = (uint32_t)N * 4u;
  // byte offset of this lane's vectors inside a B row (columns >= N: clamped, never stored)
  uint32_t lane_off[NV];
#pragma unroll
  for (int q = 0; q < NV; ++q)
    lane_off[q] = (uint32_t)min<int64_t>(ncol0 + q * 16 * V, N - V) * 4u;
  const uint32_t perm_base = 4u * (uint32_t)kq;  // ds_bpermute byte address of lane kq

  float4_t acc[T];
#pragma unroll
  for (int u = 0; u < T; ++u) acc[u] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (b_begin < b_end) {
    const uint32_t nbricks = b_end - b_begin;
    const char* Bbytes = reinterpret_cast<const char*>(B);

    struct Meta { uint64_t mask[CH]; uint32_t off[CH]; };
    auto load_meta = [&](uint32_t base) {   // uniform addresses: scalar loads
      // one pointer per array, constant offsets: lets the loads merge into wide scalar loads
      const uint64_t* __restrict__ mp = brick_mask + base;
      const uint32_t* __restrict__ op = brick_valptr + base;
      Meta m;
#pragma unroll
      for (int i = 0; i < CH; ++i) { m.mask[i] = mp[i]; m.off[i] = op[i]; }
      return m;
    };
    // lane 4*i + c: byte offset of B row brick_cols[4*(base+i) + c]; pad columns
    // (0xFFFFFFFF) clamp to the last row, which is harmless since A is 0 there
    auto load_col = [&](uint32_t base) {
      // steps past the work item's last brick re-read that brick's rows (cache hits) instead
      // of pulling the next panel's B rows through the memory system for nothing
      const uint32_t slot = (uint32_t)lane & (CH * kBrickK - 1);
      const uint32_t idx = min(base * kBrickK + slot, (b_end - 1) * kBrickK + (slot & (kBrickK - 1)));
      return brick_cols[idx];
    };
    auto row_offset = [&](uint32_t col) { return min(col, k_last) * row_bytes; };

    uint64_t st_mask[R];
    float st_a[R];
    float st_b[R][T];
    // Decode (the prefix-count decode of Algorithm 1) in pattern-bit order, then transpose:
    // lane l first acts for pattern bit l.  Its value index is the number of pattern bits
    // below bit l, which is what v_mbcnt computes from the wave-uniform pattern in two
    // instructions; the gather that fetches it has addresses that never decrease from lane
    // to lane, which the vector-memory pipe handles as cheaply as a contiguous load (a gather
    // in MFMA lane order costs it as much as a dwordx4 load).  Lanes whose bit is clear are
    // zeroed with the pattern itself as the select mask.  One ds_bpermute (LDS port, no
    // vector-ALU slot) then moves element (row r, column c) from lane 4r + c to the lane the
    // MFMA wants it in, 16c + r.
    auto issue = [&](uint64_t mask, uint32_t off, uint32_t ro, int s) {
      st_mask[s] = mask;
      const uint32_t cnt = __builtin_amdgcn_mbcnt_hi(
          (uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
      // scalar base + 32-bit byte offset (the launcher checks that the values fit 4 GiB)
      st_a[s] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(vals) +
                                                (off * 4u + cnt * 4u));
      const char* brow = Bbytes + (ro + lane_off[0]);
#pragma unroll
      for (int q = 0; q < NV; ++q) {
        float tmp[V];
        // whole tiles: the q-th vector lies a constant distance behind the first
        if constexpr (FULL) load_vec<V>(reinterpret_cast<const float*>(brow + q * 16 * V * 4), tmp);
        else load_vec<V>(reinterpret_cast<const float*>(Bbytes + (ro + lane_off[q])), tmp);
#pragma unroll
        for (int w = 0; w < V; ++w) st_b[s][q * V + w] = tmp[w];
      }
    };
    // the A operand of the brick in stage s: zero fill, then the transposition
    auto operand = [&](int s) {
      float in_bit_order;
      asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(in_bit_order) : "v"(st_a[s]), "s"(st_mask[s]));
      return __builtin_bit_cast(
          float, __builtin_amdgcn_ds_bpermute(perm_transpose, __builtin_bit_cast(int, in_bit_order)));
    };
    auto multiply = [&](float a, int s) {
#pragma unroll
      for (int u = 0; u < T; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, st_b[s][u], acc[u], 0, 0, 0);
    };
    auto compute = [&](int s) { multiply(operand(s), s); };
    float a_ahead = 0.f;   // steady chunks: the next step's A operand, made one step early

    Meta cur = load_meta(b_begin);
    uint32_t ro_cur = row_offset(load_col(b_begin));
    const uint32_t off_last = brick_valptr[b_end - 1];
    // keep the first fetch from being merged with the in-loop fetch into one
    // load at the top of the loop (which would expose its latency every chunk)
    asm volatile("" : "+v"(ro_cur));
#pragma unroll
    for (int i = 0; i < CH; ++i) asm volatile("" : "+s"(cur.mask[i]), "+s"(cur.off[i]));

    // Step g computes brick g-R from stage g%R and then refills that stage with
    // brick g, so R bricks' loads are in flight while the MFMAs issue.  Refills
    // are unconditional up to the next multiple of R past the end (keeps the
    // compiler's count of outstanding loads exact); only MFMAs are skipped for
    // steps that hold no brick.
    const uint32_t total = nbricks + R;
    uint32_t ro_next = __builtin_amdgcn_ds_bpermute(perm_base, ro_cur);
    // `steady`: the chunk lies entirely inside the work item and behind its first R steps, so
    // every step has a brick to compute and a brick to fetch and needs none of the checks
    // col_following: the next chunk's columns as loaded at the start of this chunk; they are
    // turned into row offsets in the chunk's last step, so that nothing waits for that load
    // while the ring's loads are younger than it
    uint32_t ro_following = 0;
    auto step = [&](auto steady, int i, uint32_t g, const Meta& m, uint32_t ro_this,
                    uint32_t col_following) {
      constexpr bool kSteady = decltype(steady)::value;
      if constexpr (kSteady) {
        // the cross-lane move of the next brick's operand runs under this brick's MFMAs
        const float a = a_ahead;
        a_ahead = operand((i + 1) % R);
        multiply(a, i % R);
      } else {
        if (g >= (uint32_t)R && g - R < nbricks) compute(i % R);
      }
      // this lane's row offset was fetched across lanes one step ago (its LDS-port latency
      // hides behind the MFMAs above); fetch the next brick's now
      const uint32_t ro = ro_next;
      if (i + 1 < CH) {
        ro_next = __builtin_amdgcn_ds_bpermute(perm_base + 16u * (i + 1), ro_this);
      } else {
        ro_following = row_offset(col_following);
        ro_next = __builtin_amdgcn_ds_bpermute(perm_base, ro_following);
      }
      const bool live = kSteady || g < nbricks;   // uniform: scalar selects
      issue(live ? m.mask[i] : 0ull, live ? m.off[i] : off_last, ro, i % R);
      // without the branches of the checked variant the steps of a chunk are one basic block;
      // keep the scheduler from sinking a step's loads down to their use R steps later
      if constexpr (kSteady) __builtin_amdgcn_sched_barrier(0);
    };
    // Whole chunks run in loops whose only exit is at their top; the last, partial chunk is
    // straight-line code after them.  With an exit in the middle of a loop body the compiler
    // must assume, at the loop head, that the steps after that exit issued no loads (it
    // cannot see that the loop ends on that path), and it then waits for all but the newest
    // load at the start of every chunk, which empties the ring every CH bricks.
    // Three phases: the first chunk (its first R steps have nothing to compute), the chunks
    // that lie entirely inside the work item (no checks), and the one or two chunks around its
    // end.  Every chunk issues the same loads in the same order, so the count of loads in
    // flight is the same on every path into a loop head.
    uint32_t c = 0;
    auto chunk = [&](auto steady) {
      const Meta nxt = load_meta(b_begin + c + CH);
      const uint32_t col_nxt = load_col(b_begin + c + CH);
#pragma unroll
      for (int i = 0; i < CH; ++i) step(steady, i, c + i, cur, ro_cur, col_nxt);
      cur = nxt;
      ro_cur = ro_following;
    };
    if (c + CH <= total) {
      chunk(std::false_type{});
      c += CH;
    }
    if (c + CH <= nbricks) a_ahead = operand(0);   // c is a multiple of CH, so stage 0 is next
    for (; c + CH <= nbricks; c += CH) chunk(std::true_type{});
    for (; c + CH <= total; c += CH) chunk(std::false_type{});
    if (c < total) {
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        if (i % R == 0 && i > 0 && c + i >= total) break;
        step(std::false_type{}, i, c + i, cur, ro_cur, 0u);   // its last step fetches nothing real
      }
    }
  }

  // acc[q*V + w][v] = C[row 4*kq + v][ncol0 + q*16*V + w]
  float* out;
  int64_t rows_left;
  if (slot == kNoSlot) {
    const int64_t row0 = (int64_t)panel * kPanel + 4 * kq;
    out = C + row0 * N;
    rows_left = M - row0;
  } else {
    out = partial + ((int64_t)slot * kPanel + 4 * kq) * N;
    rows_left = 4;
  }
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    if (v < rows_left) {
#pragma unroll
      for (int q = 0; q < NV; ++q) {
        const int64_t ncol = ncol0 + q * 16 * V;
        if (ncol < N) {
          typedef typename Vec<V>::type vt;
          vt t;
          if constexpr (V == 1) t = acc[q][v];
          else {
#pragma unroll
            for (int w = 0; w < V; ++w) t[w] = acc[q * V + w][v];
          }
          // C is written once and not read again here: stream it past the caches
          __builtin_nontemporal_store(t, reinterpret_cast<vt*>(out + v * N + ncol));
        }
      }
    }
  }
}

// ------------------------------------------------------------------ VALU CSR
template <int V, bool ALIGNED>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_spmm_valu(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
    const float* __restrict__ vals, const uint32_t* __restrict__ panels, int64_t n_panels,
    const float* __restrict__ B, float* __restrict__ C, int64_t M, int64_t N) {
  const int lane = threadIdx.x & 63;
  const int64_t wid = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t pslot = wid / kPanel;
  if (pslot >= n_panels) return;
  const uint32_t panel = __builtin_amdgcn_readfirstlane(panels[pslot]);
  const int64_t row = (int64_t)panel * kPanel + (wid % kPanel);
  if (row >= M) return;
  const int32_t s = __builtin_amdgcn_readfirstlane(rowptr[row]);
  const int32_t t = __builtin_amdgcn_readfirstlane(rowptr[row + 1]);
  const int64_t n = (int64_t)blockIdx.y * (64 * V) + V * lane;

  float acc[V];
#pragma unroll
  for (int w = 0; w < V; ++w) acc[w] = 0.f;

  // columns >= N are read from a clamped address and never stored
  const int64_t n_ld = ALIGNED ? min(n, N - V) : n;
  auto load_row = [&](int32_t col, float (&bv)[V]) {
    const float* brow = B + (int64_t)col * N;
    if constexpr (ALIGNED) load_vec<V>(brow + n_ld, bv);
    else {
#pragma unroll
      for (int w = 0; w < V; ++w) bv[w] = brow[min(n + w, N - 1)];
    }
  };

  int32_t e = s;
  for (; e + 4 <= t; e += 4) {
    int32_t c[4];
    float a[4];
    float bv[4][V];
#pragma unroll
    for (int x = 0; x < 4; ++x) { c[x] = colind[e + x]; a[x] = vals[e + x]; }
#pragma unroll
    for (int x = 0; x < 4; ++x) load_row(c[x], bv[x]);
#pragma unroll
    for (int x = 0; x < 4; ++x)
#pragma unroll
      for (int w = 0; w < V; ++w) acc[w] = fmaf(a[x], bv[x][w], acc[w]);
  }
  for (; e < t; ++e) {
    float bv[V];
    load_row(colind[e], bv);
    const float a = vals[e];
#pragma unroll
    for (int w = 0; w < V; ++w) acc[w] = fmaf(a, bv[w], acc[w]);
  }

  float* out = C + row * N;
  if constexpr (ALIGNED) {
    if (n < N) store_vec<V>(out + n, acc);
  } else {
#pragma unroll
    for (int w = 0; w < V; ++w)
      if (n + w < N) out[n + w] = acc[w];
  }
}

// ------------------------------------------------------------------ VALU CSR, rows side by side
// Several rows per wavefront: a group of LPR lanes owns one row and covers 4*LPR columns of C
// (one dwordx4 per lane and stored entry), so a wavefront works on 64/LPR rows at once: two rows
// at N = 128, eight at N = 32, a whole panel at N = 16.  Column index and value of an entry are
// fetched LPR at a time with coalesced loads and handed out across the group's lanes.
// Four entries are in flight per group and iteration; past the end of a row the last entry is
// re-read with a zero multiplier.  Rows longer than kLongRow entries are left to
// k_spmm_valu_long, which spreads one row over a whole workgroup.
constexpr int kLongRow = 256;   // == long_row_threshold()

template <int LPR>
__global__ __launch_bounds__(64 * kWavesPerBlock) void k_spmm_valu_rows(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
    const float* __restrict__ vals, const uint32_t* __restrict__ panels, int64_t n_panels,
    const float* __restrict__ B, float* __restrict__ C, int64_t M, int64_t N) {
  constexpr int R = 64 / LPR;              // rows per wavefront
  constexpr int WPP = kPanel / R;          // wavefronts per panel (R <= 16)
  const int lane = threadIdx.x & 63;
  const int64_t wid = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
  const int64_t pslot = wid / WPP;
  if (pslot >= n_panels) return;
  const uint32_t panel = __builtin_amdgcn_readfirstlane(panels[pslot]);
  const int64_t row = (int64_t)panel * kPanel + (wid % WPP) * R + lane / LPR;
  const int64_t n = (int64_t)blockIdx.y * (4 * LPR) + 4 * (lane % LPR);
  if (row >= M) return;                    // the whole group leaves together
  // Lanes whose columns lie past N (N is a multiple of 4: whole vectors only) stay: they hold
  // entries that the other lanes of the group fetch from them.  They read a clamped address
  // and store nothing.
  const bool in_range = n < N;
  const int32_t s = rowptr[row], t = rowptr[row + 1];
  if (t - s > kLongRow) return;
  const float* __restrict__ Bn = B + (in_range ? n : N - 4);
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  // The group fetches LPR entries of its row with one coalesced load each for column and
  // value (lane i of the group takes entry i) and hands them out across lanes, four at a
  // time: one B-row load per entry is then the only traffic through the vector-memory pipe.
  const int gl = lane % LPR;               // lane inside the group
  const int g0 = lane - gl;                // first lane of the group
  for (int32_t e0 = s; e0 < t; e0 += LPR) {
    const int32_t me = min(e0 + gl, t - 1);
    const int32_t cv = colind[me];                      // past the end: the last entry again,
    const float av = e0 + gl < t ? vals[me] : 0.f;      // with a zero multiplier
    const int cnt = min(LPR, t - e0);
    for (int x0 = 0; x0 < cnt; x0 += 4) {
      float4_t b[4];
      float a[4];
#pragma unroll
      for (int x = 0; x < 4; ++x) {
        const int src = g0 + min(x0 + x, LPR - 1);
        const int32_t c = __shfl(cv, src, 64);
        a[x] = __shfl(av, src, 64);
        b[x] = *reinterpret_cast<const float4_t*>(Bn + (int64_t)c * N);
      }
#pragma unroll
      for (int x = 0; x < 4; ++x) {
#pragma unroll
        for (int w = 0; w < 4; ++w) acc[w] = fmaf(a[x], b[x][w], acc[w]);
      }
    }
  }
  if (in_range) __builtin_nontemporal_store(acc, reinterpret_cast<float4_t*>(C + row * N + n));
}

// One workgroup of kLongWaves wavefronts per long row: its kLongWaves * (64/LPR) lane groups
// take the row's entries in turn, four at a time, with the next four columns and values
// fetched while the current B rows are in flight; the partial sums are added in group order
// through LDS (deterministic).  `long_rows` lists every row of the matrix with more than
// kLongRow entries; rows whose panel is not in the sorted list `panels` belong to the brick
// kernel and are skipped.
constexpr int kLongWaves = 16;

template <int LPR>
__global__ __launch_bounds__(64 * kLongWaves) void k_spmm_valu_long(
    const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
    const float* __restrict__ vals, const uint32_t* __restrict__ long_rows,
    const uint32_t* __restrict__ panels, int64_t n_panels, const float* __restrict__ B,
    float* __restrict__ C, int64_t N) {
  constexpr int R = 64 / LPR;
  constexpr int G = R * kLongWaves;        // lane groups of the workgroup
  __shared__ float4_t part[G][LPR];
  const int64_t row = long_rows[blockIdx.x];
  const uint32_t panel = (uint32_t)(row / kPanel);
  {   // is the row's panel routed here?  (uniform binary search in the sorted panel list)
    int64_t lo = 0, hi = n_panels;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if (panels[mid] < panel) lo = mid + 1; else hi = mid;
    }
    if (lo >= n_panels || panels[lo] != panel) return;
  }
  const int lane = threadIdx.x & 63;
  const int grp = (threadIdx.x >> 6) * R + lane / LPR;
  const int gl = lane % LPR;
  const int64_t n = (int64_t)blockIdx.y * (4 * LPR) + 4 * gl;
  const bool active = n < N;
  const int32_t s = rowptr[row], t = rowptr[row + 1];
  const float* __restrict__ Bn = B + (active ? n : 0);
  float4_t acc = {0.f, 0.f, 0.f, 0.f};
  int32_t c[4];
  float a[4];
  auto fetch = [&](int32_t e, int32_t (&cc)[4], float (&aa)[4]) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {   // past the end: the last entry again, with a zero multiplier
      const int32_t ex = min(e + x, t - 1);
      cc[x] = colind[ex];
      aa[x] = e + x < t ? vals[ex] : 0.f;
    }
  };
  int32_t e = s + 4 * grp;
  if (e < t) fetch(e, c, a);
  for (; e < t; e += 4 * G) {
    float4_t b[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) b[x] = *reinterpret_cast<const float4_t*>(Bn + (int64_t)c[x] * N);
    int32_t cn[4];
    float an[4];
    fetch(e + 4 * G, cn, an);
#pragma unroll
    for (int x = 0; x < 4; ++x) {
#pragma unroll
      for (int w = 0; w < 4; ++w) acc[w] = fmaf(a[x], b[x][w], acc[w]);
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) { c[x] = cn[x]; a[x] = an[x]; }
  }
  part[grp][gl] = acc;
  __syncthreads();
  if (grp == 0 && active) {
    float4_t sum = part[0][gl];
    for (int q = 1; q < G; ++q) sum += part[q][gl];
    __builtin_nontemporal_store(sum, reinterpret_cast<float4_t*>(C + row * N + n));
  }
}

// ------------------------------------------------------------------ merge (a8)
// Sum the partial 16 x N tiles of a split panel in part order and store to C.
// One workgroup per split panel; VEC floats per thread per step.
template <int VEC>
__global__ __launch_bounds__(256) void k_merge(const MergeItem* __restrict__ items,
                                               const float* __restrict__ partial,
                                               float* __restrict__ C, int64_t M, int64_t N) {
  const MergeItem it = items[blockIdx.x];
  const int64_t row0 = (int64_t)it.panel * kPanel;
  const int64_t rows = min<int64_t>(kPanel, M - row0);
  const int64_t tile = (int64_t)kPanel * N;
  const float* src = partial + (int64_t)it.slot_begin * tile;
  float* dst = C + row0 * N;
  for (int64_t x = (int64_t)threadIdx.x * VEC; x < rows * N; x += (int64_t)blockDim.x * VEC) {
    float s[VEC];
    load_vec<VEC>(src + x, s);
    for (uint32_t q = 1; q < it.nparts; ++q) {
      float t[VEC];
      load_vec<VEC>(src + (int64_t)q * tile + x, t);
#pragma unroll
      for (int w = 0; w < VEC; ++w) s[w] += t[w];
    }
    store_vec<VEC>(dst + x, s);
  }
}

template <int T, bool ALIGNED>
hipError_t launch_mfma_t(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                         const float* B, float* C, float* partial, int64_t M, int64_t N,
                         hipStream_t s) {
  unsigned gx = (unsigned)((n_items + kWavesPerBlock - 1) / kWavesPerBlock);
  gx = (gx + kXcds - 1) / kXcds * kXcds;  // whole rounds over the XCDs
  const unsigned gy = (unsigned)((N + 16 * T - 1) / (16 * T));
  hipLaunchKernelGGL((k_spmm_mfma<T, ALIGNED>), dim3(gx, gy), dim3(64 * kWavesPerBlock), 0, s, f,
                     items, n_items, B, C, partial, M, N);
  return hipGetLastError();
}

template <int T, bool ALIGNED>
int occupancy_t() {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_spmm_mfma<T, ALIGNED>,
                                                   64 * kWavesPerBlock, 0) != hipSuccess || nb < 1)
    nb = 1;
  return nb * kWavesPerBlock;
}

template <int T>
int occupancy_fast_t() {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_spmm_mfma_fast<T, false>, 64 * kWavesPerBlock,
                                                   0) != hipSuccess || nb < 1)
    nb = 1;
  return nb * kWavesPerBlock;
}

}  // namespace

// the fast kernel serves N that is a multiple of the vector width with B below 4 GiB
bool mfma_fast_shape(int64_t N, int64_t K) {
  const int tile = mfma_tile_for(N);
  const int V = tile >= 64 ? 4 : tile / 16;
  return N % V == 0 && K > 0 && (double)K * (double)N * 4.0 < 4294967296.0;
}


// Wavefronts of the MFMA kernel that fit on one CU at a time, for the kernel variant that
// (N, K) selects when the operands are 16-byte aligned: the "thread blocks per SM" of Eq. 7.
int mfma_resident_waves_per_cu(int64_t N, int64_t K) {
  const int tile = mfma_tile_for(N);
  const int V = tile >= 64 ? 4 : tile / 16;
  if (mfma_fast_shape(N, K)) {
    switch (tile) {
      case 16: return occupancy_fast_t<1>();
      case 32: return occupancy_fast_t<2>();
      case 64: return occupancy_fast_t<4>();
      default: return occupancy_fast_t<8>();
    }
  }
  const bool aligned = N % V == 0;
  switch (tile) {
    case 16: return occupancy_t<1, true>();
    case 32: return aligned ? occupancy_t<2, true>() : occupancy_t<2, false>();
    case 64: return aligned ? occupancy_t<4, true>() : occupancy_t<4, false>();
    default: return aligned ? occupancy_t<8, true>() : occupancy_t<8, false>();
  }
}

hipError_t launch_spmm_mfma(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                            const float* B, float* C, float* partial, int64_t M, int64_t N,
                            int64_t K, int64_t nnz, hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  const int tile = mfma_tile_for(N);
  const int V = tile >= 64 ? 4 : tile / 16;
  const bool al = (N % V == 0) && ptr_aligned16(B) && ptr_aligned16(C) &&
                  (partial == nullptr || ptr_aligned16(partial));
  // the fast kernel addresses the packed values (and their 64 spare floats) by 32-bit byte offsets
  if (al && mfma_fast_shape(N, K) && nnz + 64 < (int64_t(1) << 30)) {
    unsigned gx = (unsigned)((n_items + kWavesPerBlock - 1) / kWavesPerBlock);
    gx = (gx + kXcds - 1) / kXcds * kXcds;  // whole rounds over the XCDs
    const dim3 grid(gx, (unsigned)((N + tile - 1) / tile)), block(64 * kWavesPerBlock);
    const uint32_t k_last = (uint32_t)(K - 1);
#define SPMM_LAUNCH_FAST(TT, FF)                                                                \
  hipLaunchKernelGGL((k_spmm_mfma_fast<TT, FF>), grid, block, 0, s, f.brick_cols, f.brick_mask, \
                     f.brick_valptr, f.vals, items, n_items, B, C, partial, M, N, k_last)
    switch (tile) {
      case 16: SPMM_LAUNCH_FAST(1, false); break;
      case 32: SPMM_LAUNCH_FAST(2, false); break;
      case 64: SPMM_LAUNCH_FAST(4, false); break;
      default:   // whole 128-column tiles: the second vector of a B row at a constant offset
        if (N % 128 == 0) SPMM_LAUNCH_FAST(8, true); else SPMM_LAUNCH_FAST(8, false);
        break;
    }
#undef SPMM_LAUNCH_FAST
    return hipGetLastError();
  }
  switch (tile) {
    case 16: return launch_mfma_t<1, true>(f, items, n_items, B, C, partial, M, N, s);
    case 32: return al ? launch_mfma_t<2, true>(f, items, n_items, B, C, partial, M, N, s)
                       : launch_mfma_t<2, false>(f, items, n_items, B, C, partial, M, N, s);
    case 64: return al ? launch_mfma_t<4, true>(f, items, n_items, B, C, partial, M, N, s)
                       : launch_mfma_t<4, false>(f, items, n_items, B, C, partial, M, N, s);
    default: return al ? launch_mfma_t<8, true>(f, items, n_items, B, C, partial, M, N, s)
                       : launch_mfma_t<8, false>(f, items, n_items, B, C, partial, M, N, s);
  }
}

hipError_t launch_spmm_valu(const int32_t* rowptr, const int32_t* colind, const float* vals,
                            const uint32_t* panels, int64_t n_panels, const uint32_t* long_rows,
                            int64_t n_long_rows, const float* B, float* C, int64_t M, int64_t N,
                            hipStream_t s) {
  if (n_panels == 0 || N == 0) return hipSuccess;
  const bool a16 = ptr_aligned16(B) && ptr_aligned16(C);
  if (a16 && N % 4 == 0) {
    // lanes per row: the smallest power of two that covers N in vectors of four, at most 64
    int lpr = 4;
    while (lpr < 64 && 4 * lpr < N) lpr *= 2;
    const unsigned gy = (unsigned)((N + 4 * lpr - 1) / (4 * lpr));
    const int wpp = kPanel / (64 / lpr);
    const unsigned gx = (unsigned)((n_panels * wpp + kWavesPerBlock - 1) / kWavesPerBlock);
#define SPMM_LAUNCH_ROWS(L)                                                                     \
  do {                                                                                          \
    hipLaunchKernelGGL(k_spmm_valu_rows<L>, dim3(gx, gy), dim3(64 * kWavesPerBlock), 0, s,      \
                       rowptr, colind, vals, panels, n_panels, B, C, M, N);                     \
    if (n_long_rows > 0)                                                                        \
      hipLaunchKernelGGL(k_spmm_valu_long<L>, dim3((unsigned)n_long_rows, gy),                  \
                         dim3(64 * kLongWaves), 0, s, rowptr, colind, vals, long_rows,          \
                         panels, n_panels, B, C, N);                                            \
  } while (0)
    switch (lpr) {
      case 4: SPMM_LAUNCH_ROWS(4); break;
      case 8: SPMM_LAUNCH_ROWS(8); break;
      case 16: SPMM_LAUNCH_ROWS(16); break;
      case 32: SPMM_LAUNCH_ROWS(32); break;
      default: SPMM_LAUNCH_ROWS(64); break;
    }
#undef SPMM_LAUNCH_ROWS
    return hipGetLastError();
  }
  // any N, any alignment: one wavefront per row
  const unsigned gx = (unsigned)((n_panels * kPanel + kWavesPerBlock - 1) / kWavesPerBlock);
  const unsigned gy = (unsigned)((N + 63) / 64);
  hipLaunchKernelGGL((k_spmm_valu<1, true>), dim3(gx, gy), dim3(64 * kWavesPerBlock), 0, s, rowptr,
                     colind, vals, panels, n_panels, B, C, M, N);
  return hipGetLastError();
}

hipError_t launch_merge(const MergeItem* items, int64_t n_items, const float* partial, float* C,
                        int64_t M, int64_t N, hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  // rows * N is a multiple of 4 whenever N is, so whole vectors never straddle the end
  if (N % 4 == 0 && ptr_aligned16(partial) && ptr_aligned16(C))
    hipLaunchKernelGGL(k_merge<4>, dim3((unsigned)n_items), dim3(256), 0, s, items, partial, C, M, N);
  else
    hipLaunchKernelGGL(k_merge<1>, dim3((unsigned)n_items), dim3(256), 0, s, items, partial, C, M, N);
  return hipGetLastError();
}

}  // namespace spmm
