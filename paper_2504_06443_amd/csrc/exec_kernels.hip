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
// Loads are software-pipelined: while the MFMAs of brick b issue, the values
// and B rows of brick b+1 and the metadata of brick b+2 are in flight.
//
// Vector-ALU CSR kernel (the paper's "scalar core" path): one wavefront per
// row, one coalesced B-row load and one FMA per stored entry.  Used for panels
// whose brick density is in the Low class of Table 1, and for empty panels.
#include "spmm_internal.h"

namespace spmm {

namespace {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));

constexpr int kWavesPerBlock = 4;

template <int V> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<2> { typedef float2_t type; };
template <> struct Vec<4> { typedef float4_t type; };

template <int V>
__device__ inline void load_vec(const float* __restrict__ p, float (&out)[V]) {
  typedef typename Vec<V>::type vt;
  const vt v = *reinterpret_cast<const vt*>(p);
  if constexpr (V == 1) out[0] = v;
  else {
#pragma unroll
    for (int w = 0; w < V; ++w) out[w] = v[w];
  }
}

template <int V>
__device__ inline void store_vec(float* __restrict__ p, const float (&in)[V]) {
  typedef typename Vec<V>::type vt;
  vt v;
  if constexpr (V == 1) v = in[0];
  else {
#pragma unroll
    for (int w = 0; w < V; ++w) v[w] = in[w];
  }
  *reinterpret_cast<vt*>(p) = v;
}

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
  const int64_t item_id = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
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
    struct Meta { uint64_t mask; uint32_t off; uint32_t col; };
    struct Stage { uint64_t mask; float a_raw; float bv[T]; };
    auto load_meta = [&](uint32_t b) {
      return Meta{f.brick_mask[b], f.brick_valptr[b], f.brick_cols[(int64_t)b * kBrickK + kq]};
    };
    // Issue the loads of one brick.  The value index is the number of pattern
    // bits below this lane's bit; lanes whose bit is clear read a neighbouring
    // value (vals has one pad element) that compute() discards.
    auto issue = [&](const Meta& m, Stage& st) {
      st.mask = m.mask;
      st.a_raw = f.vals[(int64_t)m.off + __popcll(m.mask & below)];
      load_b<T, ALIGNED>(B + (int64_t)(m.col == kPadCol ? 0u : m.col) * N, N, ncol0, st.bv);
    };
    auto compute = [&](const Stage& st) {
      const float a = ((st.mask >> bit) & 1ull) ? st.a_raw : 0.f;
#pragma unroll
      for (int u = 0; u < T; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, st.bv[u], acc[u], 0, 0, 0);
    };
    // While brick b computes, the loads of brick b+1 and the metadata of brick
    // b+2 are in flight (indices clamped to the last brick: harmless re-reads).
    // The prologue values pass through empty asm statements so that they are
    // not plain loads: otherwise the compiler merges each prologue load with its
    // in-loop twin into one load at the top of the loop, which undoes the
    // prefetch distance.
    Stage cur;
    issue(load_meta(b_begin), cur);
    asm volatile("" : "+v"(cur.a_raw));
    Meta m1 = load_meta(min(b_begin + 1, last));
    asm volatile("" : "+v"(m1.col));
    m1.off = __builtin_amdgcn_readfirstlane(m1.off);
    m1.mask = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(m1.mask >> 32)) << 32) |
              (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)m1.mask);
    for (uint32_t b = b_begin; b < b_end; ++b) {
      const Meta m2 = load_meta(min(b + 2, last));
      Stage nxt;
      issue(m1, nxt);
      compute(cur);
      cur = nxt;
      m1 = m2;
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

// ------------------------------------------------------------------ merge (a8)
// Sum the partial 16 x N tiles of a split panel in part order and store to C.
__global__ __launch_bounds__(256) void k_merge(const MergeItem* __restrict__ items,
                                               const float* __restrict__ partial,
                                               float* __restrict__ C, int64_t M, int64_t N) {
  const MergeItem it = items[blockIdx.x];
  const int64_t row0 = (int64_t)it.panel * kPanel;
  const int64_t rows = min<int64_t>(kPanel, M - row0);
  const int64_t tile = (int64_t)kPanel * N;
  for (int64_t x = threadIdx.x; x < rows * N; x += blockDim.x) {
    float s = 0.f;
    for (uint32_t q = 0; q < it.nparts; ++q) s += partial[((int64_t)it.slot_begin + q) * tile + x];
    C[row0 * N + x] = s;
  }
}

template <int T, bool ALIGNED>
hipError_t launch_mfma_t(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                         const float* B, float* C, float* partial, int64_t M, int64_t N,
                         hipStream_t s) {
  const unsigned gx = (unsigned)((n_items + kWavesPerBlock - 1) / kWavesPerBlock);
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

bool ptr_aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace

int mfma_tile_for(int64_t N) { return N <= 16 ? 16 : (N <= 32 ? 32 : (N <= 64 ? 64 : 128)); }

int mfma_resident_waves_per_cu(int n_tile, bool aligned) {
  switch (n_tile) {
    case 16: return occupancy_t<1, true>();
    case 32: return aligned ? occupancy_t<2, true>() : occupancy_t<2, false>();
    case 64: return aligned ? occupancy_t<4, true>() : occupancy_t<4, false>();
    default: return aligned ? occupancy_t<8, true>() : occupancy_t<8, false>();
  }
}

hipError_t launch_spmm_mfma(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                            const float* B, float* C, float* partial, int64_t M, int64_t N,
                            hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  const int tile = mfma_tile_for(N);
  const int V = tile >= 64 ? 4 : tile / 16;
  const bool al = (N % V == 0) && ptr_aligned16(B) && ptr_aligned16(C) &&
                  (partial == nullptr || ptr_aligned16(partial));
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
                            const uint32_t* panels, int64_t n_panels, const float* B, float* C,
                            int64_t M, int64_t N, hipStream_t s) {
  if (n_panels == 0 || N == 0) return hipSuccess;
  const bool a16 = ptr_aligned16(B) && ptr_aligned16(C);
  const unsigned gx = (unsigned)((n_panels * kPanel + kWavesPerBlock - 1) / kWavesPerBlock);
  auto go = [&](auto kernel, int V) {
    const unsigned gy = (unsigned)((N + 64 * V - 1) / (64 * V));
    hipLaunchKernelGGL(kernel, dim3(gx, gy), dim3(64 * kWavesPerBlock), 0, s, rowptr, colind, vals,
                       panels, n_panels, B, C, M, N);
    return hipGetLastError();
  };
  if (a16 && N % 4 == 0 && N > 128) return go(k_spmm_valu<4, true>, 4);
  if (a16 && N % 2 == 0 && N > 64) return go(k_spmm_valu<2, true>, 2);
  return go(k_spmm_valu<1, true>, 1);
}

hipError_t launch_merge(const MergeItem* items, int64_t n_items, const float* partial, float* C,
                        int64_t M, int64_t N, hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  hipLaunchKernelGGL(k_merge, dim3((unsigned)n_items), dim3(256), 0, s, items, partial, C, M, N);
  return hipGetLastError();
}

}  // namespace spmm
