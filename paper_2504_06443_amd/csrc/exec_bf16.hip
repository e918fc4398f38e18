// Reduced-input-precision variant of the MFMA brick kernel: split-bf16 products on
// v_mfma_f32_16x16x32_bf16 (one instruction covers EIGHT bricks of a panel).
//
// The paper feeds its tensor cores FP32 inputs rounded to TF32 (10-bit mantissa) and
// accumulates in FP32 (Section 2, "Background"); the eightfold tensor-core advantage that
// rounding buys on its A100 is what makes Medium-synergy matrices profitable there
// (Section 1).  gfx950 has no TF32 matrix instruction and its FP32 MFMA is no faster than the
// vector ALUs, so the counterpart here keeps far more mantissa than TF32 instead: every FP32
// input x is written as a sum of NP bf16 numbers (x = x1 + x2 (+ x3), each the bf16 rounding
// of what the earlier ones left), and a product a.b is assembled from the leading partial
// products on the bf16 matrix cores, accumulated in FP32:
//   NP = 2:  a1 b1 + a1 b2 + a2 b1                  (3 MFMAs; drops three terms of at most
//                                                    2^-16 |a b| each: bf16 has 8 significant bits)
//   NP = 3:  + a1 b3 + a2 b2 + a3 b1               (6 MFMAs; drops terms of at most 2^-24 |a b|)
// Eight bricks (32 columns of the compacted panel) form one K = 32 step.
//
// Operand layout of v_mfma_f32_16x16x32_bf16 (wave64): lane l holds row/column l % 16 and the
// eight k-values of group g = l / 16; A and B pair up element e of group g with element e of
// group g, so the k-numbering inside is free.  Here group g stands for bricks 2g and 2g+1 of
// the step, element e = 4 h + c for column c of brick 2g + h.
//   A: the bricks are decoded as in the FP32 kernel (prefix count of the pattern with v_mbcnt,
//      one value gather per brick, lane i acting for pattern bit i), split into bf16 planes and
//      zero-filled into LDS in the paper's row-major element order; lane (r, g) then reads
//      row r of its two bricks back as two 8-byte loads per plane, which is exactly the
//      operand register layout.
//   B: lane (j, g) loads T consecutive floats of each of its eight B rows (the rows named by
//      the eight brick columns of group g), splits them in registers and packs pairs of rows
//      into the operand.  Element u of every row feeds MFMA u, so the accumulators hold T
//      consecutive columns per lane as in the FP32 kernel and the epilogue is the same.
// The vector ALU does the splitting (6 instructions per pair of B elements and plane beyond
// the first); together with the path of the B rows through the vector-memory pipe (2 KB per
// brick at N = 128 against 64 bytes per clock and CU) that, not the matrix core, bounds this
// kernel: the MFMAs disappear behind the other work.
#include "exec_common.h"

namespace spmm {

namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef uint32_t uint4_t __attribute__((ext_vector_type(4)));
typedef uint32_t uint2_t __attribute__((ext_vector_type(2)));

constexpr int kStepBricks = 8;   // bricks per K = 32 step

// two floats -> one register of two bf16 (round to nearest even), first in the low half
__device__ inline uint32_t pack_bf16(float lo, float hi) {
  const float2_t f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}
__device__ inline float bf16_lo_as_float(uint32_t p) { return __builtin_bit_cast(float, p << 16); }
__device__ inline float bf16_hi_as_float(uint32_t p) {
  return __builtin_bit_cast(float, p & 0xFFFF0000u);
}

// x0, x1 -> NP registers of packed bf16 pairs: plane p holds (bf16 of the p-th residual of x0,
// of x1).  Each residual is exact in FP32 (it has fewer significant bits than x).
template <int NP>
__device__ inline void split_pair(float x0, float x1, uint32_t (&planes)[NP]) {
#pragma unroll
  for (int p = 0; p < NP; ++p) {
    planes[p] = pack_bf16(x0, x1);
    if (p + 1 < NP) {
      x0 -= bf16_lo_as_float(planes[p]);
      x1 -= bf16_hi_as_float(planes[p]);
    }
  }
}

template <int T, int NP>
__global__ __launch_bounds__(64 * kWavesPerBlock) __attribute__((amdgpu_waves_per_eu(2))) void k_spmm_bf16(
    const uint32_t* __restrict__ brick_cols, const uint64_t* __restrict__ brick_mask,
    const uint32_t* __restrict__ brick_valptr, const float* __restrict__ vals,
    const WorkItem* __restrict__ items, int64_t n_items, const float* __restrict__ B,
    float* __restrict__ C, float* __restrict__ partial, int64_t M, int64_t N, uint32_t k_last,
    uint32_t /* reserved */) {
  constexpr int V = T < 4 ? T : 4;
  constexpr int NV = T / V;
  constexpr int SB = kStepBricks;
  // zero-filled bricks of one step, one bf16 plane after the other: [plane][brick][row][col]
  __shared__ __attribute__((aligned(16))) unsigned short lds_a[kWavesPerBlock][NP][SB * 64];

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const uint32_t vblock = xcd_contiguous_block();
  const int64_t item_id = (int64_t)vblock * kWavesPerBlock + wave;
  if (item_id >= n_items) return;  // whole wavefront leaves together
  const WorkItem it = items[item_id];
  const uint32_t panel = __builtin_amdgcn_readfirstlane(it.panel);
  const uint32_t b_begin = __builtin_amdgcn_readfirstlane(it.brick_begin);
  const uint32_t b_end = __builtin_amdgcn_readfirstlane(it.brick_end);
  const uint32_t slot = __builtin_amdgcn_readfirstlane(it.slot);

  const int j = lane & 15;   // MFMA row (A) / column (B, D)
  const int g = lane >> 4;   // k-group: bricks 2g, 2g+1 of a step
  const int64_t ncol0 = (int64_t)blockIdx.y * (16 * T) + V * j;
  const uint32_t row_bytes = (uint32_t)N * 4u;
  uint32_t lane_off[NV];   // byte offset of this lane's vectors inside a B row (clamped past N)
#pragma unroll
  for (int q = 0; q < NV; ++q)
    lane_off[q] = (uint32_t)min<int64_t>(ncol0 + q * 16 * V, N - V) * 4u;

  float4_t acc[T];
#pragma unroll
  for (int u = 0; u < T; ++u) acc[u] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (b_begin < b_end) {
    const uint32_t nbricks = b_end - b_begin;
    const uint32_t nsteps = (nbricks + SB - 1) / SB;
    const char* Bbytes = reinterpret_cast<const char*>(B);
    unsigned short* my_lds = &lds_a[wave][0][0];

    struct Meta { uint64_t mask[SB]; uint32_t off[SB]; };   // wave-uniform: scalar registers
    // Patterns and value offsets of the step's bricks.  Bricks past the item's end belong to
    // the next panel (or to the arrays' padding): their pattern is forced to zero, which makes
    // their A operand zero.
    auto load_meta = [&](uint32_t step) {
      const uint32_t base = b_begin + step * SB;
      const uint64_t* __restrict__ mp = brick_mask + base;
      const uint32_t* __restrict__ op = brick_valptr + base;
      Meta m;
#pragma unroll
      for (int i = 0; i < SB; ++i) { m.mask[i] = mp[i]; m.off[i] = op[i]; }   // wide scalar loads
      const uint32_t first = step * SB;
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        const bool live = first + (uint32_t)i < nbricks;   // uniform: scalar selects
        m.mask[i] = live ? m.mask[i] : 0ull;
      }
      return m;
    };
    // The eight brick columns of this lane's k-group (two adjacent bricks = 32 contiguous
    // bytes); bricks past the item's end are replaced by its last brick (valid rows, A is 0).
    auto load_cols = [&](uint32_t step, uint32_t (&cols)[8]) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint32_t b = min(b_begin + step * SB + 2 * g + h, b_end - 1);
        const uint4_t c = *reinterpret_cast<const uint4_t*>(brick_cols + (size_t)b * kBrickK);
#pragma unroll
        for (int x = 0; x < 4; ++x) cols[4 * h + x] = c[x];
      }
    };
    // B rows and brick values of one step into a register stage.  Lane i acts for pattern bit
    // i of every brick: its value index is the prefix count of the pattern (Algorithm 1's
    // decode), so the gather addresses never decrease from lane to lane, which the
    // vector-memory pipe serves as cheaply as a contiguous load; lanes whose bit is clear
    // fetch a neighbour's value and are zeroed when the brick is staged.
    auto issue = [&](const Meta& m, const uint32_t (&cols)[8], float (&raw)[8][T], float (&val)[SB]) {
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        const uint32_t cnt = __builtin_amdgcn_mbcnt_hi(
            (uint32_t)(m.mask[i] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m.mask[i], 0u));
        val[i] = (vals + m.off[i])[cnt];
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        // pad columns (0xFFFFFFFF) clamp to the last row of B; their A elements are zero
        const uint32_t ro = __umul24(min(cols[e], k_last), row_bytes);
#pragma unroll
        for (int q = 0; q < NV; ++q) {
          float tmp[V];
          load_vec<V>(reinterpret_cast<const float*>(Bbytes + (ro + lane_off[q])), tmp);
#pragma unroll
          for (int w = 0; w < V; ++w) raw[e][q * V + w] = tmp[w];
        }
      }
    };
    struct AOp { bf16x8_t p[NP]; };
    // A: split the zero-filled elements (lane i = element i of the brick), put them to LDS in
    // the paper's row-major order and read this lane's operand back
    auto stage_a = [&](const float (&val)[SB], const uint64_t (&mask)[SB]) {
#pragma unroll
      for (int i = 0; i < SB; ++i) {
        float a;   // zero fill: the pattern itself is the select mask (lane i <-> bit i)
        asm("v_cndmask_b32_e64 %0, 0, %1, %2" : "=v"(a) : "v"(val[i]), "s"(mask[i]));
        uint32_t pl[NP];
        split_pair<NP>(a, 0.f, pl);
#pragma unroll
        for (int p = 0; p < NP; ++p) my_lds[p * (SB * 64) + i * 64 + lane] = (unsigned short)pl[p];
      }
      __builtin_amdgcn_wave_barrier();
      AOp a;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const unsigned short* base = my_lds + p * (SB * 64) + (2 * g) * 64 + j * 4;
        const uint2_t lo = *reinterpret_cast<const uint2_t*>(base);
        const uint2_t hi = *reinterpret_cast<const uint2_t*>(base + 64);
        const uint4_t r = {lo[0], lo[1], hi[0], hi[1]};
        a.p[p] = __builtin_bit_cast(bf16x8_t, r);
      }
      __builtin_amdgcn_wave_barrier();
      return a;
    };
    // B: split element u of the eight rows into operand planes
    struct BOp { bf16x8_t p[NP]; };
    auto split_b = [&](const float (&raw)[8][T], int u) {
      uint32_t bp[4][NP];   // [pair of rows][plane]
#pragma unroll
      for (int x = 0; x < 4; ++x) split_pair<NP>(raw[2 * x][u], raw[2 * x + 1][u], bp[x]);
      BOp b;
#pragma unroll
      for (int p = 0; p < NP; ++p) {
        const uint4_t r = {bp[0][p], bp[1][p], bp[2][p], bp[3][p]};
        b.p[p] = __builtin_bit_cast(bf16x8_t, r);
      }
      return b;
    };
    // Partial products in order of increasing magnitude: planes (pa, pb) with pa + pb < NP.
    // The operand of column u+1 is split between the MFMAs of column u, which all add to one
    // accumulator and would otherwise wait for each other.
    auto multiply = [&](const AOp& a, const float (&raw)[8][T]) {
      BOp cur = split_b(raw, 0);
#pragma unroll
      for (int u = 0; u < T; ++u) {
        BOp nxt = cur;
        bool first = true;
#pragma unroll
        for (int s = NP - 1; s >= 0; --s)
#pragma unroll
          for (int pa = 0; pa <= s; ++pa) {
            acc[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.p[pa], cur.p[s - pa], acc[u], 0, 0, 0);
            if (first && u + 1 < T) nxt = split_b(raw, u + 1);
            first = false;
          }
        cur = nxt;
      }
    };

    // Two register stages: while step s is split and multiplied, the loads of step s+1 are in
    // flight.  The scalar loads of
    // the metadata of step s+2 are issued after the LDS round trip of step s (both count in
    // the same hardware counter, so a wait for the LDS would otherwise wait for the scalar
    // cache as well) and have the whole multiply phase to land.
    float raw0[8][T], raw1[8][T], val0[SB], val1[SB];
    uint64_t mk0[SB], mk1[SB];
    uint32_t cn[8];
    {
      const Meta m = load_meta(0);
      load_cols(0, cn);
      issue(m, cn, raw0, val0);
#pragma unroll
      for (int i = 0; i < SB; ++i) mk0[i] = m.mask[i];
    }
    Meta mn = load_meta(1);
    load_cols(1, cn);
    for (uint32_t s = 0; s < nsteps; s += 2) {
      // stage 1 <- step s+1 (harmless re-read of the last brick's rows when past the end)
      issue(mn, cn, raw1, val1);
#pragma unroll
      for (int i = 0; i < SB; ++i) mk1[i] = mn.mask[i];
      {
        const AOp a = stage_a(val0, mk0);
        __builtin_amdgcn_sched_barrier(0);
        mn = load_meta(s + 2);
        load_cols(s + 2, cn);
        multiply(a, raw0);
      }
      if (s + 1 >= nsteps) break;
      issue(mn, cn, raw0, val0);
#pragma unroll
      for (int i = 0; i < SB; ++i) mk0[i] = mn.mask[i];
      {
        const AOp a = stage_a(val1, mk1);
        __builtin_amdgcn_sched_barrier(0);
        mn = load_meta(s + 3);
        load_cols(s + 3, cn);
        multiply(a, raw1);
      }
    }
  }

  // acc[q*V + w][v] = C[row 4*g + v][ncol0 + q*16*V + w]
  float* out;
  int64_t rows_left;
  if (slot == kNoSlot) {
    const int64_t row0 = (int64_t)panel * kPanel + 4 * g;
    out = C + row0 * N;
    rows_left = M - row0;
  } else {
    out = partial + ((int64_t)slot * kPanel + 4 * g) * N;
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
          __builtin_nontemporal_store(t, reinterpret_cast<vt*>(out + v * N + ncol));
        }
      }
    }
  }
}

template <int T, int NP>
int occupancy_bf16_t() {
  int nb = 0;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, k_spmm_bf16<T, NP>, 64 * kWavesPerBlock,
                                                   0) != hipSuccess || nb < 1)
    nb = 1;
  return nb * kWavesPerBlock;
}

}  // namespace

// The split-bf16 kernel serves what the fast FP32 kernel serves (N a multiple of the vector
// width, 16-byte aligned operands, B below 4 GiB) with K below 2^24 (24-bit multiply for the
// row offsets).  Other shapes run the FP32 kernels, which are at least as accurate.
bool bf16_path_shape(int64_t N, int64_t K) {
  const int tile = mfma_tile_for(N);
  const int V = tile >= 64 ? 4 : tile / 16;
  return N % V == 0 && K > 0 && K <= (int64_t(1) << 24) && N < (int64_t(1) << 22) &&
         (double)K * (double)N * 4.0 < 4294967296.0;
}

int bf16_resident_waves_per_cu(int64_t N, int planes) {
  switch (mfma_tile_for(N)) {
    case 16: return planes == 2 ? occupancy_bf16_t<1, 2>() : occupancy_bf16_t<1, 3>();
    case 32: return planes == 2 ? occupancy_bf16_t<2, 2>() : occupancy_bf16_t<2, 3>();
    case 64: return planes == 2 ? occupancy_bf16_t<4, 2>() : occupancy_bf16_t<4, 3>();
    default: return planes == 2 ? occupancy_bf16_t<8, 2>() : occupancy_bf16_t<8, 3>();
  }
}

hipError_t launch_spmm_bf16(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                            const float* B, float* C, float* partial, int64_t M, int64_t N,
                            int64_t K, int planes, int64_t nnz, hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  const uint32_t zero_idx = (uint32_t)nnz;   // vals[nnz .. nnz+63] are zeros
  const int tile = mfma_tile_for(N);
  unsigned gx = (unsigned)((n_items + kWavesPerBlock - 1) / kWavesPerBlock);
  gx = (gx + kXcds - 1) / kXcds * kXcds;  // whole rounds over the XCDs
  const dim3 grid(gx, (unsigned)((N + tile - 1) / tile)), block(64 * kWavesPerBlock);
  const uint32_t k_last = (uint32_t)(K - 1);
#define SPMM_LAUNCH_BF16(TT, PP)                                                            \
  hipLaunchKernelGGL((k_spmm_bf16<TT, PP>), grid, block, 0, s, f.brick_cols, f.brick_mask,  \
                     f.brick_valptr, f.vals, items, n_items, B, C, partial, M, N, k_last, zero_idx)
  if (planes == 2) {
    switch (tile) {
      case 16: SPMM_LAUNCH_BF16(1, 2); break;
      case 32: SPMM_LAUNCH_BF16(2, 2); break;
      case 64: SPMM_LAUNCH_BF16(4, 2); break;
      default: SPMM_LAUNCH_BF16(8, 2); break;
    }
  } else {
    switch (tile) {
      case 16: SPMM_LAUNCH_BF16(1, 3); break;
      case 32: SPMM_LAUNCH_BF16(2, 3); break;
      case 64: SPMM_LAUNCH_BF16(4, 3); break;
      default: SPMM_LAUNCH_BF16(8, 3); break;
    }
  }
#undef SPMM_LAUNCH_BF16
  return hipGetLastError();
}

}  // namespace spmm
