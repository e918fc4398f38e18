// Wide-N variant of the FP32 MFMA brick kernel (Section 3.3: for large N several thread
// blocks work on one row panel and the decoded A bricks are shared among them).
//
// One workgroup of W wavefronts takes one work item; wavefront w multiplies the item's
// bricks with the w-th 128-column tile of B, so a workgroup covers 128*W columns.  In the
// one-wavefront-per-tile kernel every tile fetches the patterns and values of the same bricks
// and decodes them again.  Here each brick is decoded once per workgroup: for every chunk of
// 8 bricks, wavefront w decodes bricks 8/W*w .. 8/W*(w+1)-1 (prefix count, value gather, zero
// fill) and writes the 64 elements of each in MFMA lane order into LDS; after a barrier all W
// wavefronts read their A operands from there with one ds_read per brick.  Two LDS buffers
// alternate, so the decode of chunk c+1 overlaps the multiplication of chunk c and there is
// one barrier per 8 bricks.  B rows, the ring of register stages and the stores are those of
// the one-wavefront kernel.
#include "exec_common.h"

namespace spmm {
namespace {

constexpr int kStages = 4;   // register stages of the B-row ring
constexpr int kChunk = 8;    // bricks per decode chunk

template <int W>
__global__ __launch_bounds__(64 * W) void k_spmm_mfma_wide(
    const uint32_t* __restrict__ brick_cols, const uint64_t* __restrict__ brick_mask,
    const uint32_t* __restrict__ brick_valptr, const float* __restrict__ vals,
    const WorkItem* __restrict__ items, int64_t n_items, const float* __restrict__ B,
    float* __restrict__ C, float* __restrict__ partial, int64_t M, int64_t N, uint32_t k_last) {
  constexpr int T = 8, V = 4, NV = 2;
  constexpr int R = kStages;
  constexpr int CH = kChunk;
  constexpr int PER = CH / W;          // bricks each wavefront decodes per chunk
  static_assert(CH % R == 0 && CH % W == 0 && CH * kBrickK <= 64, "stage and lane mapping");

  __shared__ float lds_a[2][CH][64];   // decoded bricks in MFMA lane order

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t item_id = xcd_contiguous_block();   // one work item per workgroup
  if (item_id >= n_items) return;                   // the whole workgroup leaves together
  const WorkItem it = items[item_id];   // uniform index: through the scalar cache
  const uint32_t panel = it.panel;
  const uint32_t b_begin = it.brick_begin;
  const uint32_t b_end = it.brick_end;
  const uint32_t slot = it.slot;

  const int j = lane & 15;
  const int kq = lane >> 4;
  const int64_t ncol0 = ((int64_t)blockIdx.y * W + wave) * (16 * T) + V * j;
  const uint32_t row_bytes = (uint32_t)N * 4u;
  uint32_t lane_off[NV];
#pragma unroll
  for (int q = 0; q < NV; ++q)
    lane_off[q] = (uint32_t)min<int64_t>(ncol0 + q * 16 * V, N - V) * 4u;
  const uint32_t perm_base = 4u * (uint32_t)kq;   // ds_bpermute byte address of lane kq
  // lane l = 4r + c decodes element (row r, column c); the MFMA wants it in lane 16c + r
  const int lds_slot = 16 * (lane & 3) + (lane >> 2);

  float4_t acc[T];
#pragma unroll
  for (int u = 0; u < T; ++u) acc[u] = float4_t{0.f, 0.f, 0.f, 0.f};

  if (b_begin < b_end) {
    const uint32_t nbricks = b_end - b_begin;
    const char* Bbytes = reinterpret_cast<const char*>(B);
    const uint32_t off_last = brick_valptr[b_end - 1];

    // this wavefront's share of a chunk's decode: gather (needs the patterns and offsets),
    // then, later, zero fill and the write to LDS
    struct Mine { uint64_t mask[PER]; float v[PER]; };
    auto gather_mine = [&](uint32_t rel) {   // rel: chunk start relative to b_begin
      Mine m;
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const uint32_t g = rel + (uint32_t)(wave * PER + e);
        const bool live = g < nbricks;       // uniform
        const uint32_t b = b_begin + g;      // the arrays carry spare bricks past the end
        const uint64_t mask = live ? brick_mask[b] : 0ull;
        const uint32_t off = live ? brick_valptr[b] : off_last;
        m.mask[e] = mask;
        const uint32_t cnt = __builtin_amdgcn_mbcnt_hi(
            (uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
        m.v[e] = vals[(int64_t)off + cnt];
      }
      return m;
    };
    auto write_mine = [&](const Mine& m, int buf) {
#pragma unroll
      for (int e = 0; e < PER; ++e) {
        const float a = ((m.mask[e] >> lane) & 1ull) ? m.v[e] : 0.f;
        lds_a[buf][wave * PER + e][lds_slot] = a;
      }
    };
    // lane 4*i + c: byte offset of B row brick_cols[4*(base+i) + c]; pad columns clamp to the
    // last row (A is 0 there); steps past the item's last brick repeat that brick's rows
    auto load_rowoff = [&](uint32_t base) {
      const uint32_t sl = (uint32_t)lane & (CH * kBrickK - 1);
      const uint32_t idx = min(base * kBrickK + sl, (b_end - 1) * kBrickK + (sl & (kBrickK - 1)));
      const uint32_t c = brick_cols[idx];
      return min(c, k_last) * row_bytes;
    };

    float st_a[R];
    float st_b[R][T];
    auto issue = [&](int buf, int i, uint32_t ro, int s) {
      st_a[s] = lds_a[buf][i][lane];
#pragma unroll
      for (int q = 0; q < NV; ++q) {
        float tmp[V];
        load_vec<V>(reinterpret_cast<const float*>(Bbytes + (ro + lane_off[q])), tmp);
#pragma unroll
        for (int w = 0; w < V; ++w) st_b[s][q * V + w] = tmp[w];
      }
    };
    auto compute = [&](int s) {
#pragma unroll
      for (int u = 0; u < T; ++u)
        acc[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(st_a[s], st_b[s][u], acc[u], 0, 0, 0);
    };

    // chunk 0 decoded up front
    {
      const Mine m0 = gather_mine(0);
      write_mine(m0, 0);
    }
    uint32_t ro_cur = load_rowoff(b_begin);
    asm volatile("" : "+v"(ro_cur));
    __syncthreads();

    // Step g computes brick g-R from stage g%R and refills that stage with brick g.  Every
    // wavefront of the workgroup runs the same number of chunks (they share the item), so
    // the barriers match.
    const uint32_t total = nbricks + R;
    uint32_t ro_next = __builtin_amdgcn_ds_bpermute(perm_base, ro_cur);
    int buf = 0;
    for (uint32_t c = 0; c < total; c += CH) {
      const Mine mine = gather_mine(c + CH);
      const uint32_t ro_nxt = load_rowoff(b_begin + c + CH);
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        const uint32_t g = c + i;
        if (g >= (uint32_t)R && g - R < nbricks) compute(i % R);
        const uint32_t ro = ro_next;
        ro_next = (i + 1 < CH) ? __builtin_amdgcn_ds_bpermute(perm_base + 16u * (i + 1), ro_cur)
                               : __builtin_amdgcn_ds_bpermute(perm_base, ro_nxt);
        issue(buf, i, ro, i % R);
      }
      write_mine(mine, buf ^ 1);
      ro_cur = ro_nxt;
      buf ^= 1;
      __syncthreads();   // next chunk's operands written; this chunk's all read
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
          float4_t t;
#pragma unroll
          for (int w = 0; w < V; ++w) t[w] = acc[q * V + w][v];
          __builtin_nontemporal_store(t, reinterpret_cast<float4_t*>(out + v * N + ncol));
        }
      }
    }
  }
}

}  // namespace

// N a multiple of 4 with at least two 128-column tiles, whose number is a multiple of the
// workgroup's wavefront count (so no wavefront of a workgroup is without a tile), B < 4 GiB
int mfma_wide_waves(int64_t N, int64_t K) {
  if (N < 256 || N % 4 != 0 || K <= 0 || (double)K * (double)N * 4.0 >= 4294967296.0) return 0;
  const int64_t tiles = (N + 127) / 128;
  if (tiles % 4 == 0) return 4;
  if (tiles % 2 == 0) return 2;
  return 0;
}

hipError_t launch_spmm_mfma_wide(const BrickFormat& f, const WorkItem* items, int64_t n_items,
                                 const float* B, float* C, float* partial, int64_t M, int64_t N,
                                 int64_t K, hipStream_t s) {
  if (n_items == 0 || N == 0) return hipSuccess;
  const int W = mfma_wide_waves(N, K);
  if (W == 0 || !ptr_aligned16(B) || !ptr_aligned16(C) ||
      (partial != nullptr && !ptr_aligned16(partial)))
    return hipErrorInvalidValue;
  const int64_t tiles = (N + 127) / 128;
  const unsigned gx = (unsigned)((n_items + kXcds - 1) / kXcds * kXcds);
  const dim3 grid(gx, (unsigned)(tiles / W));
  const uint32_t k_last = (uint32_t)(K - 1);
  if (W == 4)
    hipLaunchKernelGGL(k_spmm_mfma_wide<4>, grid, dim3(256), 0, s, f.brick_cols, f.brick_mask,
                       f.brick_valptr, f.vals, items, n_items, B, C, partial, M, N, k_last);
  else
    hipLaunchKernelGGL(k_spmm_mfma_wide<2>, grid, dim3(128), 0, s, f.brick_cols, f.brick_mask,
                       f.brick_valptr, f.vals, items, n_items, B, C, partial, M, N, k_last);
  return hipGetLastError();
}

}  // namespace spmm
