// Small helpers shared by the SpMM kernels (device code only).
#pragma once
#include "spmm_internal.h"

namespace spmm {

typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));

constexpr int kWavesPerBlock = 4;
constexpr int kXcds = 8;     // accelerator complex dies of an MI355X, each with its own L2

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

// Workgroups are handed to the 8 XCDs round-robin, and each XCD has its own L2.  This maps a
// workgroup to a "virtual" index such that each XCD works through a contiguous range of work
// items: neighbouring panels -- which share most of their B rows in banded matrices -- then
// meet in one L2 instead of every XCD fetching every B row.  gridDim.x is a multiple of 8.
__device__ inline uint32_t xcd_contiguous_block() {
  const uint32_t per_xcd = gridDim.x / kXcds;
  return (blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
}

inline bool ptr_aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace spmm
