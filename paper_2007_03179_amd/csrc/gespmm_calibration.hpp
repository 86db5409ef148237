// Measurement helpers of the library (not part of the method): a plain copy, the yardstick hardware
// traffic counters are scaled by, and plain gathers, the yardsticks for the inner loop of the SpMM kernels.
#pragma once

#include "gespmm_kernels.hpp"

namespace gespmm_detail {

// Plain 16-byte-per-lane copy of a known size: the yardstick that hardware traffic
// counters (FETCH_SIZE / WRITE_SIZE) are scaled by.
static __global__ void __launch_bounds__(kBlock) copy_f4(const float4* __restrict__ src, float4* __restrict__ dst, int64_t n4) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  for (; i + 3 * stride < n4; i += 4 * stride) {   // four independent 16-byte loads in flight per lane
    const float4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < n4; i += stride) dst[i] = src[i];
}

// Plain gather of 128-byte lines: 8 lanes read line idx[e] of the table (16 bytes each), eight
// gathers in flight per lane, indices read coalesced; every group of 8 lanes folds what it read
// into one float4 so that the loads stay live.  It does what the chunk kernel's inner loop does
// to memory and nothing else, so its rate is the ceiling for that loop on a table of that size.
static __global__ void __launch_bounds__(kBlock) gather_lines(const float4* __restrict__ table, const int32_t* __restrict__ idx,
                                                              int64_t n, float4* __restrict__ out) {
  const int g = threadIdx.x & 7;
  const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) >> 3;
  const int64_t groups = ((int64_t)gridDim.x * kBlock) >> 3;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int64_t e = group * 8; e < n; e += groups * 8) {
    int k[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) k[u] = idx[e + u < n ? e + u : n - 1];
    float4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = table[(int64_t)k[u] * 8 + g];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (e + u < n) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }   // padded gathers do not count
    }
  }
  out[(int64_t)blockIdx.x * kBlock + threadIdx.x] = acc;
}


// The same gather with its shape as parameters: LANES lanes read WORDS 4-byte words each of row idx[e]
// (rows are row_bytes apart; LANES * WORDS * 4 <= row_bytes), FLIGHT rows in flight per lane.
// POLICY: 0 = plain global loads; 1 = buffer loads that bypass the L1 (agent scope); 2 = non-temporal
// buffer loads.  The buffer forms address at most 4 GB.
typedef unsigned int gather_u4 __attribute__((ext_vector_type(4)));
typedef unsigned int gather_u2 __attribute__((ext_vector_type(2)));

template <int WORDS> struct GatherLoad;
template <> struct GatherLoad<4> {
  using T = gather_u4;
  template <int POLICY> __device__ static T load(const char* base, __amdgpu_buffer_rsrc_t r, uint64_t off) {
    if (POLICY == 0) return *reinterpret_cast<const gather_u4*>(base + off);
    return __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, POLICY == 1 ? 16 : 2);
  }
  __device__ static float sum(T v) { return __uint_as_float(v.x) + __uint_as_float(v.y) + __uint_as_float(v.z) + __uint_as_float(v.w); }
};
template <> struct GatherLoad<2> {
  using T = gather_u2;
  template <int POLICY> __device__ static T load(const char* base, __amdgpu_buffer_rsrc_t r, uint64_t off) {
    if (POLICY == 0) return *reinterpret_cast<const gather_u2*>(base + off);
    return __builtin_amdgcn_raw_buffer_load_b64(r, (int)off, 0, POLICY == 1 ? 16 : 2);
  }
  __device__ static float sum(T v) { return __uint_as_float(v.x) + __uint_as_float(v.y); }
};
template <> struct GatherLoad<1> {
  using T = unsigned;
  template <int POLICY> __device__ static T load(const char* base, __amdgpu_buffer_rsrc_t r, uint64_t off) {
    if (POLICY == 0) return *reinterpret_cast<const unsigned*>(base + off);
    return __builtin_amdgcn_raw_buffer_load_b32(r, (int)off, 0, POLICY == 1 ? 16 : 2);
  }
  __device__ static float sum(T v) { return __uint_as_float(v); }
};

template <int LANES, int WORDS, int FLIGHT, int POLICY>
__global__ void __launch_bounds__(kBlock) gather_rows(const char* __restrict__ table, uint32_t table_bytes, int row_bytes,
                                                      const int32_t* __restrict__ idx, int64_t n, float* __restrict__ out) {
  const int g = threadIdx.x % LANES;
  const int64_t group = ((int64_t)blockIdx.x * kBlock + threadIdx.x) / LANES;
  const int64_t groups = ((int64_t)gridDim.x * kBlock) / LANES;
  __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)table, 0, (int)table_bytes, 0x00020000);
  float acc = 0.f;
  for (int64_t e = group * FLIGHT; e < n; e += groups * FLIGHT) {
    int k[FLIGHT];
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) k[u] = idx[e + u < n ? e + u : n - 1];
    typename GatherLoad<WORDS>::T v[FLIGHT];
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u)
      v[u] = GatherLoad<WORDS>::template load<POLICY>(table, rsrc, (uint64_t)k[u] * row_bytes + g * (WORDS * 4));
#pragma unroll
    for (int u = 0; u < FLIGHT; ++u) acc += GatherLoad<WORDS>::sum(v[u]);
  }
  out[(int64_t)blockIdx.x * kBlock + threadIdx.x] = acc;
}

using GatherKernel = void (*)(const char*, uint32_t, int, const int32_t*, int64_t, float*);

template <int LANES, int WORDS, int POLICY>
GatherKernel pick_gather_flight(int flight) {
  switch (flight) {
    case 2: return gather_rows<LANES, WORDS, 2, POLICY>;
    case 4: return gather_rows<LANES, WORDS, 4, POLICY>;
    case 8: return gather_rows<LANES, WORDS, 8, POLICY>;
    case 16: return gather_rows<LANES, WORDS, 16, POLICY>;
    default: return nullptr;
  }
}

inline GatherKernel pick_gather(int lanes, int words, int flight, int policy) {
  if (policy != 0) {                               // the cache policies exist for the kernel's own shape only
    if (lanes != 8 || words != 4) return nullptr;
    return policy == 1 ? pick_gather_flight<8, 4, 1>(flight) : (policy == 2 ? pick_gather_flight<8, 4, 2>(flight) : nullptr);
  }
#define GESPMM_CASE(LL, WW) if (lanes == LL && words == WW) return pick_gather_flight<LL, WW, 0>(flight);
  GESPMM_CASE(8, 4) GESPMM_CASE(16, 2) GESPMM_CASE(32, 1) GESPMM_CASE(4, 4) GESPMM_CASE(2, 4) GESPMM_CASE(4, 2)
  GESPMM_CASE(8, 1) GESPMM_CASE(16, 4) GESPMM_CASE(32, 4) GESPMM_CASE(64, 4)
#undef GESPMM_CASE
  return nullptr;
}

}  // namespace gespmm_detail
