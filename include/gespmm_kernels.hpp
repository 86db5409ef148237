// Launch helpers over the kernels of gespmm_device.hpp: the small helper kernels, the kernel tables, the
// launch-shape choice (make_plan) and the launch sequences.  The C ABI over them is in
// paper_2007_03179_amd/csrc/gespmm.hip; gespmm_custom.hpp includes this file for user-defined
// reduce operations, which is why it lives beside the public headers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <vector>

#include "gespmm.h"
#include "gespmm_device.hpp"

namespace gespmm_detail {

// -------------------------------------------------- small helper kernels -----
// dst[0..n) = value (a row-major matrix seen as a flat array)
static __global__ void __launch_bounds__(kBlock) fill_f32(float* __restrict__ dst, int64_t n, float value) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) dst[i] = value;
}

// Gradient of max / min w.r.t. B: element (i, j) adds val[p] * dC[i, j] into dB[colind[p], j]
// for p = arg[i, j] >= 0.  One lane per element, reads coalesced, atomics scattered.
static __global__ void __launch_bounds__(kBlock) pool_backward_scatter(int64_t total, int32_t N, const int32_t* __restrict__ colind,
                                                               const float* __restrict__ vals,
                                                               const int32_t* __restrict__ arg,
                                                               const float* __restrict__ dC, float* __restrict__ dB) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t e = (int64_t)blockIdx.x * kBlock + threadIdx.x; e < total; e += stride) {
    const int p = arg[e];
    if (p >= 0) {
      const float w = vals ? vals[p] : 1.0f;
      __hip_atomic_fetch_add(dB + (int64_t)colind[p] * N + (e % N), w * dC[e], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// ------------------------------------------- column counts and their scan ----
constexpr int kScanTile = 4 * kBlock;             // elements one workgroup scans

static __global__ void __launch_bounds__(kBlock) count_columns(int64_t nnz, const int32_t* __restrict__ colind, int32_t* __restrict__ counts) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t p = (int64_t)blockIdx.x * kBlock + threadIdx.x; p < nnz; p += stride)
    __hip_atomic_fetch_add(counts + colind[p], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Exclusive scan of one tile held as 4 values per thread; returns this thread's prefix and
// leaves the tile total in *total (same for all threads).
__device__ __forceinline__ int tile_exclusive_scan(const int (&v)[4], int* total) {
  __shared__ int wave_sums[kWavesPerBlock];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int mine = v[0] + v[1] + v[2] + v[3];
  int incl = mine;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int up = __shfl_up(incl, off, kWave);
    if (lane >= off) incl += up;
  }
  __syncthreads();                                 // previous use of wave_sums is over
  if (lane == kWave - 1) wave_sums[wave] = incl;
  __syncthreads();
  int before = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kWavesPerBlock; ++w) {
    if (w < wave) before += wave_sums[w];
    all += wave_sums[w];
  }
  *total = all;
  return before + incl - mine;
}

// In-place exclusive scan inside every tile of kScanTile elements; tile totals to sums[].
static __global__ void __launch_bounds__(kBlock) scan_tiles(int32_t* __restrict__ data, int64_t n, int32_t* __restrict__ sums) {
  const int64_t base = (int64_t)blockIdx.x * kScanTile + threadIdx.x * 4;
  int v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = base + j < n ? data[base + j] : 0;
  int total;
  int prefix = tile_exclusive_scan(v, &total);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (base + j < n) data[base + j] = prefix;
    prefix += v[j];
  }
  if (threadIdx.x == 0) sums[blockIdx.x] = total;
}

// One workgroup: in-place exclusive scan of the tile totals, tile after tile with a carry.
static __global__ void __launch_bounds__(kBlock) scan_sums(int32_t* __restrict__ sums, int64_t count) {
  int carry = 0;
  for (int64_t tile = 0; tile < count; tile += kScanTile) {
    const int64_t base = tile + threadIdx.x * 4;
    int v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = base + j < count ? sums[base + j] : 0;
    int total;
    int prefix = carry + tile_exclusive_scan(v, &total);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (base + j < count) sums[base + j] = prefix;
      prefix += v[j];
    }
    carry += total;
  }
}

// data[i] += (scanned) total of the tiles before i's tile; cursor[i] = data[i] for i < K.
static __global__ void __launch_bounds__(kBlock) add_tile_offsets(int32_t* __restrict__ data, int64_t n, const int32_t* __restrict__ sums,
                                                          int32_t* __restrict__ cursor, int64_t K) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += stride) {
    const int value = data[i] + sums[i / kScanTile];
    data[i] = value;
    if (i < K) cursor[i] = value;
  }
}

// ----------------------------------------------- kernels of the K-phased path --
// The K-phased path (launch_phased) cuts the column range [0, K) into Q equal parts and runs the
// whole operation once per part, one launch after the other, so that at any time the gathers touch
// only K / Q rows of B.  For that every row is cut into Q consecutive pieces: piece q of row r
// starts at the first stored position of the row whose column is >= q * cols_per_part.  With
// columns sorted inside the rows (what CSR builders produce) piece q holds exactly the entries of
// part q; with any other order the pieces still partition the row, so the result is the same and
// only the locality is lost.
//   piece_start[q * M + r]        = that stored position
//   piece_len[q * (M + 1) + r]    = length of the piece (entry M of every part is 0), which an
//                                    exclusive scan over all Q * (M + 1) numbers turns into the
//                                    virtual row starts of part q
// Lanes that sit side by side search the SAME row for consecutive parts (their probes fall into the
// same few cache lines); a wavefront takes 64 / lanes_per_row rows, lanes_per_row = Q rounded up to a
// power of two.
static __global__ void __launch_bounds__(kBlock) phase_pieces(int32_t M, int32_t Q, int32_t lanes_shift, int32_t cols_per_part,
                                                             const int32_t* __restrict__ rowptr, const int32_t* __restrict__ colind,
                                                             int32_t* __restrict__ piece_start, int32_t* __restrict__ piece_len) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  const int64_t row = t >> lanes_shift;
  const int q = (int)(t & ((1 << lanes_shift) - 1));
  const bool live = row < M && q < Q;
  const int r = (int)(row < M ? row : M - 1);
  const int s = rowptr[r], e = rowptr[r + 1];
  // Eight-way search over the whole row: seven probes per round, all in flight together, three rounds
  // for a row of 500 entries where a binary search makes nine dependent loads.  The interval becomes the
  // gap before the LEFTMOST probe whose column is >= the one searched for.  For any data, sorted or not,
  // that choice is monotone in the column searched for as long as every search starts from the same
  // interval (a larger column can only move the leftmost such probe to the right, and equal intervals
  // are probed alike), which is what makes the pieces a partition of the row: the end of piece q IS the
  // start of piece q + 1.
  int lo = s, hi = e;                               // the answer lies in [lo, hi]
  const int64_t column = (int64_t)q * cols_per_part;
  if (q == 0 || !live) hi = lo;                     // piece 0 starts where the row starts
  while (lo < hi) {
    const int step = (hi - lo + 7) >> 3;
    int seen[7];
#pragma unroll
    for (int i = 0; i < 7; ++i) {
      const int p = lo + (i + 1) * step - 1;        // a probe at or beyond hi does not exist
      seen[i] = colind[p < hi ? p : hi - 1];
    }
    int new_lo = lo, new_hi = hi;
    bool found = false;
#pragma unroll
    for (int i = 0; i < 7; ++i) {
      const int p = lo + (i + 1) * step - 1;
      if (!found && p < hi) {
        if (seen[i] < column) new_lo = p + 1;
        else {
          new_hi = p;
          found = true;
        }
      }
    }
    lo = new_lo;
    hi = new_hi;
  }
  const int begin = lo;
  const int next_begin = __shfl_down(begin, 1, kWave);    // the lane to the right holds part q + 1 of the same row
  const int end = q == Q - 1 ? e : next_begin;
  if (live) {
    piece_start[(int64_t)q * M + r] = begin;
    piece_len[(int64_t)q * (M + 1) + r] = end - begin;
    if (r == 0) piece_len[(int64_t)q * (M + 1) + M] = 0;
  }
}

// piece_start[q * M + r] -= virtual_start[q * (M + 1) + r]: what is left is the number a virtual
// position of row r in part q needs added to become the stored position.
static __global__ void __launch_bounds__(kBlock) phase_deltas(int32_t M, int32_t Q, const int32_t* __restrict__ virtual_start,
                                                             int32_t* __restrict__ piece_start) {
  const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
  if (t >= (int64_t)Q * M) return;
  const int64_t q = t / M, r = t % M;
  piece_start[t] -= virtual_start[q * (M + 1) + r];
}

// C[r, :] /= stored length of row r (the mean, after the phases have summed); empty rows stay 0.
static __global__ void __launch_bounds__(kBlock) divide_rows_by_length(int32_t M, int32_t N, const int32_t* __restrict__ rowptr,
                                                                      float* __restrict__ C) {
  const int64_t total = (int64_t)M * N;
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t i = (int64_t)blockIdx.x * kBlock + threadIdx.x; i < total; i += stride) {
    const int64_t r = i / N;
    const int len = rowptr[r + 1] - rowptr[r];
    if (len > 1) C[i] = C[i] / (float)len;
  }
}

// --------------------------------------------------------------- host side --
using MainKernel = void (*)(const KernelArgs);

enum Job { kJobAdd = kAdd, kJobMax = kMax, kJobMin = kMin, kJobArg = 3, kJobTransposed = 4, kJobScatter = 5,
           kJobMaxWithArg = 6, kJobMinWithArg = 7 };

template <template <int, int> class P, int V>
MainKernel pick_gt(int G, int T) {
#define GESPMM_CASE(GG, TT) if (G == GG && T == TT) return chunk_kernel<P<V, TT>, V, GG, TT, false>;
  GESPMM_CASE(1, 1) GESPMM_CASE(2, 1) GESPMM_CASE(4, 1) GESPMM_CASE(8, 1)
  GESPMM_CASE(16, 1) GESPMM_CASE(32, 1) GESPMM_CASE(64, 1)
  GESPMM_CASE(4, 2) GESPMM_CASE(8, 2) GESPMM_CASE(16, 2) GESPMM_CASE(32, 2) GESPMM_CASE(64, 2)
  GESPMM_CASE(8, 4) GESPMM_CASE(16, 4) GESPMM_CASE(32, 4) GESPMM_CASE(64, 4)
#undef GESPMM_CASE
  return nullptr;
}

template <int V, int T> using AddRows = FoldRows<kAdd, V, T>;
template <int V, int T> using MaxRows = FoldRows<kMax, V, T>;
template <int V, int T> using MinRows = FoldRows<kMin, V, T>;
template <int V, int T> using MaxArgRows = FoldArgRows<kMax, V, T>;
template <int V, int T> using MinArgRows = FoldArgRows<kMin, V, T>;
template <int V, int T> using PlainArgRows = ArgRows<V, T>;

template <int V>
MainKernel pick_job(int job, int G, int T) {
  switch (job) {
    case kJobAdd: return pick_gt<AddRows, V>(G, T);
    case kJobMax: return pick_gt<MaxRows, V>(G, T);
    case kJobMin: return pick_gt<MinRows, V>(G, T);
    case kJobArg: return pick_gt<PlainArgRows, V>(G, T);
    case kJobMaxWithArg: return pick_gt<MaxArgRows, V>(G, T);
    case kJobMinWithArg: return pick_gt<MinArgRows, V>(G, T);
    case kJobTransposed: return pick_gt<TransposedRows, V>(G, T);
    case kJobScatter: return (V == 1 && G == 1 && T == 1) ? chunk_kernel<ScatterRows<1, 1>, 1, 1, 1, false> : nullptr;
    default: return nullptr;
  }
}

inline MainKernel pick_kernel(int job, int vec, int G, int T) {
  return vec == 4 ? pick_job<4>(job, G, T) : pick_job<1>(job, G, T);
}

// 16-bit feature matrices: the three folds, one tile per lane; four columns per lane (one
// 8-byte load, the same four fp32 accumulators per lane as the fp32 kernels; measured 10-40 %
// faster than eight columns per lane with 16-byte loads) in slots of up to 32 lanes, or one
// column per lane in slots of any width.
template <int F, class BT>
MainKernel pick_b16_fold(int vec, int G, int T) {
  if (T != 1) return nullptr;
#define GESPMM_CASE(VV, GG) if (vec == VV && G == GG) return chunk_kernel<FoldRows<F, VV, 1, BT>, VV, GG, 1, false>;
  GESPMM_CASE(4, 1) GESPMM_CASE(4, 2) GESPMM_CASE(4, 4) GESPMM_CASE(4, 8) GESPMM_CASE(4, 16) GESPMM_CASE(4, 32)
  GESPMM_CASE(1, 1) GESPMM_CASE(1, 2) GESPMM_CASE(1, 4) GESPMM_CASE(1, 8) GESPMM_CASE(1, 16) GESPMM_CASE(1, 32) GESPMM_CASE(1, 64)
#undef GESPMM_CASE
  return nullptr;
}

template <class P4, class P1>
MainKernel pick_b16_shapes(int vec, int G, int T) {      // P4 / P1: the policy for 4 columns / 1 column per lane
  if (T != 1) return nullptr;
#define GESPMM_CASE4(GG) if (vec == 4 && G == GG) return chunk_kernel<P4, 4, GG, 1, false>;
#define GESPMM_CASE1(GG) if (vec == 1 && G == GG) return chunk_kernel<P1, 1, GG, 1, false>;
  GESPMM_CASE4(1) GESPMM_CASE4(2) GESPMM_CASE4(4) GESPMM_CASE4(8) GESPMM_CASE4(16) GESPMM_CASE4(32)
  GESPMM_CASE1(1) GESPMM_CASE1(2) GESPMM_CASE1(4) GESPMM_CASE1(8) GESPMM_CASE1(16) GESPMM_CASE1(32) GESPMM_CASE1(64)
#undef GESPMM_CASE4
#undef GESPMM_CASE1
  return nullptr;
}

template <class BT>
MainKernel pick_b16(int job, int vec, int G, int T) {
  switch (job) {
    case kJobAdd: return pick_b16_fold<kAdd, BT>(vec, G, T);
    case kJobMax: return pick_b16_fold<kMax, BT>(vec, G, T);
    case kJobMin: return pick_b16_fold<kMin, BT>(vec, G, T);
    case kJobMaxWithArg: return pick_b16_shapes<FoldArgRows<kMax, 4, 1, BT>, FoldArgRows<kMax, 1, 1, BT>>(vec, G, T);
    case kJobMinWithArg: return pick_b16_shapes<FoldArgRows<kMin, 4, 1, BT>, FoldArgRows<kMin, 1, 1, BT>>(vec, G, T);
    case kJobArg: return pick_b16_shapes<ArgRows<4, 1, BT>, ArgRows<1, 1, BT>>(vec, G, T);
    default: return nullptr;
  }
}

// Kernels of the K-phased path: the three folds with four columns per lane; slots of 8, 16 or 32
// lanes with one tile per lane, slots of 8 or 16 lanes with two.
inline bool has_phased_kernel(int G, int T) { return (T == 1 && (G == 8 || G == 16 || G == 32)) || (T == 2 && (G == 8 || G == 16)); }

template <class BT>
MainKernel pick_phased(int job, int vec, int G, int T) {
  if (vec != 4) return nullptr;
#define GESPMM_CASE(FF, GG, TT) if (job == FF && G == GG && T == TT) return chunk_kernel<FoldRows<FF, 4, TT, BT>, 4, GG, TT, true>;
  GESPMM_CASE(kAdd, 8, 1) GESPMM_CASE(kAdd, 16, 1) GESPMM_CASE(kAdd, 32, 1) GESPMM_CASE(kAdd, 8, 2) GESPMM_CASE(kAdd, 16, 2)
  GESPMM_CASE(kMax, 8, 1) GESPMM_CASE(kMax, 16, 1) GESPMM_CASE(kMax, 32, 1) GESPMM_CASE(kMax, 8, 2) GESPMM_CASE(kMax, 16, 2)
  GESPMM_CASE(kMin, 8, 1) GESPMM_CASE(kMin, 16, 1) GESPMM_CASE(kMin, 32, 1) GESPMM_CASE(kMin, 8, 2) GESPMM_CASE(kMin, 16, 2)
#undef GESPMM_CASE
  return nullptr;
}

// max / min with positions on the K-phased path (fp32 features, four columns per lane)
inline MainKernel pick_phased_arg(int job, int vec, int G, int T) {
  if (vec != 4) return nullptr;
#define GESPMM_CASE(JOB, FF, GG, TT) if (job == JOB && G == GG && T == TT) return chunk_kernel<FoldArgRows<FF, 4, TT>, 4, GG, TT, true>;
  GESPMM_CASE(kJobMaxWithArg, kMax, 8, 1) GESPMM_CASE(kJobMaxWithArg, kMax, 16, 1) GESPMM_CASE(kJobMaxWithArg, kMax, 32, 1)
  GESPMM_CASE(kJobMaxWithArg, kMax, 8, 2) GESPMM_CASE(kJobMaxWithArg, kMax, 16, 2)
  GESPMM_CASE(kJobMinWithArg, kMin, 8, 1) GESPMM_CASE(kJobMinWithArg, kMin, 16, 1) GESPMM_CASE(kJobMinWithArg, kMin, 32, 1)
  GESPMM_CASE(kJobMinWithArg, kMin, 8, 2) GESPMM_CASE(kJobMinWithArg, kMin, 16, 2)
#undef GESPMM_CASE
  return nullptr;
}

// Kernels of the whole-row path, one tile per lane: the three folds and max / min with positions on fp32 features ...
inline bool has_owned_kernel(int G, int T) { return T == 1 && G >= 1 && G <= kWave; }

template <class P4, class P1>
MainKernel pick_owned_shapes(int vec, int G) {      // P4 / P1: the policy for 4 columns / 1 column per lane
#define GESPMM_CASE(GG)                                                         \
  if (vec == 4 && G == GG) return chunk_kernel<P4, 4, GG, 1, false, true>;      \
  if (vec == 1 && G == GG) return chunk_kernel<P1, 1, GG, 1, false, true>;
  GESPMM_CASE(1) GESPMM_CASE(2) GESPMM_CASE(4) GESPMM_CASE(8) GESPMM_CASE(16) GESPMM_CASE(32) GESPMM_CASE(64)
#undef GESPMM_CASE
  return nullptr;
}

// ... and the three folds on 16-bit features (slots of up to 32 lanes with four columns per lane)
template <int F, class BT>
MainKernel pick_owned_b16_fold(int vec, int G) {
  if (vec == 4 && G > 32) return nullptr;
  return pick_owned_shapes<FoldRows<F, 4, 1, BT>, FoldRows<F, 1, 1, BT>>(vec, G);
}

template <class BT>
MainKernel pick_owned_b16(int job, int vec, int G, int T) {
  if (T != 1) return nullptr;
  switch (job) {
    case kJobAdd: return pick_owned_b16_fold<kAdd, BT>(vec, G);
    case kJobMax: return pick_owned_b16_fold<kMax, BT>(vec, G);
    case kJobMin: return pick_owned_b16_fold<kMin, BT>(vec, G);
    default: return nullptr;
  }
}

inline MainKernel pick_owned(int job, int vec, int G, int T) {
  if (T != 1) return nullptr;
  switch (job) {
    case kJobAdd: return pick_owned_shapes<FoldRows<kAdd, 4, 1>, FoldRows<kAdd, 1, 1>>(vec, G);
    case kJobMax: return pick_owned_shapes<FoldRows<kMax, 4, 1>, FoldRows<kMax, 1, 1>>(vec, G);
    case kJobMin: return pick_owned_shapes<FoldRows<kMin, 4, 1>, FoldRows<kMin, 1, 1>>(vec, G);
    case kJobMaxWithArg: return pick_owned_shapes<FoldArgRows<kMax, 4, 1>, FoldArgRows<kMax, 1, 1>>(vec, G);
    case kJobMinWithArg: return pick_owned_shapes<FoldArgRows<kMin, 4, 1>, FoldArgRows<kMin, 1, 1>>(vec, G);
    default: return nullptr;
  }
}

inline bool has_kernel(int G, int T) { return pick_gt<AddRows, 4>(G, T) != nullptr; }

inline int next_pow2(int64_t x) {
  int p = 1;
  while (p < x && p < 64) p <<= 1;
  return p;
}

// Per-call overrides of the automatic launch shape (-1 = automatic), checked copy of gespmm_tuning_t.
struct Tuning {
  int g = -1, t = -1, remap = -1, shift = -1, short_len = -1, k_parts = -1;
  int longest_row = -1;       // the caller's upper bound on the stored entries of a row; -1 = not known
  bool wide_addresses = false;   // 64-bit addresses for the gathers even where 32-bit offsets would do
};

inline int parse_tuning(const gespmm_tuning_t* in, Tuning* out) {
  *out = Tuning{};
  if (!in) return GESPMM_OK;
  const int G = in->lanes_per_row, T = in->tiles_per_lane;
  if (G > 0 && (G > kWave || (G & (G - 1)) != 0)) return GESPMM_ERR_BAD_ARG;
  if (T > 0 && T != 1 && T != 2 && T != 4) return GESPMM_ERR_BAD_ARG;
  if (G > 0 && T > 0 && !has_kernel(G, T)) return GESPMM_ERR_BAD_ARG;
  if (in->xcd_remap > 4096) return GESPMM_ERR_BAD_ARG;
  int shift = -1;
  if (in->chunk_nnz > 0) {
    for (int sh = kMinChunkShift; sh <= kMaxChunkShift; ++sh)
      if (in->chunk_nnz == (1 << sh)) shift = sh;
    if (shift < 0) return GESPMM_ERR_BAD_ARG;
  }
  if (in->short_len > (1 << kMaxChunkShift)) return GESPMM_ERR_BAD_ARG;
  if (in->k_parts > kMaxParts) return GESPMM_ERR_BAD_ARG;
  out->g = G > 0 ? G : -1;
  out->t = T > 0 ? T : -1;
  out->remap = in->xcd_remap >= 0 ? in->xcd_remap : -1;
  out->shift = shift;
  out->short_len = in->short_len >= 0 ? in->short_len : -1;
  out->k_parts = in->k_parts >= 0 ? (in->k_parts < 2 ? 1 : in->k_parts) : -1;
  out->longest_row = in->longest_row > 0 ? in->longest_row : -1;
  out->wide_addresses = in->wide_addresses > 0;
  return GESPMM_OK;
}

// A problem that yields fewer wavefronts than this (8 per compute unit) gets smaller chunks,
// so that its rows are spread over more of the chip.  Measured on matrices of 10^4 .. 10^6
// entries: below this count halving the chunk pays; above it the extra split rows (finished
// by atomics) and the extra row searches cost more than the added parallelism brings.
constexpr int64_t kMinWaves = 2048;
// chunks of a quarter of the size at the end of every phase of the K-phased path: two per wavefront the chip holds
constexpr int kTaperChunks = 2 * 256 * 20;

// Workspace of the K-phased path for Q parts: virtual row starts Q * (M + 1), deltas Q * M, scan totals.
inline size_t phased_workspace_bytes(int64_t M, int Q) {
  const int64_t n = (int64_t)Q * (M + 1);
  const int64_t tiles = (n + kScanTile - 1) / kScanTile;
  return (size_t)(n + (int64_t)Q * M + tiles + 4) * sizeof(int32_t);
}

// Number of parts the K range is cut into (1 = the plain path).  The phases pay when the rows of B
// a column block touches (K x block bytes) are several times larger than one L2 (4 MB per XCD) and
// the rows of A are long enough that a piece of a row still holds a few dozen entries.  A part is
// sized to about 7.5 MB of B rows: measured on the 233k-vertex workload (60 MB of B), 8 parts beat
// 6, 10, 14, 20 and 28; smaller parts raise the L2 hit rate further (65 % -> 84 %) but every phase
// re-reads and re-writes C and walks all rows again, which costs more than the hits bring.  The
// phases start to pay where the rows the PLAIN path's own column block touches (plain_block_bytes per
// row) reach about twice an L2: a 40k-row matrix of mean row 130 at N = 512 (10 MB per block of 256
// bytes) is 15 % faster in two parts, the same matrix at N = 128 (5 MB per block of 128 bytes) is
// slower.  Needs the vector kernels and, unless forced, a workspace that is large enough.
inline int choose_parts(int64_t M, int64_t K, int64_t nnz, int vec, int block_bytes, int plain_block_bytes, const Tuning& tune,
                        size_t workspace_bytes, int64_t part_bytes = 15ll << 19) {
  if (vec != 4 || M <= 0 || K <= 0 || nnz <= 0) return 1;
  if (tune.k_parts >= 0) return tune.k_parts < 2 ? 1 : (int)(tune.k_parts < K ? tune.k_parts : (K < 2 ? 1 : K));
  const int64_t live = K * block_bytes;
  const int64_t mean_row = nnz / M;
  if (K * plain_block_bytes < (8ll << 20) || mean_row < 128) return 1;
  int64_t q = (live + part_bytes / 2) / part_bytes;        // nearest multiple of 7.5 MB (10 MB with positions)
  if (q < 2) q = 2;
  while (q > 2 && mean_row / q < 32) --q;
  if (q > kMaxParts) q = kMaxParts;
  if (q < 2) return 1;
  if (workspace_bytes < phased_workspace_bytes(M, (int)q)) return 1;
  return (int)q;
}

// elem_bytes: size of one element of the dense input (4, or 2 for the 16-bit formats); a lane
// loads four columns at once when the width and the alignment allow it, one otherwise.
// whole_rows_allowed: the job has kernels of the whole-row path (the forward folds; max / min with positions and
// user-defined reduces on fp32 features).
// with_positions: max / min that also record positions; their phases move twice the bytes per output, so the
// parts are a third larger (measured on the 233k-vertex workload: 2.86 / 2.77 / 2.91 ms with 4 / 6 / 8 parts).
inline void make_plan(int64_t M, int64_t K, int64_t N, int64_t nnz, bool aligned16, int elem_bytes, const Tuning& tune,
                      size_t workspace_bytes, gespmm_plan_t* p, bool whole_rows_allowed = true, bool with_positions = false) {
  int vec = 1;
  if (aligned16 && N > 0) vec = N % 4 == 0 ? 4 : 1;        // 16-byte loads of fp32, 8-byte loads of 16-bit elements
  const int64_t ncv = N > 0 ? (N + vec - 1) / vec : 1;     // vector columns to cover
  // Column blocks of one 128-byte line (8 lanes x 16 bytes) up to N = 128, of two lines
  // beyond; wider N is covered by grid.y.  The blocks of one grid.y index run together in
  // time, so the part of B that is live at any moment is K x 128 (or 256) bytes, which the
  // L2s keep far better than whole rows of B; the sparse arrays are re-read per block,
  // which costs 8 bytes per entry against 128 gathered.
  int G = next_pow2(ncv), T = 1;
  int parts = 1;
  if (vec > 1) {
    const int line = 128 / (vec * elem_bytes);  // lanes that cover one 128-byte line of a row of B
    // the K-phased path keeps B in L2 by its own means and takes two lines per block
    const int wide = G > 2 * line ? 2 * line : G;
    // One line per block up to four lines of columns, two beyond.  Exactly four lines (N = 128 in fp32) go either
    // way: with short rows the per-row work of a column block weighs more than the L2 residency of a narrower
    // slice of B, and two blocks of two lines beat four blocks of one (13 of 16 suite matrices, by up to 31 % on
    // 27-point stencils; the three that lose, by 1-7 %, have mean rows of 30 and more).
    const bool two_lines = ncv > 4 * line || (elem_bytes == 4 && ncv == 4 * line && M > 0 && nnz / M < 28);
    const int plain = G > line ? (two_lines ? 2 * line : line) : G;            // what the plain path would take
    parts = choose_parts(M, K, nnz, vec, wide * vec * elem_bytes, plain * vec * elem_bytes, tune, workspace_bytes,
                         with_positions ? (10ll << 20) : (15ll << 19));
    if (parts > 1) G = wide < 8 ? 8 : wide;
    else G = plain;
  } else if (elem_bytes == 2) {
    if (G > 64) G = 64;                         // one column per lane, one tile: up to 64 columns per block
  } else if (G > 16) {
    G /= 2;
    T = 2;
    if (ncv > 64 && G * T < 128) { G = 64; T = 2; }
  }
  if (tune.g > 0) G = tune.g;
  if (tune.t > 0) T = tune.t;
  if (parts > 1 && !has_phased_kernel(G, T)) parts = 1;   // no phased kernel of that shape
  // chunk size: 256 items (stored entries and row ends); 512 for column blocks of up to 64
  // bytes (less data per entry) and for matrices with long rows (fewer split rows); halved
  // while the problem has too few chunks to fill the chip
  const int64_t col_blocks = (ncv + (int64_t)G * T - 1) / ((int64_t)G * T);
  const int64_t items = nnz + M;
  int shift = ((int64_t)vec * G * T * elem_bytes <= 64 || (M > 0 && nnz / M >= 128)) ? 9 : 8;
  // (the phases: 256 is 10 % slower than 512; 1024 is 3 % faster than 512 on the 233k-vertex workload, whose phases
  //  hold 14,000 chunks of that size, and 5 % slower on a 40k-row matrix whose phases are left with 2,500)
  //  (max / min with positions: 2 % slower with 1024, they keep 512)
  if (parts > 1) shift = (!with_positions && ((nnz / parts + M) >> 10) >= 8192) ? 10 : 9;
  // Narrow column blocks gather so little per entry that the fixed work of a chunk (row search, first row bounds)
  // weighs most: chunks of 1024 items where the problem still has thousands of them.  Up to 32 bytes per row of B
  // (N <= 8 in fp32): 4-7 % faster on R-MAT and power-law graphs of 10^6 rows, 15-27 % on a 27-point stencil and a
  // uniform graph of mean degree 4; but 6 % slower on a 170k-row graph that is left with 2400 chunks, hence the
  // floor of 4096.  Up to 128 bytes (one column block) when the caller has said that no row is longer than 64 entries (such matrices are
  // balanced whatever the chunk size): 1-19 % faster at N = 16 / 32 on the stencil and the uniform graph, where
  // graphs with hub rows lose 1-5 %.
  if (parts == 1 && vec == 4) {
    const int64_t block_bytes = (int64_t)vec * G * T * elem_bytes;
    const int64_t big_chunks = items >> 10;
    if (block_bytes <= 32 && big_chunks >= 4096) shift = 10;
    if (block_bytes <= 128 && col_blocks == 1 && tune.longest_row > 0 && tune.longest_row <= 64 && big_chunks >= 2048) shift = 10;
  }
  // ... but not below 512 when the mean row is that long: every chunk such a row crosses adds one fp32
  // rounding to each of its outputs (the atomic add), in an order the hardware picks.  A row of 10^5 ones
  // against an integer ramp (sums near 5 * 10^9: every rounding is a systematic half-way case) summed in
  // 10^4 random orders on the CPU: worst error 0.91 of the tolerance with 1563 chunks of 64, 0.62 with
  // chunks of 256, 0.25 with 512; rows of random values stay near 0.001 of it.
  const int floor_shift = (M > 0 && nnz / M >= 512) ? 9 : 6;
  while (shift > floor_shift && ((items / parts + (1ll << shift) - 1) >> shift) * col_blocks < kMinWaves) --shift;
  if (tune.shift >= kMinChunkShift) shift = tune.shift;
  p->vec = vec;
  p->lanes_per_row = G;
  p->tiles_per_lane = T;
  p->slots = kWave / G;
  p->chunk_nnz = 1 << shift;
  p->col_blocks = (int32_t)col_blocks;
  p->chunks = (items + p->chunk_nnz - 1) >> shift;
  p->grid_x = (p->chunks + kWavesPerBlock - 1) / kWavesPerBlock;
  p->block_threads = kBlock;
  // rows much longer than a chunk are finished by atomics from many consecutive chunks:
  // keep those chunks on one XCD (one L2); otherwise deal the chunks round-robin
  const bool long_rows = M > 0 && nnz / M >= p->chunk_nnz / 2;
  // Everything else on the plain path: runs of up to 32 consecutive workgroups per XCD, the runs dealt round-robin.
  // Neighbouring chunks (neighbouring rows of A, which in meshes and many graphs gather the same rows of B) then
  // share an L2, and every XCD still takes an even share of any stretch of the matrix: against chunk-by-chunk
  // round-robin 24 % / 11 % / 5 % / 3 % faster on 2-D and 3-D stencils of 90 k to 1 M rows, 1-3 % on small
  // power-law and uniform graphs, 1-2 % slower on unpermuted R-MAT graphs (whose heavy rows sit together; one
  // contiguous range per XCD costs 6 % there).  Shorter runs for grids of few workgroups, so that at least four
  // rounds of runs exist.
  int runs = 32;
  const int64_t groups = (p->chunks + kWavesPerBlock - 1) / kWavesPerBlock;
  while (runs > 1 && groups < (int64_t)8 * runs * 4) runs /= 2;
  p->xcd_remap = tune.remap >= 0 ? tune.remap : (parts > 1 ? 0 : (long_rows ? 1 : (runs > 1 ? runs : 0)));
  // Rows up to short_len entries are walked one per slot, longer ones by all slots together
  // (with a cross-slot combine per row).  Where the mean row has 17 .. 48 entries, as in
  // stencil and finite-element matrices whose rows all have about that length, one slot per
  // row up to 32 entries avoids that combine for most rows (measured: up to 22 % on a
  // 27-point stencil, within 3 % either way on power-law graphs of the same mean).
  const int64_t mean_row = M > 0 ? nnz / M / parts : 0;
  // (four slots: 16 beats 8 by 0-5 % on twelve matrices at N = 256 / 512; sixteen slots and more, N <= 16: 32 beats
  //  16 by 5-15 % on a 170k-vertex power-law graph and by 2 % on the R-MAT workload, and is neutral on nine others)
  int auto_short = p->slots >= 16 ? 32 : (p->slots >= 4 ? 16 : 2 * p->slots);
  if (mean_row > 16 && mean_row <= 48) auto_short = 32;
  p->short_len = tune.short_len >= 0 ? tune.short_len : auto_short;
  // The whole-row path (one launch, no presetting, no atomics) when the caller has said how long the
  // longest row is and that is short against a chunk: a wavefront then walks at most S + L entries
  // instead of S.  For problems that do not fill the chip anyway (where the second launch is a large
  // share of the call) rows of up to 1024 entries are accepted.  The hint only selects the path and
  // sizes the LDS slice; the result is right whatever it says.
  p->row_window = 0;
  if (whole_rows_allowed && parts == 1 && tune.longest_row > 0 && has_owned_kernel(G, T)) {
    const int64_t waves = ((items + p->chunk_nnz - 1) >> shift) * col_blocks;
    const bool small = waves <= 2 * kMinWaves;
    const int64_t accepted = small ? (p->chunk_nnz > 1024 ? p->chunk_nnz : 1024) : p->chunk_nnz;
    // (a large matrix whose mean row is below 8 has so few rows on chunk borders that nothing is gained: measured
    //  -3 % on a 5-point stencil of 10^6 rows, +-1 % on a uniform graph of mean degree 4, against +5 .. +14 % on
    //  27-point stencils and graphs of mean degree 10)
    if (tune.longest_row <= accepted && (small || nnz / M >= 8)) p->row_window = p->chunk_nnz + tune.longest_row;
    if (p->row_window > 1984) p->row_window = 0;   // 64 KB of LDS per workgroup; offsets into the slice are kept in 12 bits
  }
  const int slice = p->row_window > 0 ? p->row_window : p->chunk_nnz;
  p->lds_bytes = (int32_t)(kWavesPerBlock * (slice + (parts > 1 ? 2 : 1) * kWave) * sizeof(int2));
  p->k_parts = parts;
  p->workspace_bytes = parts > 1 ? (int64_t)phased_workspace_bytes(M, parts) : 0;
  if (parts > 1) {
    // a phase is launched with 5/4 of the wavefronts it needs when the parts hold equal shares of
    // the entries (counting the small chunks at its end); a part that holds more is finished by
    // the same wavefronts taking further chunks
    const int64_t phase_items = (nnz / parts) * 5 / 4 + M;
    int64_t small_items = (int64_t)kTaperChunks << (shift - 2);
    if (small_items > phase_items / 4) small_items = phase_items / 4;
    const int64_t phase_chunks = ((phase_items - small_items) >> shift) + ((small_items + (p->chunk_nnz >> 2) - 1) >> (shift - 2)) + 1;
    p->grid_x = (phase_chunks + kWavesPerBlock - 1) / kWavesPerBlock;
    if (p->grid_x < 1) p->grid_x = 1;
  }
}

// Event pairs around main-kernel launches, owned by the caller through an opaque handle.
struct Profiler {
  std::vector<hipEvent_t> start, stop;
  int used = 0;
};

inline int validate(int64_t M, int64_t K, int64_t N, int64_t nnz, const void* rowptr, const void* colind,
             const void* B, const void* C, int op) {
  if (M < 0 || K < 0 || N < 0 || nnz < 0) return GESPMM_ERR_BAD_ARG;
  if (op < GESPMM_SUM || op > GESPMM_MIN) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX || K > INT32_MAX || nnz > INT32_MAX - (1 << kMaxChunkShift) || N > INT32_MAX / 8) return GESPMM_ERR_TOO_LARGE;
  if (nnz > 0 && (M == 0 || K == 0)) return GESPMM_ERR_BAD_ARG;
  if (M == 0 || N == 0) return GESPMM_OK;
  if (!rowptr || !C) return GESPMM_ERR_NULL;
  if (nnz > 0 && (!colind || !B)) return GESPMM_ERR_NULL;
  return GESPMM_OK;
}

inline float bits_as_float(int32_t bits) {
  float f;
  std::memcpy(&f, &bits, sizeof(f));
  return f;
}

inline int launch_fill(float* dst, int64_t n, float value, hipStream_t stream) {
  if (n <= 0) return GESPMM_OK;
  int64_t blocks = (n + kBlock - 1) / kBlock;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(fill_f32, dim3((unsigned)blocks), dim3(kBlock), 0, stream, dst, n, value);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

// In-place exclusive scan of data[0 .. n) on the device; sums: scratch of ceil(n / kScanTile) numbers.
inline int launch_exclusive_scan(int32_t* data, int64_t n, int32_t* sums, hipStream_t stream) {
  const int64_t tiles = (n + kScanTile - 1) / kScanTile;
  hipLaunchKernelGGL(scan_tiles, dim3((unsigned)tiles), dim3(kBlock), 0, stream, data, n, sums);
  hipLaunchKernelGGL(scan_sums, dim3(1), dim3(kBlock), 0, stream, sums, tiles);
  int64_t blocks = (n + kBlock - 1) / kBlock;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(add_tile_offsets, dim3((unsigned)blocks), dim3(kBlock), 0, stream, data, n, sums, (int32_t*)nullptr, (int64_t)0);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

// One pass of the chunk kernel over the matrix, preceded (when init_target is set) by the
// row-initialisation kernel for that output.
struct ChunkLaunch {
  int job = kJobAdd;
  int64_t M = 0, K = 0, N = 0, nnz = 0;
  const int32_t* rowptr = nullptr;
  const int32_t* colind = nullptr;
  const float* vals = nullptr;
  const float* dense_in = nullptr;     // B, or dC
  float* dense_out = nullptr;          // C, or dB
  const float* result_in = nullptr;    // finished C for the position job
  int32_t* arg = nullptr;
  const void* also_aligned = nullptr;  // further buffer that must be 16-byte aligned for the vector kernels
  bool is_mean = false;
  float* init_target = nullptr;        // M x N output preset by init_rows, or nullptr
  float empty_value = 0.0f, split_value = 0.0f;
  float* init2_target = nullptr;       // a second M x N output to preset (positions of the fused pass)
  float empty2_value = 0.0f, split2_value = 0.0f;
  bool only_split = false;             // position job: leave rows that lie inside one chunk alone
  bool packed_split = false;           // fused value+position job: packed words for split rows, unpacked at the end
  MainKernel (*picker)(int vec, int G, int T) = nullptr;   // user-defined reduce: its own kernel table
  MainKernel (*owned_picker)(int vec, int G, int T) = nullptr;   // ... and its kernels of the whole-row path
  // user-defined reduce compiled at run time: launches the chunk kernel of the planned shape itself
  int (*launcher)(void* context, const gespmm_plan_t& plan, const KernelArgs& args, hipStream_t stream) = nullptr;
  void* launcher_context = nullptr;
  int32_t* cursor = nullptr;           // structure-transpose job only
  bool one_lane_per_entry = false;     // use the <V=1, G=1, T=1> instance whatever N is
  int b_dtype = GESPMM_F32;            // element type of dense_in (16-bit types: fold jobs only)
  Tuning tuning;                       // the caller's overrides
  Profiler* profiler = nullptr;        // brackets every main-kernel launch with an event pair while it has pairs left
  void* workspace = nullptr;           // enables the K-phased path (fold jobs only)
  size_t workspace_bytes = 0;
};

inline bool record_start(Profiler* prof, hipStream_t stream, bool* timed, int* status) {
  *timed = prof && prof->used < (int)prof->start.size();
  if (*timed && hipEventRecord(prof->start[prof->used], stream) != hipSuccess) {
    *status = GESPMM_ERR_HIP;
    return false;
  }
  return true;
}

inline bool record_stop(Profiler* prof, hipStream_t stream, bool timed, int* status) {
  if (!timed) return true;
  if (hipEventRecord(prof->stop[prof->used], stream) != hipSuccess) {
    *status = GESPMM_ERR_HIP;
    return false;
  }
  ++prof->used;
  return true;
}

inline void launch_init_rows(int vec, int64_t M, int64_t N, const int32_t* rowptr, float* target, float empty_value,
                             float split_value, int shift, hipStream_t stream) {
  int lanes_shift = 0;                          // lanes that write one row in init_rows
  while ((1 << lanes_shift) < kWave && ((int64_t)vec << lanes_shift) < N) ++lanes_shift;
  const unsigned init_blocks = (unsigned)((M + kBlock - 1) / kBlock);
  if (vec == 4)
    hipLaunchKernelGGL(init_rows<4>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)M, (int32_t)N, rowptr, target,
                       empty_value, split_value, shift, lanes_shift);
  else
    hipLaunchKernelGGL(init_rows<1>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)M, (int32_t)N, rowptr, target,
                       empty_value, split_value, shift, lanes_shift);
}

// Fold jobs gather through a buffer descriptor with 32-bit byte offsets when B is smaller than 2 GiB (and, for
// the scalar kernels, holds 4-byte elements: a 2-byte buffer load would need a 2-byte aligned descriptor path
// of its own); otherwise the kernels compute 64-bit addresses.
inline void set_narrow_b(const ChunkLaunch& L, int vec, KernelArgs* a) {
  const int64_t elem = L.b_dtype == GESPMM_F32 ? 4 : 2;
  const int64_t bytes = L.K * L.N * elem;
  a->b_row_bytes = 0;
  a->b_bytes = 0;
  if (bytes > 0 && bytes < (int64_t)0x7ff00000 && (vec == 4 || elem == 4) && !L.tuning.wide_addresses) {
    a->b_row_bytes = (uint32_t)(L.N * elem);
    a->b_bytes = (uint32_t)bytes;
  }
}

// Unpacks the (value, position) words that rows hold after a fused pass: the rows shared by several chunks of
// 2^shift items, or every row (shift < 0).
inline int launch_finish_rows(bool is_max, int64_t M, int64_t N, const int32_t* rowptr, float* C, int32_t* arg, int shift,
                              hipStream_t stream) {
  const unsigned blocks = (unsigned)((M + kBlock - 1) / kBlock);
  int words = 1;
  while (words * kWave < N) words *= 2;
#define GESPMM_FINISH(WW)                                                                                                \
  if (words == WW) {                                                                                                     \
    if (is_max)                                                                                                          \
      hipLaunchKernelGGL((finish_split_rows<kMax, WW>), dim3(blocks), dim3(kBlock), 0, stream, (int32_t)M, (int32_t)N, rowptr, \
                         C, arg, shift);                                                                                 \
    else                                                                                                                 \
      hipLaunchKernelGGL((finish_split_rows<kMin, WW>), dim3(blocks), dim3(kBlock), 0, stream, (int32_t)M, (int32_t)N, rowptr, \
                         C, arg, shift);                                                                                 \
  }
  GESPMM_FINISH(1) GESPMM_FINISH(2) GESPMM_FINISH(4) GESPMM_FINISH(8) GESPMM_FINISH(16)
#undef GESPMM_FINISH
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

// The K-phased path: C = A (x) B as plan.k_parts launches, part q of the column range after part q - 1.
// Every launch gathers from K / k_parts rows of B only, which the L2s hold, instead of from all of B.
//   1. every non-empty row of C is preset to the reduce identity (empty rows to 0);
//   2. phase_pieces cuts every row into k_parts pieces, an exclusive scan numbers the entries of every
//      part consecutively (its virtual row starts), phase_deltas keeps what leads back to the stored
//      positions: Q * (2 M + 1) numbers in the caller's workspace;
//   3. one launch of the chunk kernel per part on that part's virtual CSR, folding into C; launches on
//      one stream run one after the other, so no two wavefronts that may touch the same row with plain
//      loads and stores are ever in flight together;
//   4. mean: the phases sum, a last kernel divides the rows by their stored length.
inline int launch_phased(const ChunkLaunch& L, const gespmm_plan_t& plan, MainKernel kernel, int shift, hipStream_t stream) {
  const int Q = plan.k_parts;
  const int64_t M = L.M;
  if (((uintptr_t)L.workspace & 3u) != 0 || L.workspace_bytes < phased_workspace_bytes(M, Q)) return GESPMM_ERR_WORKSPACE;
  int32_t* virtual_start = static_cast<int32_t*>(L.workspace);          // Q * (M + 1)
  int32_t* delta = virtual_start + (int64_t)Q * (M + 1);                // Q * M
  int32_t* sums = delta + (int64_t)Q * M;
  const int cols_per_part = (int)((L.K + Q - 1) / Q);

  const bool with_positions = L.job == kJobMaxWithArg || L.job == kJobMinWithArg;
  if (with_positions) {
    // value and position travel as one 64-bit word per output, kept in the row's own C and arg storage through
    // all phases (zero: no entry yet) and unpacked by one kernel after the last phase
    if (!L.arg || L.N > kWave * kFinishWords || plan.vec != 4) return GESPMM_ERR_BAD_ARG;
    int filled = launch_fill(L.dense_out, M * L.N, 0.0f, stream);
    if (filled == GESPMM_OK) filled = launch_fill(reinterpret_cast<float*>(L.arg), M * L.N, 0.0f, stream);
    if (filled != GESPMM_OK) return filled;
  } else {
    launch_init_rows(plan.vec, M, L.N, L.rowptr, L.dense_out, L.empty_value, L.split_value, -1, stream);
  }
  const unsigned piece_blocks = (unsigned)(((int64_t)Q * M + kBlock - 1) / kBlock);
  int lanes_shift = 0;                              // lanes that share a row in phase_pieces
  while ((1 << lanes_shift) < Q) ++lanes_shift;
  const unsigned search_blocks = (unsigned)(((M << lanes_shift) + kBlock - 1) / kBlock);
  hipLaunchKernelGGL(phase_pieces, dim3(search_blocks), dim3(kBlock), 0, stream, (int32_t)M, Q, lanes_shift, cols_per_part, L.rowptr,
                     L.colind, delta, virtual_start);
  if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  const int scanned = launch_exclusive_scan(virtual_start, (int64_t)Q * (M + 1), sums, stream);
  if (scanned != GESPMM_OK) return scanned;
  hipLaunchKernelGGL(phase_deltas, dim3(piece_blocks), dim3(kBlock), 0, stream, (int32_t)M, Q, virtual_start, delta);
  if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;

  KernelArgs a{};
  a.M = (int32_t)M;
  a.N = (int32_t)L.N;
  a.nnz = (int32_t)L.nnz;
  a.is_mean = 0;
  a.chunks = 0;
  a.chunk_blocks = plan.grid_x;
  a.xcd_remap = plan.xcd_remap;
  a.chunk_shift = shift;
  a.short_len = plan.short_len;
  a.colind = L.colind;
  a.vals = L.vals;
  a.B = L.dense_in;
  a.C = L.dense_out;
  a.accumulate = 1;
  a.taper_chunks = kTaperChunks;
  if (with_positions) {
    a.arg = L.arg;
    a.packed_split = 1;
  }
  set_narrow_b(L, plan.vec, &a);
  // with one column block every stored entry is read once per call (measured: 1.3 % faster on the 233k-vertex workload;
  // with several blocks the re-reads of the entries would miss: 6 % slower on a 40k-row matrix at N = 512)
  a.stream_entries = plan.col_blocks == 1 ? 1 : 0;
  int status = GESPMM_OK;
  for (int q = 0; q < Q; ++q) {
    a.rowptr = virtual_start + (int64_t)q * (M + 1);
    a.delta = delta + (int64_t)q * M;
    bool timed = false;
    if (!record_start(L.profiler, stream, &timed, &status)) return status;
    hipLaunchKernelGGL(kernel, dim3((unsigned)plan.grid_x, (unsigned)plan.col_blocks), dim3(kBlock), (size_t)plan.lds_bytes, stream, a);
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
    if (!record_stop(L.profiler, stream, timed, &status)) return status;
  }
  if (with_positions) return launch_finish_rows(L.job == kJobMaxWithArg, M, L.N, L.rowptr, L.dense_out, L.arg, -1, stream);
  if (L.is_mean) {
    int64_t blocks = (M * L.N + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(divide_rows_by_length, dim3((unsigned)blocks), dim3(kBlock), 0, stream, (int32_t)M, (int32_t)L.N, L.rowptr,
                       L.dense_out);
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  }
  return GESPMM_OK;
}

// took_whole_rows (optional): set when the whole-row path ran, i.e. every row is final and nothing is left to combine.
inline int launch_chunks(const ChunkLaunch& L, hipStream_t stream, bool* took_whole_rows = nullptr) {
  if (took_whole_rows) *took_whole_rows = false;
  const bool aligned16 = (((uintptr_t)L.dense_in | (uintptr_t)L.dense_out | (uintptr_t)L.result_in |
                           (uintptr_t)L.also_aligned) & 15u) == 0;
  const bool fold_job = !L.picker && !L.launcher && (L.job == kJobAdd || L.job == kJobMax || L.job == kJobMin) && !L.one_lane_per_entry;
  const bool arg_job = !L.picker && !L.launcher && (L.job == kJobMaxWithArg || L.job == kJobMinWithArg) && L.arg && !L.one_lane_per_entry;
  // jobs that have kernels of the K-phased path: the folds, and max / min with positions on fp32 features of up to 1024 columns
  const bool phases_possible = fold_job || (arg_job && L.b_dtype == GESPMM_F32 && L.N <= kWave * kFinishWords);
  Tuning tune = L.tuning;
  if (!phases_possible || !L.workspace) {
    if (tune.k_parts > 1 && phases_possible) return GESPMM_ERR_WORKSPACE;   // phases were asked for but there is nowhere to put their row starts
    tune.k_parts = 1;
  }
  gespmm_plan_t plan;
  const bool custom_job = (L.picker && L.owned_picker) || L.launcher;
  const bool whole_rows_allowed = (fold_job || ((arg_job || custom_job) && L.b_dtype == GESPMM_F32)) && L.init_target == L.dense_out;
  make_plan(L.M, L.K, L.N, L.nnz, aligned16, L.b_dtype == GESPMM_F32 ? 4 : 2, tune, L.workspace_bytes, &plan, whole_rows_allowed, arg_job);
  if (L.one_lane_per_entry) {
    plan.vec = 1;
    plan.lanes_per_row = 1;
    plan.tiles_per_lane = 1;
    plan.slots = kWave;
    plan.col_blocks = 1;
    plan.short_len = 16;
  }
  if (plan.col_blocks > 65535) return GESPMM_ERR_TOO_LARGE;   // grid.y limit (N beyond ~33 million)
  int shift = 0;
  while ((1 << shift) < plan.chunk_nnz) ++shift;

  if (plan.k_parts > 1 && L.nnz > 0) {
    MainKernel phased = nullptr;
    if (arg_job) phased = pick_phased_arg(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else if (L.b_dtype == GESPMM_BF16) phased = pick_phased<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else if (L.b_dtype == GESPMM_F16) phased = pick_phased<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else phased = pick_phased<float>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    if (!phased) return GESPMM_ERR_BAD_ARG;
    return launch_phased(L, plan, phased, shift, stream);
  }

  MainKernel kernel = nullptr;
  if (L.launcher) kernel = nullptr;
  else if (L.picker) kernel = L.picker(plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_BF16) kernel = pick_b16<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_F16) kernel = pick_b16<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else kernel = pick_kernel(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  if (plan.row_window > 0 && L.launcher) {
    kernel = nullptr;
  } else if (plan.row_window > 0 && L.picker) {
    kernel = L.owned_picker(plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  } else if (plan.row_window > 0) {
    if (L.b_dtype == GESPMM_BF16) kernel = pick_owned_b16<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else if (L.b_dtype == GESPMM_F16) kernel = pick_owned_b16<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else kernel = pick_owned(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  }
  if (!kernel && !L.launcher) return GESPMM_ERR_BAD_ARG;

  // (a) empty rows and rows shared by several chunks are preset (the whole-row path writes every row itself)
  if (L.init_target && plan.row_window == 0) {
    launch_init_rows(plan.vec, L.M, L.N, L.rowptr, L.init_target, L.empty_value, L.split_value, shift, stream);
    if (L.init2_target)
      launch_init_rows(plan.vec, L.M, L.N, L.rowptr, L.init2_target, L.empty2_value, L.split2_value, shift, stream);
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  }
  if (L.nnz == 0 && plan.row_window == 0) return GESPMM_OK;

  // (b) the chunks
  KernelArgs a{};
  a.M = (int32_t)L.M;
  a.N = (int32_t)L.N;
  a.nnz = (int32_t)L.nnz;
  a.is_mean = L.is_mean ? 1 : 0;
  a.chunks = plan.chunks;
  a.chunk_blocks = plan.grid_x;
  a.xcd_remap = plan.xcd_remap;
  a.chunk_shift = shift;
  a.short_len = plan.short_len;
  a.rowptr = L.rowptr;
  a.delta = nullptr;
  a.colind = L.colind;
  a.vals = L.vals;
  a.B = L.dense_in;
  a.C = L.dense_out;
  a.Cin = L.result_in;
  a.arg = L.arg;
  a.cursor = L.cursor;
  a.only_split = L.only_split ? 1 : 0;
  a.packed_split = L.packed_split ? 1 : 0;
  a.accumulate = 0;
  a.row_window = plan.row_window;
  if (fold_job || arg_job) set_narrow_b(L, plan.vec, &a);
  // Rows of C written once, in whole 128-byte lines per slot: streaming stores leave more of the L2s to B (2-5 %
  // on matrices of short rows at N >= 128; narrower slots write part of a line and lose 2 % with them).
  a.stream_stores = (fold_job || arg_job) && plan.vec == 4 && plan.lanes_per_row * 16 >= 128 ? 1 : 0;
  if (plan.row_window > 0) a.packed_split = 0;    // no row is split
  else if (L.packed_split && (plan.vec != 4 || L.N > kWave * kFinishWords || !L.arg)) return GESPMM_ERR_BAD_ARG;
  int status = GESPMM_OK;
  bool timed = false;
  if (!record_start(L.profiler, stream, &timed, &status)) return status;
  if (L.launcher) {
    const int launched = L.launcher(L.launcher_context, plan, a, stream);
    if (launched != GESPMM_OK) return launched;
  } else {
    hipLaunchKernelGGL(kernel, dim3((unsigned)plan.grid_x, (unsigned)plan.col_blocks), dim3(kBlock), (size_t)plan.lds_bytes, stream, a);
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  }
  if (!record_stop(L.profiler, stream, timed, &status)) return status;
  if (plan.row_window > 0) {
    if (took_whole_rows) *took_whole_rows = true;
    return GESPMM_OK;
  }
  if (L.packed_split) return launch_finish_rows(L.job == kJobMaxWithArg, L.M, L.N, L.rowptr, L.dense_out, L.arg, shift, stream);
  return GESPMM_OK;
}

template <class R>
struct CustomBind {
  template <int V, int T> using Rows = CustomRows<R, V, T>;
};

template <class R>
MainKernel pick_custom_owned(int vec, int G, int T) {
  return T == 1 ? pick_owned_shapes<CustomRows<R, 4, 1>, CustomRows<R, 1, 1>>(vec, G) : nullptr;
}

template <class R>
MainKernel pick_custom(int vec, int G, int T) {
  return vec == 4 ? pick_gt<CustomBind<R>::template Rows, 4>(G, T) : pick_gt<CustomBind<R>::template Rows, 1>(G, T);
}

}  // namespace gespmm_detail

namespace gespmm {

// C = A (x) B with the user-defined reduce R (see CustomRows for what R must provide).
// Same arguments, layout, ownership and errors as gespmm_csr; an empty row yields 0;
// `tuning` as in gespmm_csr_ex (NULL = automatic).
template <class R>
int csr_custom(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
               const float* vals, const float* B, float* C, hipStream_t stream, const gespmm_tuning_t* tuning = nullptr) {
  using namespace gespmm_detail;
  const int st = validate(M, K, N, nnz, rowptr, colind, B, C, GESPMM_SUM);
  if (st != GESPMM_OK || M == 0 || N == 0) return st;
  ChunkLaunch L;
  const int parsed = parse_tuning(tuning, &L.tuning);
  if (parsed != GESPMM_OK) return parsed;
  L.picker = &pick_custom<R>;
  L.owned_picker = &pick_custom_owned<R>;
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = B; L.dense_out = C;
  L.init_target = C; L.empty_value = 0.0f; L.split_value = R::identity();
  return launch_chunks(L, stream);
}

}  // namespace gespmm
