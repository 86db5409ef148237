// CSR SpMM / SpMM-like kernels for gfx950 (MI355X): device code and launch helpers.
// (The C ABI over them is in gespmm.hip; user-defined reduce operations include this
// file through include/gespmm_custom.hpp.)
//
// Result computed (paper: Algorithm 1, Section III-A; general reduce: Eq. 1, Section IV-A):
//     C[i, j] = reduce_p  vals[p] * B[colind[p], j],   p over the stored entries of row i.
//
// How the work is laid out (what is kept from the paper and what is not):
//  * The paper gives one thread block to each sparse row (Algorithms 2 and 3).  Here the
//    unit of work is a CHUNK of S consecutive stored entries, one per 64-lane wavefront,
//    so every wavefront has the same amount of gather work whatever the row lengths are.
//    A row that crosses a chunk border is finished with atomics (add, or integer
//    max/min on the ordered bit pattern of the float); rows inside one chunk are
//    written with plain stores by exactly one wavefront.
//  * Kept from Coalesced Row Caching (Section III-B): a wavefront first pulls its chunk
//    of (colind, val) with fully coalesced loads into LDS, then every lane reads the
//    entries it needs from LDS (broadcast reads), so sparse data crosses HBM once.
//  * Kept from Coarse-grained Warp Merging (Section III-C): one lane owns T column tiles
//    of 4 floats (one 16-byte load each), so the sparse chunk is read once for
//    4*G*T output columns and several independent B loads are in flight per lane.
//  * New for 64 lanes: the wavefront is cut into 64/G slots of G lanes; the G lanes of a
//    slot cover the column block.  Short row segments are handled one per slot, 64/G
//    rows at a time (no cross-lane traffic at all); long segments are handled by all
//    slots together, each slot taking every (64/G)-th entry, and the slot partials are
//    folded with cross-lane exchanges at the end of the row.
//  * A first small kernel zero-fills empty rows and writes the reduce identity into the
//    rows that will be finished with atomics.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstring>
#include <vector>

#include "gespmm.h"

namespace gespmm_detail {


constexpr int kWave = 64;
constexpr int kWavesPerBlock = 4;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kMinChunkShift = 4;               // chunks hold 16 .. 1024 stored entries
constexpr int kMaxChunkShift = 10;
constexpr int kXcds = 8;
// 16-byte gathers a lane issues before it waits (measured: 8 beats 4 and 16 for slots of
// up to 16 lanes; wider slots already move 512 B and more per load instruction)
constexpr int loads_in_flight(int G) { return G <= 16 ? 8 : 4; }

enum Fold { kAdd = 0, kMax = 1, kMin = 2 };

struct KernelArgs {
  int32_t M;
  int32_t N;
  int32_t nnz;
  int32_t is_mean;
  int64_t chunks;
  int64_t chunk_blocks;   // grid.x
  int32_t xcd_remap;
  int32_t chunk_shift;    // log2(S), S = stored entries per wavefront
  int32_t short_len;      // row segments up to this length are handled one per slot
  const int32_t* rowptr;
  const int32_t* colind;
  const float* vals;
  const float* B;         // dense input (the gradient dC for the transposed job)
  float* C;               // dense output (dB for the transposed job)
  const float* Cin;       // finished max/min result, read by the position job
  int32_t* arg;           // output of the position job; row indices of the transposed arrays
  int32_t* cursor;        // next free place of every transposed row (structure-transpose job)
  int32_t only_split;     // position job: rows inside one chunk were already done by the fused pass
  int32_t packed_split;   // fused value+position pass: split rows collect (value, position) pairs in 64-bit slots
};

// ------------------------------------------------------------------ vectors --
template <int V> struct Vec;
template <> struct Vec<4> {
  float v[4];
  __device__ static Vec load(const float* p) {
    const float4 t = *reinterpret_cast<const float4*>(p);
    return Vec{{t.x, t.y, t.z, t.w}};
  }
  __device__ void store(float* p) const { *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]); }
};
template <> struct Vec<1> {
  float v[1];
  __device__ static Vec load(const float* p) { return Vec{{*p}}; }
  __device__ void store(float* p) const { *p = v[0]; }
};
// Element types of the dense input.  The 16-bit types are storage formats only: every
// value is widened to fp32 (exactly) before the multiply, and products and sums are fp32.
struct bf16_t { uint16_t bits; };               // 1 sign, 8 exponent, 7 fraction bits: the top half of an fp32
struct f16_t { uint16_t bits; };                // IEEE binary16

// BLoad<V, BT>: one load of V consecutive elements of type BT, kept as loaded (Raw) until
// it is used, so that all loads of a pass can be in flight together; unpack widens to fp32.
template <int V, class BT> struct BLoad;
template <> struct BLoad<4, float> {
  using Raw = float4;
  __device__ static Raw load(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static void unpack(const Raw& r, float (&o)[4]) { o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w; }
};
template <> struct BLoad<1, float> {
  using Raw = float;
  __device__ static Raw load(const float* p) { return *p; }
  __device__ static void unpack(const Raw& r, float (&o)[1]) { o[0] = r; }
};
__device__ __forceinline__ void widen_pair(bf16_t, unsigned w, float& lo, float& hi) {
  lo = __uint_as_float(w << 16);
  hi = __uint_as_float(w & 0xffff0000u);
}
__device__ __forceinline__ void widen_pair(f16_t, unsigned w, float& lo, float& hi) {
  typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
  const half2_t h = __builtin_bit_cast(half2_t, w);
  lo = (float)h.x;
  hi = (float)h.y;
}
template <class BT> struct BLoad<4, BT> {       // BT = bf16_t or f16_t: 8 bytes = 4 elements
  using Raw = uint2;
  __device__ static Raw load(const BT* p) { return *reinterpret_cast<const uint2*>(p); }
  __device__ static void unpack(const Raw& r, float (&o)[4]) {
    widen_pair(BT{}, r.x, o[0], o[1]);
    widen_pair(BT{}, r.y, o[2], o[3]);
  }
};
template <> struct BLoad<1, bf16_t> {
  using Raw = uint16_t;
  __device__ static Raw load(const bf16_t* p) { return p->bits; }
  __device__ static void unpack(const Raw& r, float (&o)[1]) { o[0] = __uint_as_float((unsigned)r << 16); }
};
template <> struct BLoad<1, f16_t> {
  using Raw = uint16_t;
  __device__ static Raw load(const f16_t* p) { return p->bits; }
  __device__ static void unpack(const Raw& r, float (&o)[1]) { o[0] = (float)__builtin_bit_cast(_Float16, r); }
};

template <int F> __device__ __forceinline__ float fold_identity() {
  return F == kAdd ? 0.0f : (F == kMax ? -__builtin_inff() : __builtin_inff());
}
template <int F> __device__ __forceinline__ float fold(float acc, float a, float b) {
  if (F == kAdd) return __builtin_fmaf(a, b, acc);
  const float x = a * b;                     // one correctly rounded fp32 product, then compare
  return F == kMax ? __builtin_fmaxf(acc, x) : __builtin_fminf(acc, x);
}
template <int F> __device__ __forceinline__ float fold2(float x, float y) {
  return F == kAdd ? x + y : (F == kMax ? __builtin_fmaxf(x, y) : __builtin_fminf(x, y));
}

// Combine a partial result into C[ptr] when several wavefronts share the row.
// max/min use integer atomics on the float's bit pattern: for non-negative floats the
// signed-int order equals the float order, for negative floats the unsigned order is
// the reverse of the float order; -0 < +0 comes out as IEEE maximum/minimum want it.
template <int F> __device__ __forceinline__ void atomic_fold(float* ptr, float x) {
  if (F == kAdd) {
    __hip_atomic_fetch_add(ptr, x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  } else {
    const int bits = __float_as_int(x);
    if (F == kMax) {
      if (bits >= 0) __hip_atomic_fetch_max(reinterpret_cast<int*>(ptr), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else __hip_atomic_fetch_min(reinterpret_cast<unsigned*>(ptr), (unsigned)bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      if (bits >= 0) __hip_atomic_fetch_min(reinterpret_cast<int*>(ptr), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      else __hip_atomic_fetch_max(reinterpret_cast<unsigned*>(ptr), (unsigned)bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Workgroup id -> logical block id such that each XCD (workgroups are dealt to the 8
// XCDs round-robin) walks one contiguous range of chunks: a row split over several
// chunks then meets its atomics in one L2, and neighbouring rows of C stay together.
__device__ __forceinline__ int64_t logical_block(int64_t b, int64_t nb, int remap) {
  if (!remap) return b;
  const int64_t xcd = b % kXcds, within = b / kXcds;
  const int64_t q = nb / kXcds, r = nb % kXcds;
  return xcd * q + (xcd < r ? xcd : r) + within;
}

// ------------------------------------------------------------- init kernel --
// One lane per row decides; then groups of 2^lanes_shift lanes write one row each:
// empty rows get `empty_value` (0 for the result, the bits of -1 for positions); rows whose
// entries lie in more than one chunk get `split_value` (the reduce identity, or the bits
// of INT_MAX for positions): they are completed by atomics in the chunk kernel.
template <int V>
__global__ void __launch_bounds__(kBlock) init_rows(int32_t M, int32_t N, const int32_t* __restrict__ rowptr,
                                                   float* __restrict__ C, float empty_value, float split_value,
                                                   int chunk_shift, int lanes_shift) {
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t base = ((int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * kWave;
  if (base >= M) return;
  const int64_t r = base + lane;
  int flag = 0;
  if (r < M) {
    const int s = rowptr[r], e = rowptr[r + 1];
    if (s == e) flag = 1;
    else if ((s >> chunk_shift) != ((e - 1) >> chunk_shift)) flag = 2;
  }
  const unsigned long long todo = __ballot(flag != 0);
  if (todo == 0ull) return;
  const int lanes = 1 << lanes_shift;             // lanes per row
  const int rows_per_step = kWave >> lanes_shift;
  const int sub = lane >> lanes_shift;            // which row of the step this lane writes
  const int c0 = (lane & (lanes - 1)) * V;
  for (int j = 0; j < kWave; j += rows_per_step) {
    const unsigned long long window = rows_per_step == kWave ? ~0ull : (((1ull << rows_per_step) - 1ull) << j);
    if ((todo & window) == 0ull) continue;
    const int f = __shfl(flag, j + sub, kWave);
    if (f != 0) {
      float* row = C + (base + j + sub) * (int64_t)N;
      Vec<V> out;
#pragma unroll
      for (int x = 0; x < V; ++x) out.v[x] = f == 1 ? empty_value : split_value;
      for (int c = c0; c < N; c += lanes * V) out.store(row + c);
    }
  }
}

// ------------------------------------------------------- calibration copy --
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

// ------------------------------------------------------------ chunk kernel --
// The walk over chunks, rows and row segments is the same for every job; what is done
// with a row segment is a policy:
//   FoldRows        the SpMM-like operation itself            C = A (x) B   (B in fp32, bf16 or half)
//   FoldArgRows     max / min together with its position      C and arg[i,j] = first entry that gives C[i,j]
//   ArgRows         positions only, from a finished C         (split rows of the scalar / very wide cases)
//   TransposedRows  gradient of sum / mean w.r.t. B           dB += A^T (x) dC, by scatter-add
//   ScatterRows     structure transpose                       every entry takes a place in its column's row
//   CustomRows      a user-defined reduce                     (include/gespmm_custom.hpp)
// A policy has a per-row State and four steps: begin (per row), pass (U entries of the
// segment for the lane's column tiles), combine (fold the slots that shared a long row),
// end (write the row).  In `pass`, `first` is the LDS index of the lane's first entry,
// `stride` the distance to its next one, `left` how many of the U entries exist (<= 0:
// none); `first` itself always is a valid index.

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int F, int V, int T, class BT = float>
struct FoldRows {
  static constexpr bool kCanSkipWholeRows = false;
  struct State { Vec<V> acc[T]; };

  __device__ static void begin(State& s, const KernelArgs&, int64_t, int, const int (&)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int x = 0; x < V; ++x) s.acc[t].v[x] = fold_identity<F>();
  }

  // An entry that does not exist re-reads the last one that does: harmless for max/min
  // (idempotent) and given weight 0 for the sum, so the pass is straight-line code with
  // all gathers issued before the first use.
  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int, int first, int stride, int left,
                              const int (&)[T], const int (&colc)[T]) {
    using Load = BLoad<V, BT>;
    int2 e2[U];
    typename Load::Raw b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      e2[u] = ka[first + uu * stride];
      if (F == kAdd && u >= left) e2[u].y = 0;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
      for (int t = 0; t < T; ++t) b[u][t] = Load::load(brow + colc[t]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < T; ++t) {
        float bx[V];
        Load::unpack(b[u][t], bx);
#pragma unroll
        for (int x = 0; x < V; ++x) s.acc[t].v[x] = fold<F>(s.acc[t].v[x], __int_as_float(e2[u].y), bx[x]);
      }
  }

  template <int G>
  __device__ static void combine(State& s) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int x = 0; x < V; ++x) s.acc[t].v[x] = fold2<F>(s.acc[t].v[x], __shfl_xor(s.acc[t].v[x], off, kWave));
  }

  // Plain store when the whole row lay in this chunk, atomics otherwise (the row was
  // preset to the identity by init_rows).
  __device__ static void end(State& s, const KernelArgs& a, int64_t row, bool whole, int row_len, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    const float len = (float)row_len;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (col[t] < a.N) {
        if (whole) {
          if (a.is_mean) {
#pragma unroll
            for (int x = 0; x < V; ++x) s.acc[t].v[x] = s.acc[t].v[x] / len;
          }
          s.acc[t].store(crow + col[t]);
        } else {
          const float w = a.is_mean ? 1.0f / len : 1.0f;
#pragma unroll
          for (int x = 0; x < V; ++x) atomic_fold<F>(crow + col[t] + x, F == kAdd ? s.acc[t].v[x] * w : s.acc[t].v[x]);
        }
      }
    }
  }
};

// max / min that also tracks WHERE the extreme came from, for rows that lie inside one
// chunk: value and entry index travel together through the fold, the slot combine and the
// store.  The order is the total order of the float bit patterns (so +0 is above -0, as in
// the plain fold) and ties go to the smaller entry index, which is exactly "the first entry
// whose product has the bits of the result".
// Rows split across chunks are combined in one of two ways.  packed_split: value and position
// are packed into one 64-bit word, ordered so that an unsigned atomic max keeps the better
// value and, among equal values, the smaller position; the N words of row i live in the
// storage of the row itself (the first N/2 in C[i, :], the rest in arg[i, :], both preset to
// zero, which is below every packed word) and finish_split_rows unpacks them in place
// afterwards.  Otherwise split rows only get their value here (by atomics, as in FoldRows)
// and their positions are found by ArgRows in a second pass over the matrix.
template <int F, int V, int T, class BT = float>
struct FoldArgRows {
  static constexpr bool kCanSkipWholeRows = false;
  static_assert(F == kMax || F == kMin, "positions exist for max and min only");
  struct State { float best[T][V]; int where[T][V]; };

  // monotone map float bits -> signed int (larger float <=> larger key; -0 below +0)
  __device__ static int key_of(float x) {
    const int b = __float_as_int(x);
    return b ^ ((b >> 31) & 0x7fffffff);
  }
  __device__ static float value_of(int key) { return __int_as_float(key ^ ((key >> 31) & 0x7fffffff)); }
  __device__ static bool better(int k, int w, int best_k, int best_w) {
    return F == kMax ? (k > best_k || (k == best_k && w < best_w)) : (k < best_k || (k == best_k && w < best_w));
  }

  __device__ static void begin(State& s, const KernelArgs&, int64_t, int, const int (&)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int x = 0; x < V; ++x) {
        s.best[t][x] = fold_identity<F>();
        s.where[t][x] = INT32_MAX;
      }
  }

  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int cs, int first, int stride, int left,
                              const int (&)[T], const int (&colc)[T]) {
    using Load = BLoad<V, BT>;
    int2 e2[U];
    typename Load::Raw b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) {          // a missing entry repeats an existing one: same value, same index
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      e2[u] = ka[first + uu * stride];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
      for (int t = 0; t < T; ++t) b[u][t] = Load::load(brow + colc[t]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      const int where_u = cs + first + uu * stride;      // recomputed here rather than kept in registers across the loads
#pragma unroll
      for (int t = 0; t < T; ++t) {
        float bx[V];
        Load::unpack(b[u][t], bx);
#pragma unroll
        for (int x = 0; x < V; ++x) {
          // A lane meets its entries in increasing index order, so "first among equals" is
          // "replace on strict improvement only".  The hardware max / min orders the zeros
          // (+0 above -0), so the running value changes its bits exactly when the entry improves it.
          const float product = __int_as_float(e2[u].y) * bx[x];
          const float next = F == kMax ? __builtin_fmaxf(s.best[t][x], product) : __builtin_fminf(s.best[t][x], product);
          s.where[t][x] = __float_as_int(next) != __float_as_int(s.best[t][x]) ? where_u : s.where[t][x];
          s.best[t][x] = next;
        }
      }
    }
  }

  template <int G>
  __device__ static void combine(State& s) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int x = 0; x < V; ++x) {
          const float v = __shfl_xor(s.best[t][x], off, kWave);
          const int w = __shfl_xor(s.where[t][x], off, kWave);
          if (better(key_of(v), w, key_of(s.best[t][x]), s.where[t][x])) {
            s.best[t][x] = v;
            s.where[t][x] = w;
          }
        }
  }

  __device__ static void end(State& s, const KernelArgs& a, int64_t row, bool whole, int, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    int32_t* arow = a.arg + row * (int64_t)a.N;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (col[t] < a.N) {
        if (whole) {
          Vec<V> value, place;
#pragma unroll
          for (int x = 0; x < V; ++x) {
            value.v[x] = s.best[t][x];
            place.v[x] = __int_as_float(s.where[t][x]);
          }
          value.store(crow + col[t]);
          place.store(reinterpret_cast<float*>(arow + col[t]));
        } else if (a.packed_split) {
          const int half = a.N >> 1;         // N is even; a lane's V words can straddle the two halves
#pragma unroll
          for (int x = 0; x < V; ++x) {
            const int j = col[t] + x;
            unsigned long long* slot = j < half ? reinterpret_cast<unsigned long long*>(crow) + j
                                                : reinterpret_cast<unsigned long long*>(arow) + (j - half);
            __hip_atomic_fetch_max(slot, pack(key_of(s.best[t][x]), s.where[t][x]), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
        } else {
#pragma unroll
          for (int x = 0; x < V; ++x) atomic_fold<F>(crow + col[t] + x, s.best[t][x]);
        }
      }
    }
  }

  // (value key, position) -> 64-bit word whose unsigned order is "better value first, then
  // smaller position"; every word of a real entry is > 0.  unpack is the inverse.
  __device__ static unsigned long long pack(int key, int where) {
    unsigned ukey = (unsigned)key ^ 0x80000000u;            // signed order -> unsigned order
    if (F == kMin) ukey = ~ukey;                            // smaller value <=> larger word
    return ((unsigned long long)ukey << 32) | (unsigned)~where;
  }
  __device__ static void unpack(unsigned long long word, float& value, int& where) {
    unsigned ukey = (unsigned)(word >> 32);
    if (F == kMin) ukey = ~ukey;
    value = value_of((int)(ukey ^ 0x80000000u));
    where = (int)~(unsigned)word;
  }
};

// After the fused value+position pass with packed_split: every row whose entries lie in more
// than one chunk holds N packed words in its C and arg storage; one wavefront per such row
// reads them all, then writes the row's values and positions over them.  N <= 64 * kFinishWords.
constexpr int kFinishWords = 16;
// WORDS: packed words one lane holds per row (N <= 64 * WORDS); rows are taken kFinishWords / WORDS at
// a time so that their loads are in flight together.
template <int F, int WORDS>
__global__ void __launch_bounds__(kBlock) finish_split_rows(int32_t M, int32_t N, const int32_t* __restrict__ rowptr,
                                                           float* C, int32_t* arg, int chunk_shift) {
  using Rows = FoldArgRows<F, 4, 1>;
  constexpr int BATCH = kFinishWords / WORDS;
  const int lane = threadIdx.x & (kWave - 1);
  const int64_t base = ((int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6)) * kWave;
  if (base >= M) return;
  const int64_t r = base + lane;
  bool split = false;
  if (r < M) {
    const int s = rowptr[r], e = rowptr[r + 1];
    split = e > s && (s >> chunk_shift) != ((e - 1) >> chunk_shift);
  }
  unsigned long long todo = __ballot(split);
  const int half = N >> 1;
  while (todo) {
    int64_t row[BATCH];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {                  // the next BATCH split rows (-1: none left)
      row[q] = -1;
      if (todo) {
        row[q] = base + __builtin_ctzll(todo);
        todo &= todo - 1;
      }
    }
    unsigned long long word[BATCH][WORDS];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      if (row[q] < 0) continue;
      const unsigned long long* cslots = reinterpret_cast<const unsigned long long*>(C + row[q] * (int64_t)N);
      const unsigned long long* aslots = reinterpret_cast<const unsigned long long*>(arg + row[q] * (int64_t)N);
#pragma unroll
      for (int k = 0; k < WORDS; ++k) {
        const int j = lane + k * kWave;
        word[q][k] = j < N ? (j < half ? cslots[j] : aslots[j - half]) : 0ull;
      }
    }
    // every word of these rows has been read (by all lanes) before any lane overwrites a row:
    // a workgroup-scope fence waits for this wavefront's outstanding loads and keeps the
    // compiler from moving memory operations across it (no cache maintenance is needed, the
    // rows belong to this wavefront alone)
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "workgroup");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      if (row[q] < 0) continue;
      float* crow = C + row[q] * (int64_t)N;
      int32_t* arow = arg + row[q] * (int64_t)N;
#pragma unroll
      for (int k = 0; k < WORDS; ++k) {
        const int j = lane + k * kWave;
        if (j < N) {
          float value;
          int where;
          Rows::unpack(word[q][k], value, where);
          crow[j] = value;
          arow[j] = where;
        }
      }
    }
  }
}

// Position of the extreme (run after the max / min result C is complete): an entry whose
// product has exactly the bits of C[i, j] is a candidate; the smallest entry index wins,
// i.e. the first in storage order.  Rows inside one chunk are stored, split rows are
// combined with an integer atomic min on a row preset to INT_MAX.
template <int V, int T, class BT = float>
struct ArgRows {
  static constexpr bool kCanSkipWholeRows = true;
  struct State { int best[T][V]; int want[T][V]; };

  __device__ static void begin(State& s, const KernelArgs& a, int64_t row, int, const int (&colc)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t) {
      const Vec<V> c = Vec<V>::load(a.Cin + row * (int64_t)a.N + colc[t]);
#pragma unroll
      for (int x = 0; x < V; ++x) {
        s.want[t][x] = __float_as_int(c.v[x]);
        s.best[t][x] = INT32_MAX;
      }
    }
  }

  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int cs, int first, int stride, int left,
                              const int (&)[T], const int (&colc)[T]) {
    using Load = BLoad<V, BT>;
    int2 e2[U];
    int where[U];
    typename Load::Raw b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) {          // a missing entry repeats an existing one: same index, harmless
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      e2[u] = ka[first + uu * stride];
      where[u] = cs + first + uu * stride;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
      for (int t = 0; t < T; ++t) b[u][t] = Load::load(brow + colc[t]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < T; ++t) {
        float bx[V];
        Load::unpack(b[u][t], bx);
#pragma unroll
        for (int x = 0; x < V; ++x) {
          const float prod = __int_as_float(e2[u].y) * bx[x];
          if (__float_as_int(prod) == s.want[t][x] && where[u] < s.best[t][x]) s.best[t][x] = where[u];
        }
      }
  }

  template <int G>
  __device__ static void combine(State& s) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int x = 0; x < V; ++x) {
          const int other = __shfl_xor(s.best[t][x], off, kWave);
          s.best[t][x] = other < s.best[t][x] ? other : s.best[t][x];
        }
  }

  __device__ static void end(State& s, const KernelArgs& a, int64_t row, bool whole, int, const int (&col)[T]) {
    int32_t* arow = a.arg + row * (int64_t)a.N;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (col[t] < a.N) {
        if (whole) {
          Vec<V> out;
#pragma unroll
          for (int x = 0; x < V; ++x) out.v[x] = __int_as_float(s.best[t][x]);
          out.store(reinterpret_cast<float*>(arow + col[t]));
        } else {
#pragma unroll
          for (int x = 0; x < V; ++x)
            if (s.best[t][x] != INT32_MAX)
              __hip_atomic_fetch_min(arow + col[t] + x, s.best[t][x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
    }
  }
};

// Gradient of sum / mean with respect to B from the CSR of A itself: every stored entry
// (i, k) adds  w * dC[i, :]  into dB[k, :]  (w = val, or val / row length for mean) with
// fp32 atomic adds; dB was zero-filled before.  Here KernelArgs::B is dC and ::C is dB.
template <int V, int T>
struct TransposedRows {
  static constexpr bool kCanSkipWholeRows = false;
  struct State { Vec<V> d[T]; };

  __device__ static void begin(State& s, const KernelArgs& a, int64_t row, int row_len, const int (&colc)[T]) {
    const float w = a.is_mean ? 1.0f / (float)row_len : 1.0f;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      s.d[t] = Vec<V>::load(a.B + row * (int64_t)a.N + colc[t]);
#pragma unroll
      for (int x = 0; x < V; ++x) s.d[t].v[x] *= w;
    }
  }

  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int, int first, int stride, int left,
                              const int (&col)[T], const int (&)[T]) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (u < left) {                      // no padding here: every atomic must be a real entry
        const int2 e = ka[first + u * stride];
        float* out = a.C + (int64_t)e.x * a.N;
#pragma unroll
        for (int t = 0; t < T; ++t)
          if (col[t] < a.N) {
#pragma unroll
            for (int x = 0; x < V; ++x)
              __hip_atomic_fetch_add(out + col[t] + x, __int_as_float(e.y) * s.d[t].v[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          }
      }
    }
  }

  template <int G> __device__ static void combine(State&) {}
  __device__ static void end(State&, const KernelArgs&, int64_t, bool, int, const int (&)[T]) {}
};

// Building the CSR of the transposed matrix: every stored entry (i, k, val) takes the next
// free place of transposed row k (an atomic counter per row, preset to the row's start)
// and writes (i, val) there - val divided by the length of row i when the weights are
// wanted for the gradient of mean.  Runs as the <V=1, G=1, T=1> instance: 64 slots, one
// lane per entry.  KernelArgs::C is the value array and ::arg the index array written.
template <int V, int T>
struct ScatterRows {
  static constexpr bool kCanSkipWholeRows = false;
  struct State { float len; int row; };

  __device__ static void begin(State& s, const KernelArgs&, int64_t row, int row_len, const int (&)[T]) {
    s.len = (float)row_len;
    s.row = (int)row;
  }

  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int cs, int first, int stride, int left,
                              const int (&col)[T], const int (&)[T]) {
    int2 e[U];
    int place[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {          // all counters first: the returns come back together
      const bool live = u < left && col[0] == 0;
      e[u] = ka[first + (live ? u * stride : 0)];
      place[u] = -1;
      if (live) {                            // no cursors: the entry stays where it is (row ids and weights in entry order)
        if (a.cursor) place[u] = __hip_atomic_fetch_add(a.cursor + e[u].x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        else place[u] = cs + first + u * stride;
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (place[u] >= 0) {
        a.arg[place[u]] = s.row;
        a.C[place[u]] = a.is_mean ? __int_as_float(e[u].y) / s.len : __int_as_float(e[u].y);
      }
    }
  }

  template <int G> __device__ static void combine(State&) {}
  __device__ static void end(State&, const KernelArgs&, int64_t, bool, int, const int (&)[T]) {}
};

// A user-defined SpMM-like operation (paper, Section IV-A: the user supplies an initial
// value and a reduce function, both inlined at compile time).  R provides
//   static __host__ __device__ float identity();            initial accumulator
//   static __device__ float step(float acc, float a, float b);   fold in one stored entry
//                                                           (a = stored value, b = B element)
//   static __device__ float merge(float x, float y);        combine two partial accumulators
// merge must be associative and commutative and step(acc, a, b) == merge(acc, step(identity(), a, b)).
// Split rows are combined in memory with a compare-and-swap loop around merge.
template <class R, int V, int T>
struct CustomRows {
  static constexpr bool kCanSkipWholeRows = false;
  struct State { Vec<V> acc[T]; };

  __device__ static void begin(State& s, const KernelArgs&, int64_t, int, const int (&)[T]) {
#pragma unroll
    for (int t = 0; t < T; ++t)
#pragma unroll
      for (int x = 0; x < V; ++x) s.acc[t].v[x] = R::identity();
  }

  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int, int first, int stride, int left,
                              const int (&)[T], const int (&colc)[T]) {
    int2 e2[U];
    Vec<V> b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      e2[u] = ka[first + uu * stride];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float* brow = a.B + (int64_t)e2[u].x * a.N;
#pragma unroll
      for (int t = 0; t < T; ++t) b[u][t] = Vec<V>::load(brow + colc[t]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int x = 0; x < V; ++x) {   // a padded step (u >= left) must leave the accumulator alone
          const float next = R::step(s.acc[t].v[x], __int_as_float(e2[u].y), b[u][t].v[x]);
          s.acc[t].v[x] = u < left ? next : s.acc[t].v[x];
        }
  }

  template <int G>
  __device__ static void combine(State& s) {
#pragma unroll
    for (int off = G; off < kWave; off <<= 1)
#pragma unroll
      for (int t = 0; t < T; ++t)
#pragma unroll
        for (int x = 0; x < V; ++x) s.acc[t].v[x] = R::merge(s.acc[t].v[x], __shfl_xor(s.acc[t].v[x], off, kWave));
  }

  __device__ static void end(State& s, const KernelArgs& a, int64_t row, bool whole, int, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (col[t] < a.N) {
        if (whole) {
          s.acc[t].store(crow + col[t]);
        } else {
#pragma unroll
          for (int x = 0; x < V; ++x) {
            unsigned* cell = reinterpret_cast<unsigned*>(crow + col[t] + x);
            unsigned seen = __hip_atomic_load(cell, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            for (;;) {
              const unsigned want = __float_as_uint(R::merge(__uint_as_float(seen), s.acc[t].v[x]));
              if (__hip_atomic_compare_exchange_strong(cell, &seen, want, __ATOMIC_RELAXED, __ATOMIC_RELAXED,
                                                       __HIP_MEMORY_SCOPE_AGENT))
                break;                   // on failure `seen` holds the value found: merge again
            }
          }
        }
      }
    }
  }
};

// The value+position fold carries twice the state per column; with half as many gathers in flight it
// fits 76 registers (6 waves per SIMD instead of 4) and is 3-9 % faster.
template <class P> struct FlightDivisor { static constexpr int value = 1; };
template <int F, int V, int T, class BT> struct FlightDivisor<FoldArgRows<F, V, T, BT>> { static constexpr int value = 2; };

// P: row policy; V: floats per lane per load; G: lanes per slot; T: column tiles per lane.
template <class P, int V, int G, int T>
__global__ void __launch_bounds__(kBlock) chunk_kernel(const KernelArgs a) {
  constexpr int NS = kWave / G;                 // slots
  constexpr int kFlight = loads_in_flight(G) / FlightDivisor<P>::value;
  constexpr int U = kFlight / T > 0 ? kFlight / T : 1;   // entries per lane per pass
  extern __shared__ int2 s_dyn[];               // per wavefront: S entries (colind, val) + 64 row descriptors

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int slot = lane / G;
  const int g = lane % G;
  const int S = 1 << a.chunk_shift;

  const int64_t chunk = logical_block(blockIdx.x, a.chunk_blocks, a.xcd_remap) * kWavesPerBlock + wave;
  if (chunk >= a.chunks) return;                // whole wavefront leaves; no block barrier is used
  const int cs = (int)(chunk << a.chunk_shift); // first stored entry of this chunk (< 2^31)
  const int cnt = (a.nnz - cs) < S ? (a.nnz - cs) : S;
  const int ce = cs + cnt;
  int2* ka = s_dyn + wave * (S + kWave);
  int2* short_rows = ka + S;

  // (1) coalesced load of the chunk's (colind, val) into this wavefront's LDS slice, in groups
  //     of four loads per array (indices past the end repeat the last entry; those copies
  //     are never consumed).  The first group is issued before the row search below and
  //     written to LDS after it, so its latency overlaps the search's.
  auto load_group = [&](int u0, int (&k)[4], float (&v)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = u0 + u * kWave + lane;
      k[u] = a.colind[cs + (idx < cnt ? idx : cnt - 1)];
    }
    if (a.vals) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int idx = u0 + u * kWave + lane;
        v[u] = a.vals[cs + (idx < cnt ? idx : cnt - 1)];
      }
    } else {
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u] = 1.0f;
    }
  };
  auto store_group = [&](int u0, const int (&k)[4], const float (&v)[4]) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int idx = u0 + u * kWave + lane;
      if (idx < S) ka[idx] = make_int2(k[u], __float_as_int(v[u]));
    }
  };
  int k0[4];
  float v0[4];
  load_group(0, k0, v0);

  // (2) first row of the chunk: the last r with rowptr[r] <= cs, found by a 64-way search
  int lo = 0, hi = a.M;                          // rowptr[lo] <= cs < rowptr[hi]
  while (hi - lo > 1) {
    const int64_t step = ((int64_t)(hi - lo) + kWave - 1) / kWave;
    int64_t probe = lo + (int64_t)(lane + 1) * step;
    if (probe > hi) probe = hi;
    const int below = __builtin_popcountll(__ballot(a.rowptr[probe] <= cs));   // probes are monotone
    const int64_t nlo = lo + below * step;       // below <= 63 because rowptr[hi] > cs
    int64_t nhi = nlo + step;
    if (nhi > hi) nhi = hi;
    lo = (int)nlo;
    hi = (int)nhi;
  }

  store_group(0, k0, v0);
  for (int u0 = 4 * kWave; u0 < cnt; u0 += 4 * kWave) {
    int k[4];
    float v[4];
    load_group(u0, k, v);
    store_group(u0, k, v);
  }

  // column tiles of this lane (loads use a clamped column so they are never masked)
  const int colbase = blockIdx.y * (V * G * T);
  int col[T];
  int colc[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    col[t] = colbase + (t * G + g) * V;
    colc[t] = col[t] < a.N ? col[t] : a.N - V;
  }

  wave_lds_fence();

  // (3) walk the rows that have entries in [cs, ce), 64 row bounds at a time (lane <-> row)
  for (int64_t rbase = lo;; rbase += kWave) {
    int64_t rr = rbase + lane;
    if (rr > a.M) rr = a.M;
    const int my_s = a.rowptr[rr];
    const int my_e = a.rowptr[rr < a.M ? rr + 1 : a.M];
    const bool my_whole = my_s >= cs && my_e <= ce;
    const bool valid = rbase + lane < a.M && my_e > my_s && my_s < ce &&
                       !(P::kCanSkipWholeRows && a.only_split && my_whole);
    const int my_ps = (my_s > cs ? my_s : cs) - cs;     // the row's segment inside the chunk,
    const int my_pe = (my_e < ce ? my_e : ce) - cs;     // as offsets into the LDS slice
    const bool is_short = NS > 1 && valid && (my_pe - my_ps) <= a.short_len;

    // (3a) short segments: one per slot, 64/G rows at a time, no cross-lane exchange
    if (NS > 1) {
      const unsigned long long smask = __ballot(is_short);
      const int nshort = __builtin_popcountll(smask);
      if (nshort > 0) {
        const int rank = __builtin_amdgcn_mbcnt_hi((unsigned)(smask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)smask, 0u));
        if (is_short)   // lane | offset << 6 | length << 18 | whole << 30 ; full row length
          short_rows[rank] = make_int2(lane | (my_ps << 6) | ((my_pe - my_ps) << 18) | ((int)my_whole << 30), my_e - my_s);
        wave_lds_fence();
        for (int t0 = 0; t0 < nshort; t0 += NS) {
          const bool have = t0 + slot < nshort;
          const int2 d = short_rows[have ? t0 + slot : nshort - 1];   // an idle slot shadows the last row
          const int r_ps = (d.x >> 6) & 4095;
          const int r_len = have ? (d.x >> 18) & 4095 : 0;
          const int64_t row = rbase + (d.x & 63);
          typename P::State st;
          P::begin(st, a, row, d.y, colc);
          // U entries per step; a last step with at most U / 2 entries left in every slot takes
          // the half-size pass (fewer padded gathers: up to 7 % on matrices of short rows)
          for (int it = 0; __ballot(it < r_len) != 0ull;) {
            if (U >= 4 && __ballot(r_len - it > U / 2) == 0ull) {
              P::template pass<(U >= 4 ? U / 2 : U)>(st, a, ka, cs, r_ps + (it < r_len ? it : 0), 1, r_len - it, col, colc);
              it += U / 2;
            } else {
              P::template pass<U>(st, a, ka, cs, r_ps + (it < r_len ? it : 0), 1, r_len - it, col, colc);
              it += U;
            }
          }
          if (have) P::end(st, a, row, (d.x >> 30) & 1, d.y, col);
        }
        wave_lds_fence();
      }
    }

    // (3b) long segments: all slots work on one row, slot s takes entries s, s+NS, ...
    unsigned long long todo = __ballot(valid && !is_short);
    while (todo) {
      const int i = __builtin_ctzll(todo);
      todo &= todo - 1;
      const int ps = __builtin_amdgcn_readlane(my_ps, i);
      const int pe = __builtin_amdgcn_readlane(my_pe, i);
      const int s = __builtin_amdgcn_readlane(my_s, i);
      const int e = __builtin_amdgcn_readlane(my_e, i);
      typename P::State st;
      P::begin(st, a, rbase + i, e - s, colc);
      for (int base = ps; base < pe; base += U * NS) {
        const int first = base + slot;
        const int left = (pe - first + NS - 1) / NS;       // entries first, first+NS, ... below pe
        P::template pass<U>(st, a, ka, cs, left > 0 ? first : pe - 1, NS, left, col, colc);
      }
      P::template combine<G>(st);
      if (slot == 0) P::end(st, a, rbase + i, s >= cs && e <= ce, e - s, col);
    }
    // the next batch of rows is needed only if it still starts inside the chunk
    const int next_start = __builtin_amdgcn_readlane(my_e, kWave - 1);
    if (rbase + kWave >= a.M || next_start >= ce) break;
  }
}

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

// --------------------------------------------------------------- host side --
using MainKernel = void (*)(const KernelArgs);

enum Job { kJobAdd = kAdd, kJobMax = kMax, kJobMin = kMin, kJobArg = 3, kJobTransposed = 4, kJobScatter = 5,
           kJobMaxWithArg = 6, kJobMinWithArg = 7 };

template <template <int, int> class P, int V>
MainKernel pick_gt(int G, int T) {
#define GESPMM_CASE(GG, TT) if (G == GG && T == TT) return chunk_kernel<P<V, TT>, V, GG, TT>;
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
    case kJobScatter: return (V == 1 && G == 1 && T == 1) ? chunk_kernel<ScatterRows<1, 1>, 1, 1, 1> : nullptr;
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
#define GESPMM_CASE(VV, GG) if (vec == VV && G == GG) return chunk_kernel<FoldRows<F, VV, 1, BT>, VV, GG, 1>;
  GESPMM_CASE(4, 1) GESPMM_CASE(4, 2) GESPMM_CASE(4, 4) GESPMM_CASE(4, 8) GESPMM_CASE(4, 16) GESPMM_CASE(4, 32)
  GESPMM_CASE(1, 1) GESPMM_CASE(1, 2) GESPMM_CASE(1, 4) GESPMM_CASE(1, 8) GESPMM_CASE(1, 16) GESPMM_CASE(1, 32) GESPMM_CASE(1, 64)
#undef GESPMM_CASE
  return nullptr;
}

template <class P4, class P1>
MainKernel pick_b16_shapes(int vec, int G, int T) {      // P4 / P1: the policy for 4 columns / 1 column per lane
  if (T != 1) return nullptr;
#define GESPMM_CASE4(GG) if (vec == 4 && G == GG) return chunk_kernel<P4, 4, GG, 1>;
#define GESPMM_CASE1(GG) if (vec == 1 && G == GG) return chunk_kernel<P1, 1, GG, 1>;
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

inline bool has_kernel(int G, int T) { return pick_gt<AddRows, 4>(G, T) != nullptr; }

inline int next_pow2(int64_t x) {
  int p = 1;
  while (p < x && p < 64) p <<= 1;
  return p;
}

// process-wide tuning overrides (-1 = automatic)
inline int g_force_g = -1, g_force_t = -1, g_force_remap = -1, g_force_shift = -1, g_force_short = -1;

// A problem that yields fewer wavefronts than this (8 per compute unit) gets smaller chunks,
// so that its rows are spread over more of the chip.  Measured on matrices of 10^4 .. 10^6
// entries: below this count halving the chunk pays; above it the extra split rows (finished
// by atomics) and the extra row searches cost more than the added parallelism brings.
constexpr int64_t kMinWaves = 2048;

// elem_bytes: size of one element of the dense input (4, or 2 for the 16-bit formats); a lane
// loads four columns at once when the width and the alignment allow it, one otherwise.
inline void make_plan(int64_t M, int64_t N, int64_t nnz, bool aligned16, gespmm_plan_t* p, int elem_bytes = 4) {
  int vec = 1;
  if (aligned16 && N > 0) {
    if (elem_bytes == 4) vec = N % 4 == 0 ? 4 : 1;
    else vec = N % 4 == 0 ? 4 : 1;              // 16-bit elements: 8-byte loads
  }
  const int64_t ncv = N > 0 ? (N + vec - 1) / vec : 1;     // vector columns to cover
  // Column blocks of one 128-byte line (8 lanes x 16 bytes) up to N = 128, of two lines
  // beyond; wider N is covered by grid.y.  The blocks of one grid.y index run together in
  // time, so the part of B that is live at any moment is K x 128 (or 256) bytes, which the
  // L2s keep far better than whole rows of B; the sparse arrays are re-read per block,
  // which costs 8 bytes per entry against 128 gathered.
  int G = next_pow2(ncv), T = 1;
  if (vec > 1) {
    const int line = 128 / (vec * elem_bytes);  // lanes that cover one 128-byte line of a row of B
    if (G > line) G = ncv <= 4 * line ? line : 2 * line;   // one line; two lines for wide N
  } else if (elem_bytes == 2) {
    if (G > 64) G = 64;                         // one column per lane, one tile: up to 64 columns per block
  } else if (G > 16) {
    G /= 2;
    T = 2;
    if (ncv > 64 && G * T < 128) { G = 64; T = 2; }
  }
  if (g_force_g > 0) G = g_force_g;
  if (g_force_t > 0) T = g_force_t;
  // chunk size: 256 stored entries; 512 for column blocks of up to 64 bytes (less data
  // per entry) and for matrices with long rows (fewer split rows); halved while the
  // problem has too few chunks to fill the chip
  const int64_t col_blocks = (ncv + (int64_t)G * T - 1) / ((int64_t)G * T);
  int shift = ((int64_t)vec * G * T * elem_bytes <= 64 || (M > 0 && nnz / M >= 128)) ? 9 : 8;
  while (shift > 6 && ((nnz + (1ll << shift) - 1) >> shift) * col_blocks < kMinWaves) --shift;
  if (g_force_shift >= kMinChunkShift) shift = g_force_shift;
  p->vec = vec;
  p->lanes_per_row = G;
  p->tiles_per_lane = T;
  p->slots = kWave / G;
  p->chunk_nnz = 1 << shift;
  p->col_blocks = (int32_t)col_blocks;
  p->chunks = (nnz + p->chunk_nnz - 1) >> shift;
  p->grid_x = (p->chunks + kWavesPerBlock - 1) / kWavesPerBlock;
  p->block_threads = kBlock;
  // rows much longer than a chunk are finished by atomics from many consecutive chunks:
  // keep those chunks on one XCD (one L2); otherwise deal the chunks round-robin
  const bool long_rows = M > 0 && nnz / M >= p->chunk_nnz / 2;
  p->xcd_remap = g_force_remap >= 0 ? g_force_remap : (long_rows ? 1 : 0);
  // Rows up to short_len entries are walked one per slot, longer ones by all slots together
  // (with a cross-slot combine per row).  Where the mean row has 17 .. 48 entries, as in
  // stencil and finite-element matrices whose rows all have about that length, one slot per
  // row up to 32 entries avoids that combine for most rows (measured: up to 22 % on a
  // 27-point stencil, within 3 % either way on power-law graphs of the same mean).
  const int64_t mean_row = M > 0 ? nnz / M : 0;
  int auto_short = 2 * p->slots < 16 ? 2 * p->slots : 16;
  if (mean_row > 16 && mean_row <= 48) auto_short = 32;
  p->short_len = g_force_short >= 0 ? g_force_short : auto_short;
  p->lds_bytes = (int32_t)(kWavesPerBlock * (p->chunk_nnz + kWave) * sizeof(int2));
}

// profiling state
inline std::vector<hipEvent_t> g_ev_start, g_ev_stop;
inline int g_ev_used = 0;
inline bool g_profiling = false;

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

// One pass of the chunk kernel over the matrix, preceded (when init_target is set) by the
// row-initialisation kernel for that output.
struct ChunkLaunch {
  int job = kJobAdd;
  int64_t M = 0, N = 0, nnz = 0;
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
  bool timed = false;                  // bracket the chunk kernel with profiling events
  MainKernel (*picker)(int vec, int G, int T) = nullptr;   // user-defined reduce: its own kernel table
  int32_t* cursor = nullptr;           // structure-transpose job only
  bool one_lane_per_entry = false;     // use the <V=1, G=1, T=1> instance whatever N is
  int b_dtype = GESPMM_F32;            // element type of dense_in (16-bit types: fold jobs only)
};

inline int launch_chunks(const ChunkLaunch& L, hipStream_t stream) {
  const bool aligned16 = (((uintptr_t)L.dense_in | (uintptr_t)L.dense_out | (uintptr_t)L.result_in |
                           (uintptr_t)L.also_aligned) & 15u) == 0;
  gespmm_plan_t plan;
  make_plan(L.M, L.N, L.nnz, aligned16, &plan, L.b_dtype == GESPMM_F32 ? 4 : 2);
  if (L.one_lane_per_entry) {
    plan.vec = 1;
    plan.lanes_per_row = 1;
    plan.tiles_per_lane = 1;
    plan.slots = kWave;
    plan.col_blocks = 1;
    plan.short_len = 16;
  }
  MainKernel kernel = nullptr;
  if (L.picker) kernel = L.picker(plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_BF16) kernel = pick_b16<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_F16) kernel = pick_b16<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else kernel = pick_kernel(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  if (!kernel) return GESPMM_ERR_BAD_ARG;
  if (plan.col_blocks > 65535) return GESPMM_ERR_TOO_LARGE;   // grid.y limit (N beyond ~33 million)
  int shift = 0;
  while ((1 << shift) < plan.chunk_nnz) ++shift;

  // (a) empty rows and rows shared by several chunks are preset
  if (L.init_target) {
    int lanes_shift = 0;                          // lanes that write one row in init_rows
    while ((1 << lanes_shift) < kWave && ((int64_t)plan.vec << lanes_shift) < L.N) ++lanes_shift;
    const unsigned init_blocks = (unsigned)((L.M + kBlock - 1) / kBlock);
    if (plan.vec == 4)
      hipLaunchKernelGGL(init_rows<4>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, L.rowptr,
                         L.init_target, L.empty_value, L.split_value, shift, lanes_shift);
    else
      hipLaunchKernelGGL(init_rows<1>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, L.rowptr,
                         L.init_target, L.empty_value, L.split_value, shift, lanes_shift);
    if (L.init2_target) {
      if (plan.vec == 4)
        hipLaunchKernelGGL(init_rows<4>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, L.rowptr,
                           L.init2_target, L.empty2_value, L.split2_value, shift, lanes_shift);
      else
        hipLaunchKernelGGL(init_rows<1>, dim3(init_blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, L.rowptr,
                           L.init2_target, L.empty2_value, L.split2_value, shift, lanes_shift);
    }
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  }
  if (L.nnz == 0) return GESPMM_OK;

  // (b) the chunks
  KernelArgs a;
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
  a.colind = L.colind;
  a.vals = L.vals;
  a.B = L.dense_in;
  a.C = L.dense_out;
  a.Cin = L.result_in;
  a.arg = L.arg;
  a.cursor = L.cursor;
  a.only_split = L.only_split ? 1 : 0;
  a.packed_split = L.packed_split ? 1 : 0;
  if (L.packed_split && (plan.vec != 4 || L.N > kWave * kFinishWords || !L.arg)) return GESPMM_ERR_BAD_ARG;
  const bool timed = L.timed && g_profiling && g_ev_used < (int)g_ev_start.size();
  if (timed && hipEventRecord(g_ev_start[g_ev_used], stream) != hipSuccess) return GESPMM_ERR_HIP;
  hipLaunchKernelGGL(kernel, dim3((unsigned)plan.grid_x, (unsigned)plan.col_blocks), dim3(kBlock), (size_t)plan.lds_bytes, stream, a);
  if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  if (timed) {
    if (hipEventRecord(g_ev_stop[g_ev_used], stream) != hipSuccess) return GESPMM_ERR_HIP;
    ++g_ev_used;
  }
  if (L.packed_split) {
    const unsigned blocks = (unsigned)((L.M + kBlock - 1) / kBlock);
    int words = 1;
    while (words * kWave < L.N) words *= 2;
    const bool is_max = L.job == kJobMaxWithArg;
#define GESPMM_FINISH(WW)                                                                                             \
  if (words == WW) {                                                                                                  \
    if (is_max)                                                                                                       \
      hipLaunchKernelGGL((finish_split_rows<kMax, WW>), dim3(blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, \
                         L.rowptr, L.dense_out, L.arg, shift);                                                        \
    else                                                                                                              \
      hipLaunchKernelGGL((finish_split_rows<kMin, WW>), dim3(blocks), dim3(kBlock), 0, stream, (int32_t)L.M, (int32_t)L.N, \
                         L.rowptr, L.dense_out, L.arg, shift);                                                        \
  }
    GESPMM_FINISH(1) GESPMM_FINISH(2) GESPMM_FINISH(4) GESPMM_FINISH(8) GESPMM_FINISH(16)
#undef GESPMM_FINISH
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  }
  return GESPMM_OK;
}

template <class R>
struct CustomBind {
  template <int V, int T> using Rows = CustomRows<R, V, T>;
};

template <class R>
MainKernel pick_custom(int vec, int G, int T) {
  return vec == 4 ? pick_gt<CustomBind<R>::template Rows, 4>(G, T) : pick_gt<CustomBind<R>::template Rows, 1>(G, T);
}

}  // namespace gespmm_detail

namespace gespmm {

// C = A (x) B with the user-defined reduce R (see CustomRows for what R must provide).
// Same arguments, layout, ownership and errors as gespmm_csr; an empty row yields 0.
template <class R>
int csr_custom(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
               const float* vals, const float* B, float* C, hipStream_t stream) {
  using namespace gespmm_detail;
  const int st = validate(M, K, N, nnz, rowptr, colind, B, C, GESPMM_SUM);
  if (st != GESPMM_OK || M == 0 || N == 0) return st;
  ChunkLaunch L;
  L.picker = &pick_custom<R>;
  L.M = M; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = B; L.dense_out = C;
  L.init_target = C; L.empty_value = 0.0f; L.split_value = R::identity();
  return launch_chunks(L, stream);
}

}  // namespace gespmm
