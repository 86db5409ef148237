// CSR SpMM / SpMM-like kernels for gfx950 (MI355X): device code and launch helpers.
// (The C ABI over them is in paper_2007_03179_amd/csrc/gespmm.hip; user-defined reduce
// operations include this file through gespmm_custom.hpp, which is why it lives beside
// the public headers.)
//
// Result computed (paper: Algorithm 1, Section III-A; general reduce: Eq. 1, Section IV-A):
//     C[i, j] = reduce_p  vals[p] * B[colind[p], j],   p over the stored entries of row i.
//
// How the work is laid out (what is kept from the paper and what is not):
//  * The paper gives one thread block to each sparse row (Algorithms 2 and 3).  Here the
//    unit of work is a CHUNK of S consecutive ITEMS, one per 64-lane wavefront, where the
//    items are the stored entries and the row ends merged into one sequence: row r
//    contributes its entries and then one row-end item, so entry p of row r is item p + r.
//    A wavefront therefore never has more than S entries to gather NOR more than S rows to
//    walk, whatever the row lengths are (a stretch of thousands of empty or one-entry rows
//    is spread over many wavefronts instead of trailing behind one).
//    A row whose entries fall into more than one chunk is finished with atomics (add, or
//    integer max/min on the ordered bit pattern of the float); rows inside one chunk are
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
constexpr int kMaxParts = 64;                     // most parts the K-phased path cuts the column range into
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
  const int32_t* rowptr;  // row starts; in a phase of the K-phased path: the phase's virtual row starts
  const int32_t* delta;   // K-phased path: stored position = virtual position + delta[row]; otherwise nullptr
  const int32_t* colind;
  const float* vals;
  const float* B;         // dense input (the gradient dC for the transposed job)
  float* C;               // dense output (dB for the transposed job)
  const float* Cin;       // finished max/min result, read by the position job
  int32_t* arg;           // output of the position job; row indices of the transposed arrays
  int32_t* cursor;        // next free place of every transposed row (structure-transpose job)
  int32_t only_split;     // position job: rows inside one chunk were already done by the fused pass
  int32_t packed_split;   // fused value+position pass: split rows collect (value, position) pairs in 64-bit slots
  int32_t accumulate;     // K-phased path: fold the row's result into what C already holds
  int32_t taper_chunks;   // K-phased path: this many chunks at the end of a launch hold S / 4 items only
  int32_t row_window;     // whole-row path: entries one wavefront's LDS slice holds (>= S)
};

// Entry p of row r is item p + r of the merged sequence of entries and row ends; chunk c owns the
// items [c * S, (c + 1) * S).  A non-empty row [s, e) is shared by several chunks exactly when its
// first and its last entry are owned by different chunks.
__device__ __forceinline__ bool row_is_shared(int s, int e, int64_t r, int chunk_shift) {
  return (((int64_t)s + r) >> chunk_shift) != (((int64_t)e - 1 + r) >> chunk_shift);
}

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

// Zeros: what the sum's gathers read for entries that do not exist.
__device__ float4 kZeroLine[4] = {};      // never written (not const: a const array would live in another address space than B)

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
// chunk_shift < 0: every non-empty row gets `split_value` (the K-phased path, whose phases
// all fold into what C holds).
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
    else if (chunk_shift < 0 || row_is_shared(s, e, r, chunk_shift)) flag = 2;
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

  // All gathers of a pass are issued before the first use, in straight-line code.  An entry that
  // does not exist: max / min re-read the last one that does (idempotent, whatever the values
  // are); the sum reads a line of zeros instead of B and gives it weight 0, so that a non-finite
  // element of B reaches exactly the rows that store an entry for it, as in Algorithm 1.
  template <int U>
  __device__ static void pass(State& s, const KernelArgs& a, const int2* ka, int, int first, int stride, int left,
                              const int (&)[T], const int (&colc)[T]) {
    using Load = BLoad<V, BT>;
    int2 e2[U];
    typename Load::Raw b[U][T];
    const BT* nothing = reinterpret_cast<const BT*>(kZeroLine);      // the same 16 bytes for every lane: a uniform address
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
      for (int t = 0; t < T; ++t) b[u][t] = Load::load(F == kAdd && u >= left ? nothing : brow + colc[t]);
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

  // A row without stored entries yields 0 (whole-row path, where no other kernel presets it).
  __device__ static void store_empty(const KernelArgs& a, int64_t row, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    Vec<V> zero;
#pragma unroll
    for (int x = 0; x < V; ++x) zero.v[x] = 0.0f;
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (col[t] < a.N) zero.store(crow + col[t]);
  }

  // Plain store when the whole row lay in this chunk, atomics otherwise (the row was
  // preset to the identity by init_rows).  In a phase of the K-phased path the row's part
  // of this phase is folded into what the earlier phases left in C: by this wavefront
  // alone when the part lay in one chunk (nobody else touches the row during the launch).
  __device__ static void end(State& s, const KernelArgs& a, int64_t row, bool whole, int row_len, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    const float len = (float)row_len;
#pragma unroll
    for (int t = 0; t < T; ++t) {
      if (col[t] < a.N) {
        if (whole) {
          if (a.accumulate) {
            const Vec<V> before = Vec<V>::load(crow + col[t]);
#pragma unroll
            for (int x = 0; x < V; ++x) s.acc[t].v[x] = fold2<F>(before.v[x], s.acc[t].v[x]);
          } else if (a.is_mean) {
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

  // A row without stored entries: value 0, position -1 (whole-row path).
  __device__ static void store_empty(const KernelArgs& a, int64_t row, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    int32_t* arow = a.arg + row * (int64_t)a.N;
    Vec<V> value, place;
#pragma unroll
    for (int x = 0; x < V; ++x) {
      value.v[x] = 0.0f;
      place.v[x] = __int_as_float(-1);
    }
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (col[t] < a.N) {
        value.store(crow + col[t]);
        place.store(reinterpret_cast<float*>(arow + col[t]));
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
    split = e > s && row_is_shared(s, e, r, chunk_shift);
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
// kPhased: the kernel runs one phase of the K-phased path (see launch_phased): `rowptr` holds the
// phase's virtual row starts (consecutive numbers for the entries the phase owns, row after row),
// `delta[r]` turns a virtual position of row r into the stored position, the number of chunks is
// read from the device, a wavefront takes chunks c, c + (wavefronts launched), ... and the result
// of a row is folded into C.
// kOwned: the whole-row path.  A row belongs to the chunk that owns its FIRST item (its first entry, or
// its end when it stores nothing) and that chunk's wavefront walks all of it, also the part that lies
// beyond the chunk's own items: every row is written exactly once, by plain stores, empty rows
// included, so nothing has to be preset and nothing is combined by atomics: one launch per call.
// The LDS slice holds `row_window` >= S entries; with the longest row L of the matrix, S + L entries
// cover everything a chunk can own.  A row that still reaches beyond the slice is necessarily the
// last one the chunk owns and is walked in windows, each staged over the slice: correct for any
// matrix, fast when rows are short against S.
template <class P, int V, int G, int T, bool kPhased, bool kOwned = false>
__global__ void __launch_bounds__(kBlock) chunk_kernel(const KernelArgs a) {
  static_assert(!(kPhased && kOwned), "a phase folds into C; the whole-row path writes every row once");
  constexpr int NS = kWave / G;                 // slots
  constexpr int kFlight = loads_in_flight(G) / FlightDivisor<P>::value;
  constexpr int U = kFlight / T > 0 ? kFlight / T : 1;   // entries per lane per pass
  extern __shared__ int2 s_dyn[];               // per wavefront: S entries (colind, val) + 64 row descriptors (+ 64 row records)

  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  const int slot = lane / G;
  const int g = lane % G;
  const int S = 1 << a.chunk_shift;
  const int slice = kOwned ? a.row_window : S;  // entries the LDS slice of this wavefront holds
  int2* ka = s_dyn + wave * (slice + (kPhased ? 2 : 1) * kWave);
  int2* short_rows = ka + slice;
  int2* row_info = short_rows + kWave;          // kPhased only: (row start relative to the chunk's first entry, delta)

  // column tiles of this lane (loads use a clamped column so they are never masked)
  const int colbase = blockIdx.y * (V * G * T);
  int col[T];
  int colc[T];
#pragma unroll
  for (int t = 0; t < T; ++t) {
    col[t] = colbase + (t * G + g) * V;
    colc[t] = col[t] < a.N ? col[t] : a.N - V;
  }

  // Items are numbered from `first_item`; a phase's entries carry the numbers rowptr[0] .. rowptr[M].
  const int64_t first_item = kPhased ? (int64_t)a.rowptr[0] : 0;
  const int64_t end_entry = kPhased ? (int64_t)a.rowptr[a.M] : (int64_t)a.nnz;
  const int64_t end_item = end_entry + a.M;
  // A phase ends with chunks of S / 4 items (at most a quarter of its items): the wavefronts that are
  // dispatched last finish four times sooner, which shortens the time the launch spends draining.
  const int small_shift = a.chunk_shift - 2;
  int64_t small_items = kPhased ? (int64_t)a.taper_chunks << small_shift : 0;
  if (small_items > (end_item - first_item) >> 2) small_items = (end_item - first_item) >> 2;
  const int64_t big_chunks = kPhased ? (end_item - first_item - small_items) >> a.chunk_shift : 0;   // chunks of S items
  const int64_t first_small_item = first_item + (big_chunks << a.chunk_shift);
  const int64_t nchunks = kPhased ? big_chunks + ((end_item - first_small_item + (S >> 2) - 1) >> small_shift) : a.chunks;
  const int64_t wave_stride = a.chunk_blocks * kWavesPerBlock;

  for (int64_t chunk = logical_block(blockIdx.x, a.chunk_blocks, a.xcd_remap) * kWavesPerBlock + wave; chunk < nchunks;
       chunk += wave_stride) {
    const bool small = kPhased && chunk >= big_chunks;
    const int64_t d0 = small ? first_small_item + ((chunk - big_chunks) << small_shift)
                             : first_item + (chunk << a.chunk_shift);    // items [d0, d1) are this chunk's
    const int64_t span = small ? S >> 2 : S;
    const int64_t d1 = d0 + span < end_item ? d0 + span : end_item;

    // (1) first row of the chunk: the last r with rowptr[r] + r <= d0 (that function of r is strictly
    //     increasing), found by a 64-way search
    int lo = 0, hi = a.M;                          // rowptr[lo] + lo <= d0 < rowptr[hi] + hi
    while (hi - lo > 1) {
      const int64_t step = ((int64_t)(hi - lo) + kWave - 1) / kWave;
      int64_t probe = lo + (int64_t)(lane + 1) * step;
      if (probe > hi) probe = hi;
      const int below = __builtin_popcountll(__ballot((int64_t)a.rowptr[probe] + probe <= d0));   // probes are monotone
      const int64_t nlo = lo + below * step;       // below <= 63 because the item of row `hi` lies beyond d0
      int64_t nhi = nlo + step;
      if (nhi > hi) nhi = hi;
      lo = (int)nlo;
      hi = (int)nhi;
    }
    const int64_t r0 = lo;
    const int cs = (int)(d0 - r0);                 // first entry the chunk can own (rowptr[r0] <= cs <= rowptr[r0 + 1])
    const int cnt = (int)(end_entry - cs < slice ? end_entry - cs : slice);   // entries [cs, cs + cnt) cover everything it owns
    if (!kOwned && cnt <= 0) {                     // only the ends of trailing empty rows: nothing to compute
      if (!kPhased) break;
      continue;
    }

    // row bounds, 64 rows at a time (lane <-> row); the next batch is requested before the current one is worked on
    auto load_bounds = [&](int64_t rbase, int& s, int& e, int& dl) {
      int64_t rr = rbase + lane;
      if (rr > a.M) rr = a.M;
      s = a.rowptr[rr];
      e = a.rowptr[rr < a.M ? rr + 1 : a.M];
      if (kPhased) dl = a.delta[rr < a.M ? rr : a.M - 1];
    };
    int next_s, next_e, next_delta = 0;
    load_bounds(r0, next_s, next_e, next_delta);

    // (2) plain path: coalesced load of the entries [cs, cs + cnt) into this wavefront's LDS slice.
    //     The K-phased path stages its entries batch by batch below.
    auto stage = [&](int from, int count) {        // entries [from, from + count) -> ka[0 .. count), count <= slice
      // up to eight loads per array are issued before the first is waited for (a whole chunk of 512 in one
      // round trip); a group of 64 that lies wholly beyond `count` is skipped (the test is wave-uniform)
      for (int u0 = 0; u0 < count; u0 += 8 * kWave) {
        int k[8];
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int idx = u0 + u * kWave + lane;
          k[u] = 0;
          if (u0 + u * kWave < count) k[u] = a.colind[from + (idx < count ? idx : count - 1)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int idx = u0 + u * kWave + lane;
          v[u] = 1.0f;
          if (a.vals && u0 + u * kWave < count) v[u] = a.vals[from + (idx < count ? idx : count - 1)];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int idx = u0 + u * kWave + lane;
          if (idx < count) ka[idx] = make_int2(k[u], __float_as_int(v[u]));
        }
      }
      wave_lds_fence();
    };
    if (!kPhased) stage(cs, cnt);

    // (3) walk the rows that have entries among the chunk's items
    for (int64_t rbase = r0;; rbase += kWave) {
      const int my_s = next_s, my_e = next_e, my_delta = next_delta;
      // another batch follows if its first row still starts inside the chunk
      const bool more = rbase + kWave < a.M && (int64_t)__builtin_amdgcn_readlane(my_e, kWave - 1) + rbase + kWave < d1;
      if (more) load_bounds(rbase + kWave, next_s, next_e, next_delta);

      const int64_t rr = rbase + lane;
      const int64_t limit = d1 - rr;                       // the chunk owns the row's entries below this number ...
      int own_s = my_s > cs ? my_s : cs;                   // ... and from this one on
      int own_e = (int64_t)my_e <= limit ? my_e : (limit > own_s ? (int)limit : own_s);
      bool my_whole = own_s == my_s && own_e == my_e;
      bool valid = rr < a.M && own_e > own_s && !(P::kCanSkipWholeRows && a.only_split && my_whole);
      bool is_empty = false;                               // whole-row path: a row of this chunk without entries
      if (kOwned) {
        const int64_t first_item_of_row = (int64_t)my_s + rr;
        const bool mine = rr < a.M && first_item_of_row >= d0 && first_item_of_row < d1;
        own_s = my_s;
        own_e = my_e;
        my_whole = true;
        valid = mine && my_e > my_s;
        is_empty = mine && my_e == my_s;
      }
      const int my_ps = own_s - cs;                        // the row's segment inside the chunk,
      const int my_pe = own_e - cs;                        // as offsets into the LDS slice
      // (whole-row path: a row counts as short only when the slice holds all of it; an empty one is a short row of length 0)
      const bool is_short = NS > 1 && ((valid && (my_pe - my_ps) <= a.short_len && (!kOwned || my_pe <= slice)) || is_empty);

      if (kPhased) {
        // stage the entries of this batch's segments: they are consecutive virtual positions [bs, be);
        // a lane finds the row of its position by a search over the batch's row starts, then reads
        // the stored entry at position + delta[row]
        const unsigned long long vmask = __ballot(valid);
        if (vmask) {
          const int bs = __builtin_amdgcn_readlane(my_ps, __builtin_ctzll(vmask));
          const int be = __builtin_amdgcn_readlane(my_pe, 63 - __builtin_clzll(vmask));
          row_info[lane] = make_int2(rr < a.M ? my_s - cs : INT32_MAX, my_delta);
          wave_lds_fence();
          for (int x0 = bs; x0 < be; x0 += 4 * kWave) {
            int k[4];
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int x = x0 + u * kWave + lane;
              const int xc = x < be ? x : be - 1;
              int pos = 0;                                 // last row of the batch that starts at or before xc
#pragma unroll
              for (int step = kWave / 2; step > 0; step >>= 1)
                if (row_info[pos + step].x <= xc) pos += step;
              const int p = xc + cs + row_info[pos].y;
              k[u] = a.colind[p];
              v[u] = a.vals ? a.vals[p] : 1.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
              const int x = x0 + u * kWave + lane;
              if (x < be) ka[x] = make_int2(k[u], __float_as_int(v[u]));
            }
          }
          wave_lds_fence();
        }
      }

      // (3a) short segments: one per slot, 64/G rows at a time, no cross-lane exchange
      if (NS > 1) {
        const unsigned long long smask = __ballot(is_short);
        const int nshort = __builtin_popcountll(smask);
        if (nshort > 0) {
          const int rank = __builtin_amdgcn_mbcnt_hi((unsigned)(smask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)smask, 0u));
          // an empty row's offset is only ever used for padded gathers: it is moved onto a staged entry
          const int desc_ps = is_empty ? (my_ps < cnt ? my_ps : (cnt > 0 ? cnt - 1 : 0)) : my_ps;
          if (is_short)   // lane | offset << 6 | length << 18 | whole << 30 ; full row length
            short_rows[rank] = make_int2(lane | (desc_ps << 6) | ((my_pe - my_ps) << 18) | ((int)my_whole << 30), my_e - my_s);
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
            if constexpr (kOwned) {
              if (have && r_len == 0) P::store_empty(a, row, col);
              else if (have) P::end(st, a, row, true, d.y, col);
            } else {
              if (have) P::end(st, a, row, (d.x >> 30) & 1, d.y, col);
            }
          }
          wave_lds_fence();
        }
      }

      // (3b) long segments: all slots work on one row, slot s takes entries s, s+NS, ...
      unsigned long long todo = __ballot((valid || is_empty) && !is_short);
      while (todo) {
        const int i = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int ps = __builtin_amdgcn_readlane(my_ps, i);
        const int pe = __builtin_amdgcn_readlane(my_pe, i);
        const int s = __builtin_amdgcn_readlane(my_s, i);
        const int e = __builtin_amdgcn_readlane(my_e, i);
        const bool whole = __builtin_amdgcn_readlane((int)my_whole, i) != 0;
        typename P::State st;
        if constexpr (kOwned) {
          if (e == s) {                                      // (only reached when a slot is the whole wavefront)
            if (slot == 0) P::store_empty(a, rbase + i, col);
            continue;
          }
          if (pe > slice) {
            // the row reaches beyond the staged entries: it is the last row of this chunk (every later row
            // starts beyond the chunk's items), so the slice can be reused for windows of the row
            P::begin(st, a, rbase + i, e - s, colc);
            for (int w = s; w < e; w += slice) {
              const int wn = e - w < slice ? e - w : slice;
              wave_lds_fence();                              // earlier reads of the slice are done
              stage(w, wn);
              for (int base = 0; base < wn; base += U * NS) {
                const int first = base + slot;
                const int left = (wn - first + NS - 1) / NS;
                P::template pass<U>(st, a, ka, w, left > 0 ? first : wn - 1, NS, left, col, colc);
              }
            }
            P::template combine<G>(st);
            if (slot == 0) P::end(st, a, rbase + i, true, e - s, col);
            continue;
          }
        }
        P::begin(st, a, rbase + i, e - s, colc);
        for (int base = ps; base < pe; base += U * NS) {
          const int first = base + slot;
          const int left = (pe - first + NS - 1) / NS;       // entries first, first+NS, ... below pe
          P::template pass<U>(st, a, ka, cs, left > 0 ? first : pe - 1, NS, left, col, colc);
        }
        P::template combine<G>(st);
        if (slot == 0) P::end(st, a, rbase + i, whole, e - s, col);
      }
      if (!more) break;
    }
    if (!kPhased) break;
    wave_lds_fence();                              // the LDS slice is reused by the next chunk
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
  // Binary search over the whole row.  For any data, sorted or not, the result is monotone in the
  // column searched for as long as every search starts from the same interval, which is what makes
  // the pieces a partition of the row: the end of piece q IS the start of piece q + 1.
  int lo = s, hi = e;
  const int64_t column = (int64_t)q * cols_per_part;
  if (q == 0 || !live) hi = lo;                     // piece 0 starts where the row starts
  while (lo < hi) {
    const int mid = lo + ((hi - lo) >> 1);
    if (colind[mid] < column) lo = mid + 1;
    else hi = mid;
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

// Kernels of the whole-row path: the three folds and max / min with positions, on fp32 features, one tile per lane.
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
};

inline int parse_tuning(const gespmm_tuning_t* in, Tuning* out) {
  *out = Tuning{};
  if (!in) return GESPMM_OK;
  const int G = in->lanes_per_row, T = in->tiles_per_lane;
  if (G > 0 && (G > kWave || (G & (G - 1)) != 0)) return GESPMM_ERR_BAD_ARG;
  if (T > 0 && T != 1 && T != 2 && T != 4) return GESPMM_ERR_BAD_ARG;
  if (G > 0 && T > 0 && !has_kernel(G, T)) return GESPMM_ERR_BAD_ARG;
  if (in->xcd_remap > 1) return GESPMM_ERR_BAD_ARG;
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
// re-reads and re-writes C and walks all rows again, which costs more than the hits bring.  Needs
// the vector kernels and, unless forced, a workspace that is large enough.
inline int choose_parts(int64_t M, int64_t K, int64_t nnz, int vec, int block_bytes, const Tuning& tune,
                        size_t workspace_bytes) {
  if (vec != 4 || M <= 0 || K <= 0 || nnz <= 0) return 1;
  if (tune.k_parts >= 0) return tune.k_parts < 2 ? 1 : (int)(tune.k_parts < K ? tune.k_parts : (K < 2 ? 1 : K));
  const int64_t live = K * block_bytes;
  const int64_t mean_row = nnz / M;
  if (live < (12ll << 20) || mean_row < 128) return 1;
  int64_t q = (live + (15ll << 18)) / (15ll << 19);        // nearest multiple of 7.5 MB
  while (q > 2 && mean_row / q < 32) --q;
  if (q > kMaxParts) q = kMaxParts;
  if (q < 2) return 1;
  if (workspace_bytes < phased_workspace_bytes(M, (int)q)) return 1;
  return (int)q;
}

// elem_bytes: size of one element of the dense input (4, or 2 for the 16-bit formats); a lane
// loads four columns at once when the width and the alignment allow it, one otherwise.
// whole_rows_allowed: the job has kernels of the whole-row path (the forward folds on fp32 features).
inline void make_plan(int64_t M, int64_t K, int64_t N, int64_t nnz, bool aligned16, int elem_bytes, const Tuning& tune,
                      size_t workspace_bytes, gespmm_plan_t* p, bool whole_rows_allowed = true) {
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
    parts = choose_parts(M, K, nnz, vec, wide * vec * elem_bytes, tune, workspace_bytes);
    if (parts > 1) G = wide < 8 ? 8 : wide;
    else if (G > line) G = ncv <= 4 * line ? line : 2 * line;   // one line; two lines for wide N
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
  if (parts > 1) shift = 9;                     // measured: 512 and 1024 within 1 %, 256 is 10 % slower
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
  p->xcd_remap = tune.remap >= 0 ? tune.remap : (long_rows && parts == 1 ? 1 : 0);
  // Rows up to short_len entries are walked one per slot, longer ones by all slots together
  // (with a cross-slot combine per row).  Where the mean row has 17 .. 48 entries, as in
  // stencil and finite-element matrices whose rows all have about that length, one slot per
  // row up to 32 entries avoids that combine for most rows (measured: up to 22 % on a
  // 27-point stencil, within 3 % either way on power-law graphs of the same mean).
  const int64_t mean_row = M > 0 ? nnz / M / parts : 0;
  int auto_short = 2 * p->slots < 16 ? 2 * p->slots : 16;
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

  launch_init_rows(plan.vec, M, L.N, L.rowptr, L.dense_out, L.empty_value, L.split_value, -1, stream);
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
  const bool fold_job = !L.picker && (L.job == kJobAdd || L.job == kJobMax || L.job == kJobMin) && !L.one_lane_per_entry;
  Tuning tune = L.tuning;
  if (!fold_job || !L.workspace) {
    if (tune.k_parts > 1 && fold_job) return GESPMM_ERR_WORKSPACE;   // phases were asked for but there is nowhere to put their row starts
    tune.k_parts = 1;
  }
  gespmm_plan_t plan;
  const bool arg_job = !L.picker && (L.job == kJobMaxWithArg || L.job == kJobMinWithArg) && L.arg && !L.one_lane_per_entry;
  const bool whole_rows_allowed = (fold_job || arg_job) && L.b_dtype == GESPMM_F32 && L.init_target == L.dense_out;
  make_plan(L.M, L.K, L.N, L.nnz, aligned16, L.b_dtype == GESPMM_F32 ? 4 : 2, tune, L.workspace_bytes, &plan, whole_rows_allowed);
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
    if (L.b_dtype == GESPMM_BF16) phased = pick_phased<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else if (L.b_dtype == GESPMM_F16) phased = pick_phased<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    else phased = pick_phased<float>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
    if (!phased) return GESPMM_ERR_BAD_ARG;
    return launch_phased(L, plan, phased, shift, stream);
  }

  MainKernel kernel = nullptr;
  if (L.picker) kernel = L.picker(plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_BF16) kernel = pick_b16<bf16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else if (L.b_dtype == GESPMM_F16) kernel = pick_b16<f16_t>(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  else kernel = pick_kernel(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  if (plan.row_window > 0) kernel = pick_owned(L.job, plan.vec, plan.lanes_per_row, plan.tiles_per_lane);
  if (!kernel) return GESPMM_ERR_BAD_ARG;

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
  if (plan.row_window > 0) a.packed_split = 0;    // no row is split
  else if (L.packed_split && (plan.vec != 4 || L.N > kWave * kFinishWords || !L.arg)) return GESPMM_ERR_BAD_ARG;
  int status = GESPMM_OK;
  bool timed = false;
  if (!record_start(L.profiler, stream, &timed, &status)) return status;
  hipLaunchKernelGGL(kernel, dim3((unsigned)plan.grid_x, (unsigned)plan.col_blocks), dim3(kBlock), (size_t)plan.lds_bytes, stream, a);
  if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  if (!record_stop(L.profiler, stream, timed, &status)) return status;
  if (plan.row_window > 0) {
    if (took_whole_rows) *took_whole_rows = true;
    return GESPMM_OK;
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
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = B; L.dense_out = C;
  L.init_target = C; L.empty_value = 0.0f; L.split_value = R::identity();
  return launch_chunks(L, stream);
}

}  // namespace gespmm
