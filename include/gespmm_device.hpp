// CSR SpMM / SpMM-like kernels for gfx950 (MI355X): the device code.
// (The launch helpers are in gespmm_kernels.hpp, the C ABI over them in
// paper_2007_03179_amd/csrc/gespmm.hip.  User-defined reduce operations instantiate these
// templates in their own translation unit through gespmm_custom.hpp, or at run time through
// gespmm_custom_op_create, which hands this very file to the run-time compiler: it therefore
// holds device code only and includes nothing but the HIP runtime header.)
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

#ifdef __HIPCC_RTC__
// the run-time compiler brings the HIP device runtime with it and has no C library headers
typedef unsigned short uint16_t;
typedef signed int int32_t;
typedef unsigned int uint32_t;
typedef long long int64_t;
typedef unsigned long long uint64_t;
typedef unsigned long uintptr_t;
#ifndef INT32_MAX
#define INT32_MAX 2147483647
#endif
#else
#include <hip/hip_runtime.h>

#include <cstdint>
#endif

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
  uint32_t b_row_bytes;   // fold jobs on a B below 2 GiB: bytes of one row of B (the staged key of an entry is then
                          // the byte offset of its row of B, and the gathers are buffer loads); 0 = 64-bit addresses
  uint32_t b_bytes;       // ... and the size of B in bytes
  int32_t stream_stores;  // finished rows of C are written with streaming stores (whole 128-byte lines, written once)
  int32_t stream_entries; // K-phased path: colind / vals are loaded with the streaming hint (one column block: read once)
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
  // a store that tells the caches the line will not be read again soon (results that are written once)
  __device__ void store_streaming(float* p) const {
    typedef float f4 __attribute__((ext_vector_type(4)));
    f4 t = {v[0], v[1], v[2], v[3]};
    __builtin_nontemporal_store(t, reinterpret_cast<f4*>(p));
  }
};
template <> struct Vec<1> {
  float v[1];
  __device__ static Vec load(const float* p) { return Vec{{*p}}; }
  __device__ void store(float* p) const { *p = v[0]; }
  __device__ void store_streaming(float* p) const { __builtin_nontemporal_store(v[0], p); }
};
// Element types of the dense input.  The 16-bit types are storage formats only: every
// value is widened to fp32 (exactly) before the multiply, and products and sums are fp32.
struct bf16_t { uint16_t bits; };               // 1 sign, 8 exponent, 7 fraction bits: the top half of an fp32
struct f16_t { uint16_t bits; };                // IEEE binary16

// Gathers through a buffer descriptor of B (base, size): the address of a load is base + a 32-bit byte
// offset, which costs one 32-bit add per gather where a 64-bit address costs a 64-bit multiply-add and a
// 64-bit shift-add, and a load whose offset lies beyond the size returns zeros instead of faulting - the
// sum uses that for entries that do not exist (kPastTheEnd).  Limited to 2 GiB of B by the 32-bit offsets.
using BufferOfB = __amdgpu_buffer_rsrc_t;
constexpr uint32_t kPastTheEnd = 0x80000000u;     // plus any offset inside a row: still beyond every B this path takes
__device__ __forceinline__ BufferOfB buffer_of(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);   // untyped 32-bit data, no swizzle
}

// BLoad<V, BT>: one load of V consecutive elements of type BT, kept as loaded (Raw) until
// it is used, so that all loads of a pass can be in flight together; unpack widens to fp32.
// load_at is the same load through the buffer descriptor, at a byte offset.
template <int V, class BT> struct BLoad;
template <> struct BLoad<4, float> {
  using Raw = float4;
  __device__ static Raw load(const float* p) { return *reinterpret_cast<const float4*>(p); }
  __device__ static Raw load_at(BufferOfB b, uint32_t offset) {
    const auto w = __builtin_amdgcn_raw_buffer_load_b128(b, (int)offset, 0, 0);
    return make_float4(__uint_as_float(w[0]), __uint_as_float(w[1]), __uint_as_float(w[2]), __uint_as_float(w[3]));
  }
  __device__ static void unpack(const Raw& r, float (&o)[4]) { o[0] = r.x; o[1] = r.y; o[2] = r.z; o[3] = r.w; }
};
template <> struct BLoad<1, float> {
  using Raw = float;
  __device__ static Raw load(const float* p) { return *p; }
  __device__ static Raw load_at(BufferOfB b, uint32_t offset) { return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(b, (int)offset, 0, 0)); }
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
  __device__ static Raw load_at(BufferOfB b, uint32_t offset) {
    const auto w = __builtin_amdgcn_raw_buffer_load_b64(b, (int)offset, 0, 0);
    return make_uint2(w[0], w[1]);
  }
  __device__ static void unpack(const Raw& r, float (&o)[4]) {
    widen_pair(BT{}, r.x, o[0], o[1]);
    widen_pair(BT{}, r.y, o[2], o[3]);
  }
};
template <> struct BLoad<1, bf16_t> {
  using Raw = uint16_t;
  __device__ static Raw load(const bf16_t* p) { return p->bits; }
  __device__ static Raw load_at(BufferOfB b, uint32_t offset) { return __builtin_amdgcn_raw_buffer_load_b16(b, (int)offset, 0, 0); }
  __device__ static void unpack(const Raw& r, float (&o)[1]) { o[0] = __uint_as_float((unsigned)r << 16); }
};
template <> struct BLoad<1, f16_t> {
  using Raw = uint16_t;
  __device__ static Raw load(const f16_t* p) { return p->bits; }
  __device__ static Raw load_at(BufferOfB b, uint32_t offset) { return __builtin_amdgcn_raw_buffer_load_b16(b, (int)offset, 0, 0); }
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
  if (remap > 1) {
    // runs of `remap` consecutive workgroups per XCD, the runs dealt round-robin: neighbours share an L2 and
    // every XCD still gets an even share of every stretch of 8 * remap workgroups
    const int64_t period = (int64_t)kXcds * remap;
    if (b >= nb / period * period) return b;          // (the last, incomplete period stays as dispatched)
    const int64_t w = b % period;
    return b - w + (w % kXcds) * remap + w / kXcds;
  }
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

template <bool B> struct BoolTag { static constexpr bool value = B; };

// The same address as a pointer into global memory (which is what the arrays of this library are).
template <class T>
__device__ __forceinline__ const __attribute__((address_space(1))) T* global_pointer(const T* p) {
  return (const __attribute__((address_space(1))) T*)p;
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int F, int V, int T, class BT = float>
struct FoldRows {
  static constexpr bool kCanSkipWholeRows = false;
  static constexpr bool kHasFullPass = true;
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
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      e2[u] = ka[first + uu * stride];
      if (F == kAdd && u >= left) e2[u].y = 0;
    }
    if (a.b_row_bytes != 0) {
      // the staged key is the byte offset of the entry's row of B; an entry that does not exist reads past the end (zeros)
      const BufferOfB whole_b = buffer_of(a.B, a.b_bytes);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t row_offset = F == kAdd && u >= left ? kPastTheEnd : (uint32_t)e2[u].x;
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load_at(whole_b, row_offset + (uint32_t)colc[t] * (uint32_t)sizeof(BT));
      }
    } else {
      const BT* nothing = reinterpret_cast<const BT*>(kZeroLine);      // the same 16 bytes for every lane: a uniform address
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load(F == kAdd && u >= left ? nothing : brow + colc[t]);
      }
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

  // The same for a pass in which every lane has all U entries (the usual case inside a long row): the
  // entries sit at fixed distances from `first`, nothing is clamped, masked or replaced.
  template <int U>
  __device__ static void pass_full(State& s, const KernelArgs& a, const int2* ka, int, int first, int stride, const int (&colc)[T]) {
    using Load = BLoad<V, BT>;
    int2 e2[U];
    typename Load::Raw b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) e2[u] = ka[first + u * stride];
    if (a.b_row_bytes != 0) {
      const BufferOfB whole_b = buffer_of(a.B, a.b_bytes);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load_at(whole_b, (uint32_t)e2[u].x + (uint32_t)colc[t] * (uint32_t)sizeof(BT));
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load(brow + colc[t]);
      }
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
          if (a.stream_stores) s.acc[t].store_streaming(crow + col[t]);
          else s.acc[t].store(crow + col[t]);
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
    gather<U>(a, e2, colc, b);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int uu = u < left ? u : (left > 0 ? left - 1 : 0);
      fold_entry(s, e2[u], b[u], cs + first + uu * stride);      // (the index is recomputed here rather than kept in registers across the loads)
    }
  }

  // A pass in which every lane has all U entries: fixed distances from `first`, nothing clamped.
  static constexpr bool kHasFullPass = true;
  template <int U>
  __device__ static void pass_full(State& s, const KernelArgs& a, const int2* ka, int cs, int first, int stride, const int (&colc)[T]) {
    int2 e2[U];
    typename BLoad<V, BT>::Raw b[U][T];
#pragma unroll
    for (int u = 0; u < U; ++u) e2[u] = ka[first + u * stride];
    gather<U>(a, e2, colc, b);
#pragma unroll
    for (int u = 0; u < U; ++u) fold_entry(s, e2[u], b[u], cs + first + u * stride);
  }

  // The rows of B of U staged entries (the staged key is the row's byte offset when B is gathered through a buffer
  // descriptor, the column index otherwise).
  template <int U>
  __device__ static void gather(const KernelArgs& a, const int2 (&e2)[U], const int (&colc)[T], typename BLoad<V, BT>::Raw (&b)[U][T]) {
    using Load = BLoad<V, BT>;
    if (a.b_row_bytes != 0) {
      const BufferOfB whole_b = buffer_of(a.B, a.b_bytes);
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load_at(whole_b, (uint32_t)e2[u].x + (uint32_t)colc[t] * (uint32_t)sizeof(BT));
    } else {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const BT* brow = reinterpret_cast<const BT*>(a.B) + (int64_t)e2[u].x * a.N;
#pragma unroll
        for (int t = 0; t < T; ++t) b[u][t] = Load::load(brow + colc[t]);
      }
    }
  }

  __device__ static void fold_entry(State& s, const int2 entry, const typename BLoad<V, BT>::Raw (&b)[T], int where_u) {
#pragma unroll
    for (int t = 0; t < T; ++t) {
      float bx[V];
      BLoad<V, BT>::unpack(b[t], bx);
#pragma unroll
      for (int x = 0; x < V; ++x) {
        // A lane meets its entries in increasing index order, so "first among equals" is
        // "replace on strict improvement only".  The hardware max / min orders the zeros
        // (+0 above -0), so the running value changes its bits exactly when the entry improves it.
        const float product = __int_as_float(entry.y) * bx[x];
        const float next = F == kMax ? __builtin_fmaxf(s.best[t][x], product) : __builtin_fminf(s.best[t][x], product);
        s.where[t][x] = __float_as_int(next) != __float_as_int(s.best[t][x]) ? where_u : s.where[t][x];
        s.best[t][x] = next;
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
        if (whole && a.accumulate) {
          // A phase of the K-phased path: during all phases every row holds packed words (zero: nothing yet).
          // This wavefront alone touches the row in this launch, so the better of (what the earlier phases
          // left, this phase's piece) goes back with plain loads and stores.
          const int half = a.N >> 1;
          if (V == 4 && (half & 3) == 0) {
            // the lane's four words lie side by side in one of the two arrays: two 16-byte loads and stores
            const int j = col[t];
            ulonglong2* words = reinterpret_cast<ulonglong2*>(j < half ? reinterpret_cast<unsigned long long*>(crow) + j
                                                                       : reinterpret_cast<unsigned long long*>(arow) + (j - half));
            ulonglong2 lo = words[0], hi = words[1];
            const unsigned long long m0 = pack(key_of(s.best[t][0]), s.where[t][0]), m1 = pack(key_of(s.best[t][1 % V]), s.where[t][1 % V]);
            const unsigned long long m2 = pack(key_of(s.best[t][2 % V]), s.where[t][2 % V]), m3 = pack(key_of(s.best[t][3 % V]), s.where[t][3 % V]);
            lo.x = m0 > lo.x ? m0 : lo.x;
            lo.y = m1 > lo.y ? m1 : lo.y;
            hi.x = m2 > hi.x ? m2 : hi.x;
            hi.y = m3 > hi.y ? m3 : hi.y;
            words[0] = lo;
            words[1] = hi;
            continue;
          }
          unsigned long long* slot[V];
          unsigned long long before[V];
#pragma unroll
          for (int x = 0; x < V; ++x) {
            const int j = col[t] + x;
            slot[x] = j < half ? reinterpret_cast<unsigned long long*>(crow) + j
                               : reinterpret_cast<unsigned long long*>(arow) + (j - half);
            before[x] = *slot[x];
          }
#pragma unroll
          for (int x = 0; x < V; ++x) {
            const unsigned long long mine = pack(key_of(s.best[t][x]), s.where[t][x]);
            if (mine > before[x]) *slot[x] = mine;
          }
        } else if (whole) {
          Vec<V> value, place;
#pragma unroll
          for (int x = 0; x < V; ++x) {
            value.v[x] = s.best[t][x];
            place.v[x] = __int_as_float(s.where[t][x]);
          }
          if (a.stream_stores) {
            value.store_streaming(crow + col[t]);
            place.store_streaming(reinterpret_cast<float*>(arow + col[t]));
          } else {
            value.store(crow + col[t]);
            place.store(reinterpret_cast<float*>(arow + col[t]));
          }
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
  // (the wavefront's number as a scalar: everything derived from it and from the ballot below stays in scalar registers)
  const int64_t base = (int64_t)__builtin_amdgcn_readfirstlane((int)(blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6))) * kWave;
  if (base >= M) return;
  const int64_t r = base + lane;
  bool split = false;
  if (r < M) {
    const int s = rowptr[r], e = rowptr[r + 1];
    split = chunk_shift < 0 || (e > s && row_is_shared(s, e, r, chunk_shift));   // (chunk_shift < 0: every row holds packed words)
  }
  unsigned long long todo = __ballot(split);
  const int half = N >> 1;
  // where this lane's words sit inside a row: 8-byte word `place[k]` of the row's C storage, or of its arg storage
  bool in_c[WORDS];
  int place[WORDS];
#pragma unroll
  for (int k = 0; k < WORDS; ++k) {
    const int j = lane + k * kWave;
    const int jj = j < N ? j : N - 1;                  // lanes beyond the row re-read its last word (and store nothing)
    in_c[k] = jj < half;
    place[k] = jj < half ? jj : jj - half;
  }
  while (todo) {
    // the next BATCH rows; when fewer are left the last one is repeated (its loads are harmless, its stores skipped).
    // All loads are unconditional, so that they are in flight together: one round trip per batch.
    int pick[BATCH];
    int rows_here = 0;
    const int first = __builtin_ctzll(todo);
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      pick[q] = first;
      if (todo) {
        pick[q] = __builtin_ctzll(todo);
        todo &= todo - 1;
        ++rows_here;
      }
    }
    unsigned long long word[BATCH][WORDS];
#pragma unroll
    for (int q = 0; q < BATCH; ++q) {
      const int64_t at = (base + pick[q]) * (int64_t)N;
      const unsigned long long* cwords = reinterpret_cast<const unsigned long long*>(C + at);
      const unsigned long long* awords = reinterpret_cast<const unsigned long long*>(arg + at);
#pragma unroll
      for (int k = 0; k < WORDS; ++k) {
        const unsigned long long* src = (in_c[k] ? cwords : awords) + place[k];
        word[q][k] = *src;
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
      if (q >= rows_here) break;                        // (wave-uniform)
      float* crow = C + (base + pick[q]) * (int64_t)N;
      int32_t* arow = arg + (base + pick[q]) * (int64_t)N;
#pragma unroll
      for (int k = 0; k < WORDS; ++k) {
        const int j = lane + k * kWave;
        if (j < N) {
          float value;
          int where;
          Rows::unpack(word[q][k], value, where);
          if (word[q][k] == 0ull) {          // below every word of a real entry: the row stores nothing
            value = 0.0f;
            where = -1;
          }
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

  // A row without stored entries yields 0 (whole-row path).
  __device__ static void store_empty(const KernelArgs& a, int64_t row, const int (&col)[T]) {
    float* crow = a.C + row * (int64_t)a.N;
    Vec<V> zero;
#pragma unroll
    for (int x = 0; x < V; ++x) zero.v[x] = 0.0f;
#pragma unroll
    for (int t = 0; t < T; ++t)
      if (col[t] < a.N) zero.store(crow + col[t]);
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
// Policies that have a pass_full<U>() say so with a member `kHasFullPass = true`.
template <bool B> struct enable_if_true {};
template <> struct enable_if_true<true> { using type = void; };
template <class P, class = void> struct has_full_pass { static constexpr bool value = false; };
template <class P> struct has_full_pass<P, typename enable_if_true<P::kHasFullPass>::type> { static constexpr bool value = true; };

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
          // (the key becomes the row's byte offset in B, which fits 31 bits on this path, only here: used right
          //  after its load it would make every load wait for the one before)
          if (idx < count) ka[idx] = make_int2(a.b_row_bytes != 0 ? k[u] * (int)a.b_row_bytes : k[u], __float_as_int(v[u]));
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
          // Entries that the call reads exactly once (one column block) are loaded with the streaming hint: they
          // then take less of the L2s away from the part of B the phase gathers from.  Two copies of the loop, so
          // that neither carries a branch per load.
          auto stage_batch = [&](auto streaming) {
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
                if constexpr (decltype(streaming)::value) {
                  k[u] = __builtin_nontemporal_load(global_pointer(a.colind + p));
                  v[u] = a.vals ? __builtin_nontemporal_load(global_pointer(a.vals + p)) : 1.0f;
                } else {
                  k[u] = a.colind[p];
                  v[u] = a.vals ? a.vals[p] : 1.0f;
                }
                if (a.b_row_bytes != 0) k[u] *= (int)a.b_row_bytes;
              }
#pragma unroll
              for (int u = 0; u < 4; ++u) {
                const int x = x0 + u * kWave + lane;
                if (x < be) ka[x] = make_int2(k[u], __float_as_int(v[u]));
              }
            }
          };
          if (a.stream_entries) stage_batch(BoolTag<true>{});
          else stage_batch(BoolTag<false>{});
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
            // (stored position of a slice entry = cs + its offset, in a phase plus the row's delta)
            const int r_cs = kPhased ? cs + row_info[d.x & 63].y : cs;
            typename P::State st;
            P::begin(st, a, row, d.y, colc);
            // U entries per step; a last step with at most U / 2 entries left in every slot takes
            // the half-size pass (fewer padded gathers: up to 7 % on matrices of short rows)
            for (int it = 0; __ballot(it < r_len) != 0ull;) {
              if (U >= 4 && __ballot(r_len - it > U / 2) == 0ull) {
                P::template pass<(U >= 4 ? U / 2 : U)>(st, a, ka, r_cs, r_ps + (it < r_len ? it : 0), 1, r_len - it, col, colc);
                it += U / 2;
              } else {
                P::template pass<U>(st, a, ka, r_cs, r_ps + (it < r_len ? it : 0), 1, r_len - it, col, colc);
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
                if constexpr (has_full_pass<P>::value) {
                  if (base + U * NS <= wn) {
                    P::template pass_full<U>(st, a, ka, w, first, NS, colc);
                    continue;
                  }
                }
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
        // (stored position of a slice entry = cs + its offset, in a phase plus the row's delta)
        const int row_cs = kPhased ? cs + __builtin_amdgcn_readlane(my_delta, i) : cs;
        for (int base = ps; base < pe; base += U * NS) {
          const int first = base + slot;
          if constexpr (has_full_pass<P>::value) {
            if (base + U * NS <= pe) {                       // (wave-uniform) every lane has all its U entries
              P::template pass_full<U>(st, a, ka, row_cs, first, NS, colc);
              continue;
            }
          }
          const int left = (pe - first + NS - 1) / NS;       // entries first, first+NS, ... below pe
          P::template pass<U>(st, a, ka, row_cs, left > 0 ? first : pe - 1, NS, left, col, colc);
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

}  // namespace gespmm_detail
