// Structure transpose by a stable least-significant-digit radix sort on the column index.
//
// The transposed CSR arrays are the stored entries of A ordered by (column, original position).
// gespmm_csr_transpose gets there with one counter per column and one scattered atomic plus two
// scattered 4-byte writes per entry, which is bound by the rate of scattered L2 requests.  Here
// every pass streams: a tile of 4096 consecutive entries is read with coalesced loads, ranked
// inside the workgroup, reordered through LDS and written out as one run per digit value, so
// the traffic is 28 bytes per entry and pass whatever the column distribution is (a hub
// column is just a long run).  Two passes cover up to 2^20 columns, three up to 2^30.
// The sort is stable, so inside a transposed row the entries keep the order of A's rows: the
// result is unique and equals a stable counting sort on the CPU bit for bit.
#pragma once

#include "gespmm_kernels.hpp"

namespace gespmm_detail {

constexpr int kSortItems = 16;                          // entries per thread
constexpr int kSortTile = kBlock * kSortItems;          // 4096 entries per workgroup
constexpr int kSortWaveSpan = kWave * kSortItems;       // 1024 consecutive entries per wavefront
constexpr int kSortMaxBits = 10;                        // digit width: up to 1024 bins
constexpr int kSortMaxBins = 1 << kSortMaxBits;

// counts[d * tiles + tile] = entries of the tile whose digit is d
static __global__ void __launch_bounds__(kBlock) radix_histogram(const int32_t* __restrict__ keys, int64_t n, int shift,
                                                                 int bits, int64_t tiles, int32_t* __restrict__ counts) {
  __shared__ int bins[kSortMaxBins];
  const int nbins = 1 << bits;
  for (int d = threadIdx.x; d < nbins; d += kBlock) bins[d] = 0;
  __syncthreads();
  const int64_t tile = logical_block(blockIdx.x, gridDim.x, 1);   // neighbouring tiles on one XCD, as in radix_scatter
  const int64_t base = tile * kSortTile;
  int key[kSortItems];
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {                   // all loads first
    const int64_t idx = base + j * kBlock + threadIdx.x;
    key[j] = idx < n ? keys[idx] : -1;
  }
#pragma unroll
  for (int j = 0; j < kSortItems; ++j)
    if (key[j] >= 0) atomicAdd(&bins[(key[j] >> shift) & (nbins - 1)], 1);
  __syncthreads();
  for (int d = threadIdx.x; d < nbins; d += kBlock) counts[(int64_t)d * tiles + tile] = bins[d];
}

// One pass: entries of tile `blockIdx.x` go to out[...] ordered by digit, ties in input order.
// starts[d * tiles + tile] is the exclusive scan of radix_histogram's counts (digit-major), i.e.
// the first output position of the tile's entries with digit d.
static __global__ void __launch_bounds__(kBlock) radix_scatter(const int32_t* __restrict__ keys_in, const int32_t* __restrict__ rows_in,
                                                               const float* __restrict__ vals_in, int64_t n, int shift, int bits,
                                                               int64_t tiles, const int32_t* __restrict__ starts,
                                                               int32_t* __restrict__ keys_out, int32_t* __restrict__ rows_out,
                                                               float* __restrict__ vals_out) {
  // (16-bit counters: a tile holds 4096 entries; everything together stays below 64 KB of LDS)
  __shared__ unsigned short wave_count[kWavesPerBlock][kSortMaxBins];   // per wavefront: entries seen per digit, then its offset
  __shared__ unsigned short tile_first[kSortMaxBins];       // first position of the digit inside the sorted tile
  __shared__ int out_first[kSortMaxBins];                    // first output position of the digit for this tile
  __shared__ int s_buf[kSortTile];                          // the tile in sorted order, one array at a time

  const int nbins = 1 << bits;
  const int lane = threadIdx.x & (kWave - 1);
  const int wave = threadIdx.x >> 6;
  // Neighbouring tiles continue each other's runs (tile t + 1 writes right behind tile t in every
  // digit's region), a few entries each: keeping them on one XCD lets its L2 complete the 128-byte
  // lines before they are written back.
  const int64_t tile = logical_block(blockIdx.x, gridDim.x, 1);
  const int64_t base = tile * kSortTile;
  const int tile_count = (int)((n - base) < kSortTile ? (n - base) : kSortTile);

  for (int d = threadIdx.x; d < nbins; d += kBlock) {
#pragma unroll
    for (int w = 0; w < kWavesPerBlock; ++w) wave_count[w][d] = 0;
    out_first[d] = starts[(int64_t)d * tiles + tile];
  }
  __syncthreads();

  // (1) every wavefront ranks its 1024 consecutive entries, 64 at a time in input order:
  //     rank = entries of the same digit seen earlier by this wavefront
  int key[kSortItems], row[kSortItems], rank[kSortItems];
  float val[kSortItems];
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int local = wave * kSortWaveSpan + j * kWave + lane;
    const bool live = local < tile_count;
    key[j] = live ? keys_in[base + local] : 0;
    row[j] = live ? rows_in[base + local] : 0;
    val[j] = live ? vals_in[base + local] : 0.0f;
  }
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int local = wave * kSortWaveSpan + j * kWave + lane;
    const bool live = local < tile_count;
    const int d = (key[j] >> shift) & (nbins - 1);
    unsigned long long peers = __ballot(live);             // lanes of this step with my digit
    for (int b = 0; b < bits; ++b) {
      const unsigned long long vote = __ballot((d >> b) & 1);
      peers &= ((d >> b) & 1) ? vote : ~vote;
    }
    const int before = __builtin_popcountll(peers & ((1ull << lane) - 1ull));
    const int leader = __builtin_ctzll(peers | (1ull << 63));
    int seen = 0;
    if (live && lane == leader) {                          // one lane per distinct digit updates the counter
      seen = wave_count[wave][d];
      wave_count[wave][d] = (unsigned short)(seen + __builtin_popcountll(peers));
    }
    seen = __shfl(seen, leader, kWave);
    rank[j] = seen + before;
    wave_lds_fence();                                      // the next step sees this step's counters
  }
  __syncthreads();

  // (2) per digit: offsets of the four wavefronts, then first position inside the sorted tile
  {
    int total[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int d = threadIdx.x * 4 + q;
      int run = 0;
      if (d < nbins) {
#pragma unroll
        for (int w = 0; w < kWavesPerBlock; ++w) {
          const int c = wave_count[w][d];
          wave_count[w][d] = (unsigned short)run;
          run += c;
        }
      }
      total[q] = run;
    }
    int all;
    int prefix = tile_exclusive_scan(total, &all);
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int d = threadIdx.x * 4 + q;
      if (d < nbins) tile_first[d] = (unsigned short)prefix;
      prefix += total[q];
    }
  }
  __syncthreads();

  // (3) through LDS in sorted order, one array at a time (16 KB instead of 48 KB keeps more
  //     workgroups on a compute unit); consecutive threads write consecutive places of a digit's run
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int local = wave * kSortWaveSpan + j * kWave + lane;
    if (local < tile_count) {
      const int d = (key[j] >> shift) & (nbins - 1);
      rank[j] = tile_first[d] + wave_count[wave][d] + rank[j];      // place inside the sorted tile
      s_buf[rank[j]] = key[j];
    }
  }
  __syncthreads();
  int to[kSortItems];                                       // output places (all below 2^31)
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int pos = j * kBlock + threadIdx.x;
    to[j] = -1;
    if (pos < tile_count) {
      const int k = s_buf[pos];
      const int d = (k >> shift) & (nbins - 1);
      to[j] = out_first[d] + (pos - tile_first[d]);
      keys_out[to[j]] = k;
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int local = wave * kSortWaveSpan + j * kWave + lane;
    if (local < tile_count) s_buf[rank[j]] = row[j];
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortItems; ++j)
    if (to[j] >= 0) rows_out[to[j]] = s_buf[j * kBlock + threadIdx.x];
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortItems; ++j) {
    const int local = wave * kSortWaveSpan + j * kWave + lane;
    if (local < tile_count) s_buf[rank[j]] = __float_as_int(val[j]);
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kSortItems; ++j)
    if (to[j] >= 0) vals_out[to[j]] = __int_as_float(s_buf[j * kBlock + threadIdx.x]);
}

// rowptrT[k] = number of entries whose column is below k = first place of k in the sorted keys
static __global__ void __launch_bounds__(kBlock) row_starts_from_sorted_keys(const int32_t* __restrict__ keys, int64_t n, int64_t K,
                                                                             int32_t* __restrict__ rowptrT) {
  const int64_t stride = (int64_t)gridDim.x * kBlock;
  for (int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x; k <= K; k += stride) {
    int64_t lo = 0, hi = n;                                // first p with keys[p] >= k
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if (keys[mid] < k) lo = mid + 1; else hi = mid;
    }
    rowptrT[k] = (int32_t)lo;
  }
}

struct SortPlan {
  int bits_total, passes, bits_per_pass;
  int64_t tiles, count_len, count_tiles;
  size_t off_rowid, off_val, off_keys_a, off_keys_x, off_rows_x, off_vals_x, off_counts, off_sums, bytes;
};

inline SortPlan make_sort_plan(int64_t K, int64_t nnz) {
  SortPlan p;
  p.bits_total = 1;
  while (p.bits_total < 31 && (1ll << p.bits_total) < K) ++p.bits_total;
  p.passes = (p.bits_total + kSortMaxBits - 1) / kSortMaxBits;
  p.bits_per_pass = (p.bits_total + p.passes - 1) / p.passes;
  p.tiles = nnz > 0 ? (nnz + kSortTile - 1) / kSortTile : 1;
  p.count_len = p.tiles << p.bits_per_pass;
  p.count_tiles = (p.count_len + kScanTile - 1) / kScanTile;
  const size_t n4 = ((size_t)(nnz > 0 ? nnz : 1) * 4 + 255) & ~(size_t)255;   // one int/float array, 256-byte aligned
  size_t at = 0;
  p.off_rowid = at; at += n4;
  p.off_val = at; at += n4;
  p.off_keys_a = at; at += n4;
  p.off_keys_x = at; at += n4;
  p.off_rows_x = at; at += n4;
  p.off_vals_x = at; at += n4;
  p.off_counts = at; at += ((size_t)p.count_len * 4 + 255) & ~(size_t)255;
  p.off_sums = at; at += ((size_t)(p.count_tiles + 4) * 4 + 255) & ~(size_t)255;
  p.bytes = at;
  return p;
}

}  // namespace gespmm_detail
