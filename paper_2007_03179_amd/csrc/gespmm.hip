// C ABI of the MI355X (gfx950) CSR SpMM / SpMM-like library (declared in include/gespmm.h).
// The kernels and launch helpers are in gespmm_kernels.hpp; this file validates arguments,
// fills the launch descriptions and owns no device code of its own.
#include "gespmm_kernels.hpp"
#include "gespmm_sort.hpp"
#include "gespmm_calibration.hpp"
#include "gespmm_rtc.hpp"

#include <mutex>
#include <new>

using namespace gespmm_detail;

extern "C" {

struct gespmm_profiler : gespmm_detail::Profiler {};

static int element_bytes(int b_dtype) { return b_dtype == GESPMM_F32 ? 4 : 2; }
static bool known_dtype(int b_dtype) { return b_dtype == GESPMM_F32 || b_dtype == GESPMM_BF16 || b_dtype == GESPMM_F16; }

int gespmm_plan_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, int aligned16, int b_dtype, size_t workspace_bytes,
                   const gespmm_tuning_t* tuning, gespmm_plan_t* out) {
  if (!out) return GESPMM_ERR_NULL;
  if (M < 0 || K < 0 || N < 0 || nnz < 0 || !known_dtype(b_dtype)) return GESPMM_ERR_BAD_ARG;
  Tuning tune;
  const int parsed = parse_tuning(tuning, &tune);
  if (parsed != GESPMM_OK) return parsed;
  make_plan(M, K, N, nnz, aligned16 != 0, element_bytes(b_dtype), tune, workspace_bytes, out);
  return GESPMM_OK;
}

int gespmm_plan(int64_t M, int64_t N, int64_t nnz, int aligned16, gespmm_plan_t* out) {
  return gespmm_plan_ex(M, 0, N, nnz, aligned16, GESPMM_F32, 0, nullptr, out);
}

int gespmm_plan_b16(int64_t M, int64_t N, int64_t nnz, int aligned16, int b_dtype, gespmm_plan_t* out) {
  return gespmm_plan_ex(M, 0, N, nnz, aligned16, b_dtype, 0, nullptr, out);
}

size_t gespmm_csr_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t nnz, int b_dtype, const gespmm_tuning_t* tuning) {
  gespmm_plan_t plan;
  if (gespmm_plan_ex(M, K, N, nnz, 1, b_dtype, (size_t)-1, tuning, &plan) != GESPMM_OK) return 0;
  return (size_t)plan.workspace_bytes;
}

int gespmm_profiler_create(int capacity, gespmm_profiler_t** out) {
  if (!out) return GESPMM_ERR_NULL;
  *out = nullptr;
  if (capacity <= 0) return GESPMM_ERR_BAD_ARG;
  gespmm_profiler* p = new (std::nothrow) gespmm_profiler();
  if (!p) return GESPMM_ERR_HIP;
  p->start.assign(capacity, nullptr);
  p->stop.assign(capacity, nullptr);
  for (int i = 0; i < capacity; ++i) {
    if (hipEventCreate(&p->start[i]) != hipSuccess || hipEventCreate(&p->stop[i]) != hipSuccess) {
      for (int j = 0; j <= i; ++j) {              // release what was created before the failure
        if (p->start[j]) (void)hipEventDestroy(p->start[j]);
        if (p->stop[j]) (void)hipEventDestroy(p->stop[j]);
      }
      delete p;
      return GESPMM_ERR_HIP;
    }
  }
  *out = p;
  return GESPMM_OK;
}

int gespmm_profiler_finish(gespmm_profiler_t* p, double* main_kernel_ms_sum, int* launches) {
  if (!p) return GESPMM_ERR_NULL;
  double total = 0.0;
  int status = GESPMM_OK;
  for (int i = 0; i < p->used; ++i) {
    float ms = 0.0f;
    if (hipEventSynchronize(p->stop[i]) != hipSuccess || hipEventElapsedTime(&ms, p->start[i], p->stop[i]) != hipSuccess)
      status = GESPMM_ERR_HIP;
    total += ms;
  }
  for (size_t i = 0; i < p->start.size(); ++i) {
    (void)hipEventDestroy(p->start[i]);
    (void)hipEventDestroy(p->stop[i]);
  }
  if (main_kernel_ms_sum) *main_kernel_ms_sum = total;
  if (launches) *launches = p->used;
  delete p;
  return status;
}

int gespmm_csr_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                  const float* vals, const void* B, int b_dtype, float* C, int op, void* workspace,
                  size_t workspace_bytes, const gespmm_tuning_t* tuning, gespmm_profiler_t* profiler, void* stream_) {
  if (!known_dtype(b_dtype)) return GESPMM_ERR_BAD_ARG;
  const int st = validate(M, K, N, nnz, rowptr, colind, B, C, op);
  if (st != GESPMM_OK || M == 0 || N == 0) return st;
  ChunkLaunch L;
  const int parsed = parse_tuning(tuning, &L.tuning);
  if (parsed != GESPMM_OK) return parsed;
  const int job = op == GESPMM_MAX ? kJobMax : (op == GESPMM_MIN ? kJobMin : kJobAdd);
  float identity = 0.0f;
  if (job == kJobMax) identity = -__builtin_inff();
  if (job == kJobMin) identity = __builtin_inff();
  L.job = job;
  L.b_dtype = b_dtype;
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = static_cast<const float*>(B); L.dense_out = C;
  L.is_mean = op == GESPMM_MEAN;
  L.init_target = C; L.empty_value = 0.0f; L.split_value = identity;
  L.profiler = profiler;
  L.workspace = workspace; L.workspace_bytes = workspace ? workspace_bytes : 0;
  return launch_chunks(L, (hipStream_t)stream_);
}

int gespmm_csr(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
               const int32_t* colind, const float* vals, const float* B, float* C, int op,
               void* stream_) {
  return gespmm_csr_ex(M, K, N, nnz, rowptr, colind, vals, B, GESPMM_F32, C, op, nullptr, 0, nullptr, nullptr, stream_);
}

int gespmm_csr_b16(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                   const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                   int op, void* stream_) {
  return gespmm_csr_ex(M, K, N, nnz, rowptr, colind, vals, B, b_dtype, C, op, nullptr, 0, nullptr, nullptr, stream_);
}

int gespmm_csr_arg(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                   const int32_t* colind, const float* vals, const float* B, float* C, int32_t* arg,
                   int op, void* stream_) {
  return gespmm_csr_arg_ex(M, K, N, nnz, rowptr, colind, vals, B, GESPMM_F32, C, arg, op, nullptr, stream_);
}

int gespmm_csr_arg_b16(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                       const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                       int32_t* arg, int op, void* stream_) {
  return gespmm_csr_arg_ex(M, K, N, nnz, rowptr, colind, vals, B, b_dtype, C, arg, op, nullptr, stream_);
}

int gespmm_csr_arg_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                      int32_t* arg, int op, const gespmm_tuning_t* tuning, void* stream) {
  gespmm_tuning_t no_phases;
  if (tuning) {
    no_phases = *tuning;
    no_phases.k_parts = 1;
  }
  return gespmm_csr_arg_ws(M, K, N, nnz, rowptr, colind, vals, B, b_dtype, C, arg, op, nullptr, 0, tuning ? &no_phases : nullptr, stream);
}

int gespmm_csr_arg_ws(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const void* B_, int b_dtype, float* C,
                      int32_t* arg, int op, void* workspace, size_t workspace_bytes,
                      const gespmm_tuning_t* tuning, void* stream_) {
  if (!known_dtype(b_dtype)) return GESPMM_ERR_BAD_ARG;
  const float* B = static_cast<const float*>(B_);
  if (op != GESPMM_MAX && op != GESPMM_MIN) return GESPMM_ERR_BAD_ARG;
  const int st = validate(M, K, N, nnz, rowptr, colind, B, C, op);
  if (st != GESPMM_OK || M == 0 || N == 0) return st;
  if (!arg) return GESPMM_ERR_NULL;
  // One fused pass gives value and position for every row that lies inside one chunk.
  hipStream_t stream = (hipStream_t)stream_;
  ChunkLaunch L;
  const int parsed = parse_tuning(tuning, &L.tuning);
  if (parsed != GESPMM_OK) return parsed;
  L.job = op == GESPMM_MAX ? kJobMaxWithArg : kJobMinWithArg;
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = B; L.dense_out = C; L.arg = arg;
  L.b_dtype = b_dtype;
  L.also_aligned = arg;
  L.init_target = C;
  L.init2_target = reinterpret_cast<float*>(arg);
  L.empty_value = 0.0f;
  L.empty2_value = bits_as_float(-1);
  // Rows split across chunks.  Vector kernels, N <= 1024: their (value, position) pairs are
  // combined as packed 64-bit words kept in the row's own C and arg storage (preset to zero)
  // and unpacked by a small kernel after the pass.  Otherwise: values by atomics in this pass
  // (rows preset to the reduce identity / INT_MAX), positions by a second pass over the matrix.
  const bool vector = N % 4 == 0 && (((uintptr_t)B | (uintptr_t)C | (uintptr_t)arg) & 15u) == 0;
  L.packed_split = vector && N <= kWave * kFinishWords && nnz > 0;
  const bool phases_possible = L.packed_split && b_dtype == GESPMM_F32;
  if (L.tuning.k_parts > 1 && nnz > 0) {            // phases were asked for
    if (!phases_possible) return GESPMM_ERR_BAD_ARG;
    if (!workspace) return GESPMM_ERR_WORKSPACE;
  }
  if (!phases_possible || !workspace) L.tuning.k_parts = 1;
  if (L.packed_split) {
    L.split_value = 0.0f;
    L.split2_value = 0.0f;
    if (phases_possible && workspace) {
      L.workspace = workspace;
      L.workspace_bytes = workspace_bytes;
    }
    return launch_chunks(L, stream);
  }
  L.split_value = op == GESPMM_MAX ? -__builtin_inff() : __builtin_inff();
  L.split2_value = bits_as_float(INT32_MAX);
  bool whole_rows = false;
  const int fused = launch_chunks(L, stream, &whole_rows);
  if (fused != GESPMM_OK || nnz == 0 || whole_rows) return fused;
  // Second pass, split rows only (their values are final once the first kernel has ended):
  // entries whose product has the bits of C[i, j] compete by atomic min on their index.
  ChunkLaunch S;
  S.tuning = L.tuning;
  S.job = kJobArg;
  S.M = M; S.K = K; S.N = N; S.nnz = nnz;
  S.rowptr = rowptr; S.colind = colind; S.vals = vals;
  S.dense_in = B; S.result_in = C; S.arg = arg;
  S.b_dtype = b_dtype;
  S.also_aligned = arg;
  S.only_split = true;
  return launch_chunks(S, stream);
}

int gespmm_csr_transposed(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                          const int32_t* colind, const float* vals, const float* dC, float* dB, int op,
                          void* stream_) {
  if (op != GESPMM_SUM && op != GESPMM_MEAN) return GESPMM_ERR_BAD_ARG;
  if (M < 0 || K < 0 || N < 0 || nnz < 0) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX || K > INT32_MAX || nnz > INT32_MAX - (1 << kMaxChunkShift) || N > INT32_MAX / 8) return GESPMM_ERR_TOO_LARGE;
  if (nnz > 0 && (M == 0 || K == 0)) return GESPMM_ERR_BAD_ARG;
  if (K == 0 || N == 0) return GESPMM_OK;
  if (!dB) return GESPMM_ERR_NULL;
  if (nnz > 0 && (!rowptr || !colind || !dC)) return GESPMM_ERR_NULL;
  hipStream_t stream = (hipStream_t)stream_;
  const int fill = launch_fill(dB, K * N, 0.0f, stream);
  if (fill != GESPMM_OK || nnz == 0) return fill;
  ChunkLaunch L;
  L.job = kJobTransposed;
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = dC; L.dense_out = dB;
  L.is_mean = op == GESPMM_MEAN;
  return launch_chunks(L, stream);
}

size_t gespmm_csr_transpose_workspace_bytes(int64_t K) {
  if (K < 0) return 0;
  const int64_t tiles = (K + 1 + kScanTile - 1) / kScanTile;
  return (size_t)(K + tiles + 4) * sizeof(int32_t);
}

// Argument checks shared by the two counter-based transpose entry points (everything but the scratch memory).
static int check_transpose_args(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                int32_t* rowptrT, int32_t* colindT, float* valsT) {
  if (M < 0 || K < 0 || nnz < 0) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX || K >= INT32_MAX || nnz > INT32_MAX - (1 << kMaxChunkShift)) return GESPMM_ERR_TOO_LARGE;
  if (nnz > 0 && (M == 0 || K == 0)) return GESPMM_ERR_BAD_ARG;
  if (!rowptrT) return GESPMM_ERR_NULL;
  if (nnz > 0 && (!rowptr || !colind || !colindT || !valsT)) return GESPMM_ERR_NULL;
  return GESPMM_OK;
}

// The counter-based transpose on a scratch buffer of gespmm_csr_transpose_workspace_bytes(K) bytes
// (cursors, then one total per scan tile).  Every word of the scratch that is read was written earlier
// in the same call, so stale contents do no harm.
static int transpose_with_counters(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                   const float* vals, int scale_by_row_length, int32_t* rowptrT, int32_t* colindT,
                                   float* valsT, void* scratch_memory, hipStream_t stream) {
  int32_t* cursor = static_cast<int32_t*>(scratch_memory);     // K entries
  int32_t* sums = cursor + K;                                  // one per scan tile
  const int64_t n = K + 1;
  const int64_t tiles = (n + kScanTile - 1) / kScanTile;

  // column counts -> exclusive scan -> row starts of the transposed matrix (and the cursors)
  int st = launch_fill(reinterpret_cast<float*>(rowptrT), n, 0.0f, stream);
  if (st != GESPMM_OK) return st;
  if (nnz > 0) {
    int64_t blocks = (nnz + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(count_columns, dim3((unsigned)blocks), dim3(kBlock), 0, stream, nnz, colind, rowptrT);
  }
  hipLaunchKernelGGL(scan_tiles, dim3((unsigned)tiles), dim3(kBlock), 0, stream, rowptrT, n, sums);
  hipLaunchKernelGGL(scan_sums, dim3(1), dim3(kBlock), 0, stream, sums, tiles);
  {
    int64_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(add_tile_offsets, dim3((unsigned)blocks), dim3(kBlock), 0, stream, rowptrT, n, sums, cursor, K);
  }
  if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
  if (nnz == 0) return GESPMM_OK;

  // every stored entry takes the next free place of its column's row
  ChunkLaunch L;
  L.job = kJobScatter;
  L.M = M; L.K = K; L.N = 1; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_out = valsT; L.arg = colindT; L.cursor = cursor;
  L.is_mean = scale_by_row_length != 0;
  L.one_lane_per_entry = true;
  return launch_chunks(L, stream);
}

int gespmm_csr_transpose(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                         const float* vals, int scale_by_row_length, int32_t* rowptrT, int32_t* colindT,
                         float* valsT, void* workspace, size_t workspace_bytes, void* stream_) {
  const int st = check_transpose_args(M, K, nnz, rowptr, colind, rowptrT, colindT, valsT);
  if (st != GESPMM_OK) return st;
  if (!workspace) return GESPMM_ERR_NULL;
  if (workspace_bytes < gespmm_csr_transpose_workspace_bytes(K) || ((uintptr_t)workspace & 3u) != 0) return GESPMM_ERR_WORKSPACE;
  return transpose_with_counters(M, K, nnz, rowptr, colind, vals, scale_by_row_length, rowptrT, colindT, valsT,
                                 workspace, (hipStream_t)stream_);
}

// ---- the entry point that allocates nothing ---------------------------------------------------
// Scratch memory of the counter-based transpose for up to GESPMM_NOALLOC_TRANSPOSE_MAX_K columns, held
// by every GPU the library runs on until the process ends.  In host code the array's name is only a
// stand-in for the symbol; its device address comes from hipGetSymbolAddress, once per device.
constexpr int64_t kNoAllocMaxK = GESPMM_NOALLOC_TRANSPOSE_MAX_K;
constexpr size_t kNoAllocScratchBytes =
    (size_t)(kNoAllocMaxK + (kNoAllocMaxK + 1 + kScanTile - 1) / kScanTile + 4) * sizeof(int32_t);
static __device__ __align__(256) unsigned char scratch[(kNoAllocScratchBytes + 255) / 256 * 256];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_address[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call on that device).
static int scratch_of_current_device(void** out) {
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return GESPMM_ERR_HIP;
  std::lock_guard<std::mutex> hold(g_scratch_mutex);
  if (!g_scratch_address[device]) {
    void* address = nullptr;
    if (hipGetSymbolAddress(&address, HIP_SYMBOL(scratch)) != hipSuccess || !address) return GESPMM_ERR_HIP;
    g_scratch_address[device] = address;
  }
  *out = g_scratch_address[device];
  return GESPMM_OK;
}

int gespmm_csr_transpose_noalloc(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                 const float* vals, int scale_by_row_length, int32_t* rowptrT, int32_t* colindT,
                                 float* valsT, void* stream_) {
  const int st = check_transpose_args(M, K, nnz, rowptr, colind, rowptrT, colindT, valsT);
  if (st != GESPMM_OK) return st;
  if (K > kNoAllocMaxK) return GESPMM_ERR_SCRATCH_LIMIT;
  static_assert(sizeof(scratch) >= kNoAllocScratchBytes, "scratch array too small for the stated maximum");
  void* memory = nullptr;
  const int found = scratch_of_current_device(&memory);
  if (found != GESPMM_OK) return found;
  return transpose_with_counters(M, K, nnz, rowptr, colind, vals, scale_by_row_length, rowptrT, colindT, valsT,
                                 memory, (hipStream_t)stream_);
}

size_t gespmm_csr_transpose_sorted_workspace_bytes(int64_t K, int64_t nnz) {
  if (K < 0 || nnz < 0) return 0;
  return make_sort_plan(K, nnz).bytes;
}

int gespmm_csr_transpose_sorted(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                const float* vals, int scale_by_row_length, int32_t* rowptrT, int32_t* colindT,
                                float* valsT, void* workspace, size_t workspace_bytes, void* stream_) {
  if (M < 0 || K < 0 || nnz < 0) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX || K >= INT32_MAX || nnz > INT32_MAX - (1 << kMaxChunkShift)) return GESPMM_ERR_TOO_LARGE;
  if (nnz > 0 && (M == 0 || K == 0)) return GESPMM_ERR_BAD_ARG;
  if (!rowptrT) return GESPMM_ERR_NULL;
  if (nnz > 0 && (!rowptr || !colind || !colindT || !valsT)) return GESPMM_ERR_NULL;
  if (!workspace) return GESPMM_ERR_NULL;
  const SortPlan plan = make_sort_plan(K, nnz);
  if (workspace_bytes < plan.bytes || ((uintptr_t)workspace & 3u) != 0) return GESPMM_ERR_WORKSPACE;
  hipStream_t stream = (hipStream_t)stream_;
  if (nnz == 0) return launch_fill(reinterpret_cast<float*>(rowptrT), K + 1, 0.0f, stream);

  char* ws = static_cast<char*>(workspace);
  int32_t* rowid = reinterpret_cast<int32_t*>(ws + plan.off_rowid);
  float* weight = reinterpret_cast<float*>(ws + plan.off_val);
  int32_t* keys_a = reinterpret_cast<int32_t*>(ws + plan.off_keys_a);
  int32_t* keys_x = reinterpret_cast<int32_t*>(ws + plan.off_keys_x);
  int32_t* rows_x = reinterpret_cast<int32_t*>(ws + plan.off_rows_x);
  float* vals_x = reinterpret_cast<float*>(ws + plan.off_vals_x);
  int32_t* counts = reinterpret_cast<int32_t*>(ws + plan.off_counts);
  int32_t* sums = reinterpret_cast<int32_t*>(ws + plan.off_sums);

  // (1) row index and weight of every stored entry, in entry order (the chunk walk, one lane per entry)
  ChunkLaunch L;
  L.job = kJobScatter;
  L.M = M; L.K = K; L.N = 1; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_out = weight; L.arg = rowid; L.cursor = nullptr;
  L.is_mean = scale_by_row_length != 0;
  L.one_lane_per_entry = true;
  int st = launch_chunks(L, stream);
  if (st != GESPMM_OK) return st;

  // (2) stable radix sort of (column, row, weight) by column, least significant digit first; the buffers
  //     alternate so that the last pass writes the caller's arrays
  const int32_t* keys_in = colind;
  const int32_t* rows_in = rowid;
  const float* vals_in = weight;
  bool to_caller = plan.passes % 2 == 1;
  const unsigned tiles = (unsigned)plan.tiles;
  for (int pass = 0; pass < plan.passes; ++pass) {
    const int shift = pass * plan.bits_per_pass;
    int32_t* keys_out = to_caller ? keys_a : keys_x;
    int32_t* rows_out = to_caller ? colindT : rows_x;
    float* vals_out = to_caller ? valsT : vals_x;
    hipLaunchKernelGGL(radix_histogram, dim3(tiles), dim3(kBlock), 0, stream, keys_in, nnz, shift, plan.bits_per_pass,
                       plan.tiles, counts);
    hipLaunchKernelGGL(scan_tiles, dim3((unsigned)plan.count_tiles), dim3(kBlock), 0, stream, counts, plan.count_len, sums);
    hipLaunchKernelGGL(scan_sums, dim3(1), dim3(kBlock), 0, stream, sums, plan.count_tiles);
    {
      int64_t blocks = (plan.count_len + kBlock - 1) / kBlock;
      if (blocks > 256 * 32) blocks = 256 * 32;
      hipLaunchKernelGGL(add_tile_offsets, dim3((unsigned)blocks), dim3(kBlock), 0, stream, counts, plan.count_len, sums,
                         (int32_t*)nullptr, (int64_t)0);
    }
    hipLaunchKernelGGL(radix_scatter, dim3(tiles), dim3(kBlock), 0, stream, keys_in, rows_in, vals_in, nnz, shift,
                       plan.bits_per_pass, plan.tiles, counts, keys_out, rows_out, vals_out);
    if (hipGetLastError() != hipSuccess) return GESPMM_ERR_HIP;
    keys_in = keys_out; rows_in = rows_out; vals_in = vals_out;
    to_caller = !to_caller;
  }

  // (3) row starts of the transposed matrix from the sorted columns
  {
    int64_t blocks = (K + 1 + kBlock - 1) / kBlock;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(row_starts_from_sorted_keys, dim3((unsigned)blocks), dim3(kBlock), 0, stream, keys_in, nnz, K, rowptrT);
  }
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

int gespmm_pool_backward(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* colind,
                         const float* vals, const int32_t* arg, const float* dC, float* dB,
                         void* stream_) {
  if (M < 0 || K < 0 || N < 0 || nnz < 0) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX || K > INT32_MAX || nnz > INT32_MAX || N > INT32_MAX / 8) return GESPMM_ERR_TOO_LARGE;
  if (K == 0 || N == 0) return GESPMM_OK;
  if (!dB) return GESPMM_ERR_NULL;
  if (M > 0 && (!arg || !dC)) return GESPMM_ERR_NULL;
  if (nnz > 0 && M > 0 && !colind) return GESPMM_ERR_NULL;
  hipStream_t stream = (hipStream_t)stream_;
  const int fill = launch_fill(dB, K * N, 0.0f, stream);
  if (fill != GESPMM_OK || M == 0 || nnz == 0) return fill;
  const int64_t total = M * N;
  int64_t blocks = (total + kBlock - 1) / kBlock;
  if (blocks > 256 * 64) blocks = 256 * 64;
  hipLaunchKernelGGL(pool_backward_scatter, dim3((unsigned)blocks), dim3(kBlock), 0, stream, total, (int32_t)N,
                     colind, vals, arg, dC, dB);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

int gespmm_csr_simple(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colind,
                      const float* vals, const float* B, float* C, int op, void* stream_) {
  if (M < 0 || K < 0 || N < 0) return GESPMM_ERR_BAD_ARG;
  if (M >= INT32_MAX) return GESPMM_ERR_TOO_LARGE;
  if (M == 0 || N == 0) return validate(M, K, N, 0, rowptr, colind, B, C, op);
  if (!rowptr) return GESPMM_ERR_NULL;
  hipStream_t stream = (hipStream_t)stream_;
  int32_t nnz = 0;
  if (hipMemcpyAsync(&nnz, rowptr + M, sizeof(nnz), hipMemcpyDeviceToHost, stream) != hipSuccess) return GESPMM_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return GESPMM_ERR_HIP;
  return gespmm_csr(M, K, N, nnz, rowptr, colind, vals, B, C, op, stream_);
}

int gespmm_calibration_copy(const void* src, void* dst, int64_t bytes, void* stream_) {
  if (bytes < 0 || bytes % 16 != 0) return GESPMM_ERR_BAD_ARG;
  if (bytes == 0) return GESPMM_OK;
  if (!src || !dst) return GESPMM_ERR_NULL;
  if ((((uintptr_t)src | (uintptr_t)dst) & 15u) != 0) return GESPMM_ERR_BAD_ARG;
  const int64_t n4 = bytes / 16;
  int64_t blocks = (n4 + kBlock - 1) / kBlock;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(copy_f4, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream_,
                     (const float4*)src, (float4*)dst, n4);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

int gespmm_calibration_gather(const void* table, int64_t table_lines, const int32_t* idx, int64_t n, void* out,
                              int64_t out_bytes, void* stream_) {
  if (table_lines < 0 || n < 0 || out_bytes < 0) return GESPMM_ERR_BAD_ARG;
  if (n == 0) return GESPMM_OK;
  if (!table || !idx || !out) return GESPMM_ERR_NULL;
  if (table_lines == 0 || table_lines > INT32_MAX) return GESPMM_ERR_BAD_ARG;
  if ((((uintptr_t)table | (uintptr_t)out) & 15u) != 0) return GESPMM_ERR_BAD_ARG;
  int64_t blocks = (n + kBlock - 1) / kBlock;              // 8 lanes per gather, 8 gathers per step
  if (blocks > 256 * 32) blocks = 256 * 32;
  if (out_bytes < blocks * kBlock * 16) return GESPMM_ERR_BAD_ARG;
  hipLaunchKernelGGL(gather_lines, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream_,
                     (const float4*)table, idx, n, (float4*)out);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

int gespmm_calibration_gather_shape(const void* table, int64_t table_bytes, int row_bytes, const int32_t* idx, int64_t n,
                                    int lanes_per_row, int load_bytes, int in_flight, int cache_policy, void* out,
                                    int64_t out_bytes, void* stream_) {
  if (table_bytes < 0 || n < 0 || out_bytes < 0 || row_bytes <= 0 || row_bytes % 4 != 0) return GESPMM_ERR_BAD_ARG;
  if (n == 0) return GESPMM_OK;
  if (!table || !idx || !out) return GESPMM_ERR_NULL;
  if (load_bytes != 4 && load_bytes != 8 && load_bytes != 16) return GESPMM_ERR_BAD_ARG;
  if (lanes_per_row <= 0 || (int64_t)lanes_per_row * load_bytes > row_bytes) return GESPMM_ERR_BAD_ARG;
  if (table_bytes < row_bytes || table_bytes % row_bytes != 0 || table_bytes >= (4ll << 30)) return GESPMM_ERR_BAD_ARG;
  if ((((uintptr_t)table | (uintptr_t)out) & 15u) != 0 || row_bytes % load_bytes != 0) return GESPMM_ERR_BAD_ARG;
  GatherKernel kernel = pick_gather(lanes_per_row, load_bytes / 4, in_flight, cache_policy);
  if (!kernel) return GESPMM_ERR_BAD_ARG;
  const int64_t blocks = 256 * 8;                  // eight workgroups per compute unit
  if (out_bytes < blocks * kBlock * 4) return GESPMM_ERR_BAD_ARG;
  hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream_, (const char*)table,
                     (uint32_t)table_bytes, row_bytes, idx, n, (float*)out);
  return hipGetLastError() == hipSuccess ? GESPMM_OK : GESPMM_ERR_HIP;
}

static void copy_log(const std::string& text, char* log, size_t log_bytes) {
  if (!log || log_bytes == 0) return;
  const size_t n = text.size() < log_bytes - 1 ? text.size() : log_bytes - 1;
  std::memcpy(log, text.data(), n);
  log[n] = '\0';
}

int gespmm_custom_op_create(const char* source, const char* name, gespmm_custom_op_t** out, char* log, size_t log_bytes) {
  if (log && log_bytes > 0) log[0] = '\0';
  if (!source || !name || !out) return GESPMM_ERR_NULL;
  *out = nullptr;
  if (!is_identifier(name)) return GESPMM_ERR_BAD_ARG;
  gespmm_custom_op* op = new (std::nothrow) gespmm_custom_op;
  if (!op) return GESPMM_ERR_HIP;
  hipDeviceProp_t prop;
  if (hipGetDevice(&op->device) != hipSuccess || hipGetDeviceProperties(&prop, op->device) != hipSuccess) {
    delete op;
    return GESPMM_ERR_HIP;
  }
  op->arch = prop.gcnArchName;
  op->name = name;
  op->source = std::string("#include \"gespmm_device.hpp\"\n#line 1 \"user_reduce\"\n") + source + "\n";
  // identity(): read back once through a one-thread kernel (also the first check that the text compiles)
  std::string text;
  std::vector<char> code;
  std::string symbol;
  const std::string probe = op->source + "extern \"C\" __global__ void gespmm_identity_of(float* out) { *out = " + op->name +
                            "::identity(); }\n";
  int status = rtc_compile(probe, op->arch, "", "gespmm_identity_of", &code, &symbol, &text);
  if (status == GESPMM_OK) {
    hipModule_t module = nullptr;
    hipFunction_t function = nullptr;
    float* device_value = nullptr;
    status = GESPMM_ERR_HIP;
    if (hipModuleLoadData(&module, code.data()) == hipSuccess) {
      if (hipModuleGetFunction(&function, module, symbol.c_str()) == hipSuccess &&
          hipMalloc(reinterpret_cast<void**>(&device_value), sizeof(float)) == hipSuccess) {
        void* params[] = {&device_value};
        if (hipModuleLaunchKernel(function, 1, 1, 1, 1, 1, 1, 0, nullptr, params, nullptr) == hipSuccess &&
            hipMemcpy(&op->identity, device_value, sizeof(float), hipMemcpyDeviceToHost) == hipSuccess)
          status = GESPMM_OK;
        (void)hipFree(device_value);
      }
      (void)hipModuleUnload(module);
    }
  }
  // step() and merge(): build the most common kernel shape now, so that a mistake in them is reported here
  if (status == GESPMM_OK) {
    hipFunction_t function = nullptr;
    status = op->kernel_for(4, 8, 1, false, &function, &text);
  }
  copy_log(text, log, log_bytes);
  if (status != GESPMM_OK) {
    gespmm_custom_op_destroy(op);
    return status;
  }
  *out = op;
  return GESPMM_OK;
}

int gespmm_custom_op_check(const char* source, const char* name, const char* arch, char* log, size_t log_bytes) {
  if (log && log_bytes > 0) log[0] = '\0';
  if (!source || !name) return GESPMM_ERR_NULL;
  if (!is_identifier(name)) return GESPMM_ERR_BAD_ARG;
  const std::string text = std::string("#include \"gespmm_device.hpp\"\n#line 1 \"user_reduce\"\n") + source + "\n" +
                           "extern \"C\" __global__ void gespmm_identity_of(float* out) { *out = " + name + "::identity(); }\n";
  const std::string expression = std::string("gespmm_detail::chunk_kernel<gespmm_detail::CustomRows<") + name + ", 4, 1>, 4, 8, 1, false, false>";
  std::vector<char> code;
  std::string symbol, messages;
  const int status = rtc_compile(text, arch && *arch ? arch : "gfx950", expression, "", &code, &symbol, &messages);
  copy_log(messages, log, log_bytes);
  return status;
}

int gespmm_custom_op_destroy(gespmm_custom_op_t* op) {
  if (!op) return GESPMM_OK;
  int status = GESPMM_OK;
  for (auto& entry : op->kernels)
    if (hipModuleUnload(entry.second.module) != hipSuccess) status = GESPMM_ERR_HIP;
  delete op;
  return status;
}

int gespmm_csr_custom(gespmm_custom_op_t* op, int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const float* B, float* C,
                      const gespmm_tuning_t* tuning, void* stream_) {
  if (!op) return GESPMM_ERR_NULL;
  const int st = validate(M, K, N, nnz, rowptr, colind, B, C, GESPMM_SUM);
  if (st != GESPMM_OK || M == 0 || N == 0) return st;
  int device = -1;
  if (hipGetDevice(&device) != hipSuccess) return GESPMM_ERR_HIP;
  if (device != op->device) return GESPMM_ERR_BAD_ARG;      // its kernels are loaded on the device it was created on
  ChunkLaunch L;
  const int parsed = parse_tuning(tuning, &L.tuning);
  if (parsed != GESPMM_OK) return parsed;
  L.launcher = &rtc_launch;
  L.launcher_context = op;
  L.M = M; L.K = K; L.N = N; L.nnz = nnz;
  L.rowptr = rowptr; L.colind = colind; L.vals = vals;
  L.dense_in = B; L.dense_out = C;
  L.init_target = C; L.empty_value = 0.0f; L.split_value = op->identity;
  return launch_chunks(L, (hipStream_t)stream_);
}

const char* gespmm_status_string(int status) {
  switch (status) {
    case GESPMM_OK: return "ok";
    case GESPMM_ERR_BAD_ARG: return "bad argument (negative size, unknown op, or no kernel for the forced tuning)";
    case GESPMM_ERR_NULL: return "a required pointer is NULL";
    case GESPMM_ERR_TOO_LARGE: return "M, K or nnz does not fit 32-bit indices";
    case GESPMM_ERR_WORKSPACE: return "the workspace is too small or misaligned";
    case GESPMM_ERR_HIP: return "a HIP call failed";
    case GESPMM_ERR_SCRATCH_LIMIT:
      return "the problem needs more scratch memory than the built-in buffer of the no-allocation entry point holds";
    case GESPMM_ERR_COMPILE: return "the source of a user-defined reduce operation did not compile (see the log)";
    case GESPMM_ERR_NO_RTC: return "the run-time compiler library (libhiprtc.so) could not be loaded";
    default: return "unknown status";
  }
}

int gespmm_version(void) { return 100; }

}  // extern "C"
