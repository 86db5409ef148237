// Two user-defined SpMM-like operations built on include/gespmm_custom.hpp; used by
// tests/test_gpu_custom_op.py to check the compile-time reduce mechanism end to end.
#include "gespmm_custom.hpp"

namespace {

// C[i, j] = sum_p (vals[p] * B[colind[p], j])^2
struct SumOfSquares {
  static __host__ __device__ float identity() { return 0.0f; }
  static __device__ float step(float acc, float a, float b) {
    const float x = a * b;
    return acc + x * x;
  }
  static __device__ float merge(float x, float y) { return x + y; }
};

// C[i, j] = max_p |vals[p] * B[colind[p], j]|
struct MaxMagnitude {
  static __host__ __device__ float identity() { return 0.0f; }      // |x| >= 0
  static __device__ float step(float acc, float a, float b) { return __builtin_fmaxf(acc, __builtin_fabsf(a * b)); }
  static __device__ float merge(float x, float y) { return __builtin_fmaxf(x, y); }
};

}  // namespace

extern "C" {

int custom_sum_of_squares(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                          const float* vals, const float* B, float* C, void* stream) {
  return gespmm::csr_custom<SumOfSquares>(M, K, N, nnz, rowptr, colind, vals, B, C, (hipStream_t)stream);
}

// the same with the caller's bound on the longest row: the whole-row path (one launch, no compare-and-swap combine)
int custom_sum_of_squares_bounded(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                                  const float* vals, const float* B, float* C, void* stream, int longest_row) {
  gespmm_tuning_t tuning = {-1, -1, -1, -1, -1, -1, longest_row, -1};
  return gespmm::csr_custom<SumOfSquares>(M, K, N, nnz, rowptr, colind, vals, B, C, (hipStream_t)stream, &tuning);
}

int custom_max_magnitude(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                         const float* vals, const float* B, float* C, void* stream) {
  return gespmm::csr_custom<MaxMagnitude>(M, K, N, nnz, rowptr, colind, vals, B, C, (hipStream_t)stream);
}

}  // extern "C"
