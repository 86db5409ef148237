/*
 * CPU oracle for CSR SpMM and the SpMM-like reductions (sum, mean, max, min).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * GPU library is checked against; the product never calls it.  It shares no
 * code with the GPU path.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may use it.
 *
 * What it computes is the plain definition of the result (Algorithm 1 of the
 * paper, with the walk-through of Section III-A): for every output row i and
 * column j, walk the stored entries p of row i in storage order, form
 * vals[p] * B[colind[p], j], and fold the products with the reduction.  The
 * SpMM-like generalisation (Eq. 1, Section IV-A) swaps the initial value and
 * the fold, nothing else: the multiply stays for every op.
 *
 * Readings where the paper is silent:
 *   - mean divides by the number of STORED entries of the row;
 *   - an empty row yields 0 for every op;
 *   - max/min on signed zeros follow IEEE-754 maximum/minimum (+0 > -0);
 *   - columns need not be sorted or unique: repeated columns are separate terms;
 *   - vals == NULL means every stored value is 1.
 *
 * Arithmetic: every product of two fp32 numbers is formed in double (exact:
 * 24 x 24 significant bits fit in 53) and the fold runs in double.  Besides the
 * result, the oracle returns Sabs = sum_p |vals[p] * B[colind[p], j]| (divided
 * by the row length for mean), the scale of the fp32 error bound.
 *
 * The same file holds the three gradient-side references (position of the extreme for
 * max/min, the transposed product for sum/mean, the routed gradient of max/min).
 *
 * Pins (tests/test_oracle_pins.py): brute-force dense products and explicit
 * per-entry loops on tiny inputs, the identity matrix, an all-ones B, closed
 * forms, scipy's CSR product in float64, a hand-worked example, and a set of
 * planted single-token mistakes that the pins must all reject.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <omp.h>

enum { OP_SUM = 0, OP_MEAN = 1, OP_MAX = 2, OP_MIN = 3 };

/* IEEE-754 maximum / minimum on non-NaN doubles, +0 ordered above -0. */
static double fold_max(double acc, double x) {
  if (x > acc) return x;
  if (x == acc && !signbit(x)) return x;
  return acc;
}
static double fold_min(double acc, double x) {
  if (x < acc) return x;
  if (x == acc && signbit(x)) return x;
  return acc;
}

/* One output row: out_c[0..N) and out_s[0..N) for row i of A. */
static void oracle_row(int64_t i, int64_t N, const int32_t* rowptr, const int32_t* colind,
                       const float* vals, const float* B, int op, double* out_c, double* out_s) {
  const int64_t row_start = rowptr[i];
  const int64_t row_end = rowptr[i + 1];
  const int64_t len = row_end - row_start;
  for (int64_t j = 0; j < N; ++j) {
    if (len == 0) {
      out_c[j] = 0.0;
      out_s[j] = 0.0;
      continue;
    }
    double result = (op == OP_MAX) ? -INFINITY : (op == OP_MIN) ? INFINITY : 0.0;
    double sabs = 0.0;
    for (int64_t ptr = row_start; ptr < row_end; ++ptr) {
      const int64_t k = colind[ptr];
      const double a = vals ? (double)vals[ptr] : 1.0;
      const double x = a * (double)B[k * N + j];
      if (op == OP_MAX) result = fold_max(result, x);
      else if (op == OP_MIN) result = fold_min(result, x);
      else result += x;
      sabs += fabs(x);
    }
    if (op == OP_MEAN) {
      result /= (double)len;
      sabs /= (double)len;
    }
    out_c[j] = result;
    out_s[j] = sabs;
  }
}

/*
 * rows == NULL : all M rows; Cref and Sabs are M x N row-major.
 * rows != NULL : only the nrows listed rows, in list order; outputs are nrows x N.
 * threads <= 0 : use OpenMP's default.  Returns 0, or -1 on a bad argument.
 */
int spmm_oracle(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colind,
                const float* vals, const float* B, int op, const int64_t* rows, int64_t nrows,
                double* Cref, double* Sabs, int threads) {
  if (M < 0 || K < 0 || N < 0 || op < OP_SUM || op > OP_MIN) return -1;
  if (!rowptr || !Cref || !Sabs) return -1;
  const int64_t count = rows ? nrows : M;
  const int nt = threads > 0 ? threads : omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 256) num_threads(nt)
  for (int64_t r = 0; r < count; ++r) {
    const int64_t i = rows ? rows[r] : r;
    oracle_row(i, N, rowptr, colind, vals, B, op, Cref + r * N, Sabs + r * N);
  }
  return 0;
}

/*
 * max / min together with the position of the extreme: what routes the gradient of a pooling
 * aggregation (the GraphSAGE-pool use of the SpMM-like operation, Section V-E; the operator has
 * a gradient definition, Section IV-B).  The paper does not say which entry wins among equals;
 * the reading taken here refers to the fp32 result the operator returns: arg[i, j] is the index p
 * (into colind / vals) of the FIRST stored entry of row i, in storage order, whose product
 * vals[p] * B[colind[p], j], rounded once to fp32, has exactly the bits of C[i, j] rounded once to
 * fp32; -1 for an empty row.  (Two entries whose exact products differ but round to the same fp32
 * number are therefore equals, and the earlier one wins.)  The value is the same fold as above.
 */
static int same_bits32(float x, float y) {
  union { float f; uint32_t u; } ux, uy;
  ux.f = x;
  uy.f = y;
  return ux.u == uy.u;
}

static void oracle_row_arg(int64_t i, int64_t N, const int32_t* rowptr, const int32_t* colind,
                           const float* vals, const float* B, int op, double* out_c, int32_t* out_arg) {
  const int64_t row_start = rowptr[i];
  const int64_t row_end = rowptr[i + 1];
  for (int64_t j = 0; j < N; ++j) {
    if (row_end == row_start) {
      out_c[j] = 0.0;
      out_arg[j] = -1;
      continue;
    }
    double result = (op == OP_MAX) ? -INFINITY : INFINITY;
    for (int64_t ptr = row_start; ptr < row_end; ++ptr) {
      const int64_t k = colind[ptr];
      const double a = vals ? (double)vals[ptr] : 1.0;
      const double x = a * (double)B[k * N + j];
      result = (op == OP_MAX) ? fold_max(result, x) : fold_min(result, x);
    }
    const float target = (float)result;
    int64_t where = -1;
    for (int64_t ptr = row_start; ptr < row_end; ++ptr) {
      const int64_t k = colind[ptr];
      const double a = vals ? (double)vals[ptr] : 1.0;
      const double x = a * (double)B[k * N + j];
      if (where < 0 && same_bits32((float)x, target)) where = ptr;
    }
    out_c[j] = result;
    out_arg[j] = (int32_t)where;
  }
}

int spmm_oracle_arg(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colind,
                    const float* vals, const float* B, int op, const int64_t* rows, int64_t nrows,
                    double* Cref, int32_t* arg, int threads) {
  if (M < 0 || K < 0 || N < 0 || (op != OP_MAX && op != OP_MIN)) return -1;
  if (!rowptr || !Cref || !arg) return -1;
  const int64_t count = rows ? nrows : M;
  const int nt = threads > 0 ? threads : omp_get_max_threads();
#pragma omp parallel for schedule(dynamic, 256) num_threads(nt)
  for (int64_t r = 0; r < count; ++r) {
    const int64_t i = rows ? rows[r] : r;
    oracle_row_arg(i, N, rowptr, colind, vals, B, op, Cref + r * N, arg + r * N);
  }
  return 0;
}

/*
 * Gradient of sum / mean with respect to B, i.e. the product with the transposed sparse
 * matrix taken from the same CSR arrays (the backward pass of a graph convolution is again
 * an SpMM, Section I; gradient definition of the operator, Section IV-B):
 *     dB[k, j] = sum over stored entries p with colind[p] == k of  w_p * dC[row(p), j],
 *     w_p = vals[p] for sum, vals[p] / (stored length of row(p)) for mean.
 * Sabs[k, j] is the same sum over |w_p * dC|.  Columns j are independent, so the threads
 * split the columns; every thread walks all entries in storage order.
 */
int spmm_oracle_transposed(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colind,
                           const float* vals, const float* dC, int op, double* dBref, double* Sabs,
                           int threads) {
  if (M < 0 || K < 0 || N < 0 || (op != OP_SUM && op != OP_MEAN)) return -1;
  if (!rowptr || !dBref || !Sabs) return -1;
  const int nt = threads > 0 ? threads : omp_get_max_threads();
#pragma omp parallel for schedule(static) num_threads(nt)
  for (int64_t j = 0; j < N; ++j) {
    for (int64_t k = 0; k < K; ++k) {
      dBref[k * N + j] = 0.0;
      Sabs[k * N + j] = 0.0;
    }
    for (int64_t i = 0; i < M; ++i) {
      const int64_t len = rowptr[i + 1] - rowptr[i];
      for (int64_t ptr = rowptr[i]; ptr < rowptr[i + 1]; ++ptr) {
        const int64_t k = colind[ptr];
        double w = vals ? (double)vals[ptr] : 1.0;
        if (op == OP_MEAN) w /= (double)len;
        const double x = w * (double)dC[i * N + j];
        dBref[k * N + j] += x;
        Sabs[k * N + j] += fabs(x);
      }
    }
  }
  return 0;
}

/*
 * Gradient of max / min with respect to B, given the positions arg from the forward pass:
 *     dB[colind[arg[i, j]], j] += vals[arg[i, j]] * dC[i, j]     for every (i, j) with arg >= 0.
 */
int spmm_oracle_pool_backward(int64_t M, int64_t K, int64_t N, const int32_t* colind, const float* vals,
                              const int32_t* arg, const float* dC, double* dBref, double* Sabs) {
  if (M < 0 || K < 0 || N < 0 || !arg || !dBref || !Sabs) return -1;
  for (int64_t e = 0; e < K * N; ++e) {
    dBref[e] = 0.0;
    Sabs[e] = 0.0;
  }
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      const int64_t ptr = arg[i * N + j];
      if (ptr < 0) continue;
      const int64_t k = colind[ptr];
      const double x = (vals ? (double)vals[ptr] : 1.0) * (double)dC[i * N + j];
      dBref[k * N + j] += x;
      Sabs[k * N + j] += fabs(x);
    }
  }
  return 0;
}

/*
 * The transposed matrix in CSR, built from the CSR of A by a stable counting sort over the
 * column indices: row k of the result lists, in increasing row order of A, every stored
 * entry of A whose column is k, as (row index of A, weight).  weight = vals[p], divided by
 * the stored length of the entry's row when scale_by_row_length is set (then the forward
 * sum over the result is the gradient of mean).  With it the gradient of sum / mean with
 * respect to B is the forward operation on the transposed arrays (Sections I, IV-B).
 */
int spmm_oracle_csr_transpose(int64_t M, int64_t K, const int32_t* rowptr, const int32_t* colind,
                              const float* vals, int scale_by_row_length, int32_t* rowptrT,
                              int32_t* colindT, float* valsT) {
  if (M < 0 || K < 0 || !rowptr || !rowptrT) return -1;
  const int64_t nnz = rowptr[M];
  for (int64_t k = 0; k <= K; ++k) rowptrT[k] = 0;
  for (int64_t ptr = 0; ptr < nnz; ++ptr) rowptrT[colind[ptr] + 1] += 1;
  for (int64_t k = 0; k < K; ++k) rowptrT[k + 1] += rowptrT[k];
  int32_t* next = (int32_t*)malloc((size_t)(K > 0 ? K : 1) * sizeof(int32_t));
  if (!next) return -1;
  for (int64_t k = 0; k < K; ++k) next[k] = rowptrT[k];
  for (int64_t i = 0; i < M; ++i) {
    const double len = (double)(rowptr[i + 1] - rowptr[i]);
    for (int64_t ptr = rowptr[i]; ptr < rowptr[i + 1]; ++ptr) {
      const int32_t place = next[colind[ptr]]++;
      double w = vals ? (double)vals[ptr] : 1.0;
      if (scale_by_row_length) w /= len;
      colindT[place] = (int32_t)i;
      valsT[place] = (float)w;     /* the correctly rounded fp32 quotient */
    }
  }
  free(next);
  return 0;
}

/*
 * The general SpMM-like operation with a user-supplied initial value and fold (Eq. 1; Section
 * IV-A lets the user supply the initial value and the reduce step): for every output,
 * start from `init` and fold the stored entries of the row in storage order with
 * `step(acc, stored value, B element)`, all in double.  An empty row yields 0.  Serial:
 * the fold may be a callback into an interpreter.
 */
typedef double (*oracle_step_fn)(double acc, double a, double b);

int spmm_oracle_custom(int64_t M, int64_t K, int64_t N, const int32_t* rowptr, const int32_t* colind,
                       const float* vals, const float* B, double init, oracle_step_fn step, double* Cref) {
  if (M < 0 || K < 0 || N < 0 || !rowptr || !step || !Cref) return -1;
  for (int64_t i = 0; i < M; ++i) {
    for (int64_t j = 0; j < N; ++j) {
      double acc = init;
      for (int64_t ptr = rowptr[i]; ptr < rowptr[i + 1]; ++ptr) {
        const double a = vals ? (double)vals[ptr] : 1.0;
        acc = step(acc, a, (double)B[(int64_t)colind[ptr] * N + j]);
      }
      Cref[i * N + j] = rowptr[i + 1] > rowptr[i] ? acc : 0.0;
    }
  }
  return 0;
}

int spmm_oracle_max_threads(void) { return omp_get_max_threads(); }
