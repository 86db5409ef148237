/*
 * gespmm.h - C ABI of the MI355X (gfx950) CSR SpMM / SpMM-like library.
 *
 * The operation (paper: Algorithm 1 and Section III-A for the plain result,
 * Eq. 1 and Section IV-A for the general reduce):
 *
 *     C[i, j] = reduce over the stored entries p of row i of  vals[p] * B[colind[p], j]
 *
 * with A (M x K) in plain CSR exactly as the caller holds it (Section III-A:
 * rowptr / colind / vals; no preprocessing, no format conversion, no state kept
 * between calls), B (K x N) and C (M x N) dense, row-major, fp32 (Section V-C).
 * reduce is sum, mean, max or min; an empty row gives 0 for every op; mean
 * divides by the number of stored entries of the row.
 *
 * All data pointers are DEVICE pointers on the current HIP device.  The caller
 * owns every buffer.  The library allocates no device memory, frees nothing,
 * and never synchronises (except gespmm_csr_simple, see below): all work is
 * enqueued on the given stream.  Inputs are only read.  C is fully overwritten
 * and need not be initialised; C must not overlap any input.  There is no
 * process-wide mutable state: tuning overrides and timing brackets are arguments
 * of the call they apply to, so calls from several threads do not interact.
 *
 * Every function returns a gespmm_status_t (0 = success) unless stated.
 * Argument errors are detected on the host before any HIP call is made.
 * Device-side contents (colind range, rowptr monotonicity) are NOT validated:
 * violating them is undefined behaviour.
 */
#ifndef GESPMM_H
#define GESPMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { GESPMM_SUM = 0, GESPMM_MEAN = 1, GESPMM_MAX = 2, GESPMM_MIN = 3 } gespmm_op_t;

typedef enum {
  GESPMM_OK = 0,
  GESPMM_ERR_BAD_ARG = 1,   /* negative size, unknown op, nnz inconsistent       */
  GESPMM_ERR_NULL = 2,      /* a required pointer is NULL                         */
  GESPMM_ERR_TOO_LARGE = 3, /* M, K or nnz does not fit the 32-bit index arrays   */
  GESPMM_ERR_WORKSPACE = 4, /* the caller's workspace is too small or misaligned  */
  GESPMM_ERR_HIP = 5,       /* a HIP call (launch, event, copy) reported an error */
  GESPMM_ERR_SCRATCH_LIMIT = 6, /* beyond the built-in scratch buffer of the entry
                                   point that allocates nothing                   */
  GESPMM_ERR_COMPILE = 7,   /* the text of a user-defined reduce did not compile   */
  GESPMM_ERR_NO_RTC = 8     /* the run-time compiler library cannot be loaded      */
} gespmm_status_t;

/*
 * The SpMM / SpMM-like operation (Algorithm 1; Eq. 1; Section IV-A).
 *
 *   M, K, N   matrix sizes, >= 0.  M < 2^31 - 1, K < 2^31.
 *   nnz       number of stored entries, 0 <= nnz <= 2^31 - 1025; must equal rowptr[M].
 *   rowptr    device, int32[M+1], rowptr[0] == 0, non-decreasing, rowptr[M] == nnz.
 *   colind    device, int32[nnz], 0 <= colind[p] < K, any order inside a row,
 *             repeated columns allowed (each stored entry is its own term).
 *   vals      device, fp32[nnz], or NULL meaning every stored value is 1.0f.
 *   B         device, fp32[K*N], row-major, leading dimension N.
 *   C         device, fp32[M*N], row-major, leading dimension N; overwritten.
 *   op        gespmm_op_t.
 *   stream    a hipStream_t passed as void* (NULL = the default stream).
 *
 * 16-byte aligned B and C with N a multiple of 4 take the vectorised kernels;
 * anything else takes the scalar kernels.  M == 0 or N == 0 returns at once;
 * nnz == 0 fills C with zeros.  sum and mean are accurate to fp32 rounding in an
 * unspecified summation order (rows that are split across wavefronts are
 * combined with fp32 atomic adds, so the last bits can differ from run to run);
 * max and min are exact and bit-reproducible.
 * Errors: GESPMM_ERR_NULL (rowptr, B or C NULL; colind NULL with nnz > 0),
 * GESPMM_ERR_BAD_ARG, GESPMM_ERR_TOO_LARGE, GESPMM_ERR_HIP (launch failure).
 */
int gespmm_csr(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
               const int32_t* colind, const float* vals, const float* B, float* C, int op,
               void* stream);

/*
 * Same operation for callers that do not track nnz: reads rowptr[M] from the
 * device with one 4-byte copy and waits for it (this call DOES synchronise the
 * stream once), then behaves as gespmm_csr.
 */
int gespmm_csr_simple(int64_t M, int64_t K, int64_t N, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const float* B, float* C, int op,
                      void* stream);

/*
 * The same operation with B stored in a 16-bit floating-point format.  This goes beyond the
 * paper, which evaluates fp32 only (Section V-A): the result is still Algorithm 1 / Eq. 1,
 * every element of B is widened to fp32 (exactly) before use, products, sums, comparisons and
 * C are fp32, so the accuracy statement of gespmm_csr holds unchanged with respect to the
 * values B actually stores.  What changes is the traffic: a gathered row of B is half as long.
 *   B        device, 16-bit elements [K*N], row-major, leading dimension N.
 *   b_dtype  GESPMM_BF16 (1 sign, 8 exponent, 7 fraction bits) or GESPMM_F16 (IEEE binary16);
 *            GESPMM_F32 makes the call identical to gespmm_csr (B then points to fp32 data).
 * Everything else as gespmm_csr.  16-byte aligned B and C with N a multiple of 4 take the
 * vectorised kernels (4 columns per lane, 8-byte loads), anything else one column per lane.
 * Errors as gespmm_csr; GESPMM_ERR_BAD_ARG for an unknown b_dtype.
 */
typedef enum { GESPMM_F32 = 0, GESPMM_BF16 = 1, GESPMM_F16 = 2 } gespmm_dtype_t;

int gespmm_csr_b16(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                   const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                   int op, void* stream);

/*
 * max or min together with the POSITION of the extreme: what a pooling aggregation
 * (the GraphSAGE-pool use of the SpMM-like operation, Section V-E) needs in order to
 * route its gradient (the operator carries a gradient definition, Section IV-B).
 * Arguments as gespmm_csr, op must be GESPMM_MAX or GESPMM_MIN, plus
 *   arg   device, int32[M*N], row-major like C; overwritten.  arg[i*N+j] is the index p
 *         into colind / vals of the stored entry of row i whose product vals[p] *
 *         B[colind[p], j] has exactly the bits of C[i, j]; if several entries do, the
 *         smallest p (first in storage order); -1 for an empty row.
 * One fused pass carries (value, position) pairs through the reduction; rows that several
 * wavefronts share combine their pairs as packed 64-bit words held, during the call, in the
 * row's own C and arg storage, and a small kernel unpacks them at the end (1.1 to 1.4 times
 * the cost of gespmm_csr).  That route needs the vector kernels (N a multiple of 4; B, C and
 * arg 16-byte aligned) and N <= 1024; otherwise split rows get their positions from a second
 * pass over the matrix (up to 1.9 times the cost of gespmm_csr).  Same errors as gespmm_csr;
 * GESPMM_ERR_BAD_ARG for any other op; GESPMM_ERR_NULL for arg == NULL.
 */
int gespmm_csr_arg(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                   const int32_t* colind, const float* vals, const float* B, float* C, int32_t* arg,
                   int op, void* stream);
/* gespmm_csr_arg with B stored in a 16-bit format (see gespmm_csr_b16 for b_dtype and the layout
 * of B; everything else, including the exactness of values and positions with respect to the
 * stored values of B, as gespmm_csr_arg). */
int gespmm_csr_arg_b16(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                       const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                       int32_t* arg, int op, void* stream);

/*
 * Gradient of sum / mean with respect to B (the backward pass of a graph convolution is
 * again an SpMM, Section I; gradient definition, Section IV-B), taken from the SAME CSR
 * arrays, without a transposed copy of A:
 *     dB[k, j] = sum over stored entries p with colind[p] == k of  w_p * dC[row(p), j],
 *     w_p = vals[p] (GESPMM_SUM) or vals[p] / (stored length of row(p)) (GESPMM_MEAN).
 *   dC   device, fp32[M*N], row-major;  dB  device, fp32[K*N], row-major, overwritten
 *   (zero-filled by the call, then accumulated with fp32 atomic adds: the last bits can
 *   differ from run to run).  K == 0 or N == 0 returns at once; op other than SUM / MEAN
 *   is GESPMM_ERR_BAD_ARG.  This is the no-extra-memory route; fp32 atomics make it 20-30x
 *   slower than a forward call, so for repeated use build the transposed arrays once with
 *   gespmm_csr_transpose and call gespmm_csr on them (for a symmetric A with symmetric
 *   values, gespmm_csr on A itself already is the answer).
 */
int gespmm_csr_transposed(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                          const int32_t* colind, const float* vals, const float* dC, float* dB, int op,
                          void* stream);

/*
 * The CSR arrays of the transposed matrix, built on the device from the CSR arrays of A.
 * GNN frameworks keep both orientations of the graph; with this one, the gradient of
 * sum / mean with respect to B (Sections I, IV-B) is a plain gespmm_csr call,
 *     dB = gespmm_csr(K, M, N, nnz, rowptrT, colindT, valsT, dC, GESPMM_SUM),
 * at forward speed, and the arrays can be reused for every training step on the graph.
 *   scale_by_row_length   0: valsT holds vals (ones if vals is NULL);
 *                         1: vals[p] / (stored length of p's row in A): the weights of the
 *                            gradient of GESPMM_MEAN (correctly rounded fp32 quotient).
 *   rowptrT  device, int32[K+1], written;  colindT  device, int32[nnz], written (row indices
 *   of A; the ORDER inside a transposed row is unspecified and can differ from run to run);
 *   valsT  device, fp32[nnz], written.
 *   workspace  device memory of at least gespmm_csr_transpose_workspace_bytes(K) bytes,
 *   4-byte aligned, owned by the caller, contents destroyed; the library allocates nothing.
 * Errors: GESPMM_ERR_NULL (an output or the workspace is NULL), GESPMM_ERR_BAD_ARG
 * (negative size), GESPMM_ERR_WORKSPACE (workspace too small or misaligned),
 * GESPMM_ERR_TOO_LARGE, GESPMM_ERR_HIP.
 */
size_t gespmm_csr_transpose_workspace_bytes(int64_t K);   /* pure host function */
int gespmm_csr_transpose(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr,
                         const int32_t* colind, const float* vals, int scale_by_row_length,
                         int32_t* rowptrT, int32_t* colindT, float* valsT, void* workspace,
                         size_t workspace_bytes, void* stream);

/*
 * gespmm_csr_transpose for callers that cannot allocate device memory or hand in a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results, ownership and errors as gespmm_csr_transpose, minus the workspace: the
 * cursors and scan totals live in a buffer built into the library (static device memory,
 * GESPMM_NOALLOC_TRANSPOSE_MAX_K * 4 bytes plus a few KB, held by every GPU the library runs on
 * until the process ends).  The call allocates nothing, frees nothing and does not synchronise.
 * K > GESPMM_NOALLOC_TRANSPOSE_MAX_K is rejected with GESPMM_ERR_SCRATCH_LIMIT before anything
 * is launched.  All calls on one GPU share that one buffer: two calls of this function that
 * overlap in time on the same GPU (different streams or threads) race; calls on one stream,
 * or otherwise ordered, are fine, and so are calls on different GPUs.
 */
#define GESPMM_NOALLOC_TRANSPOSE_MAX_K 2097152
int gespmm_csr_transpose_noalloc(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr,
                                 const int32_t* colind, const float* vals, int scale_by_row_length,
                                 int32_t* rowptrT, int32_t* colindT, float* valsT, void* stream);

/*
 * The same transposed arrays by a stable radix sort on the column index instead of per-column
 * counters: every pass streams the entries (28 bytes per entry and pass, two passes up to 2^20
 * columns, three beyond), so the time does not depend on the column distribution, and inside
 * a transposed row the entries keep the order of A's rows: the result is unique, the same
 * from run to run, and equal to a stable counting sort.  3 to 7 times faster than
 * gespmm_csr_transpose on the graphs measured, at the price of a larger workspace:
 * gespmm_csr_transpose_sorted_workspace_bytes(K, nnz) = about 24 bytes per stored entry.
 * Arguments, ownership and errors as gespmm_csr_transpose.
 */
size_t gespmm_csr_transpose_sorted_workspace_bytes(int64_t K, int64_t nnz);   /* pure host function */
int gespmm_csr_transpose_sorted(int64_t M, int64_t K, int64_t nnz, const int32_t* rowptr,
                                const int32_t* colind, const float* vals, int scale_by_row_length,
                                int32_t* rowptrT, int32_t* colindT, float* valsT, void* workspace,
                                size_t workspace_bytes, void* stream);

/*
 * Gradient of max / min with respect to B, routed through the positions from
 * gespmm_csr_arg (Sections IV-B, V-E):
 *     dB[colind[p], j] += vals[p] * dC[i, j]   with p = arg[i*N+j], for every p >= 0.
 *   colind, vals (NULL = all ones) as in the forward call; arg int32[M*N]; dC fp32[M*N];
 *   dB fp32[K*N], overwritten (zero-filled, then fp32 atomic adds).  arg values must be
 *   -1 or valid entry indices (not validated).
 */
int gespmm_pool_backward(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* colind,
                         const float* vals, const int32_t* arg, const float* dC, float* dB,
                         void* stream);

/*
 * Per-call overrides of the automatic launch shape, for tests, benchmarks and callers who know
 * their matrix.  Every field: -1 = automatic.  lanes_per_row in {1,2,4,...,64}, tiles_per_lane
 * in {1,2,4}, xcd_remap in [0, 4096] (see gespmm_plan_t), chunk_nnz a power of two in [16, 1024], short_len in
 * [0, 1024] (0 = every row is handled by all slots together), k_parts in [0, 64] (parts the
 * column range is cut into by the K-phased path of gespmm_csr_ex; 0 or 1 = off).  A value that
 * has no kernel makes the call return GESPMM_ERR_BAD_ARG.
 * longest_row is not an override but something the caller may know about the matrix: an upper
 * bound on the stored entries of any row (-1 or 0 = not known).  With it the forward call (and the
 * value+position call and user-defined reduces on fp32 features) can take the WHOLE-ROW path when
 * rows are short against a chunk (or the problem is small): every row is computed by one wavefront
 * and written once, so the call is a single kernel launch without presetting and without atomics,
 * and sum / mean become independent of the order in which wavefronts finish.  A structure that a C
 * caller initialises with fewer fields leaves the later ones 0, which means "not known" / automatic.  The bound only selects the path: the result is right whatever it says;
 * a row much longer than stated is walked by one wavefront alone and is slow.
 * wide_addresses = 1 makes the forward kernels compute 64-bit addresses for their gathers also when B
 * is smaller than 2 GiB, where they otherwise gather through a buffer descriptor with 32-bit offsets
 * (-1 or 0 = automatic; same results either way; for tests and comparisons).
 */
typedef struct {
  int32_t lanes_per_row;
  int32_t tiles_per_lane;
  int32_t xcd_remap;
  int32_t chunk_nnz;
  int32_t short_len;
  int32_t k_parts;
  int32_t longest_row;
  int32_t wide_addresses;
} gespmm_tuning_t;

/*
 * The kernel selection of Section IV-A ("GE-SpMM for different matrix sizes"),
 * redone for 64-lane wavefronts: pure host functions, they touch no device.
 * They fill the launch shape the forward call would use for these sizes.
 */
typedef struct {
  int32_t vec;            /* columns per lane per load: 4 (vectorised) or 1 (scalar)      */
  int32_t lanes_per_row;  /* G: lanes that cover one column block of a sparse row         */
  int32_t tiles_per_lane; /* T: column tiles each lane accumulates (row loaded once)      */
  int32_t slots;          /* 64 / G: non-zeros of a row consumed per wavefront step       */
  int32_t chunk_nnz;      /* S: items (stored entries + row ends) assigned to one wavefront */
  int32_t col_blocks;     /* grid.y: ceil(N / (vec * G * T))                              */
  int64_t chunks;         /* ceil((nnz + M) / S)                                          */
  int64_t grid_x;         /* workgroups along x of one main-kernel launch                 */
  int32_t block_threads;  /* threads per workgroup                                        */
  int32_t xcd_remap;      /* workgroups -> XCDs: 0 round-robin as dispatched, 1 one contiguous range per XCD,
                             r > 1 runs of r consecutive workgroups per XCD, the runs round-robin */
  int32_t short_len;      /* row segments up to this length are handled one per slot      */
  int32_t lds_bytes;      /* dynamic LDS per workgroup                                    */
  int32_t k_parts;        /* main-kernel launches per call: 1, or the parts of the K-phased path */
  int32_t row_window;     /* whole-row path: entries a wavefront stages at once (S + longest row); 0 = rows are split among chunks */
  int64_t workspace_bytes; /* workspace the K-phased path needs for this shape (0 when k_parts == 1) */
} gespmm_plan_t;

int gespmm_plan(int64_t M, int64_t N, int64_t nnz, int aligned16, gespmm_plan_t* out);
/* The same for gespmm_csr_b16. */
int gespmm_plan_b16(int64_t M, int64_t N, int64_t nnz, int aligned16, int b_dtype, gespmm_plan_t* out);
/* The same for gespmm_csr_ex: K, the workspace the caller will pass and the tuning overrides count. */
int gespmm_plan_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, int aligned16, int b_dtype,
                   size_t workspace_bytes, const gespmm_tuning_t* tuning, gespmm_plan_t* out);

/*
 * Timing brackets for benchmarks: an object that owns `capacity` HIP event pairs.  A forward call
 * that is given the object records one pair around every main-kernel launch it makes, on the call's
 * stream, while pairs are left.  gespmm_profiler_finish waits for the recorded events, returns the
 * summed main-kernel time in milliseconds and the number of bracketed launches, and destroys the
 * object (also on error).  One object must not be used by two threads at once.
 */
typedef struct gespmm_profiler gespmm_profiler_t;
int gespmm_profiler_create(int capacity, gespmm_profiler_t** out);
int gespmm_profiler_finish(gespmm_profiler_t* profiler, double* main_kernel_ms_sum, int* launches);

/*
 * The forward operation with everything optional spelled out (Algorithm 1; Eq. 1; Sections III,
 * IV-A): gespmm_csr / gespmm_csr_b16 are this call with no workspace, tuning or profiler.
 *   b_dtype          element type of B (gespmm_dtype_t).
 *   workspace        device memory, 4-byte aligned, owned by the caller, contents destroyed, or NULL.
 *   workspace_bytes  its size.  With at least gespmm_csr_workspace_bytes(...) bytes the call may take
 *                    the K-PHASED path: the column range [0, K) is cut into k_parts equal parts and
 *                    the operation runs once per part, launch after launch, each launch folding into
 *                    C; every launch then gathers from K / k_parts rows of B only, which stay in the
 *                    L2 caches (Section III observes that the loads of B dominate; on this chip a B
 *                    that does not fit the L2s is what bounds the kernel).  The path is chosen when B
 *                    is several times larger than the L2s and the rows of A are long (mean >= 128
 *                    stored entries); it pays when columns are sorted inside the rows, as CSR builders
 *                    produce them, and is correct for any order.  No state survives the call: the
 *                    workspace is rebuilt every time (about 0.1 ms for 10^8 entries).
 *   tuning           overrides or NULL.  k_parts >= 2 forces the phased path (GESPMM_ERR_WORKSPACE if
 *                    the workspace is NULL or too small), 0 or 1 forbids it.
 *   profiler         timing brackets or NULL.
 * Everything else, including accuracy and errors, as gespmm_csr; sum and mean add one rounding per
 * part to every output.
 */
size_t gespmm_csr_workspace_bytes(int64_t M, int64_t K, int64_t N, int64_t nnz, int b_dtype,
                                  const gespmm_tuning_t* tuning);   /* pure host function */
int gespmm_csr_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                  const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C, int op,
                  void* workspace, size_t workspace_bytes, const gespmm_tuning_t* tuning,
                  gespmm_profiler_t* profiler, void* stream);

/* gespmm_csr_arg_b16 with tuning overrides (NULL = automatic; k_parts is ignored: no workspace; with longest_row and fp32
 * features the call can take the whole-row path: one launch instead of four). */
int gespmm_csr_arg_ex(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                      int32_t* arg, int op, const gespmm_tuning_t* tuning, void* stream);

/*
 * gespmm_csr_arg_ex with a workspace, which lets max / min with positions (Section V-E's pooling aggregation)
 * take the K-phased path of gespmm_csr_ex under the same rule (B several times larger than the L2 caches, mean
 * row >= 128 entries) when the features are fp32, N is a multiple of 4 and at most 1024, and B, C and arg are
 * 16-byte aligned; otherwise the call is gespmm_csr_arg_ex.  On that path every output carries (value, position)
 * as one 64-bit word, held in the row's own C and arg storage through all phases and unpacked by one kernel after
 * the last; values and positions are exactly those of gespmm_csr_arg (measured: 2.6 instead of 3.4 ms on a
 * 233k-vertex graph of mean degree 492 at N = 64).
 *   workspace        device, gespmm_csr_workspace_bytes(M, K, N, nnz, GESPMM_F32, tuning) bytes, 4-byte aligned,
 *                    or NULL (no phases); contents need not be initialised, nothing survives the call.
 *   tuning           k_parts >= 2 forces the phases (GESPMM_ERR_WORKSPACE without a large enough workspace,
 *                    GESPMM_ERR_BAD_ARG if the call cannot take them), 0 or 1 forbids them.
 */
int gespmm_csr_arg_ws(int64_t M, int64_t K, int64_t N, int64_t nnz, const int32_t* rowptr,
                      const int32_t* colind, const float* vals, const void* B, int b_dtype, float* C,
                      int32_t* arg, int op, void* workspace, size_t workspace_bytes,
                      const gespmm_tuning_t* tuning, void* stream);

/*
 * User-defined reduce operations compiled at run time (Eq. 1; Section IV-A: the user supplies an
 * initialisation and a reduce function, which are compiled into the kernel).  include/gespmm_custom.hpp is
 * the same mechanism at build time, for C++ callers; this one needs no compiler on the caller's side.
 *   source   HIP C++ text that defines a struct `name` with three static functions
 *                static __device__ float identity();                        initial value of a row
 *                static __device__ float step(float acc, float a, float b); acc joined with the entry (a = vals[p], b = B[colind[p], j])
 *                static __device__ float merge(float x, float y);           two partial results
 *            merge must be associative and commutative with identity() as neutral element, and
 *            step(acc, a, b) == merge(acc, step(identity(), a, b)): partial results of a row are combined
 *            in parallel.  The text may contain helpers of its own; it sees the HIP device runtime only.
 *   name     the struct (an identifier, optionally qualified).
 *   out      receives the operation; the caller destroys it with gespmm_custom_op_destroy once no call
 *            that uses it is in flight.
 *   log      host buffer for the compiler's messages (NUL-terminated, truncated to log_bytes) or NULL.
 * gespmm_custom_op_create compiles on the calling thread (about a second), runs a one-thread kernel on the
 * current device to read identity() and synchronises with it; kernels for further launch shapes are
 * compiled on first use inside gespmm_csr_custom (a fraction of a second each, once).  The operation is
 * bound to the device that was current at creation.  It may be used from several threads.  Creation
 * allocates and synchronises, and so does the first call with a new launch shape (it loads a module): do
 * both outside HIP graph capture; later calls only launch kernels and can be captured.
 * Errors: GESPMM_ERR_NULL, GESPMM_ERR_BAD_ARG (name is not an identifier; another device is current),
 * GESPMM_ERR_COMPILE (see log), GESPMM_ERR_NO_RTC, GESPMM_ERR_HIP.
 *
 * gespmm_csr_custom: C[i, j] = merge over the stored entries p of row i of step(identity(), vals[p],
 * B[colind[p], j]), 0 for a row that stores nothing.  Arguments, layout, ownership, stream semantics and
 * errors as gespmm_csr (fp32 features); tuning as in gespmm_csr_ex (k_parts is ignored; longest_row selects the
 * whole-row path as there, on which no compare-and-swap loop runs).
 * Rows that lie in several chunks are combined by a compare-and-swap loop around merge.
 */
typedef struct gespmm_custom_op gespmm_custom_op_t;
int gespmm_custom_op_create(const char* source, const char* name, gespmm_custom_op_t** out, char* log,
                            size_t log_bytes);
int gespmm_custom_op_destroy(gespmm_custom_op_t* op);
/* Compiles the same text for `arch` (NULL = "gfx950") without touching a device and without keeping anything:
 * GESPMM_OK, or GESPMM_ERR_COMPILE with the compiler's messages in log.  A pure host function. */
int gespmm_custom_op_check(const char* source, const char* name, const char* arch, char* log, size_t log_bytes);
int gespmm_csr_custom(gespmm_custom_op_t* op, int64_t M, int64_t K, int64_t N, int64_t nnz,
                      const int32_t* rowptr, const int32_t* colind, const float* vals, const float* B,
                      float* C, const gespmm_tuning_t* tuning, void* stream);

/*
 * Measurement helper, not part of the method: copies `bytes` (a multiple of 16, both
 * pointers 16-byte aligned, device memory, non-overlapping) from src to dst with a plain
 * copy kernel on `stream`.  It reads `bytes` and writes `bytes` of HBM and nothing else,
 * which makes it the yardstick for scaling hardware traffic counters.
 */
int gespmm_calibration_copy(const void* src, void* dst, int64_t bytes, void* stream);

/*
 * Second yardstick: a plain gather of 128-byte lines.  n times, 8 lanes read line idx[e]
 * (0 <= idx[e] < table_lines) of `table` (table_lines * 128 bytes, 16-byte aligned), eight
 * gathers in flight per lane: what the inner loop of gespmm_csr does to memory, and nothing
 * else.  Its rate on a table of the size of the live slice of B is the ceiling for that loop.
 * `out` receives one 16-byte value per launched lane (so the loads stay live): at least
 * min(ceil(n / 256), 8192) * 4096 bytes.  Values in idx are not validated.
 */
int gespmm_calibration_gather(const void* table, int64_t table_lines, const int32_t* idx, int64_t n,
                              void* out, int64_t out_bytes, void* stream);

/*
 * The same yardstick with its shape as arguments, for mapping out what the chip delivers: n times,
 * lanes_per_row lanes read load_bytes (4, 8 or 16) each of row idx[e] of `table` (rows row_bytes apart,
 * table_bytes in all, below 4 GB, 16-byte aligned; lanes_per_row * load_bytes <= row_bytes), in_flight
 * (2, 4, 8 or 16) rows in flight per lane.  cache_policy: 0 plain loads; 1 loads that bypass the L1;
 * 2 non-temporal loads (1 and 2 exist for 8 lanes x 16 bytes only).  `out`: 2048 * 256 * 4 bytes of scratch
 * output.  GESPMM_ERR_BAD_ARG for a shape that is not instantiated.  Values in idx are not validated.
 */
int gespmm_calibration_gather_shape(const void* table, int64_t table_bytes, int row_bytes, const int32_t* idx,
                                    int64_t n, int lanes_per_row, int load_bytes, int in_flight,
                                    int cache_policy, void* out, int64_t out_bytes, void* stream);

/* Static text for a status code (never NULL). */
const char* gespmm_status_string(int status);

/* Library version, major * 100 + minor. */
int gespmm_version(void);

#ifdef __cplusplus
}
#endif
#endif /* GESPMM_H */
