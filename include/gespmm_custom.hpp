// gespmm_custom.hpp - user-defined SpMM-like operations, compiled in at build time.
//
// The paper's general operation (Eq. 1; Section IV-A) lets the user provide an
// initialisation function and a reduce function that are inlined into the kernel when it
// is compiled.  This header is that mechanism for the gfx950 kernels: write a small struct,
// include this file in a .hip translation unit, and call gespmm::csr_custom<YourReduce>().
//
//   struct SumOfSquares {
//     static __host__ __device__ float identity() { return 0.0f; }                 // initial value
//     static __device__ float step(float acc, float a, float b) { float x = a * b; return acc + x * x; }
//     static __device__ float merge(float x, float y) { return x + y; }            // two partial results
//   };
//   int status = gespmm::csr_custom<SumOfSquares>(M, K, N, nnz, rowptr, colind, vals, B, C, stream);
//
// Requirements (Section IV-A asks for an associative and commutative reduce, because partial results are
// combined in parallel): merge is associative and commutative, identity() is its neutral
// element, and step(acc, a, b) == merge(acc, step(identity(), a, b)).  Arguments, layout,
// ownership and error codes are those of gespmm_csr (include/gespmm.h); an empty row yields 0;
// rows that are split across wavefronts are combined with a compare-and-swap loop around merge.
// A last argument `const gespmm_tuning_t* tuning` (default NULL = automatic) overrides the launch shape
// for this call, as in gespmm_csr_ex.  Compile with hipcc --offload-arch=gfx950 -I <this directory>:
// everything needed (this file, gespmm_kernels.hpp, gespmm_device.hpp, gespmm.h) lies here.  The same struct
// can be compiled at run time from source text instead: gespmm_custom_op_create in gespmm.h.
#pragma once

#include "gespmm_kernels.hpp"
