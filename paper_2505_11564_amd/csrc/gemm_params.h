// Kernel-side parameter block shared by the matrix-product kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hf {

struct GemmP {
  const void* A[3];  // up to three (A, B) terms accumulate into one product
  const void* B[3];
  int nterm;
  void* C;
  void* C_lo;  // bf16 C only: optional low-order part, C_lo = bf16(v - float(bf16(v)))
  const float* Cadd;
  const void* bias;
  const float* bias_t;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int transA, transB;
  int nb2;
  int divB;  // the B operand of batch entry (z1, z2) is entry (z1, z2 / divB): shared key/value heads
  int64_t sA1, sA2, sB1, sB2, sC1, sC2;
  float alpha;
  int out_bf16, bias_bf16;
  int klimit, skip_upper;
  int tiles_n;
  int vecA, vecB;  // operands satisfy the alignment the vector loaders need
};

// MFMA path with direct global->LDS loads; needs 16-byte aligned operand rows.
// force_cfg / force_ks < 0 (<= 0): choose automatically.
// c_zeroed: C is already zero, so a product that splits k (atomic accumulation) skips its own fill.
hipError_t launch_gemm_mfma(GemmP p, int nb, int allow_splitk, int force_cfg, int force_ks, hipStream_t st, int c_zeroed = 0);
// Two products of one shape (primal and tangent) in one launch; hipErrorNotSupported = launch them separately.
hipError_t launch_gemm_mfma_pair(GemmP a, GemmP b, int nb, hipStream_t st);

// Several A^T B products with fp32 results as one launch of 256 x 256 tiles with split k (atomic
// accumulation into results that are zero or hold the addend); hipErrorNotSupported = launch them separately.
hipError_t launch_gemm_mfma_group(const GemmP* ps, int n, hipStream_t st);

}  // namespace hf
