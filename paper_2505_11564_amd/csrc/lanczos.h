// Internal interface of the Lanczos vector kernels (lanczos.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hf {

// Slots of the device-resident scalar array.
enum {
  S_ALPHA = 0,       // alpha_k
  S_BETA = 1,        // current ||r|| (beta_k once the iteration's updates are done)
  S_NRM_BEFORE = 3,  // ||r|| before the orthogonalisation pass in flight
  S_REDO = 4,        // 1.0 when a second orthogonalisation pass is required
  S_Q0NORM = 5,      // ||q0|| before normalisation
  S_FLAG0 = 6,       // error bits and number of valid labels of the Hessian-vector product that made
  S_FLAG1 = 7,       //   w, copied here by the kernel that writes q_{k+1}
  S_COUNT = 8
};

constexpr int HF_MAX_M = 2000;  // most basis vectors a context may hold
constexpr int LZ_NBLK = 2048;  // upper bound on blocks (= partial sums per basis vector) of the re-orthogonalisation kernels
constexpr int LZ_NBLK_VEC = 16384;  // upper bound on blocks (= partial sums) of the read-only passes over one vector

hipError_t lz_norm_q0(const float* z, int64_t n, double* scal, double* partials, hipStream_t st);
// Iteration k of the three-term recurrence without a basis: alpha_k, beta_k into scal, and
// q_{k+1} = (w - beta_prev qp - alpha_k q) / beta_k written over qp (with its bf16 copy in vb, may be
// NULL) unless beta_k < tol or `flags` (device, may be NULL: [0] error bits, [1] valid labels)
// report a failed product.  partials: 3 * LZ_NBLK_VEC doubles.
hipError_t lz3_update(const float* w, const float* q, float* qp, bf16* vb, int64_t n, int use_prev, double beta_prev,
                      double tol, const int* flags, double* scal, double* partials, hipStream_t st);
// q_{k+1} = src / scal[idx] into dst (fp32, may be NULL), its basis row (may be NULL) and vb (bf16,
// may be NULL), under the same test.
hipError_t lz_scale(const float* src, float* dst, void* basis, int basis_bf16, bf16* vb, int64_t n, double* scal, int idx,
                    double tol, const int* flags, hipStream_t st);
// One classical Gram-Schmidt pass of r against Q[0..nq); pass 1 is a no-op
// unless pass 0 set the redo flag.
// copies (optional, fp32 basis only): bf16 copies of the rows, same row stride; the subtraction
// reads rows 0 .. nq-3 from them.
hipError_t lz_reorth_pass(const void* Q, int basis_bf16, const bf16* copies, int64_t ldq, float* r, int64_t n, int nq, int pass,
                          double* scal, double* c, double* partials, hipStream_t st);
// The first pass applied to w = H q_k itself against an fp32 basis holding q_0 .. q_k (nq = k + 1):
// also yields alpha_k, in place of lz_axpy_dot and lz_axpy_nrm.
hipError_t lz_gs_first_pass(const float* Q, const bf16* copies, int64_t ldq, float* r, int64_t n, int nq, double* scal,
                            double* c, double* partials, hipStream_t st);
// The same for a bf16 basis: q_k and q_{k-1} come from the fp32 working vectors, rows 0 .. k-2 from the basis.
hipError_t lz_gs_first_pass_bf16(const bf16* Q, int64_t ldq, const float* qkm1, const float* qk, float* r, int64_t n, int k,
                                 double* scal, double* c, double* partials, hipStream_t st);
hipError_t lz_widen(const void* src, int is_bf16, float* dst, int64_t n, hipStream_t st);

}  // namespace hf
