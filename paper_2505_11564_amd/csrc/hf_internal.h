// Internal declarations shared by the HIP sources of libhessformer_hip.
// Nothing here is part of the C ABI (see include/hessformer.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "hessformer.h"

namespace hf {

typedef __bf16 bf16;

// ---------------------------------------------------------------- errors ----

struct Err {
  int code = HF_OK;
  std::string msg;
};

#define HF_HIP_TRY(expr)                                                        \
  do {                                                                          \
    hipError_t e_ = (expr);                                                     \
    if (e_ != hipSuccess) {                                                     \
      return fail(HF_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
    }                                                                           \
  } while (0)

// ------------------------------------------------------------- GEMM ----------

// C[z] = alpha * (A0 op B0 + A1 op B1 + A2 op B2) + bias + bias_t + Cadd[z]
//   A element (m,k): transA ? A[k*lda + m] : A[m*lda + k]
//   B element (k,n): transB ? B[n*ldb + k] : B[k*ldb + n]
//   batch z = z1*nb2 + z2, operand offset z1*s?1 + z2*s?2 (elements)
//   in_bf16: A and B are bf16 (MFMA path) else fp32 (FMA path)
//   out_bf16: C is bf16 else fp32.  Cadd (fp32, same ld/strides as C, may be C
//   itself) only with fp32 C.  bias: per-column, type of the parameters;
//   bias_t: per-column fp32.
//   causal: 0 none; 1 = output tiles strictly above the diagonal are skipped
//   (left untouched); 2 = k-range limited to k <= last row of the tile (A is
//   lower triangular, e.g. P V); 3 = k-range limited to k >= first column...
struct Gemm {
  const void* A[3] = {nullptr, nullptr, nullptr};
  const void* B[3] = {nullptr, nullptr, nullptr};
  void* C = nullptr;
  void* C_lo = nullptr;  // bf16 C only: low-order part of the result
  const float* Cadd = nullptr;
  const void* bias = nullptr;
  const float* bias_t = nullptr;
  int M = 0, N = 0, K = 0;
  int64_t lda = 0, ldb = 0, ldc = 0;
  int transA = 0, transB = 0;
  int nb1 = 1, nb2 = 1;
  int divB = 1;  // batch entry (i1, i2) reads B of entry (i1, i2 / divB): grouped key/value heads
  int64_t sA1 = 0, sA2 = 0, sB1 = 0, sB2 = 0, sC1 = 0, sC2 = 0;
  float alpha = 1.f;
  int in_bf16 = 0, out_bf16 = 0;
  int klimit = 0;  // 0 none; 1: k <= row (A lower-triangular in (m,k));
                   // 2: k >= m (A upper-triangular in (m,k))
  int skip_upper = 0;  // skip output tiles with n0 > m_last (causal scores)
  int allow_splitk = 0;  // fp32 C only: few output tiles, long k -> split k with atomics
  int c_zeroed = 0;      // with allow_splitk: the caller has cleared C already
  // Dual output (Ct != nullptr): additionally Ct = alpha (At op B[0] + A[0] op Bt) + bias_t + Cadd_t in
  // the same launch; C then takes bias and Cadd only, Ct takes bias_t and Cadd_t only.
  const void* At = nullptr;
  const void* Bt = nullptr;
  void* Ct = nullptr;
  const float* Cadd_t = nullptr;
  int force_cfg = -1, force_ks = 0;  // tuning / tests: tile configuration and k-split override
  // Dual-output products with few output tiles and a long k: fp32 scratch for the partial sums
  // of a k-split (2 * splits * M * N floats are used when they fit); nullptr = never split.
  float* ws = nullptr;
  int64_t ws_elems = 0;
  // Attention epilogues of the dual-output kernel (bf16 operands, Ct != nullptr).  With them the
  // score-shaped products never go to memory in fp32: the product is formed twice, once to reduce
  // row statistics over 64-column parts and once to apply them.
  //   EPI_FWD_STATS   : part[row][N/64][3] = (max, sum exp(s - max), sum exp(s - max) s_t) of the part
  //   EPI_FWD_SOFTMAX : C = P = exp(s - m) / l, C_lo = its low-order half, Ct = P (s_t - r); rstat[row] = (m, 1/l, r)
  //   EPI_BWD_STATS   : part[row][N/64][3] = (sum P c, sum P_t c + P c_t, -) with P = E0, P_t = E1
  //   EPI_BWD_DS      : C = P (c - delta), Ct = P_t (c - delta) + P (c_t - delta_t); rstat[row] = (delta, delta_t, -)
  // s / c are the primal product, s_t / c_t its tangent; rows are batch-major (batch index * M + m);
  // entries with column > row are masked (zero) when skip_upper is set.
  int epi = 0;
  float* part = nullptr;
  const float* rstat = nullptr;
  const void* E0 = nullptr;
  const void* E1 = nullptr;
};
enum { EPI_NONE = 0, EPI_FWD_STATS = 1, EPI_FWD_SOFTMAX = 2, EPI_BWD_STATS = 3, EPI_BWD_DS = 4 };

hipError_t launch_gemm(const Gemm& g, hipStream_t st);
hipError_t launch_gemm_dual(const Gemm& g, hipStream_t st);  // bf16, aligned operands only
// gs[0..n): single-output products whose results are already zero (c_zeroed) or are added to
// (Cadd == C); launched as one grid where that is faster, else in turn.
hipError_t launch_gemm_group(const Gemm* gs, int n, hipStream_t st);
// bf16 A^T B product [M, N] over k = K with fp32 result and split-K allowed: will it accumulate with atomics?
bool gemm_mfma_splits_k(int M, int N, int K, int nterm);

// -------------------------------------------------------- row / pointwise ----
// AT = operand type of activations (float or bf16); PT = parameter type.
// Launchers take `bf` = 1 for bf16 mode (AT = PT = bf16), 0 for fp32 mode.

hipError_t launch_fill_f32(float* p, int64_t n, float val, hipStream_t st);
// Combine the per-part row statistics of the attention epilogues: forward (online softmax merge)
// -> rstat[row] = (m, 1/l, r); backward (plain sums) -> rstat[row] = (delta, delta_t, 0).
// Softmax-adjoint row statistics from dO and O (bf16 operands, head width 8 * 2^k); hipErrorNotSupported otherwise.
hipError_t launch_attn_delta(const void* dO, const void* dO_t, const void* O, const void* O_lo, const void* O_t, int T, int S,
                             int H, int dh, float* rstat, hipStream_t st);
hipError_t launch_attn_combine(int backward, const float* part, int NP, int M, int64_t rows, float* rstat, hipStream_t st);

// attn_flash.hip: causal attention with tangents, streamed over key / query tiles (bf16 operands,
// head width 32, 64 or 128).  Activations are packed rows [T, ldq] = q | k | v: head h of q at
// column h*dh, its key and value at offK + (h / grp) * dh and offV + (h / grp) * dh (grp query heads
// share one key/value head); token of (batch b, position s) is row b*S + s.
struct AttnP {
  const bf16 *qkv = nullptr, *qkv_lo = nullptr, *qkv_t = nullptr;  // primal (high, low half) and tangent
  int64_t ldq = 0;
  int offK = 0, offV = 0;
  int B = 0, H = 0, S = 0, grp = 1, dh = 0;
  float scale = 1.f;
  // forward results [T, ldo], head h at column h*dh; stat[(b*H + h)*S + s] = (m + log l, r)
  bf16 *o = nullptr, *o_lo = nullptr, *o_t = nullptr;
  int64_t ldo = 0;
  float* stat = nullptr;
  // backward: adjoint of the output and its tangent [T, lddo]; delta[(b*H + h)*S + s] = (delta, delta_t, -)
  const bf16 *dO = nullptr, *dO_t = nullptr;
  int64_t lddo = 0;
  const float* delta = nullptr;
  // results, bf16 or fp32 (x_f32), rows of ldd? elements: dq / dq_t [T, H*dh], dk, dv (and tangents)
  // [T, (H/grp)*dh] summed over the query heads of a group; the pointers address column 0 of head 0
  void *dq = nullptr, *dq_t = nullptr, *dk = nullptr, *dk_t = nullptr, *dv = nullptr, *dv_t = nullptr;
  int64_t lddq = 0, lddk = 0, lddv = 0;
  int dq_f32 = 0, dk_f32 = 0, dv_f32 = 0;
};
bool attn_flash_supported(int dh, int64_t ldq, int64_t ldo);
// measured faster than the stored-probability path at this head width and launch size (heads = batch x heads)
bool attn_flash_preferred(int dh, int64_t heads, int64_t S);
hipError_t launch_attn_fwd(const AttnP& p, hipStream_t st);
hipError_t launch_attn_bwd(const AttnP& p, hipStream_t st);  // dQ, dK, dV with tangents (needs delta)

// probe.hip: batch-loop accumulation and Hessian-column statistics
constexpr int CS_MAX_THRESHOLDS = 16, CS_MAX_BINS = 256, CS_STATS_WORDS = 32 + CS_MAX_BINS;
struct ColThresholds { float t[CS_MAX_THRESHOLDS]; };
constexpr int64_t GEMM_WS_ELEMS = 16ll << 20;  // 64 MiB of fp32: two results x up to 8 splits of a 512 x 2048 product, 2 x 2 of 512 x 4096
// One result of a k-split dual-output product: C = sum over the splits' partial sums (each
// M x N, row stride N, consecutive splits M*N apart) + bias + Cadd, written as fp32 or as bf16
// with an optional low-order half; rows of C / Cadd / C_lo have stride ldc.
struct SplitKOut {
  const float* part = nullptr;
  const bf16* bias_bf16 = nullptr;
  const float* bias_f32 = nullptr;
  const float* Cadd = nullptr;
  void* C = nullptr;
  void* C_lo = nullptr;
};
hipError_t launch_splitk_reduce(const SplitKOut& o0, const SplitKOut& o1, int splits, int M, int N, int64_t ldc, int out_bf16,
                                hipStream_t st);
hipError_t launch_scale_add(float* h, const float* u, float w, int first, int64_t n, hipStream_t st);
hipError_t launch_colstats_pass1(const float* h, int64_t n, const ColThresholds& thr, int nt, unsigned long long* stats,
                                 hipStream_t st);
hipError_t launch_colstats_hist(const float* h, int64_t n, const unsigned long long* max_bits, int nb, unsigned long long* hist,
                                hipStream_t st);
// Device address, on the current device, of the library's static array of CS_STATS_WORDS counters.
hipError_t colstats_static_counters(unsigned long long** out);
hipError_t launch_f32_to_bf16(const float* src, bf16* dst, int64_t n, hipStream_t st);
hipError_t launch_cast_pair(int bf, const float* a, const float* b, void* oa, void* ob, int64_t n, hipStream_t st);

// x[t,:] = wte[tok[t],:] (+ wpe[t % S,:]) and the same gather of the direction.
hipError_t launch_embed_fwd(int bf, const void* wte, const void* wpe, const float* wte_t, const float* wpe_t,
                            const int32_t* tok, int T, int S, int d, int vocab, float* x, float* x_t,
                            int* err_flag, hipStream_t st);
// out_wte[tok[t],:] += dx_t[t,:]; out_wpe[t % S,:] += dx_t[t,:]   (atomic adds)
hipError_t launch_embed_bwd(const float* dx_t, const int32_t* tok, int T, int S, int d, int vocab, float* out_wte,
                            float* out_wpe, hipStream_t st);

// LayerNorm (rms = 0) / RMSNorm (rms = 1) with tangent.  stats: [T,4].
hipError_t launch_norm_fwd(int bf, int rms, const float* x, const float* x_t, const void* gam, const void* bet,
                           const float* gam_t, const float* bet_t, int T, int d, float eps, void* y, void* y_t,
                           void* y_lo, float* stats, hipStream_t st);
// dx (+)= ..., dx_t (+)= ...; hv_gam / hv_bet += column sums (atomic).
constexpr int NORM_PART_BLOCKS = 1024;  // upper bound of the blocks launch_norm_bwd uses with `part`
hipError_t launch_norm_bwd(int bf, int rms, const float* dy, const float* dy_t, const float* x, const float* x_t,
                           const float* stats, const void* gam, const float* gam_t, int T, int d, int accumulate,
                           float* dx, float* dx_t, float* hv_gam, float* hv_bet, float* part, hipStream_t st,
                           void* dxb = nullptr, void* dxb_t = nullptr,  // optional bf16 copies of dx, dx_t
                           float* hv_out = nullptr);  // optional: hv_out[c] += column sums of the dx_t written

enum Act { ACT_TANH = 0, ACT_GELU = 1, ACT_GELU_TANH = 2 };
// a_lo / y_lo (nullable): low-order halves of the primal input / output.
hipError_t launch_act_fwd(int bf, int act, const void* a, const void* a_t, const void* a_lo, void* y, void* y_t,
                          void* y_lo, int64_t n, hipStream_t st);
hipError_t launch_act_bwd(int bf, int act, const void* a, const void* a_t, const void* dy, const void* dy_t, void* da,
                          void* da_t, int64_t n, hipStream_t st);
hipError_t launch_swiglu_fwd(int bf, const void* g, const void* g_t, const void* u, const void* u_t, const void* g_lo,
                             const void* u_lo, void* y, void* y_t, void* y_lo, int64_t n, hipStream_t st);
hipError_t launch_swiglu_bwd(int bf, const void* g, const void* g_t, const void* u, const void* u_t, const void* dy,
                             const void* dy_t, void* dg, void* dg_t, void* du, void* du_t, int64_t n, hipStream_t st);

// Causal softmax over rows of scores [nbh, S, S] with tangent.
hipError_t launch_softmax_fwd(int bf, const float* s, const float* s_t, void* p, void* p_t, void* p_lo, int nbh, int S,
                              hipStream_t st);
hipError_t launch_softmax_bwd(int bf, const void* p, const void* p_t, const float* dp, const float* dp_t, void* ds,
                              void* ds_t, int nbh, int S, hipStream_t st);

// Rotary embedding: src (fp32, [T, lds], n_head heads of width dh from column
// 0) rotated into dst (operand type, [T, ldd]); the tangent takes the same
// rotation; inverse = the transposed rotation (adjoints).
hipError_t launch_rope(int bf, const float* src, const float* src_t, int64_t lds, void* dst, void* dst_t, void* dst_lo,
                       int64_t ldd, int T, int S, int n_head, int dh, float theta, int inverse, hipStream_t st);

// Softmax cross-entropy with tangent: dz, dz_t (operand type) from z, z_t
// (fp32, leading dimension ldz); loss_rows[T] = per-row loss (0 if ignored);
// n_valid: device int.  err_flag: bit 1 set if a label >= V.  `scale` multiplies dz and dz_t (the
// weight |B| / N of a batch in the batch loop of Algorithm 1; the backward sweep is linear in them).
hipError_t launch_count_valid(const int32_t* labels, int T, int V, int* n_valid, int* err_flag, hipStream_t st);
hipError_t launch_ce(int bf, const float* z, const float* z_t, const int32_t* labels, const int* n_valid, int T, int V,
                     int64_t ldz, void* dz, void* dz_t, float* loss_rows, float scale, hipStream_t st);
// out[0] (+)= weight * sum(v) / n_valid; bit 2 of err_flag set when n_valid is 0.
hipError_t launch_sum_rows_f64(const float* v, int n, const int* n_valid, double* out, double weight, int accumulate,
                               int* err_flag, hipStream_t st);

// hv_b[c] = sum_rows y_t[r, c]   (y_t operand type or fp32)
hipError_t launch_colsum(int is_bf16, const void* y, int T, int N, int64_t ld, float* out, hipStream_t st);

// ------------------------------------------------------------- Lanczos ------

struct LzScalars;  // device-resident doubles, see lanczos.hip

}  // namespace hf
