// Context of libhessformer_hip: model description, canonical layout, device
// workspace, and the host-side schedules of the Hessian-vector product
// (Algorithm 1 of the paper, evaluated forward-over-reverse) and of the
// Lanczos iteration (Algorithm 2).
#pragma once

#include "hf_internal.h"
#include "lanczos.h"

namespace hf {

struct LayoutEntry {
  std::string name;
  int64_t offset;
  int64_t shape[2];
  int64_t count() const { return shape[0] * (shape[1] ? shape[1] : 1); }
};

// Fills `out` with the canonical flat order; returns HF_OK or HF_EINVAL.
int build_layout(const hf_model_desc& d, std::vector<LayoutEntry>& out, std::string* why);

// Offsets (elements) of one transformer layer's tensors in the flat vector.
struct LayerOff {
  int64_t n1g = -1, n1b = -1, wqkv = -1, bqkv = -1, wq = -1, wk = -1, wv = -1, wo = -1, bo = -1;
  int64_t n2g = -1, n2b = -1, wfc = -1, bfc = -1, wproj = -1, bproj = -1, wgate = -1, wup = -1, wdown = -1;
};

// Device buffers of one layer kept from the forward pass for the backward
// pass (each with its tangent twin `*_t`).
struct LayerBuf {
  float *x1, *x1_t, *x2, *x2_t, *st1, *st2;          // residual stream, norm statistics
  void *a, *a_t, *qkv, *qkv_t, *P, *P_t, *o, *o_t;   // attention branch
  void *m, *m_t, *f, *f_t, *g, *g_t;                 // MLP branch: norm out, pre-activation, activation out
  void *up, *up_t;                                   // LLAMA: up projection (f = gate)
  // streamed attention (bf16, head width 32 / 64 / 128): the backward sweep recomputes the scores,
  // so each layer keeps the low-order halves of q | k | v and of the attention output, and the
  // row statistics (m + log l, r) of its softmax
  void *qkv_lo, *o_lo;
  float* att_stat;
};

}  // namespace hf

struct hf_ctx {
  hf_model_desc desc;
  int device = 0;
  int max_batch = 0, max_m = 0;
  int bf = 0;  // 1: bf16 parameters / operands
  int flash = 0;  // 1: attention runs in the streamed kernels (no S x S buffers are allocated)
  int pairs = 0;  // 1: bf16 primal activations are carried as (rounded value, remainder) pairs; the *_lo buffers exist
  int64_t n = 0;
  std::vector<hf::LayoutEntry> layout;
  std::vector<hf::LayerOff> loff;
  int64_t off_wte = -1, off_wpe = -1, off_nfg = -1, off_nfb = -1, off_head = -1;
  int64_t off_w1 = -1, off_b1 = -1, off_w2 = -1, off_b2 = -1;
  std::vector<std::pair<int64_t, int64_t>> zero_ranges;  // H v regions filled by atomics
  int64_t layers_begin = 0, layers_end = 0;  // the layers' parameters (through the final norm) in the flat vector
  int dw_prezeroed = 0;  // this product cleared [layers_begin, layers_end) of H v in one pass
  std::string err;

  // device memory
  char* arena = nullptr;
  int64_t arena_bytes = 0;
  std::vector<hf::LayerBuf> lb;
  hf::bf16* vb = nullptr;  // bf16 copy of the direction (bf16 mode)
  const float* vb_of = nullptr;  // the Lanczos vector whose bf16 copy vb_cur holds (written by the update), or nullptr
  const hf::bf16* vb_cur = nullptr;   // the bf16 copy the running product multiplies with: vb, or a row of a bf16 basis
  const hf::bf16* next_vb = nullptr;  // scratch of lanczos_update
  float *xL = nullptr, *xL_t = nullptr, *stf = nullptr;
  void *xf = nullptr, *xf_t = nullptr, *xf_lo = nullptr;
  // bf16 mode: low-order halves of the primal forward activations (reused by every layer)
  void *a_lo = nullptr, *qkv_lo = nullptr, *P_lo = nullptr, *o_lo = nullptr, *f_lo = nullptr, *up_lo = nullptr, *g_lo = nullptr;
  float *rq = nullptr, *rq_t = nullptr;  // LLAMA: fp32 q|k (or their adjoints) before the rotation
  float *rv = nullptr, *rv_t = nullptr;  // grouped-query attention: fp32 dV summed over the heads of a group
  void *dvb = nullptr, *dvb_t = nullptr; //   and its operand-type copy (bf16 mode)
  float *z = nullptr, *z_t = nullptr;
  void *dz = nullptr, *dz_t = nullptr;
  int64_t ldz = 0;
  float* loss_rows = nullptr;
  float *sc = nullptr, *sc_t = nullptr;
  float* norm_part = nullptr;  // per-block column sums of the norm backward kernels
  float *att_part = nullptr, *att_rstat = nullptr;  // row statistics of the fused attention epilogues
  int64_t att_SS = 0;                                 // elements of one score-shaped buffer
  int att_zero_B = -1, att_zero_S = -1;               // shape for which the never-written score tiles were last cleared
  void *dS = nullptr, *dS_t = nullptr;
  float *dx = nullptr, *dx_t = nullptr, *tmpd = nullptr, *tmpd_t = nullptr;
  void *dxb = nullptr, *dxb_t = nullptr, *dob = nullptr, *dob_t = nullptr;
  void *dxb2 = nullptr, *dxb2_t = nullptr;  // second pair of bf16 adjoint copies (grouped weight-gradient launches)
  void *dqkv = nullptr, *dqkv_t = nullptr;
  void *dg = nullptr, *dg_t = nullptr, *dup = nullptr, *dup_t = nullptr, *dy = nullptr, *dy_t = nullptr;
  void* xin = nullptr;  // MLP input in operand type (bf16 mode)
  int* flags = nullptr;  // [0] error bits, [1] number of valid labels
  double* loss_dev = nullptr;
  unsigned long long* stats_dev = nullptr;  // column statistics counters
  float* gemm_ws = nullptr;  // fp32 scratch of the k-split dual-output products (GEMM_WS_ELEMS floats)
  float* aux_vec = nullptr;  // n floats, allocated on first use (batch-loop partial result, unit vector)
  int ensure_aux();

  // Lanczos state
  // Working vectors.  With an fp32 basis and full orthogonalisation the basis rows k and k - 1 are
  // q_k and q_{k-1} themselves (cur_q / prev_q) and lz_vec holds only r and, once the basis is
  // full, the last q; otherwise lz_vec rotates q, q_prev and r.
  float* lz_vec[3] = {nullptr, nullptr, nullptr};
  int iq = 0, iqp = 1, ir = 2;
  void* basis = nullptr;
  // bf16 copies of the rows of an fp32 basis, kept by contexts with bf16 parameters: row k is the
  // operand-type copy of q_k that the product multiplies with anyway, and the subtraction pass of
  // the orthogonalisation reads rows 0 .. k-2 from here at half the bytes (their coefficients are
  // at rounding level, so the rounding of the copies is below that of the fp32 result)
  hf::bf16* basis_bf = nullptr;
  int64_t ldq = 0;
  double *scal = nullptr, *cvec = nullptr, *partials = nullptr;
  double* host_scal = nullptr;  // pinned, S_COUNT + 2 doubles
  int lz_k = -1;                // iterations done; -1 = not initialised
  int lz_reorth = 0;
  int lz_done = 0;
  double lz_beta_prev = 0.0;    // beta_{k-1}
  bool lz_rows_are_vectors() const { return lz_reorth == HF_REORTH_FULL && desc.basis_dtype == HF_F32; }
  float* cur_q() const;         // q_k
  float* prev_q() const;        // q_{k-1} (meaningful for k >= 1)

  int fail(int code, const std::string& m) { err = m; return code; }
  int plan_and_alloc();
  // out = seed_scale * H v, or out += seed_scale * H v when accumulate (the batch loop of Algorithm 1:
  // the weight of a batch multiplies the adjoint seeds, in which the backward sweep is linear)
  int hvp_enqueue(const void* params, const void* inputs, const int32_t* labels, int batch, int seq, const float* v,
                  float* out, hipStream_t st, float seed_scale = 1.f, int accumulate = 0);
  int acc_mode = 0;   // the product being enqueued adds to out
  float seed = 1.f;   // and scales its adjoint seeds by this
  int hvp_mlp(const void* params, const void* inputs, const int32_t* labels, int B, const float* v, float* out,
              hipStream_t st);
  int hvp_transformer(const void* params, const int32_t* tok, const int32_t* labels, int B, int S, const float* v,
                      float* out, hipStream_t st);
  int finish_hvp(double* loss_host, hipStream_t st);
  // hvp_flags: the device flags of the product that made r (NULL when r came from the caller)
  int lanczos_update(float* r, double tol, double* alpha_k, double* beta_k, const int* hvp_flags, hipStream_t st);
};
