/*
 * hessformer.h -- C ABI of the single-GPU HessFormer hot path for MI355X.
 *
 * What the library computes (paper: "HessFormer: Hessians at Foundation
 * Scale", Section "Distributed Pearlmutter & Stochastic Lanczos Quadrature"):
 *
 *   hf_hvp           one batch iteration of Algorithm 1: u = d<dL/dp, v>/dp,
 *                    i.e. the exact Hessian-vector product H v of the mean
 *                    cross-entropy loss L of a model on one batch.  Computed
 *                    forward-over-reverse (a tangent pass over the forward and
 *                    the backward pass), which yields the same vector as the
 *                    double backward the paper writes.
 *   hf_lanczos_*     Algorithm 2, one iteration per call, with the optional
 *                    full orthogonalisation against a stored basis Q that
 *                    Section "Memory Compute trade off" names as the baseline.
 *   hf_slq           Algorithm 2 for every probe followed by the read-out of
 *                    Section "A note on numerical precision for the weight
 *                    value" / Table 2: Ritz values of the tridiagonal T_k and
 *                    one quadrature weight per Ritz value.
 *
 * Conventions
 *   - Pointers named *_dev are device (HBM) pointers of the GPU the context
 *     was created on; they are owned by the caller (allocate them with
 *     PyTorch-ROCm or hipMalloc), are never freed by the library and are not
 *     retained after the call returns, except q0_dev which hf_lanczos_init
 *     copies.  Pointers without _dev are host pointers.
 *   - The library owns only what hf_create allocates (activation workspace for
 *     max_batch*max_seq tokens, three fp32 Lanczos vectors (with an fp32 basis
 *     its rows k and k-1 serve as q_k and q_{k-1}), max_m basis
 *     vectors, a bf16 copy of the direction when parameters are bf16, and with
 *     bf16 parameters and an fp32 basis a bf16 copy of every basis row, i.e.
 *     half the basis again) and frees it in hf_destroy.
 *   - Work is enqueued on the HIP stream passed as `hip_stream` (a hipStream_t
 *     cast to void*, NULL = the default stream).  Calls that return host
 *     scalars synchronise that stream before returning.
 *   - Every function returns an hf_status (or a count); nothing throws or
 *     aborts.  hf_last_error(ctx) gives a message for the last failure on that
 *     context; hf_last_error(NULL) for failures of hf_create itself.
 *   - Parameters, directions, H v and all Lanczos vectors are ONE flat vector
 *     of length n = hf_num_params in the canonical order reported by
 *     hf_layout_entry: row-major tensors, matrices stored [in, out].
 *       MLP  : W1[in,hid] b1[hid] W2[hid,out] b2[out]
 *       GPT  : wte[V,d] wpe[max_seq,d], per layer { ln1.g ln1.b Wqkv[d,3d]
 *              bqkv Wo[d,d] bo ln2.g ln2.b Wfc[d,ff] bfc Wproj[ff,d] bproj },
 *              lnf.g lnf.b, lm_head[d,V] only if tie_embeddings == 0.
 *              Wqkv columns are Q|K|V; head h owns columns h*dh..(h+1)*dh of
 *              each third.
 *       LLAMA: wte[V,d], per layer { rms1.g Wq Wk Wv Wo rms2.g Wgate[d,ff]
 *              Wup[d,ff] Wdown[ff,d] }, rmsf.g, lm_head[d,V].
 *     params_dev stores that vector as fp32 (HF_F32) or bf16 (HF_BF16);
 *     v, H v and the Lanczos vectors are always fp32.
 */
#ifndef HESSFORMER_H
#define HESSFORMER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct hf_ctx hf_ctx; /* opaque */

typedef enum {
  HF_OK = 0,
  HF_EBREAKDOWN = 1, /* beta_k < tol: not an error, fewer than m iterations ran */
  HF_EINVAL = -1,    /* NULL pointer, bad enum, bad handle */
  HF_ENOMEM = -2,    /* hipMalloc failed in hf_create */
  HF_EDEVICE = -3,   /* a HIP call or kernel launch failed */
  HF_ESHAPE = -4,    /* batch/seq/m beyond what hf_create was sized for, or
                        dimensions the kernels do not support */
  HF_ESTATE = -5     /* hf_lanczos_step before hf_lanczos_init, or after the
                        iteration ended */
} hf_status;

typedef enum { HF_ARCH_MLP = 0, HF_ARCH_GPT = 1, HF_ARCH_LLAMA = 2 } hf_arch;
typedef enum { HF_F32 = 0, HF_BF16 = 1, HF_NONE = 2 /* basis_dtype only: store no basis */ } hf_dtype;
typedef enum { HF_REORTH_NONE = 0, HF_REORTH_FULL = 1 } hf_reorth;
typedef enum { HF_ACT_GELU_ERF = 0, HF_ACT_GELU_TANH = 1 } hf_activation;
/* How attention is evaluated (same result up to rounding): streamed over key / query tiles with
 * the probabilities recomputed in the backward sweep (bf16 parameters, head width 32, 64 or 128),
 * or with the S x S probabilities and score adjoints of every layer stored.  AUTO takes the
 * streamed kernels where they are supported and measured faster. */
typedef enum { HF_ATTN_AUTO = 0, HF_ATTN_STREAMED = 1, HF_ATTN_STORED = 2 } hf_attention;
/* bf16 parameters: whether the primal forward activations that feed matrix products (and the
 * attention probabilities) are carried as pairs of bf16 numbers, a rounded value and the rounding's
 * remainder, which enter the products as extra terms.  Tangents and adjoints are single bf16
 * numbers either way.  AUTO: pairs for LLAMA, whose product misses the 2e-2 bar against a float64
 * evaluation without them beyond a few layers at width 4096; single numbers for GPT, where the
 * pairs change the error of the product by less than a tenth of itself (2.2e-3 -> 2.6e-3 at 24
 * layers of width 2048) and cost a quarter more forward matrix work.  Ignored for fp32 parameters
 * and for the MLP. */
typedef enum { HF_PRIMAL_AUTO = 0, HF_PRIMAL_PAIRS = 1, HF_PRIMAL_SINGLE = 2 } hf_primal;

/* Model description.  MLP uses mlp_*; GPT/LLAMA use the transformer fields.
 * GPT: pre-LayerNorm decoder, learned positions, GELU (erf or tanh form, see
 * `activation`), causal attention
 * with scale 1/sqrt(dh).  LLAMA: RMSNorm, rotary positions on pairs
 * (i, i + dh/2) with base rope_theta, SwiGLU, no biases, optional grouped-query
 * attention (n_kv_head).
 * param_dtype HF_BF16: weights are bf16 MFMA operands, activations fed to
 * matrix products are rounded to bf16 (see `primal`), accumulation / residual stream /
 * normalisation and softmax statistics are fp32.  HF_F32: fp32 throughout. */
typedef struct {
  int32_t arch;           /* hf_arch */
  int32_t n_layer, d_model, n_head, d_ff, vocab, max_seq;
  int32_t mlp_in, mlp_hidden, mlp_out;
  int32_t tie_embeddings; /* GPT only: lm_head = wte^T */
  float norm_eps;
  float rope_theta;
  int32_t param_dtype;    /* hf_dtype of params_dev */
  int32_t basis_dtype;    /* hf_dtype of the stored Lanczos basis; HF_NONE: no basis is
                             allocated and only HF_REORTH_NONE iterations can run */
  int32_t activation;     /* GPT only: HF_ACT_GELU_ERF (0) or HF_ACT_GELU_TANH (1), the form
                             a/2 (1 + tanh(sqrt(2/pi)(a + 0.044715 a^3))) */
  int32_t n_kv_head;      /* LLAMA only: key/value heads of grouped-query attention (query head h
                             reads key/value head h / (n_head / n_kv_head)); Wk, Wv are
                             [d_model, n_kv_head * d_model / n_head].  0 = n_head.  Must divide
                             n_head; GPT takes 0 or n_head. */
  int32_t attention;      /* hf_attention; HF_ATTN_STREAMED where it is not supported: hf_create
                             returns HF_ESHAPE */
  int32_t primal;         /* hf_primal */
} hf_model_desc;

/* ---- host-only helpers (no GPU needed) ---------------------------------- */

/* Number of parameters n of the described model, or a negative hf_status. */
int64_t hf_desc_num_params(const hf_model_desc* desc);

/* Number of tensors in the canonical layout, or a negative hf_status. */
int32_t hf_layout_count(const hf_model_desc* desc);

/* Tensor `idx` of the canonical layout: its name (copied, NUL-terminated, at
 * most name_cap bytes), its offset in elements into the flat vector, and its
 * shape (shape[1] = 0 for vectors). */
int32_t hf_layout_entry(const hf_model_desc* desc, int32_t idx, char* name,
                        int32_t name_cap, int64_t* offset, int64_t shape[2]);

/* Read-out of stochastic Lanczos quadrature (Table 2): eigen-decomposition of
 * the k x k symmetric tridiagonal T with diagonal alpha[0..k) and off-diagonal
 * beta[0..k-1).  ritz[k] ascending; weights[i] = (first component of the unit
 * eigenvector of ritz[i])^2, so weights sum to 1.  All host, float64.
 * last_row (may be NULL) receives the last component of each eigenvector
 * (|beta[k-1] * last_row[i]| is the residual bound of Ritz pair i). */
int32_t hf_tridiag_readout(const double* alpha, const double* beta, int32_t k,
                           double* ritz, double* weights, double* last_row);

const char* hf_version(void);

/* ---- context ------------------------------------------------------------ */

/* Allocates every buffer the calls below need for batches of at most
 * max_batch sequences of at most desc->max_seq tokens (MLP: max_batch rows)
 * and Lanczos runs of at most max_m iterations (max_m = 0: hvp only;
 * max_m > 2000: HF_ESHAPE). */
int32_t hf_create(const hf_model_desc* desc, int32_t hip_device,
                  int32_t max_batch, int32_t max_m, hf_ctx** out);
void hf_destroy(hf_ctx* ctx);
int64_t hf_num_params(const hf_ctx* ctx);
/* Bytes of device memory the context allocated. */
int64_t hf_workspace_bytes(const hf_ctx* ctx);
const char* hf_last_error(const hf_ctx* ctx);

/* ---- Algorithm 1: Hessian-vector product on one batch ------------------- */

/* out_dev[n] (fp32) = H(params; batch) v_dev[n] (fp32).
 *   params_dev : flat parameters, fp32 or bf16 per desc.param_dtype
 *   inputs_dev : int32 tokens[batch, seq] (GPT/LLAMA) or fp32 x[batch, mlp_in]
 *   labels_dev : int32 [batch, seq] (or [batch] for MLP); -1 = position ignored.
 *                The loss is the mean cross-entropy over the other positions.
 *   seq        : ignored for MLP
 *   loss_host  : if not NULL receives L (forces a stream synchronisation)
 * out_dev must not alias v_dev or params_dev.  A label >= vocab or a token id
 * outside [0, vocab) makes the call return HF_EINVAL (checked on the device;
 * out_dev is then unspecified). */
int32_t hf_hvp(hf_ctx* ctx, const void* params_dev, const void* inputs_dev,
               const int32_t* labels_dev, int32_t batch, int32_t seq,
               const float* v_dev, float* out_dev, double* loss_host,
               void* hip_stream);

/* ---- Algorithm 2: Lanczos, one iteration per call ----------------------- */

/* Starts an iteration from q_0 = q0_dev / ||q0_dev|| (q0_dev: fp32[n], copied).
 * reorth HF_REORTH_FULL needs max_m > 0 basis vectors from hf_create. */
int32_t hf_lanczos_init(hf_ctx* ctx, const float* q0_dev, int32_t reorth,
                        void* hip_stream);

/* Iteration k of Algorithm 2: r = H q_k; r -= beta_{k-1} q_{k-1};
 * alpha_k = <q_k, r>; r -= alpha_k q_k; [full orthogonalisation of r against
 * q_0..q_k: classical Gram-Schmidt, a second pass when the first shrank ||r||
 * below 1/sqrt(2)]; beta_k = ||r||; q_{k+1} = r / beta_k unless beta_k < tol.
 * With full orthogonalisation the two subtractions are carried out by the
 * first Gram-Schmidt pass itself, applied to H q_k against q_0..q_k (alpha_k
 * is its k-th coefficient): the same r and alpha_k up to rounding.  The
 * coefficients are always formed against the stored rows; where the context
 * also holds bf16 copies of an fp32 basis, the subtraction reads rows 0..k-2
 * (whose coefficients are at rounding level) from the copies.  Without a
 * basis r is never stored: alpha_k, <r', r'> and <q_k, q_k> (r' = H q_k -
 * beta_{k-1} q_{k-1}) come from one read-only pass, beta_k^2 = <r', r'> -
 * alpha_k^2 (2 - <q_k, q_k>) (formed explicitly when that difference loses its
 * digits), and one pass writes q_{k+1} over q_{k-1}.
 * alpha_k / beta_k: host outputs.  Returns HF_EBREAKDOWN when beta_k < tol
 * (the iteration has ended), HF_ESHAPE after max_m iterations with a basis.
 * A token or label error (HF_EINVAL, as hf_hvp) leaves the iteration where it
 * was: the same step can be repeated with valid inputs.  Synchronises the
 * stream once, after all work of the iteration has been enqueued.
 * The iteration is that of one fixed operator: parameters and batch must be
 * the same in every step of a run (the library does not check this). */
int32_t hf_lanczos_step(hf_ctx* ctx, const void* params_dev,
                        const void* inputs_dev, const int32_t* labels_dev,
                        int32_t batch, int32_t seq, double tol,
                        double* alpha_k, double* beta_k, void* hip_stream);

/* Number of iterations done since hf_lanczos_init. */
int32_t hf_lanczos_iterations(const hf_ctx* ctx);

/* Copies working vector `which` (0: q_k, 1: q_{k-1}, 2: r) or, for
 * which = 16 + j, stored basis vector j widened to fp32, to dst_dev[n]. */
int32_t hf_lanczos_get_vector(hf_ctx* ctx, int32_t which, float* dst_dev,
                              void* hip_stream);

/* ---- stochastic Lanczos quadrature -------------------------------------- */

/* For each probe p (probes_dev: fp32 [n_probes, n], e.g. Rademacher vectors)
 * runs up to m Lanczos iterations and reads out T.  Host outputs, caller
 * allocated, row p at offset p*m: alpha, beta (beta[k] is the norm computed in
 * iteration k; T uses beta[0..m_eff-1)), ritz, weights (first m_eff[p]
 * entries of each row are valid).  No averaging over probes is done.
 * Returns HF_OK, or HF_EBREAKDOWN if any probe stopped early. */
int32_t hf_slq(hf_ctx* ctx, const void* params_dev, const void* inputs_dev,
               const int32_t* labels_dev, int32_t batch, int32_t seq,
               const float* probes_dev, int32_t n_probes, int32_t m,
               int32_t reorth, double tol, double* alpha, double* beta,
               double* ritz, double* weights, int32_t* m_eff, void* hip_stream);

/* ---- measurement hooks --------------------------------------------------- */

/* The Lanczos vector update of one iteration (everything in hf_lanczos_step
 * after the Hessian-vector product) applied to the current state with the
 * caller-supplied r_dev[n] standing in for H q_k.  r_dev (fp32, 16-byte
 * aligned) is used as the working vector r and may be overwritten.  Used by the
 * benchmark to time the bandwidth-bound part alone, and by tests to drive
 * Algorithm 2 with a synthetic operator. */
int32_t hf_lanczos_update(hf_ctx* ctx, float* r_dev, double tol,
                          double* alpha_k, double* beta_k, void* hip_stream);

/* ---- Widened rows ------------------------------------------------------------ */

/* Dataset-averaged Hessian-vector product: the batch loop of Algorithm 1.
 * inputs_dev / labels_dev hold n_samples samples (tokens [n_samples, seq] and
 * labels [n_samples, seq]; MLP: x [n_samples, mlp_in] and labels [n_samples]).
 * They are walked in consecutive batches of micro_batch samples (the last one
 * may be smaller, micro_batch <= max_batch of hf_create); each batch's product
 * u_B of its own mean loss is accumulated as h += u_B |B| with |B| the number of
 * samples in the batch, and out_dev (device, fp32[n], 16-byte aligned, must not
 * alias an input) receives h / n_samples.  loss_host (host, may be NULL)
 * receives the same weighted mean of the batch losses.  The weight |B| /
 * n_samples multiplies the adjoint seeds of the batch (the backward sweep is
 * linear in them) and every block of the batch's product is added to out_dev in
 * place, so no second vector is needed.  Synchronises the stream once, after
 * the last batch has been enqueued.  Errors as hf_hvp (a batch without a valid
 * label, a bad token or label in any batch: HF_EINVAL). */
int32_t hf_hvp_accumulate(hf_ctx* ctx, const void* params_dev, const void* inputs_dev,
                          const int32_t* labels_dev, int32_t n_samples, int32_t micro_batch,
                          int32_t seq, const float* v_dev, float* out_dev, double* loss_host,
                          void* hip_stream);

/* One column of the Hessian (section "Banded Hessians"): the product with the
 * vector that is 1 at `index` (0 <= index < n, canonical order) and 0
 * elsewhere.  column_dev: device, fp32[n], caller-owned, must not alias
 * params_dev.  Uses the context's auxiliary vector (see hf_hvp_accumulate).
 * Other arguments and errors as hf_hvp. */
int32_t hf_hessian_column(hf_ctx* ctx, const void* params_dev, const void* inputs_dev,
                          const int32_t* labels_dev, int32_t batch, int32_t seq, int64_t index,
                          float* column_dev, double* loss_host, void* hip_stream);

/* Sparsity summary of a vector, as tabulated in section "Banded Hessians":
 * below[k] = number of i with |h_i| < thresholds[k] (float32 comparison);
 * *max_abs = max_i |h_i|; hist = histogram of |h_i| with n_bins equal bins over
 * [0, max_abs]: entry i falls in bin floor(|h_i| * (n_bins / max_abs)), quotient
 * and product each rounded to float32, clamped to the last bin (which therefore
 * holds the maximum).  A vector of zeros puts every entry in bin 0.  NaN
 * entries are below no threshold and are left out of max_abs and hist.
 * h_dev: device, fp32[n], 4-byte aligned, read-only, n < 2^40 (n = 0 allowed).
 * thresholds (host, n_thresholds <= 16), below (host, int64[n_thresholds]),
 * max_abs (host), hist (host, int64[n_bins], 1 <= n_bins <= 256).  Two
 * streaming passes over h_dev; synchronises the stream.  HF_EINVAL on bad
 * arguments. */
int32_t hf_column_stats(hf_ctx* ctx, const float* h_dev, int64_t n, const float* thresholds,
                        int32_t n_thresholds, int32_t n_bins, int64_t* below, float* max_abs,
                        int64_t* hist, void* hip_stream);

/* hf_column_stats for callers that cannot allocate device memory or hold a
 * context: code under HIP graph capture set-up, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results and errors as
 * hf_column_stats, without a context: the counters the two passes need (2304
 * bytes) live in a fixed array inside the library's device image, one copy per
 * GPU, held until the process ends.  Limits: n < 2^40, n_thresholds <= 16,
 * n_bins <= 256 (HF_ESHAPE / HF_EINVAL beyond them).  The call allocates and
 * frees nothing.  It runs on the device that is current on the calling thread,
 * which must own h_dev.  Every call on a GPU shares that GPU's array, which
 * keeps the previous call's contents: the call clears it first (a fill kernel
 * on hip_stream), and two calls that overlap on one GPU race.  The message of a
 * failure is available from hf_last_error(NULL). */
int32_t hf_column_stats_noalloc(const float* h_dev, int64_t n, const float* thresholds,
                                int32_t n_thresholds, int32_t n_bins, int64_t* below,
                                float* max_abs, int64_t* hist, void* hip_stream);

/* Smoothed spectral density from the quadrature nodes and weights of hf_slq
 * (the smoothed densities the paper plots; Table 2 lists the underlying nodes
 * and weights): density[g] = (1/n_probes) sum_p sum_{i < m_eff[p]}
 * weights[p*m+i] N(grid[g]; ritz[p*m+i], sigma^2).  Host only, float64; all
 * arrays caller-owned.  HF_EINVAL on NULL, sigma <= 0 or m_eff[p] outside [0, m]. */
int32_t hf_slq_density(const double* ritz, const double* weights, const int32_t* m_eff,
                       int32_t n_probes, int32_t m, double sigma, const double* grid,
                       int32_t n_grid, double* density);

/* Moment estimates from the same nodes and weights: moments[q] =
 * (1/n_probes) sum_p sum_i weights[p*m+i] ritz[p*m+i]^q, q = 0..n_moments-1, the
 * quadrature estimate of tr(H^q)/n for Rademacher probes.  Host only. */
int32_t hf_slq_moments(const double* ritz, const double* weights, const int32_t* m_eff,
                       int32_t n_probes, int32_t m, int32_t n_moments, double* moments);

/* ---- Lanczos state hand-over (checkpoint / resume of Algorithm 2) ---------------
 * The state after k iterations is k, q_k, q_{k-1}, beta_{k-1}, the
 * re-orthogonalisation mode and (full mode) the stored basis q_0..q_k; the
 * coefficients alpha, beta already returned are the caller's to keep.
 * hf_lanczos_state_bytes: size of the image for the current state (negative
 * hf_status when no iteration is in progress).
 * hf_lanczos_export: writes the image to state_dev (device, caller-owned,
 * 256-byte aligned, capacity_bytes >= hf_lanczos_state_bytes).
 * hf_lanczos_import: restores an image into a context of the same parameter
 * count, basis precision and max_m >= stored rows (max_m == stored rows if the
 * image was exported after its basis had filled), replacing whatever iteration
 * it held; the next hf_lanczos_step continues at iteration k.  The image is
 * plain device memory (copy it to a file or another process as you like); it
 * is only meaningful to this library version.  Both synchronise the stream.
 * HF_ESTATE / HF_ESHAPE / HF_EINVAL as described. */
int64_t hf_lanczos_state_bytes(const hf_ctx* ctx);
int32_t hf_lanczos_export(hf_ctx* ctx, void* state_dev, int64_t capacity_bytes, void* hip_stream);
int32_t hf_lanczos_import(hf_ctx* ctx, const void* state_dev, int64_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* HESSFORMER_H */
