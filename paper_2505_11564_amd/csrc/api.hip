// C ABI of libhessformer_hip (declared in include/hessformer.h): argument
// checking, context life cycle, the Lanczos / SLQ drivers (Algorithm 2 of the
// paper and the Ritz value / weight read-out of its Table 2).
#include <algorithm>
#include <cmath>
#include <cstddef>
#include <cstring>
#include <mutex>

#include "engine.h"

using namespace hf;

namespace {
std::mutex g_err_mu;
std::string g_create_err;
void set_create_err(const std::string& m) {
  std::lock_guard<std::mutex> lk(g_err_mu);
  g_create_err = m;
}

// Eigen-decomposition of a symmetric tridiagonal matrix by cyclic Jacobi
// rotations on its dense form (k is at most a few hundred).  V's columns are
// the eigenvectors.
void jacobi_eig(std::vector<double>& A, std::vector<double>& Vm, int k) {
  Vm.assign((size_t)k * k, 0.0);
  for (int i = 0; i < k; ++i) Vm[(size_t)i * k + i] = 1.0;
  double fro = 0.0;
  for (double x : A) fro += x * x;
  if (fro == 0.0) return;
  for (int sweep = 0; sweep < 100; ++sweep) {
    double off = 0.0;
    for (int p = 0; p < k; ++p)
      for (int q = p + 1; q < k; ++q) off += A[(size_t)p * k + q] * A[(size_t)p * k + q];
    if (off <= 1e-34 * fro) break;
    for (int p = 0; p < k - 1; ++p) {
      for (int q = p + 1; q < k; ++q) {
        const double apq = A[(size_t)p * k + q];
        if (apq == 0.0) continue;
        const double app = A[(size_t)p * k + p], aqq = A[(size_t)q * k + q];
        const double tau = (aqq - app) / (2.0 * apq);
        const double t = (tau >= 0.0 ? 1.0 : -1.0) / (std::fabs(tau) + std::sqrt(1.0 + tau * tau));
        const double cs = 1.0 / std::sqrt(1.0 + t * t), sn = t * cs;
        for (int i = 0; i < k; ++i) {  // columns p, q of A
          const double aip = A[(size_t)i * k + p], aiq = A[(size_t)i * k + q];
          A[(size_t)i * k + p] = cs * aip - sn * aiq;
          A[(size_t)i * k + q] = sn * aip + cs * aiq;
        }
        for (int i = 0; i < k; ++i) {  // rows p, q of A
          const double api = A[(size_t)p * k + i], aqi = A[(size_t)q * k + i];
          A[(size_t)p * k + i] = cs * api - sn * aqi;
          A[(size_t)q * k + i] = sn * api + cs * aqi;
        }
        for (int i = 0; i < k; ++i) {
          const double vip = Vm[(size_t)i * k + p], viq = Vm[(size_t)i * k + q];
          Vm[(size_t)i * k + p] = cs * vip - sn * viq;
          Vm[(size_t)i * k + q] = sn * vip + cs * viq;
        }
      }
    }
  }
}
}  // namespace

extern "C" {

const char* hf_version(void) { return "hessformer-hip 0.1 (gfx950)"; }

int64_t hf_desc_num_params(const hf_model_desc* desc) {
  if (!desc) return HF_EINVAL;
  std::vector<LayoutEntry> lay;
  const int rc = build_layout(*desc, lay, nullptr);
  if (rc != HF_OK) return rc;
  return lay.back().offset + lay.back().count();
}

int32_t hf_layout_count(const hf_model_desc* desc) {
  if (!desc) return HF_EINVAL;
  std::vector<LayoutEntry> lay;
  const int rc = build_layout(*desc, lay, nullptr);
  if (rc != HF_OK) return rc;
  return (int32_t)lay.size();
}

int32_t hf_layout_entry(const hf_model_desc* desc, int32_t idx, char* name, int32_t name_cap, int64_t* offset,
                        int64_t shape[2]) {
  if (!desc) return HF_EINVAL;
  std::vector<LayoutEntry> lay;
  const int rc = build_layout(*desc, lay, nullptr);
  if (rc != HF_OK) return rc;
  if (idx < 0 || idx >= (int32_t)lay.size()) return HF_EINVAL;
  const LayoutEntry& e = lay[idx];
  if (name && name_cap > 0) {
    std::strncpy(name, e.name.c_str(), (size_t)name_cap - 1);
    name[name_cap - 1] = 0;
  }
  if (offset) *offset = e.offset;
  if (shape) { shape[0] = e.shape[0]; shape[1] = e.shape[1]; }
  return HF_OK;
}

int32_t hf_tridiag_readout(const double* alpha, const double* beta, int32_t k, double* ritz, double* weights,
                           double* last_row) {
  if (!alpha || !ritz || !weights || k <= 0 || (k > 1 && !beta)) return HF_EINVAL;
  if (k > 2048) return HF_ESHAPE;
  std::vector<double> A((size_t)k * k, 0.0), Vm;
  for (int i = 0; i < k; ++i) {
    A[(size_t)i * k + i] = alpha[i];
    if (i + 1 < k) A[(size_t)i * k + i + 1] = A[(size_t)(i + 1) * k + i] = beta[i];
  }
  jacobi_eig(A, Vm, k);
  std::vector<int> ord(k);
  for (int i = 0; i < k; ++i) ord[i] = i;
  std::sort(ord.begin(), ord.end(), [&](int a, int b) { return A[(size_t)a * k + a] < A[(size_t)b * k + b]; });
  for (int i = 0; i < k; ++i) {
    const int j = ord[i];
    ritz[i] = A[(size_t)j * k + j];
    const double y0 = Vm[j];  // row 0, column j
    weights[i] = y0 * y0;
    if (last_row) last_row[i] = Vm[(size_t)(k - 1) * k + j];
  }
  return HF_OK;
}

int32_t hf_create(const hf_model_desc* desc, int32_t hip_device, int32_t max_batch, int32_t max_m, hf_ctx** out) {
  if (!desc || !out) { set_create_err("hf_create: NULL argument"); return HF_EINVAL; }
  *out = nullptr;
  if (max_batch <= 0 || max_m < 0) { set_create_err("hf_create: max_batch must be > 0 and max_m >= 0"); return HF_EINVAL; }
  // the orthogonalisation kernels keep 32 bytes of LDS per basis vector, and hf_tridiag_readout stops at 2048
  if (max_m > HF_MAX_M) { set_create_err("hf_create: max_m must be at most 2000"); return HF_ESHAPE; }
  hf_ctx* c = new (std::nothrow) hf_ctx();
  if (!c) { set_create_err("hf_create: out of host memory"); return HF_ENOMEM; }
  c->desc = *desc;
  std::string why;
  int rc = build_layout(*desc, c->layout, &why);
  if (rc != HF_OK) { set_create_err("hf_create: " + why); delete c; return rc; }
  c->n = c->layout.back().offset + c->layout.back().count();
  c->bf = desc->param_dtype == HF_BF16;
  c->max_batch = max_batch;
  c->max_m = max_m;
  c->device = hip_device;
  // named offsets
  if (desc->arch != HF_ARCH_MLP) c->loff.resize(desc->n_layer);
  for (const auto& e : c->layout) {
    const std::string& nm = e.name;
    const int64_t o = e.offset;
    if (nm == "W1") c->off_w1 = o; else if (nm == "b1") c->off_b1 = o;
    else if (nm == "W2") c->off_w2 = o; else if (nm == "b2") c->off_b2 = o;
    else if (nm == "wte") c->off_wte = o; else if (nm == "wpe") c->off_wpe = o;
    else if (nm == "lnf.g" || nm == "rmsf.g") { c->off_nfg = o; c->layers_end = o + e.count(); }
    else if (nm == "lnf.b") { c->off_nfb = o; c->layers_end = o + e.count(); }
    else if (nm == "lm_head") c->off_head = o;
    else if (nm[0] == 'h') {
      const size_t dot = nm.find('.');
      const int l = std::stoi(nm.substr(1, dot - 1));
      if (c->layers_end == 0) c->layers_begin = o;
      c->layers_end = o + e.count();
      const std::string t = nm.substr(dot + 1);
      LayerOff& lo = c->loff[l];
      if (t == "ln1.g" || t == "rms1.g") lo.n1g = o; else if (t == "ln1.b") lo.n1b = o;
      else if (t == "ln2.g" || t == "rms2.g") lo.n2g = o; else if (t == "ln2.b") lo.n2b = o;
      else if (t == "Wqkv") lo.wqkv = o; else if (t == "bqkv") lo.bqkv = o;
      else if (t == "Wq") lo.wq = o; else if (t == "Wk") lo.wk = o; else if (t == "Wv") lo.wv = o;
      else if (t == "Wo") lo.wo = o; else if (t == "bo") lo.bo = o;
      else if (t == "Wfc") lo.wfc = o; else if (t == "bfc") lo.bfc = o;
      else if (t == "Wproj") lo.wproj = o; else if (t == "bproj") lo.bproj = o;
      else if (t == "Wgate") lo.wgate = o; else if (t == "Wup") lo.wup = o; else if (t == "Wdown") lo.wdown = o;
    }
    // H v blocks that are accumulated with atomics start from zero: every
    // vector parameter, the position table, and the token table unless the
    // tied head product writes it first.
    const bool tied_wte = (nm == "wte" && desc->arch == HF_ARCH_GPT && desc->tie_embeddings);
    if (e.shape[1] == 0 || nm == "wpe" || (nm == "wte" && !tied_wte)) {
      // (a range never straddles the start of the layers, which may be cleared as a whole)
      if (!c->zero_ranges.empty() && c->zero_ranges.back().first + c->zero_ranges.back().second == o && o != c->layers_begin)
        c->zero_ranges.back().second += e.count();
      else c->zero_ranges.push_back({o, e.count()});
    }
  }
  hipError_t he = hipSetDevice(hip_device);
  if (he != hipSuccess) {
    set_create_err(std::string("hf_create: hipSetDevice failed: ") + hipGetErrorString(he));
    (void)hipGetLastError();
    delete c;
    return HF_EDEVICE;
  }
  rc = c->plan_and_alloc();
  if (rc != HF_OK) { set_create_err("hf_create: " + c->err); hf_destroy(c); return rc; }
  *out = c;
  return HF_OK;
}

void hf_destroy(hf_ctx* ctx) {
  if (!ctx) return;
  if (ctx->arena) (void)hipFree(ctx->arena);
  if (ctx->host_scal) (void)hipHostFree(ctx->host_scal);
  if (ctx->aux_vec) (void)hipFree(ctx->aux_vec);
  delete ctx;
}

int64_t hf_num_params(const hf_ctx* ctx) { return ctx ? ctx->n : (int64_t)HF_EINVAL; }
int64_t hf_workspace_bytes(const hf_ctx* ctx) { return ctx ? ctx->arena_bytes : (int64_t)HF_EINVAL; }

const char* hf_last_error(const hf_ctx* ctx) {
  if (ctx) return ctx->err.c_str();
  static thread_local std::string copy;
  std::lock_guard<std::mutex> lk(g_err_mu);
  copy = g_create_err;
  return copy.c_str();
}

int32_t hf_hvp(hf_ctx* ctx, const void* params_dev, const void* inputs_dev, const int32_t* labels_dev, int32_t batch,
               int32_t seq, const float* v_dev, float* out_dev, double* loss_host, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hipStream_t st = (hipStream_t)hip_stream;
  if (out_dev == v_dev || (const void*)out_dev == params_dev) return ctx->fail(HF_EINVAL, "hf_hvp: out_dev aliases an input");
  int rc = ctx->hvp_enqueue(params_dev, inputs_dev, labels_dev, batch, seq, v_dev, out_dev, st);
  if (rc != HF_OK) return rc;
  return ctx->finish_hvp(loss_host, st);
}

int32_t hf_lanczos_init(hf_ctx* ctx, const float* q0_dev, int32_t reorth, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!q0_dev) return c->fail(HF_EINVAL, "hf_lanczos_init: NULL q0_dev");
  if (reorth != HF_REORTH_NONE && reorth != HF_REORTH_FULL) return c->fail(HF_EINVAL, "hf_lanczos_init: bad reorth");
  if (c->max_m <= 0) return c->fail(HF_ESHAPE, "hf_lanczos_init: context was created with max_m = 0");
  if (reorth == HF_REORTH_FULL && !c->basis) return c->fail(HF_ESHAPE, "hf_lanczos_init: context was created without a basis (basis_dtype HF_NONE)");
  c->lz_k = -1;
  c->iq = 0; c->iqp = 1; c->ir = 2;
  c->lz_reorth = reorth;
  const int bq = c->desc.basis_dtype == HF_BF16;
  const bool rows = c->lz_rows_are_vectors();
#define CKI(expr)                                                                                   \
  do {                                                                                              \
    hipError_t e_ = (expr);                                                                         \
    if (e_ != hipSuccess) return c->fail(HF_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)
  CKI(launch_fill_f32((float*)c->scal, S_COUNT * 2, 0.f, st));
  if ((uintptr_t)q0_dev & 15) {  // the kernels read 16 bytes at a time: stage an unaligned probe in r
    CKI(hipMemcpyAsync(c->lz_vec[c->ir], q0_dev, (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
    q0_dev = c->lz_vec[c->ir];
  }
  CKI(lz_norm_q0(q0_dev, c->n, c->scal, c->partials, st));
  CKI(hipMemcpyAsync(c->host_scal, c->scal, S_COUNT * sizeof(double), hipMemcpyDeviceToHost, st));
  CKI(hipStreamSynchronize(st));
  const double nrm = c->host_scal[S_Q0NORM];
  if (!(nrm > 0.0) || !std::isfinite(nrm)) return c->fail(HF_EINVAL, "hf_lanczos_init: q0 has zero or non-finite norm");
  // q_0 = q0 / ||q0||: row 0 of an fp32 basis is the working vector itself; a bf16 basis takes the
  // rounded copy, which is also the bf16 operand of the first product
  void* row0 = reorth == HF_REORTH_FULL ? c->basis : nullptr;
  bf16* vdst = c->bf ? ((bq && row0) ? nullptr : ((rows && c->basis_bf) ? c->basis_bf : c->vb)) : nullptr;
  CKI(lz_scale(q0_dev, rows ? nullptr : c->lz_vec[c->iq], row0, bq, vdst, c->n, c->scal, S_Q0NORM, 0.0, nullptr, st));
  c->lz_k = 0;
  c->lz_done = 0;
  c->lz_beta_prev = 0.0;
  c->vb_cur = c->bf ? ((bq && row0) ? (const bf16*)row0 : vdst) : nullptr;
  c->vb_of = c->bf ? c->cur_q() : nullptr;
  return HF_OK;
}

int32_t hf_lanczos_step(hf_ctx* ctx, const void* params_dev, const void* inputs_dev, const int32_t* labels_dev,
                        int32_t batch, int32_t seq, double tol, double* alpha_k, double* beta_k, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (c->lz_k < 0) return c->fail(HF_ESTATE, "hf_lanczos_step: call hf_lanczos_init first");
  if (c->lz_done) return c->fail(HF_ESTATE, "hf_lanczos_step: the iteration has ended (breakdown)");
  if (c->lz_reorth == HF_REORTH_FULL && c->lz_k >= c->max_m) return c->fail(HF_ESHAPE, "hf_lanczos_step: max_m iterations reached");
  float* r = c->lz_vec[c->ir];
  int rc = c->hvp_enqueue(params_dev, inputs_dev, labels_dev, batch, seq, c->cur_q(), r, st);
  if (rc != HF_OK) return rc;
  // a bad token or label (found on the device) leaves the iteration where it was
  return c->lanczos_update(r, tol, alpha_k, beta_k, c->flags, st);
}

int32_t hf_lanczos_update(hf_ctx* ctx, float* r_dev, double tol, double* alpha_k, double* beta_k,
                          void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!r_dev) return c->fail(HF_EINVAL, "hf_lanczos_update: NULL r_dev");
  if (c->lz_k < 0) return c->fail(HF_ESTATE, "hf_lanczos_update: call hf_lanczos_init first");
  if (c->lz_done) return c->fail(HF_ESTATE, "hf_lanczos_update: the iteration has ended (breakdown)");
  if (c->lz_reorth == HF_REORTH_FULL && c->lz_k >= c->max_m) return c->fail(HF_ESHAPE, "hf_lanczos_update: max_m iterations reached");
  if ((uintptr_t)r_dev & 15) return c->fail(HF_EINVAL, "hf_lanczos_update: r_dev must be 16-byte aligned");
  return c->lanczos_update(r_dev, tol, alpha_k, beta_k, nullptr, st);
}

int32_t hf_lanczos_iterations(const hf_ctx* ctx) { return ctx ? ctx->lz_k : (int32_t)HF_EINVAL; }

int32_t hf_lanczos_get_vector(hf_ctx* ctx, int32_t which, float* dst_dev, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!dst_dev) return c->fail(HF_EINVAL, "hf_lanczos_get_vector: NULL dst_dev");
  if (c->lz_k < 0) return c->fail(HF_ESTATE, "hf_lanczos_get_vector: no iteration in progress");
  if (which >= 0 && which < 3) {
    const float* src = which == 0 ? c->cur_q() : (which == 1 ? c->prev_q() : c->lz_vec[c->ir]);
    CKI(hipMemcpyAsync(dst_dev, src, (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
    return HF_OK;
  }
  const int j = which - 16;
  const int have = c->lz_reorth == HF_REORTH_FULL ? std::min(c->lz_k + 1, c->max_m) : 0;
  if (j < 0 || j >= have) return c->fail(HF_EINVAL, "hf_lanczos_get_vector: no such vector");
  const int bq = c->desc.basis_dtype == HF_BF16;
  CKI(lz_widen((char*)c->basis + (int64_t)j * c->ldq * (bq ? 2 : 4), bq, dst_dev, c->n, st));
  return HF_OK;
}

int32_t hf_slq(hf_ctx* ctx, const void* params_dev, const void* inputs_dev, const int32_t* labels_dev, int32_t batch,
               int32_t seq, const float* probes_dev, int32_t n_probes, int32_t m, int32_t reorth, double tol,
               double* alpha, double* beta, double* ritz, double* weights, int32_t* m_eff, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  if (!probes_dev || !alpha || !beta || !ritz || !weights || !m_eff) return c->fail(HF_EINVAL, "hf_slq: NULL argument");
  if (n_probes <= 0 || m <= 0) return c->fail(HF_EINVAL, "hf_slq: n_probes and m must be positive");
  if (m > c->max_m) return c->fail(HF_ESHAPE, "hf_slq: m exceeds max_m of hf_create");
  int status = HF_OK;
  for (int p = 0; p < n_probes; ++p) {
    int rc = hf_lanczos_init(c, probes_dev + (int64_t)p * c->n, reorth, hip_stream);
    if (rc != HF_OK) return rc;
    int k = 0;
    for (; k < m; ++k) {
      rc = hf_lanczos_step(c, params_dev, inputs_dev, labels_dev, batch, seq, tol, alpha + (int64_t)p * m + k,
                           beta + (int64_t)p * m + k, hip_stream);
      if (rc < 0) return rc;
      if (rc == HF_EBREAKDOWN) { status = HF_EBREAKDOWN; ++k; break; }
    }
    m_eff[p] = k;
    rc = hf_tridiag_readout(alpha + (int64_t)p * m, beta + (int64_t)p * m, k, ritz + (int64_t)p * m,
                            weights + (int64_t)p * m, nullptr);
    if (rc != HF_OK) return c->fail(rc, "hf_slq: read-out failed");
  }
  return status;
}

// ---- widened rows ---------------------------------------------------------------

int32_t hf_hvp_accumulate(hf_ctx* ctx, const void* params_dev, const void* inputs_dev, const int32_t* labels_dev,
                          int32_t n_samples, int32_t micro_batch, int32_t seq, const float* v_dev, float* out_dev,
                          double* loss_host, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!params_dev || !inputs_dev || !labels_dev || !v_dev || !out_dev) return c->fail(HF_EINVAL, "hf_hvp_accumulate: NULL argument");
  if (n_samples <= 0 || micro_batch <= 0) return c->fail(HF_EINVAL, "hf_hvp_accumulate: n_samples and micro_batch must be positive");
  if (micro_batch > c->max_batch) return c->fail(HF_ESHAPE, "hf_hvp_accumulate: micro_batch exceeds max_batch of hf_create");
  if (out_dev == v_dev || (const void*)out_dev == params_dev) return c->fail(HF_EINVAL, "hf_hvp_accumulate: out_dev aliases an input");
  if ((uintptr_t)out_dev & 15) return c->fail(HF_EINVAL, "hf_hvp_accumulate: out_dev must be 16-byte aligned");
  const bool mlp = c->desc.arch == HF_ARCH_MLP;
  const int64_t in_row = mlp ? (int64_t)c->desc.mlp_in * 4 : (int64_t)seq * 4;  // bytes per sample
  const int64_t lab_row = mlp ? 1 : seq;
  for (int b0 = 0; b0 < n_samples; b0 += micro_batch) {
    const int b = std::min(micro_batch, n_samples - b0);
    // the direction is the same for every micro-batch: its bf16 copy is made by the first product only
    if (b0 > 0 && c->bf) c->vb_of = v_dev;
    // h += u_B |B| / N: the weight goes into the adjoint seeds and every block of the product is added
    // to out_dev in place; the loss and the input checks accumulate on the device as well
    const int rc = c->hvp_enqueue(params_dev, (const char*)inputs_dev + b0 * in_row, labels_dev + b0 * lab_row, b, seq, v_dev,
                                  out_dev, st, (float)((double)b / (double)n_samples), b0 > 0);
    if (rc != HF_OK) return rc;
  }
  return c->finish_hvp(loss_host, st);
}

int32_t hf_hessian_column(hf_ctx* ctx, const void* params_dev, const void* inputs_dev, const int32_t* labels_dev,
                          int32_t batch, int32_t seq, int64_t index, float* column_dev, double* loss_host,
                          void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!column_dev) return c->fail(HF_EINVAL, "hf_hessian_column: NULL column_dev");
  if (index < 0 || index >= c->n) return c->fail(HF_EINVAL, "hf_hessian_column: index outside [0, n)");
  if ((const void*)column_dev == params_dev) return c->fail(HF_EINVAL, "hf_hessian_column: column_dev aliases params_dev");
  int rc = c->ensure_aux();
  if (rc != HF_OK) return rc;
  CKI(launch_fill_f32(c->aux_vec, c->n, 0.f, st));
  CKI(launch_fill_f32(c->aux_vec + index, 1, 1.f, st));
  rc = c->hvp_enqueue(params_dev, inputs_dev, labels_dev, batch, seq, c->aux_vec, column_dev, st);
  if (rc != HF_OK) return rc;
  return c->finish_hvp(loss_host, st);
}

// Both column-statistics entry points: `stats` is CS_STATS_WORDS device counters (the context's, or
// the library's static array); on failure *why names the reason.
static int column_stats_run(unsigned long long* stats, const float* h_dev, int64_t n, const float* thresholds,
                            int32_t n_thresholds, int32_t n_bins, int64_t* below, float* max_abs, int64_t* hist,
                            hipStream_t st, std::string* why) {
  auto bad = [&](int code, const std::string& m) { *why = m; return code; };
#define CKS(expr)                                                                                 \
  do {                                                                                            \
    hipError_t e_ = (expr);                                                                       \
    if (e_ != hipSuccess) return bad(HF_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)
  if (n < 0 || (n > 0 && !h_dev)) return bad(HF_EINVAL, "bad h_dev / n");
  if ((uintptr_t)h_dev & 3) return bad(HF_EINVAL, "h_dev must be 4-byte aligned");
  if (n_thresholds < 0 || n_thresholds > CS_MAX_THRESHOLDS) return bad(HF_EINVAL, "at most 16 thresholds");
  if (n_bins < 1 || n_bins > CS_MAX_BINS) return bad(HF_EINVAL, "n_bins must be in [1, 256]");
  if ((n_thresholds > 0 && (!thresholds || !below)) || !hist || !max_abs) return bad(HF_EINVAL, "NULL argument");
  if (n >= ((int64_t)1 << 40)) return bad(HF_ESHAPE, "n must be below 2^40");
  // sorted copy of the thresholds (padded with +inf), and where each caller threshold went
  ColThresholds thr;
  int order[CS_MAX_THRESHOLDS];
  for (int k = 0; k < n_thresholds; ++k) order[k] = k;
  std::stable_sort(order, order + n_thresholds, [&](int a, int b) { return thresholds[a] < thresholds[b]; });
  for (int k = 0; k < CS_MAX_THRESHOLDS; ++k) thr.t[k] = k < n_thresholds ? thresholds[order[k]] : INFINITY;
  for (int k = 0; k < n_thresholds; ++k)
    if (thresholds[k] != thresholds[k]) return bad(HF_EINVAL, "a threshold is NaN");
  unsigned long long hs[CS_STATS_WORDS];
  // the counters keep the previous call's values: cleared by a fill kernel, not by a memset, so that
  // the sequence stays valid under stream capture
  CKS(launch_fill_f32((float*)stats, CS_STATS_WORDS * 2, 0.f, st));
  if (n > 0) {
    CKS(launch_colstats_pass1(h_dev, n, thr, n_thresholds, stats, st));
    CKS(launch_colstats_hist(h_dev, n, stats + 24, n_bins, stats + 32, st));  // reads the maximum of the first pass
  }
  CKS(hipMemcpyAsync(hs, stats, (size_t)(32 + n_bins) * 8, hipMemcpyDeviceToHost, st));
  CKS(hipStreamSynchronize(st));
  // |h_i| < t_k (sorted) exactly when the entry reaches at most k thresholds: prefix sums of the buckets
  unsigned long long run = 0, valid = 0;
  for (int k = 0; k <= CS_MAX_THRESHOLDS; ++k) valid += hs[k];
  for (int k = 0; k < n_thresholds; ++k) {
    run += hs[k];
    below[order[k]] = (int64_t)run;
  }
  float mx;
  const unsigned bits = (unsigned)hs[24];
  memcpy(&mx, &bits, 4);
  *max_abs = mx;
  for (int k = 0; k < n_bins; ++k) hist[k] = mx > 0.f ? (int64_t)hs[32 + k] : 0;
  if (!(mx > 0.f)) hist[0] = (int64_t)valid;  // a column of zeros: every entry in the first bin
  return HF_OK;
#undef CKS
}

int32_t hf_column_stats(hf_ctx* ctx, const float* h_dev, int64_t n, const float* thresholds, int32_t n_thresholds,
                        int32_t n_bins, int64_t* below, float* max_abs, int64_t* hist, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  std::string why;
  const int rc = column_stats_run(ctx->stats_dev, h_dev, n, thresholds, n_thresholds, n_bins, below, max_abs, hist,
                                  (hipStream_t)hip_stream, &why);
  return rc == HF_OK ? rc : ctx->fail(rc, "hf_column_stats: " + why);
}

int32_t hf_column_stats_noalloc(const float* h_dev, int64_t n, const float* thresholds, int32_t n_thresholds,
                                int32_t n_bins, int64_t* below, float* max_abs, int64_t* hist, void* hip_stream) {
  unsigned long long* counters = nullptr;
  const hipError_t e = colstats_static_counters(&counters);
  if (e != hipSuccess) {
    set_create_err(std::string("hf_column_stats_noalloc: no address for the static counters: ") + hipGetErrorString(e));
    (void)hipGetLastError();
    return HF_EDEVICE;
  }
  std::string why;
  const int rc = column_stats_run(counters, h_dev, n, thresholds, n_thresholds, n_bins, below, max_abs, hist,
                                  (hipStream_t)hip_stream, &why);
  if (rc != HF_OK) set_create_err("hf_column_stats_noalloc: " + why);
  return rc;
}

int32_t hf_slq_density(const double* ritz, const double* weights, const int32_t* m_eff, int32_t n_probes, int32_t m,
                       double sigma, const double* grid, int32_t n_grid, double* density) {
  if (!ritz || !weights || !m_eff || !grid || !density || n_probes <= 0 || m <= 0 || n_grid < 0 || !(sigma > 0.0))
    return HF_EINVAL;
  for (int p = 0; p < n_probes; ++p)
    if (m_eff[p] < 0 || m_eff[p] > m) return HF_EINVAL;
  const double norm = 1.0 / (sigma * std::sqrt(2.0 * M_PI));
  for (int g = 0; g < n_grid; ++g) {
    double acc = 0.0;
    for (int p = 0; p < n_probes; ++p)
      for (int i = 0; i < m_eff[p]; ++i) {
        const double z = (grid[g] - ritz[(int64_t)p * m + i]) / sigma;
        acc += weights[(int64_t)p * m + i] * std::exp(-0.5 * z * z) * norm;
      }
    density[g] = acc / n_probes;
  }
  return HF_OK;
}

int32_t hf_slq_moments(const double* ritz, const double* weights, const int32_t* m_eff, int32_t n_probes, int32_t m,
                       int32_t n_moments, double* moments) {
  if (!ritz || !weights || !m_eff || !moments || n_probes <= 0 || m <= 0 || n_moments < 0) return HF_EINVAL;
  for (int p = 0; p < n_probes; ++p)
    if (m_eff[p] < 0 || m_eff[p] > m) return HF_EINVAL;
  for (int q = 0; q < n_moments; ++q) {
    double acc = 0.0;
    for (int p = 0; p < n_probes; ++p)
      for (int i = 0; i < m_eff[p]; ++i) acc += weights[(int64_t)p * m + i] * std::pow(ritz[(int64_t)p * m + i], (double)q);
    moments[q] = acc / n_probes;
  }
  return HF_OK;
}

// ---- Lanczos state hand-over (checkpoint / resume) --------------------------------
// Device image: 128-byte header, then q_k, q_{k-1} (fp32[n] each, 256-byte aligned
// starts), then the stored basis rows q_0 .. q_{rows-1} densely (n elements each) in the
// basis precision.
namespace {
struct LzHeader {
  int64_t magic, version, n, k, reorth, basis_dtype, done, rows;
  double beta_prev;
  int64_t pad[7];
};
static_assert(sizeof(LzHeader) == 128, "header size");
constexpr int64_t kLzMagic = 0x5a4c4648;  // "HFLZ"
int64_t lz_align(int64_t b) { return (b + 255) / 256 * 256; }
int64_t lz_rows(const hf_ctx* c) {
  return c->lz_reorth == HF_REORTH_FULL ? std::min<int64_t>(c->lz_k + 1, c->max_m) : 0;
}
int64_t lz_image_bytes(int64_t n, int64_t rows, int basis_dtype) {
  const int64_t be = basis_dtype == HF_BF16 ? 2 : 4;
  return 128 + 2 * lz_align(n * 4) + rows * n * be;
}
}  // namespace

int64_t hf_lanczos_state_bytes(const hf_ctx* ctx) {
  if (!ctx || ctx->lz_k < 0) return HF_ESTATE;
  return lz_image_bytes(ctx->n, lz_rows(ctx), ctx->desc.basis_dtype);
}

int32_t hf_lanczos_export(hf_ctx* ctx, void* state_dev, int64_t capacity_bytes, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (c->lz_k < 0) return c->fail(HF_ESTATE, "hf_lanczos_export: no iteration in progress");
  if (!state_dev || ((uintptr_t)state_dev & 255)) return c->fail(HF_EINVAL, "hf_lanczos_export: state_dev must be non-NULL and 256-byte aligned");
  const int64_t rows = lz_rows(c), need = lz_image_bytes(c->n, rows, c->desc.basis_dtype);
  if (capacity_bytes < need) return c->fail(HF_ESHAPE, "hf_lanczos_export: buffer too small (see hf_lanczos_state_bytes)");
  LzHeader h{};
  h.magic = kLzMagic; h.version = 1; h.n = c->n; h.k = c->lz_k; h.reorth = c->lz_reorth;
  h.basis_dtype = c->desc.basis_dtype; h.done = c->lz_done; h.rows = rows; h.beta_prev = c->lz_beta_prev;
  char* base = (char*)state_dev;
  CKI(hipMemcpyAsync(base, &h, sizeof(h), hipMemcpyHostToDevice, st));
  CKI(hipStreamSynchronize(st));  // h lives on this stack frame
  const int64_t vb = lz_align(c->n * 4);
  CKI(hipMemcpyAsync(base + 128, c->cur_q(), (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
  CKI(hipMemcpyAsync(base + 128 + vb, c->prev_q(), (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
  const int64_t be = c->desc.basis_dtype == HF_BF16 ? 2 : 4;
  if (rows > 0)
    CKI(hipMemcpy2DAsync(base + 128 + 2 * vb, (size_t)c->n * be, c->basis, (size_t)c->ldq * be, (size_t)c->n * be, (size_t)rows,
                         hipMemcpyDeviceToDevice, st));
  CKI(hipStreamSynchronize(st));
  return HF_OK;
}

int32_t hf_lanczos_import(hf_ctx* ctx, const void* state_dev, int64_t bytes, void* hip_stream) {
  if (!ctx) return HF_EINVAL;
  hf_ctx* c = ctx;
  hipStream_t st = (hipStream_t)hip_stream;
  if (!state_dev || ((uintptr_t)state_dev & 255) || bytes < 128) return c->fail(HF_EINVAL, "hf_lanczos_import: bad state_dev / bytes");
  if (c->max_m <= 0) return c->fail(HF_ESHAPE, "hf_lanczos_import: context was created with max_m = 0");
  LzHeader h;
  CKI(hipMemcpyAsync(&h, state_dev, sizeof(h), hipMemcpyDeviceToHost, st));
  CKI(hipStreamSynchronize(st));
  if (h.magic != kLzMagic || h.version != 1) return c->fail(HF_EINVAL, "hf_lanczos_import: not a Lanczos state image");
  if (h.n != c->n) return c->fail(HF_ESHAPE, "hf_lanczos_import: the image belongs to a model with another parameter count");
  if (h.k < 0 || h.rows < 0 || (h.reorth != HF_REORTH_NONE && h.reorth != HF_REORTH_FULL)) return c->fail(HF_EINVAL, "hf_lanczos_import: corrupt header");
  if (h.reorth == HF_REORTH_FULL) {
    if (!c->basis) return c->fail(HF_ESHAPE, "hf_lanczos_import: the image holds a basis, the context was created without one");
    if (h.basis_dtype != c->desc.basis_dtype) return c->fail(HF_ESHAPE, "hf_lanczos_import: basis precision differs from the context's");
    if (h.rows > c->max_m) return c->fail(HF_ESHAPE, "hf_lanczos_import: more basis rows than max_m of hf_create");
    // rows = k + 1, or k once the exporter's basis was full; such an image continues nowhere, and a
    // context with room for more rows would orthogonalise against a row k that was never stored
    if (h.rows != std::min<int64_t>(h.k + 1, c->max_m)) return c->fail(HF_ESHAPE, "hf_lanczos_import: the image was exported with its basis full; max_m of this context must equal its number of rows");
  } else if (h.rows != 0) {
    return c->fail(HF_EINVAL, "hf_lanczos_import: corrupt header");
  }
  if (bytes < lz_image_bytes(h.n, h.rows, (int)h.basis_dtype)) return c->fail(HF_EINVAL, "hf_lanczos_import: image is truncated");
  const char* base = (const char*)state_dev;
  const int64_t vb = lz_align(c->n * 4);
  c->iq = 0; c->iqp = 1; c->ir = 2;
  CKI(launch_fill_f32((float*)c->scal, S_COUNT * 2, 0.f, st));
  // (with an fp32 basis q_k and q_{k-1} are also rows k and k - 1 below, which is where the
  // iteration reads them; the copies in lz_vec serve a full basis, whose last q has no row)
  CKI(hipMemcpyAsync(c->lz_vec[0], base + 128, (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
  c->vb_of = nullptr;  // the imported q_k has no bf16 copy yet
  CKI(hipMemcpyAsync(c->lz_vec[1], base + 128 + vb, (size_t)c->n * 4, hipMemcpyDeviceToDevice, st));
  const int64_t be = c->desc.basis_dtype == HF_BF16 ? 2 : 4;
  if (h.rows > 0)
    CKI(hipMemcpy2DAsync(c->basis, (size_t)c->ldq * be, base + 128 + 2 * vb, (size_t)c->n * be, (size_t)c->n * be, (size_t)h.rows,
                         hipMemcpyDeviceToDevice, st));
  if (c->basis_bf)  // the bf16 copies of the rows are not part of the image
    for (int64_t j = 0; j < h.rows; ++j)
      CKI(launch_f32_to_bf16((const float*)c->basis + j * c->ldq, c->basis_bf + j * c->ldq, c->n, st));
  CKI(hipStreamSynchronize(st));
  c->lz_k = (int)h.k;
  c->lz_reorth = (int)h.reorth;
  c->lz_done = (int)h.done;
  c->lz_beta_prev = h.beta_prev;
  return HF_OK;
}

}  // extern "C"
