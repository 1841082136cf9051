// Host-side schedule of the Hessian-vector product: Algorithm 1 of the paper
// (u = d<dL/dp, v>/dp on one batch) evaluated forward-over-reverse.  One sweep
// forward computes every activation a together with its tangent a_t (its
// derivative along the parameter direction v); one sweep backward computes
// every adjoint da with its tangent da_t and emits, per parameter tensor, only
// the H v block (the tangent of the gradient); the plain gradient is never
// formed.  For a linear layer Y = X W + b:
//   Y_t = X_t W + X W_t + b_t          dX   = dY W^T
//   dX_t = dY_t W^T + dY W_t^T         (Hv)_W = X_t^T dY + X^T dY_t
//   (Hv)_b = column sums of dY_t
#include "engine.h"

#include <algorithm>
#include <cmath>

using namespace hf;

// ------------------------------------------------------------------ layout ----

int hf::build_layout(const hf_model_desc& d, std::vector<LayoutEntry>& out, std::string* why) {
  out.clear();
  int64_t off = 0;
  auto add = [&](const std::string& nm, int64_t a, int64_t b) {
    LayoutEntry e;
    e.name = nm; e.offset = off; e.shape[0] = a; e.shape[1] = b;
    off += e.count();
    out.push_back(e);
  };
  auto bad = [&](const char* m) { if (why) *why = m; return (int)HF_EINVAL; };
  if (d.param_dtype != HF_F32 && d.param_dtype != HF_BF16) return bad("param_dtype must be HF_F32 or HF_BF16");
  if (d.basis_dtype != HF_F32 && d.basis_dtype != HF_BF16 && d.basis_dtype != HF_NONE) return bad("basis_dtype must be HF_F32, HF_BF16 or HF_NONE");
  if (d.arch == HF_ARCH_MLP) {
    if (d.mlp_in <= 0 || d.mlp_hidden <= 0 || d.mlp_out <= 1) return bad("MLP sizes must be positive (mlp_out >= 2)");
    add("W1", d.mlp_in, d.mlp_hidden); add("b1", d.mlp_hidden, 0);
    add("W2", d.mlp_hidden, d.mlp_out); add("b2", d.mlp_out, 0);
    return HF_OK;
  }
  if (d.arch != HF_ARCH_GPT && d.arch != HF_ARCH_LLAMA) return bad("unknown arch");
  if (d.n_layer <= 0 || d.d_model <= 0 || d.n_head <= 0 || d.d_ff <= 0 || d.vocab <= 1 || d.max_seq <= 0)
    return bad("transformer sizes must be positive");
  if (d.d_model % d.n_head) return bad("d_model must be a multiple of n_head");
  if (d.d_model > 8192) return bad("d_model > 8192 is not supported by the norm kernels");
  if (!(d.norm_eps > 0.f)) return bad("norm_eps must be positive");
  if (d.activation != HF_ACT_GELU_ERF && d.activation != HF_ACT_GELU_TANH) return bad("activation must be HF_ACT_GELU_ERF or HF_ACT_GELU_TANH");
  if (d.attention != HF_ATTN_AUTO && d.attention != HF_ATTN_STREAMED && d.attention != HF_ATTN_STORED) return bad("attention must be HF_ATTN_AUTO, HF_ATTN_STREAMED or HF_ATTN_STORED");
  if (d.primal != HF_PRIMAL_AUTO && d.primal != HF_PRIMAL_PAIRS && d.primal != HF_PRIMAL_SINGLE) return bad("primal must be HF_PRIMAL_AUTO, HF_PRIMAL_PAIRS or HF_PRIMAL_SINGLE");
  const int64_t D = d.d_model, F = d.d_ff, V = d.vocab;
  const int hkv = d.n_kv_head > 0 ? d.n_kv_head : d.n_head;
  if (hkv > d.n_head || d.n_head % hkv) return bad("n_kv_head must divide n_head");
  if (d.arch == HF_ARCH_GPT && hkv != d.n_head) return bad("grouped-query attention (n_kv_head) is a LLAMA option");
  const int64_t Dkv = D / d.n_head * hkv;
  if (d.arch == HF_ARCH_GPT) {
    add("wte", V, D); add("wpe", d.max_seq, D);
    for (int l = 0; l < d.n_layer; ++l) {
      const std::string p = "h" + std::to_string(l) + ".";
      add(p + "ln1.g", D, 0); add(p + "ln1.b", D, 0);
      add(p + "Wqkv", D, 3 * D); add(p + "bqkv", 3 * D, 0);
      add(p + "Wo", D, D); add(p + "bo", D, 0);
      add(p + "ln2.g", D, 0); add(p + "ln2.b", D, 0);
      add(p + "Wfc", D, F); add(p + "bfc", F, 0);
      add(p + "Wproj", F, D); add(p + "bproj", D, 0);
    }
    add("lnf.g", D, 0); add("lnf.b", D, 0);
    if (!d.tie_embeddings) add("lm_head", D, V);
  } else {
    if ((d.d_model / d.n_head) % 2) return bad("rotary embedding needs an even head width");
    if (!(d.rope_theta > 0.f)) return bad("rope_theta must be positive");
    add("wte", V, D);
    for (int l = 0; l < d.n_layer; ++l) {
      const std::string p = "h" + std::to_string(l) + ".";
      add(p + "rms1.g", D, 0);
      add(p + "Wq", D, D); add(p + "Wk", D, Dkv); add(p + "Wv", D, Dkv); add(p + "Wo", D, D);
      add(p + "rms2.g", D, 0);
      add(p + "Wgate", D, F); add(p + "Wup", D, F); add(p + "Wdown", F, D);
    }
    add("rmsf.g", D, 0); add("lm_head", D, V);
  }
  return HF_OK;
}

// --------------------------------------------------------------- workspace ----

namespace {
struct Planner {
  int64_t off = 0;
  std::vector<std::pair<void**, int64_t>> fix;
  template <typename T>
  void add(T*& ptr, int64_t bytes) {
    fix.push_back({(void**)&ptr, off});
    off += (std::max<int64_t>(bytes, 1) + 255) / 256 * 256;
  }
};
int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
}  // namespace

int hf_ctx::plan_and_alloc() {
  Planner pl;
  const int64_t e = bf ? 2 : 4;
  if (desc.arch == HF_ARCH_MLP) {
    const int64_t B = max_batch, Hd = desc.mlp_hidden, O = desc.mlp_out;
    lb.resize(1);
    LayerBuf& b = lb[0];
    b = LayerBuf{};
    pl.add(b.f, B * Hd * e); pl.add(b.f_t, B * Hd * e);
    pl.add(b.g, B * Hd * e); pl.add(b.g_t, B * Hd * e);
    pl.add(dg, B * Hd * e); pl.add(dg_t, B * Hd * e);
    ldz = round_up(O, 8);
    pl.add(z, B * ldz * 4); pl.add(z_t, B * ldz * 4);
    pl.add(dz, B * ldz * e); pl.add(dz_t, B * ldz * e);
    pl.add(loss_rows, B * 4);
    if (bf) pl.add(xin, B * desc.mlp_in * e);
  } else {
    const int64_t S = desc.max_seq, B = max_batch, T = B * S, D = desc.d_model, F = desc.d_ff, H = desc.n_head;
    const int64_t SS = B * H * S * S;
    const bool llama = desc.arch == HF_ARCH_LLAMA;
    const int64_t Dkv = D / H * (desc.n_kv_head > 0 ? desc.n_kv_head : H);  // key / value width
    const int64_t W3 = D + 2 * Dkv;                                           // packed q | k | v row
    {
      const bool can = bf && attn_flash_supported((int)(D / H), W3, D);
      if (desc.attention == HF_ATTN_STREAMED && !can)
        return fail(HF_ESHAPE, "HF_ATTN_STREAMED needs bf16 parameters, a head width of 32, 64 or 128 and d_model a multiple of 8");
      flash = can && desc.attention != HF_ATTN_STORED && (desc.attention == HF_ATTN_STREAMED || attn_flash_preferred((int)(D / H), B * H, S));
    }
    pairs = bf && (desc.primal == HF_PRIMAL_PAIRS || (desc.primal == HF_PRIMAL_AUTO && llama));
    const int64_t SSa = flash ? 0 : SS;  // the S x S buffers exist only for the unstreamed paths
    lb.resize(desc.n_layer);
    for (auto& b : lb) {
      b = LayerBuf{};
      pl.add(b.x1, T * D * 4); pl.add(b.x1_t, T * D * 4); pl.add(b.x2, T * D * 4); pl.add(b.x2_t, T * D * 4);
      pl.add(b.st1, T * 16); pl.add(b.st2, T * 16);
      pl.add(b.a, T * D * e); pl.add(b.a_t, T * D * e);
      pl.add(b.qkv, T * W3 * e); pl.add(b.qkv_t, T * W3 * e);
      pl.add(b.P, SSa * e); pl.add(b.P_t, SSa * e);
      if (flash) pl.add(b.att_stat, SS / S * 2 * 4);
      if (flash && pairs) { pl.add(b.qkv_lo, T * W3 * e); pl.add(b.o_lo, T * D * e); }
      pl.add(b.o, T * D * e); pl.add(b.o_t, T * D * e);
      pl.add(b.m, T * D * e); pl.add(b.m_t, T * D * e);
      pl.add(b.f, T * F * e); pl.add(b.f_t, T * F * e);
      pl.add(b.g, T * F * e); pl.add(b.g_t, T * F * e);
      if (llama) { pl.add(b.up, T * F * e); pl.add(b.up_t, T * F * e); }
    }
    pl.add(xL, T * D * 4); pl.add(xL_t, T * D * 4); pl.add(stf, T * 16);
    pl.add(xf, T * D * e); pl.add(xf_t, T * D * e);
    if (pairs) {
      pl.add(xf_lo, T * D * e); pl.add(a_lo, T * D * e); pl.add(o_lo, T * D * e); pl.add(qkv_lo, T * W3 * e);
      pl.add(P_lo, SSa * e); pl.add(f_lo, T * F * e); pl.add(g_lo, T * F * e);
      if (llama) pl.add(up_lo, T * F * e);
    }
    if (llama) { pl.add(rq, T * (D + Dkv) * 4); pl.add(rq_t, T * (D + Dkv) * 4); }
    if (llama && Dkv != D) {  // grouped heads: dV is summed over a group in fp32, then rounded once
      pl.add(rv, T * Dkv * 4); pl.add(rv_t, T * Dkv * 4);
      if (bf) { pl.add(dvb, T * Dkv * e); pl.add(dvb_t, T * Dkv * e); }
    }
    ldz = round_up(desc.vocab, 64);
    pl.add(z, T * ldz * 4); pl.add(z_t, T * ldz * 4);
    pl.add(dz, T * ldz * e); pl.add(dz_t, T * ldz * e);
    pl.add(loss_rows, T * 4);
    pl.add(sc, SSa * 4); pl.add(sc_t, SSa * 4);
    att_SS = SSa;
    pl.add(norm_part, (int64_t)NORM_PART_BLOCKS * 3 * D * 4);
    if (bf) pl.add(gemm_ws, GEMM_WS_ELEMS * 4);
    if (bf) {
      const int64_t rows = SS / desc.max_seq, np = (desc.max_seq + 63) / 64;  // B*H*S rows
      pl.add(att_part, (flash ? 0 : rows * np) * 3 * 4); pl.add(att_rstat, rows * 3 * 4);
    }
    pl.add(dS, SSa * e); pl.add(dS_t, SSa * e);
    pl.add(dx, T * D * 4); pl.add(dx_t, T * D * 4); pl.add(tmpd, T * D * 4); pl.add(tmpd_t, T * D * 4);
    if (bf) { pl.add(dxb, T * D * e); pl.add(dxb_t, T * D * e); pl.add(dxb2, T * D * e); pl.add(dxb2_t, T * D * e); }
    pl.add(dob, T * D * e); pl.add(dob_t, T * D * e);
    pl.add(dqkv, T * W3 * e); pl.add(dqkv_t, T * W3 * e);
    pl.add(dg, T * F * e); pl.add(dg_t, T * F * e);
    if (llama) {
      pl.add(dup, T * F * e); pl.add(dup_t, T * F * e);
      pl.add(dy, T * F * e); pl.add(dy_t, T * F * e);
    }
  }
  if (bf) pl.add(vb, n * 2);
  pl.add(flags, 64);
  pl.add(loss_dev, 64);
  pl.add(stats_dev, CS_STATS_WORDS * 8);
  // Lanczos
  if (max_m > 0) {
    for (int i = 0; i < 3; ++i) pl.add(lz_vec[i], n * 4);
    ldq = round_up(n, 64);
    if (desc.basis_dtype != HF_NONE) pl.add(basis, (int64_t)max_m * ldq * (desc.basis_dtype == HF_BF16 ? 2 : 4));
    if (desc.basis_dtype == HF_F32 && bf) pl.add(basis_bf, (int64_t)max_m * ldq * 2);
    pl.add(scal, S_COUNT * 8);
    pl.add(cvec, (int64_t)(max_m + 1) * 8);
    pl.add(partials, std::max<int64_t>((int64_t)LZ_NBLK * (max_m + 1), 3 * LZ_NBLK_VEC) * 8);
  }
  arena_bytes = pl.off;
  hipError_t e1 = hipMalloc((void**)&arena, (size_t)arena_bytes);
  if (e1 != hipSuccess) {
    arena = nullptr;
    (void)hipGetLastError();
    return fail(HF_ENOMEM, "hipMalloc of " + std::to_string(arena_bytes) + " bytes failed: " + hipGetErrorString(e1));
  }
  for (auto& f : pl.fix) *f.first = arena + f.second;
  if (!bf) { dxb = dx; dxb_t = dx_t; dxb2 = dx; dxb2_t = dx_t; }
  if (max_m > 0) {
    e1 = hipHostMalloc((void**)&host_scal, (S_COUNT + 2) * sizeof(double), hipHostMallocDefault);
    if (e1 != hipSuccess) return fail(HF_ENOMEM, std::string("hipHostMalloc failed: ") + hipGetErrorString(e1));
  }
  return HF_OK;
}

// ------------------------------------------------------------ GEMM helpers ----

namespace {

#define CK(expr)                                                                                   \
  do {                                                                                             \
    hipError_t e_ = (expr);                                                                        \
    if (e_ != hipSuccess) return c->fail(HF_EDEVICE, std::string(#expr) + ": " + hipGetErrorString(e_)); \
  } while (0)

struct Lin {
  hf_ctx* c;
  const void* params;
  const float* v;
  float* out;
  hipStream_t st;
  int bf;
  const void* Wp(int64_t off) const { return (const char*)params + off * (bf ? 2 : 4); }
  const void* Wt(int64_t off) const { return bf ? (const void*)(c->vb_cur + off) : (const void*)(v + off); }

  // Y = X W (+ b) (+ add);  Y_t = X_t W + X W_t (+ b_t) (+ add_t).   W: [K, N] at woff.
  // X_t == nullptr means a zero input tangent.
  int fwd(const void* X, const void* X_t, int M, int K, int N, int64_t ldx, int64_t woff, int64_t boff, void* Y,
          void* Y_t, int64_t ldy, int out_bf16, const float* add = nullptr, const float* add_t = nullptr,
          int transW = 0, int64_t ldw = -1, const void* X_lo = nullptr, void* Y_lo = nullptr) const {
    // X_lo (bf16 mode): low-order half of the primal input, added as a second
    // term against the same (exact bf16) weights; Y_lo: low-order half of a
    // bf16 primal output.  The primal forward chain so keeps ~16 mantissa
    // bits; tangents and adjoints (linear in their inputs) use the high halves.
    Gemm g;
    g.M = M; g.N = N; g.K = K; g.lda = ldx; g.ldb = ldw < 0 ? N : ldw; g.ldc = ldy; g.transB = transW;
    g.in_bf16 = bf; g.out_bf16 = out_bf16;
    g.ws = c->gemm_ws; g.ws_elems = c->gemm_ws ? GEMM_WS_ELEMS : 0;
    g.A[0] = X; g.B[0] = Wp(woff); g.C = Y; g.Cadd = add;
    if (X_lo) { g.A[1] = X_lo; g.B[1] = g.B[0]; }
    if (out_bf16) g.C_lo = Y_lo;
    if (boff >= 0) g.bias = Wp(boff);
    if (X_t) {  // primal and tangent in one (dual-output) product
      g.At = X_t; g.Bt = Wt(woff); g.Ct = Y_t; g.Cadd_t = add_t;
      if (boff >= 0) g.bias_t = v + boff;
      CK(launch_gemm(g, st));
      return HF_OK;
    }
    CK(launch_gemm(g, st));
    Gemm t = g;
    t.A[1] = nullptr; t.B[1] = nullptr; t.C_lo = nullptr;
    t.C = Y_t; t.Cadd = add_t; t.bias = nullptr;
    if (boff >= 0) t.bias_t = v + boff;
    t.A[0] = X; t.B[0] = Wt(woff);
    CK(launch_gemm(t, st));
    return HF_OK;
  }

  // dX = dY W^T (+ add);  dX_t = dY_t W^T + dY W_t^T (+ add_t).   W: [K_in, N_out] at woff.
  int bwd_dx(const void* dY, const void* dY_t, int M, int Kin, int Nout, int64_t lddy, int64_t woff, void* dX,
             void* dX_t, int64_t lddx, int out_bf16, const float* add = nullptr, const float* add_t = nullptr,
             int transW = 0, int64_t ldw = -1) const {
    Gemm g;
    g.M = M; g.N = Kin; g.K = Nout; g.lda = lddy; g.ldb = ldw < 0 ? Nout : ldw; g.ldc = lddx; g.transB = !transW;
    g.in_bf16 = bf; g.out_bf16 = out_bf16;
    g.ws = c->gemm_ws; g.ws_elems = c->gemm_ws ? GEMM_WS_ELEMS : 0;
    g.A[0] = dY; g.B[0] = Wp(woff); g.C = dX; g.Cadd = add;
    // Few output tiles and a long contraction (the head: K = vocabulary): two
    // split-K products; otherwise one dual-output product.
    const int64_t tiles = ((int64_t)(M + 127) / 128) * ((Kin + 127) / 128);
    if (!out_bf16 && tiles < 256 && Nout >= 8192 && (tiles * 2 > 256 || !c->gemm_ws)) {
      g.allow_splitk = 1;
      CK(launch_gemm(g, st));
      Gemm t = g;
      t.C = dX_t; t.Cadd = add_t;
      t.A[0] = dY_t; t.B[0] = Wp(woff); t.A[1] = dY; t.B[1] = Wt(woff);
      CK(launch_gemm(t, st));
      return HF_OK;
    }
    g.At = dY_t; g.Bt = Wt(woff); g.Ct = dX_t; g.Cadd_t = add_t;
    CK(launch_gemm(g, st));
    return HF_OK;
  }

  // (Hv)_W = X_t^T dY + X^T dY_t  -> out[woff] as [Kin, Nout];  (Hv)_b += colsum(dY_t).
  // defer != nullptr: the product is described there instead of launched (the caller launches the
  // products of a layer together); the bias sums are still taken at once.
  int bwd_dw(const void* X, const void* X_t, const void* dY, const void* dY_t, int T, int Kin, int Nout, int64_t ldx,
             int64_t lddy, int64_t woff, int64_t boff, const void* dYt_for_bias, int bias_src_bf16, Gemm* defer = nullptr) const {
    Gemm g;
    g.M = Kin; g.N = Nout; g.K = T; g.lda = ldx; g.ldb = lddy; g.ldc = Nout; g.transA = 1;
    g.in_bf16 = bf; g.out_bf16 = 0;
    g.allow_splitk = 1;
    g.c_zeroed = c->dw_prezeroed && woff >= c->layers_begin && woff < c->layers_end;
    g.C = out + woff;
    if (c->acc_mode) g.Cadd = out + woff;
    if (X_t) { g.A[0] = X_t; g.B[0] = dY; g.A[1] = X; g.B[1] = dY_t; }
    else { g.A[0] = X; g.B[0] = dY_t; }
    if (defer) *defer = g;
    else CK(launch_gemm(g, st));
    if (boff >= 0) CK(launch_colsum(bias_src_bf16, dYt_for_bias, T, Nout, lddy, out + boff, st));
    return HF_OK;
  }
};

}  // namespace

// ------------------------------------------------------------------- common ----

int hf_ctx::hvp_enqueue(const void* params, const void* inputs, const int32_t* labels, int batch, int seq,
                        const float* v, float* out, hipStream_t st, float seed_scale, int accumulate) {
  hf_ctx* c = this;
  if (!params || !inputs || !labels || !v || !out) return fail(HF_EINVAL, "hf_hvp: NULL pointer argument");
  if (((uintptr_t)v | (uintptr_t)out | (uintptr_t)params) & 15) return fail(HF_EINVAL, "hf_hvp: params, v and out must be 16-byte aligned");
  if (batch <= 0 || batch > max_batch) return fail(HF_ESHAPE, "hf_hvp: batch outside [1, max_batch]");
  if (desc.arch != HF_ARCH_MLP && (seq <= 0 || seq > desc.max_seq)) return fail(HF_ESHAPE, "hf_hvp: seq outside [1, max_seq]");
  if (desc.arch != HF_ARCH_MLP && (int64_t)batch * seq > (int64_t)max_batch * desc.max_seq) return fail(HF_ESHAPE, "hf_hvp: too many tokens");
  // accumulate: out += seed_scale * H v (every block of H v is written through Cadd = C or added with
  // atomics, so nothing is cleared); the error bits stay, the count of valid labels starts over
  acc_mode = accumulate;
  seed = seed_scale;
  if (accumulate) CK(launch_fill_f32((float*)(flags + 1), 1, 0.f, st));
  else CK(launch_fill_f32((float*)flags, 2, 0.f, st));
  // Small models: every weight-gradient product of a layer splits k and adds into a cleared
  // result, and the vectors between them are accumulated with atomics as well.  One pass over the
  // layers' whole range then replaces a fill per matrix and per group of vectors.
  dw_prezeroed = 0;
  if (!accumulate && bf && desc.arch != HF_ARCH_MLP && layers_end > layers_begin) {
    const int T = batch * seq, D = desc.d_model, F = desc.d_ff;
    const int hkv = desc.n_kv_head > 0 ? desc.n_kv_head : desc.n_head, Dkv = D / desc.n_head * hkv;
    bool all = gemm_mfma_splits_k(D, D, T, 2) && gemm_mfma_splits_k(D, F, T, 2) && gemm_mfma_splits_k(F, D, T, 2);
    if (desc.arch == HF_ARCH_GPT) all = all && gemm_mfma_splits_k(D, 3 * D, T, 2);
    else all = all && gemm_mfma_splits_k(D, Dkv, T, 2);
    if (all) {
      CK(launch_fill_f32(out + layers_begin, layers_end - layers_begin, 0.f, st));
      dw_prezeroed = 1;
    }
  }
  if (!accumulate) for (auto& zr : zero_ranges) {
    if (dw_prezeroed && zr.first >= layers_begin && zr.first + zr.second <= layers_end) continue;
    CK(launch_fill_f32(out + zr.first, zr.second, 0.f, st));
  }
  // The Lanczos update leaves the bf16 copy of q_{k+1} in vb; every other direction is converted here.
  if (bf && !(vb_of != nullptr && vb_of == v)) {
    CK(launch_f32_to_bf16(v, vb, n, st));
    vb_cur = vb;
  }
  vb_of = nullptr;
  if (desc.arch == HF_ARCH_MLP) return hvp_mlp(params, inputs, labels, batch, v, out, st);
  return hvp_transformer(params, (const int32_t*)inputs, labels, batch, seq, v, out, st);
}

int hf_ctx::ensure_aux() {
  if (aux_vec) return HF_OK;
  hipError_t e = hipMalloc((void**)&aux_vec, (size_t)n * 4);
  if (e != hipSuccess) {
    aux_vec = nullptr;
    (void)hipGetLastError();
    return fail(HF_ENOMEM, "hipMalloc of the auxiliary vector (" + std::to_string(n * 4) + " bytes) failed");
  }
  return HF_OK;
}

int hf_ctx::finish_hvp(double* loss_host, hipStream_t st) {
  hf_ctx* c = this;
  struct { int flags[2]; double loss; } h;
  CK(hipMemcpyAsync(h.flags, flags, 2 * sizeof(int), hipMemcpyDeviceToHost, st));
  CK(hipMemcpyAsync(&h.loss, loss_dev, sizeof(double), hipMemcpyDeviceToHost, st));
  CK(hipStreamSynchronize(st));
  if (h.flags[0] & 1) return fail(HF_EINVAL, "token id outside [0, vocab)");
  if (h.flags[0] & 2) return fail(HF_EINVAL, "label >= number of classes");
  if (h.flags[1] == 0 || (h.flags[0] & 4)) return fail(HF_EINVAL, "no valid label in the batch");
  if (loss_host) *loss_host = h.loss;
  return HF_OK;
}

// ---------------------------------------------------------------------- MLP ----

int hf_ctx::hvp_mlp(const void* params, const void* inputs, const int32_t* labels, int B, const float* v, float* out,
                    hipStream_t st) {
  hf_ctx* c = this;
  const int I = desc.mlp_in, Hd = desc.mlp_hidden, O = desc.mlp_out;
  Lin L{this, params, v, out, st, bf};
  LayerBuf& b = lb[0];
  const void* X = inputs;
  if (bf) { CK(launch_f32_to_bf16((const float*)inputs, (bf16*)xin, (int64_t)B * I, st)); X = xin; }
  int rc;
  if ((rc = L.fwd(X, nullptr, B, I, Hd, I, off_w1, off_b1, b.f, b.f_t, Hd, bf))) return rc;
  CK(launch_act_fwd(bf, ACT_TANH, b.f, b.f_t, nullptr, b.g, b.g_t, nullptr, (int64_t)B * Hd, st));
  if ((rc = L.fwd(b.g, b.g_t, B, Hd, O, Hd, off_w2, off_b2, z, z_t, ldz, 0))) return rc;
  CK(launch_count_valid(labels, B, O, flags + 1, flags, st));
  CK(launch_ce(bf, z, z_t, labels, flags + 1, B, O, ldz, dz, dz_t, loss_rows, seed, st));
  CK(launch_sum_rows_f64(loss_rows, B, flags + 1, loss_dev, (double)seed, acc_mode, flags, st));
  if ((rc = L.bwd_dw(b.g, b.g_t, dz, dz_t, B, Hd, O, Hd, ldz, off_w2, off_b2, dz_t, bf))) return rc;
  if ((rc = L.bwd_dx(dz, dz_t, B, Hd, O, ldz, off_w2, dg, dg_t, Hd, bf))) return rc;
  CK(launch_act_bwd(bf, ACT_TANH, b.f, b.f_t, dg, dg_t, dg, dg_t, (int64_t)B * Hd, st));
  if ((rc = L.bwd_dw(X, nullptr, dg, dg_t, B, I, Hd, I, Hd, off_w1, off_b1, dg_t, bf))) return rc;
  return HF_OK;
}

// -------------------------------------------------------------- transformer ----

int hf_ctx::hvp_transformer(const void* params, const int32_t* tok, const int32_t* labels, int B, int S,
                            const float* v, float* out, hipStream_t st) {
  hf_ctx* c = this;
  const int D = desc.d_model, H = desc.n_head, dh = D / H, F = desc.d_ff, V = desc.vocab, NL = desc.n_layer;
  const int T = B * S;
  const bool llama = desc.arch == HF_ARCH_LLAMA;
  const int rms = llama ? 1 : 0;
  const float eps = desc.norm_eps;
  const float cs = 1.f / sqrtf((float)dh);
  const int gelu_kind = desc.activation == HF_ACT_GELU_TANH ? ACT_GELU_TANH : ACT_GELU;
  // grouped-query attention: Hkv key/value heads, query head h reads head h / grp
  const int Hkv = desc.n_kv_head > 0 ? desc.n_kv_head : H, grp = H / Hkv;
  const int Dkv = Hkv * dh, W3 = D + 2 * Dkv, offK = D, offV = D + Dkv, RQ = D + Dkv;
  const int64_t e = bf ? 2 : 4;
  Lin L{this, params, v, out, st, bf};
  auto at = [&](void* p, int64_t elems) -> void* { return (char*)p + elems * e; };
  auto cat = [&](const void* p, int64_t elems) -> const void* { return (const char*)p + elems * e; };
  int rc;

  // Batched per-(batch, head) attention products.  Scores are [B,H,S,S].
  const int64_t SS = (int64_t)S * S;
  auto att = [&](Gemm& g) {
    g.nb1 = B; g.nb2 = H; g.in_bf16 = bf;
  };
  auto set_qkv = [&](int64_t& s1, int64_t& s2) { s1 = (int64_t)S * W3; s2 = dh; };
  auto set_sc = [&](int64_t& s1, int64_t& s2) { s1 = (int64_t)H * SS; s2 = SS; };
  auto set_td = [&](int64_t& s1, int64_t& s2) { s1 = (int64_t)S * D; s2 = dh; };

  // Fused attention epilogues (bf16 operands, 16-byte aligned rows).  The fused
  // kernels write only the score tiles on and below the diagonal; tiles above it
  // are read as zeros by products that run with larger tiles, so they are
  // cleared whenever the [B,H,S,S] layout changes.
  const bool fused_att = !flash && bf && D % 8 == 0 && dh % 32 == 0 && S % 8 == 0;
  if (fused_att && (att_zero_B != B || att_zero_S != S)) {
    const int64_t words = (int64_t)B * H * SS / 2;  // bf16 pairs
    for (auto& b : lb) {
      CK(launch_fill_f32((float*)b.P, words, 0.f, st));
      CK(launch_fill_f32((float*)b.P_t, words, 0.f, st));
    }
    if (P_lo) CK(launch_fill_f32((float*)P_lo, words, 0.f, st));
    CK(launch_fill_f32((float*)dS, words, 0.f, st));
    CK(launch_fill_f32((float*)dS_t, words, 0.f, st));
    att_zero_B = B; att_zero_S = S;
  }
  // The unfused path writes whole score matrices in its own [B,H,S,S] layout, so the tiles the
  // fused kernels rely on being zero must be cleared again before their next use.
  if (bf && !fused_att) att_zero_B = att_zero_S = -1;
  AttnP ap;  // streamed attention: what every layer shares
  if (flash) {
    ap.ldq = W3; ap.offK = offK; ap.offV = offV; ap.B = B; ap.H = H; ap.S = S; ap.grp = grp; ap.dh = dh; ap.scale = cs;
    ap.ldo = D; ap.lddo = D; ap.delta = att_rstat;
  }

  // ------------------------------ forward with tangents ----------------------
  CK(launch_embed_fwd(bf, L.Wp(off_wte), llama ? nullptr : L.Wp(off_wpe), v + off_wte, llama ? nullptr : v + off_wpe,
                      tok, T, S, D, V, lb[0].x1, lb[0].x1_t, flags, st));
  for (int l = 0; l < NL; ++l) {
    LayerBuf& b = lb[l];
    const LayerOff& o = loff[l];
    float* xn = (l + 1 < NL) ? lb[l + 1].x1 : xL;
    float* xn_t = (l + 1 < NL) ? lb[l + 1].x1_t : xL_t;
    // *_lo buffers (bf16 mode, shared by all layers) hold the low-order halves
    // of the primal activations of the forward chain.
    CK(launch_norm_fwd(bf, rms, b.x1, b.x1_t, L.Wp(o.n1g), rms ? nullptr : L.Wp(o.n1b), v + o.n1g,
                       rms ? nullptr : v + o.n1b, T, D, eps, b.a, b.a_t, a_lo, b.st1, st));
    // (streamed attention keeps these two per layer: its backward sweep forms the scores again)
    void* const qkv_lo = flash ? b.qkv_lo : this->qkv_lo;
    void* const o_lo = flash ? b.o_lo : this->o_lo;
    if (!llama) {
      if ((rc = L.fwd(b.a, b.a_t, T, D, 3 * D, D, o.wqkv, o.bqkv, b.qkv, b.qkv_t, W3, bf, nullptr, nullptr, 0, -1, a_lo, qkv_lo))) return rc;
    } else {
      // q and k leave their products in fp32 and are rounded once, after the rotation
      if ((rc = L.fwd(b.a, b.a_t, T, D, D, D, o.wq, -1, rq, rq_t, RQ, 0, nullptr, nullptr, 0, -1, a_lo))) return rc;
      if ((rc = L.fwd(b.a, b.a_t, T, D, Dkv, D, o.wk, -1, rq + D, rq_t + D, RQ, 0, nullptr, nullptr, 0, -1, a_lo))) return rc;
      if ((rc = L.fwd(b.a, b.a_t, T, D, Dkv, D, o.wv, -1, at(b.qkv, offV), at(b.qkv_t, offV), W3, bf, nullptr, nullptr, 0, -1, a_lo,
                      qkv_lo ? at(qkv_lo, offV) : nullptr))) return rc;
      CK(launch_rope(bf, rq, rq_t, RQ, b.qkv, b.qkv_t, qkv_lo, W3, T, S, H + Hkv, dh, desc.rope_theta, 0, st));
    }
    if (flash) {
      AttnP a = ap;
      a.qkv = (const bf16*)b.qkv; a.qkv_lo = (const bf16*)qkv_lo; a.qkv_t = (const bf16*)b.qkv_t;
      a.o = (bf16*)b.o; a.o_lo = (bf16*)o_lo; a.o_t = (bf16*)b.o_t; a.stat = b.att_stat;
      CK(launch_attn_fwd(a, st));
    } else {
    if (fused_att) {
      // scores without a trip through memory: the product is formed twice by the
      // dual-output kernel, first to reduce (max, sum, tangent sum) per row over
      // 64-column parts, then to write P, P_lo, P_t with the combined statistics
      Gemm g; att(g);
      g.M = S; g.N = S; g.K = dh; g.lda = W3; g.ldb = W3; g.ldc = S; g.transB = 1; g.alpha = cs; g.skip_upper = 1; g.divB = grp;
      set_qkv(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_sc(g.sC1, g.sC2);
      g.A[0] = b.qkv; g.B[0] = cat(b.qkv, offK);
      if (qkv_lo) {
        g.A[1] = qkv_lo; g.B[1] = cat(b.qkv, offK);
        g.A[2] = b.qkv; g.B[2] = cat(qkv_lo, offK);
      }
      g.At = b.qkv_t; g.Bt = cat(b.qkv_t, offK);
      g.C = b.P; g.Ct = b.P_t; g.out_bf16 = 1;
      g.epi = EPI_FWD_STATS; g.part = att_part;
      CK(launch_gemm(g, st));
      CK(launch_attn_combine(0, att_part, (S + 63) / 64, S, (int64_t)B * H * S, att_rstat, st));
      g.epi = EPI_FWD_SOFTMAX; g.part = nullptr; g.rstat = att_rstat; g.C_lo = P_lo;
      CK(launch_gemm(g, st));
    } else {
    {  // scores S = c Q K^T, S_t = c (Q_t K^T + Q K_t^T); lower-triangular tiles only
      Gemm g; att(g);
      g.M = S; g.N = S; g.K = dh; g.lda = W3; g.ldb = W3; g.ldc = S; g.transB = 1; g.alpha = cs; g.skip_upper = 1; g.divB = grp;
      set_qkv(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_sc(g.sC1, g.sC2);
      g.A[0] = b.qkv; g.B[0] = cat(b.qkv, offK); g.C = sc;
      if (qkv_lo) {  // (q + q_lo)(k + k_lo)^T without the lo*lo term
        g.A[1] = qkv_lo; g.B[1] = cat(b.qkv, offK);
        g.A[2] = b.qkv; g.B[2] = cat(qkv_lo, offK);
      }
      g.At = b.qkv_t; g.Bt = cat(b.qkv_t, offK); g.Ct = sc_t;
      CK(launch_gemm(g, st));
    }
    CK(launch_softmax_fwd(bf, sc, sc_t, b.P, b.P_t, P_lo, B * H, S, st));
    }
    {  // O = P V, O_t = P_t V + P V_t
      Gemm g; att(g);
      g.M = S; g.N = dh; g.K = S; g.lda = S; g.ldb = W3; g.ldc = D; g.klimit = 1; g.out_bf16 = bf; g.divB = grp;
      set_sc(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_td(g.sC1, g.sC2);
      g.A[0] = b.P; g.B[0] = cat(b.qkv, offV); g.C = b.o;
      if (P_lo) {
        g.A[1] = P_lo; g.B[1] = cat(b.qkv, offV);
        g.A[2] = b.P; g.B[2] = cat(qkv_lo, offV);
        g.C_lo = o_lo;
      }
      g.At = b.P_t; g.Bt = cat(b.qkv_t, offV); g.Ct = b.o_t;
      CK(launch_gemm(g, st));
    }
    }
    if ((rc = L.fwd(b.o, b.o_t, T, D, D, D, o.wo, o.bo, b.x2, b.x2_t, D, 0, b.x1, b.x1_t, 0, -1, o_lo))) return rc;
    CK(launch_norm_fwd(bf, rms, b.x2, b.x2_t, L.Wp(o.n2g), rms ? nullptr : L.Wp(o.n2b), v + o.n2g,
                       rms ? nullptr : v + o.n2b, T, D, eps, b.m, b.m_t, a_lo, b.st2, st));
    if (!llama) {
      if ((rc = L.fwd(b.m, b.m_t, T, D, F, D, o.wfc, o.bfc, b.f, b.f_t, F, bf, nullptr, nullptr, 0, -1, a_lo, f_lo))) return rc;
      CK(launch_act_fwd(bf, gelu_kind, b.f, b.f_t, f_lo, b.g, b.g_t, g_lo, (int64_t)T * F, st));
      if ((rc = L.fwd(b.g, b.g_t, T, F, D, F, o.wproj, o.bproj, xn, xn_t, D, 0, b.x2, b.x2_t, 0, -1, g_lo))) return rc;
    } else {
      if ((rc = L.fwd(b.m, b.m_t, T, D, F, D, o.wgate, -1, b.f, b.f_t, F, bf, nullptr, nullptr, 0, -1, a_lo, f_lo))) return rc;
      if ((rc = L.fwd(b.m, b.m_t, T, D, F, D, o.wup, -1, b.up, b.up_t, F, bf, nullptr, nullptr, 0, -1, a_lo, up_lo))) return rc;
      CK(launch_swiglu_fwd(bf, b.f, b.f_t, b.up, b.up_t, f_lo, up_lo, b.g, b.g_t, g_lo, (int64_t)T * F, st));
      if ((rc = L.fwd(b.g, b.g_t, T, F, D, F, o.wdown, -1, xn, xn_t, D, 0, b.x2, b.x2_t, 0, -1, g_lo))) return rc;
    }
  }
  CK(launch_norm_fwd(bf, rms, xL, xL_t, L.Wp(off_nfg), rms ? nullptr : L.Wp(off_nfb), v + off_nfg,
                     rms ? nullptr : v + off_nfb, T, D, eps, xf, xf_t, xf_lo, stf, st));
  const bool tied = off_head < 0;
  // The softmax turns an absolute error of a logit into a relative error of
  // every probability, so the primal logits also take the low-order half.
  if (tied) { if ((rc = L.fwd(xf, xf_t, T, D, V, D, off_wte, -1, z, z_t, ldz, 0, nullptr, nullptr, 1, D, xf_lo))) return rc; }
  else { if ((rc = L.fwd(xf, xf_t, T, D, V, D, off_head, -1, z, z_t, ldz, 0, nullptr, nullptr, 0, -1, xf_lo))) return rc; }

  // ------------------------------ loss and adjoint seeds ----------------------
  CK(launch_count_valid(labels, T, V, flags + 1, flags, st));
  CK(launch_ce(bf, z, z_t, labels, flags + 1, T, V, ldz, dz, dz_t, loss_rows, seed, st));
  CK(launch_sum_rows_f64(loss_rows, T, flags + 1, loss_dev, (double)seed, acc_mode, flags, st));

  // ------------------------------ backward with tangents ----------------------
  if (tied) {
    // z = xf wte^T:  (Hv)_wte = dz_t^T xf + dz^T xf_t  [V, D];  dxf = dz wte
    Gemm g;
    g.M = V; g.N = D; g.K = T; g.lda = ldz; g.ldb = D; g.ldc = D; g.transA = 1; g.in_bf16 = bf;
    g.A[0] = dz_t; g.B[0] = xf; g.A[1] = dz; g.B[1] = xf_t; g.C = out + off_wte;
    if (acc_mode) g.Cadd = out + off_wte;
    CK(launch_gemm(g, st));
    if ((rc = L.bwd_dx(dz, dz_t, T, D, V, ldz, off_wte, tmpd, tmpd_t, D, 0, nullptr, nullptr, 1, D))) return rc;
  } else {
    if ((rc = L.bwd_dw(xf, xf_t, dz, dz_t, T, D, V, D, ldz, off_head, -1, nullptr, 0))) return rc;
    if ((rc = L.bwd_dx(dz, dz_t, T, D, V, ldz, off_head, tmpd, tmpd_t, D, 0))) return rc;
  }
  // each norm adjoint also leaves the bf16 copies (dxb, dxb_t) that the next products read, and adds
  // the column sums of its dx_t to the H v block of the bias that this adjoint belongs to (the output
  // bias of the linear layer applied just before, in forward order)
  CK(launch_norm_bwd(bf, rms, tmpd, tmpd_t, xL, xL_t, stf, L.Wp(off_nfg), v + off_nfg, T, D, 0, dx, dx_t,
                     out + off_nfg, rms ? nullptr : out + off_nfb, norm_part, st, bf ? dxb : nullptr, bf ? dxb_t : nullptr,
                     loff[NL - 1].bproj >= 0 ? out + loff[NL - 1].bproj : nullptr));

  for (int l = NL - 1; l >= 0; --l) {
    LayerBuf& b = lb[l];
    const LayerOff& o = loff[l];
    // ---- MLP branch
    // GPT, small models: the four weight-gradient products of a layer (few output tiles each, a long
    // contraction over the tokens) are only described here and launched together once the last of
    // their operands exists; the two norm adjoints of a layer then write their bf16 copies to
    // different buffers, so that the first is still there when the group runs.
    Gemm dw[4];
    int ndw = 0;
    const bool group_dw = bf && !llama && (dw_prezeroed || acc_mode);
    void* const dxa = dxb;                        // adjoint entering the layer (bf16 copy) and its tangent
    void* const dxa_t = dxb_t;
    void* const dxm = group_dw ? dxb2 : dxb;      // adjoint between the two branches
    void* const dxm_t = group_dw ? dxb2_t : dxb_t;
    if (!llama) {
      if ((rc = L.bwd_dw(b.g, b.g_t, dxa, dxa_t, T, F, D, F, D, o.wproj, -1, nullptr, 0, group_dw ? &dw[ndw++] : nullptr))) return rc;
      if ((rc = L.bwd_dx(dxa, dxa_t, T, F, D, D, o.wproj, dg, dg_t, F, bf))) return rc;
      CK(launch_act_bwd(bf, gelu_kind, b.f, b.f_t, dg, dg_t, dg, dg_t, (int64_t)T * F, st));
      if ((rc = L.bwd_dw(b.m, b.m_t, dg, dg_t, T, D, F, D, F, o.wfc, o.bfc, dg_t, bf, group_dw ? &dw[ndw++] : nullptr))) return rc;
      if ((rc = L.bwd_dx(dg, dg_t, T, D, F, F, o.wfc, tmpd, tmpd_t, D, 0))) return rc;
    } else {
      if ((rc = L.bwd_dw(b.g, b.g_t, dxb, dxb_t, T, F, D, F, D, o.wdown, -1, nullptr, 0))) return rc;
      if ((rc = L.bwd_dx(dxb, dxb_t, T, F, D, D, o.wdown, dy, dy_t, F, bf))) return rc;
      CK(launch_swiglu_bwd(bf, b.f, b.f_t, b.up, b.up_t, dy, dy_t, dg, dg_t, dup, dup_t, (int64_t)T * F, st));
      if ((rc = L.bwd_dw(b.m, b.m_t, dg, dg_t, T, D, F, D, F, o.wgate, -1, nullptr, 0))) return rc;
      if ((rc = L.bwd_dw(b.m, b.m_t, dup, dup_t, T, D, F, D, F, o.wup, -1, nullptr, 0))) return rc;
      if ((rc = L.bwd_dx(dg, dg_t, T, D, F, F, o.wgate, tmpd, tmpd_t, D, 0))) return rc;
      if ((rc = L.bwd_dx(dup, dup_t, T, D, F, F, o.wup, tmpd, tmpd_t, D, 0, tmpd, tmpd_t))) return rc;
    }
    CK(launch_norm_bwd(bf, rms, tmpd, tmpd_t, b.x2, b.x2_t, b.st2, L.Wp(o.n2g), v + o.n2g, T, D, 1, dx, dx_t,
                       out + o.n2g, rms ? nullptr : out + o.n2b, norm_part, st, bf ? dxm : nullptr, bf ? dxm_t : nullptr,
                       o.bo >= 0 ? out + o.bo : nullptr));
    // ---- attention branch
    if ((rc = L.bwd_dw(b.o, b.o_t, dxm, dxm_t, T, D, D, D, D, o.wo, -1, nullptr, 0, group_dw ? &dw[ndw++] : nullptr))) return rc;
    if ((rc = L.bwd_dx(dxm, dxm_t, T, D, D, D, o.wo, dob, dob_t, D, bf))) return rc;
    // Products whose result belongs to a key/value head sum over the grp query heads that share
    // it: one launch per member j of the groups (batch = key/value heads, query head kv * grp + j),
    // the first writing and the others adding to an fp32 result.
    auto grouped = [&](Gemm g, int64_t a_head, int64_t b_head, float* c, float* c_t) -> hipError_t {
      g.nb2 = Hkv; g.out_bf16 = 0; g.sA2 = grp * a_head; g.sB2 = grp * b_head;
      const char *a0 = (const char*)g.A[0], *at0 = (const char*)g.At, *b0 = (const char*)g.B[0], *bt0 = (const char*)g.Bt;
      for (int j = 0; j < grp; ++j) {
        g.A[0] = a0 + j * a_head * e; g.At = at0 + j * a_head * e;
        g.B[0] = b0 + j * b_head * e; g.Bt = bt0 + j * b_head * e;
        g.C = c; g.Ct = c_t;
        g.Cadd = j ? c : nullptr; g.Cadd_t = j ? c_t : nullptr;
        hipError_t er = launch_gemm(g, st);
        if (er != hipSuccess) return er;
      }
      return hipSuccess;
    };
    if (flash) {
      // delta, delta_t from <dO, O>, then dQ, dK, dV and their tangents with the probabilities
      // recomputed tile by tile from the saved row statistics
      CK(launch_attn_delta(dob, dob_t, b.o, b.o_lo, b.o_t, T, S, H, dh, att_rstat, st));
      AttnP a = ap;
      a.qkv = (const bf16*)b.qkv; a.qkv_lo = (const bf16*)b.qkv_lo; a.qkv_t = (const bf16*)b.qkv_t; a.stat = b.att_stat;
      a.dO = (const bf16*)dob; a.dO_t = (const bf16*)dob_t;
      a.dv = at(dqkv, offV); a.dv_t = at(dqkv_t, offV); a.lddv = W3; a.dv_f32 = 0;
      if (llama) {  // fp32 staging [T, D + Dkv]; rounded once after the inverse rotation
        a.dq = rq; a.dq_t = rq_t; a.dk = rq + D; a.dk_t = rq_t + D; a.lddq = a.lddk = RQ; a.dq_f32 = a.dk_f32 = 1;
      } else {
        a.dq = dqkv; a.dq_t = dqkv_t; a.dk = at(dqkv, offK); a.dk_t = at(dqkv_t, offK); a.lddq = a.lddk = W3;
      }
      CK(launch_attn_bwd(a, st));
    } else {
    {  // dV = P^T dO, dV_t = P_t^T dO + P^T dO_t   -> v part of dqkv
      Gemm g; att(g);
      g.M = S; g.N = dh; g.K = S; g.lda = S; g.ldb = D; g.ldc = W3; g.transA = 1; g.klimit = 2; g.out_bf16 = bf;
      set_sc(g.sA1, g.sA2); set_td(g.sB1, g.sB2); set_qkv(g.sC1, g.sC2);
      g.A[0] = b.P; g.B[0] = dob; g.C = at(dqkv, offV);
      g.At = b.P_t; g.Bt = dob_t; g.Ct = at(dqkv_t, offV);
      if (grp == 1) {
        CK(launch_gemm(g, st));
      } else {  // fp32 [T, Dkv], rounded once below
        g.ldc = Dkv; g.sC1 = (int64_t)S * Dkv; g.sC2 = dh;
        CK(grouped(g, SS, dh, rv, rv_t));
        if (bf) CK(launch_cast_pair(1, rv, rv_t, dvb, dvb_t, (int64_t)T * Dkv, st));
      }
    }
    if (fused_att) {
      // dP = dO V^T and its tangent, reduced to (delta, delta_t) per row on the
      // first pass and turned into dS, dS_t on the second; dP never reaches memory
      Gemm g; att(g);
      g.M = S; g.N = S; g.K = dh; g.lda = D; g.ldb = W3; g.ldc = S; g.transB = 1; g.skip_upper = 1; g.divB = grp;
      set_td(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_sc(g.sC1, g.sC2);
      g.A[0] = dob; g.B[0] = cat(b.qkv, offV);
      g.At = dob_t; g.Bt = cat(b.qkv_t, offV);
      g.C = dS; g.Ct = dS_t; g.out_bf16 = 1; g.E0 = b.P; g.E1 = b.P_t;
      // delta, delta_t from <dO, O> where the head width allows, else by a statistics pass
      // (the shared low-order buffer of O still holds this layer's only for the last layer)
      hipError_t ed = launch_attn_delta(dob, dob_t, b.o, l == NL - 1 ? o_lo : nullptr, b.o_t, T, S, H, dh, att_rstat, st);
      if (ed == hipErrorNotSupported) {
        g.epi = EPI_BWD_STATS; g.part = att_part;
        CK(launch_gemm(g, st));
        CK(launch_attn_combine(1, att_part, (S + 63) / 64, S, (int64_t)B * H * S, att_rstat, st));
      } else {
        CK(ed);
      }
      g.epi = EPI_BWD_DS; g.part = nullptr; g.rstat = att_rstat;
      CK(launch_gemm(g, st));
    } else {
    {  // dP = dO V^T, dP_t = dO_t V^T + dO V_t^T
      Gemm g; att(g);
      g.M = S; g.N = S; g.K = dh; g.lda = D; g.ldb = W3; g.ldc = S; g.transB = 1; g.skip_upper = 1; g.divB = grp;
      set_td(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_sc(g.sC1, g.sC2);
      g.A[0] = dob; g.B[0] = cat(b.qkv, offV); g.C = sc;
      g.At = dob_t; g.Bt = cat(b.qkv_t, offV); g.Ct = sc_t;
      CK(launch_gemm(g, st));
    }
    CK(launch_softmax_bwd(bf, b.P, b.P_t, sc, sc_t, dS, dS_t, B * H, S, st));
    }
    {  // dQ = c dS K, dQ_t = c (dS_t K + dS K_t)
      Gemm g; att(g);
      g.M = S; g.N = dh; g.K = S; g.lda = S; g.ldb = W3; g.ldc = W3; g.klimit = 1; g.alpha = cs; g.out_bf16 = bf;
      set_sc(g.sA1, g.sA2); set_qkv(g.sB1, g.sB2); set_qkv(g.sC1, g.sC2);
      void *cq = dqkv, *cq_t = dqkv_t, *ck = at(dqkv, offK), *ck_t = at(dqkv_t, offK);
      if (llama) {  // fp32 staging [T, D + Dkv]; rounded once after the inverse rotation
        g.out_bf16 = 0; g.ldc = RQ; g.sC1 = (int64_t)S * RQ; g.sC2 = dh;
        cq = rq; cq_t = rq_t; ck = rq + D; ck_t = rq_t + D;
      }
      g.A[0] = dS; g.B[0] = cat(b.qkv, offK); g.C = cq;
      g.At = dS_t; g.Bt = cat(b.qkv_t, offK); g.Ct = cq_t;
      g.divB = grp;
      CK(launch_gemm(g, st));
      // dK = c dS^T Q, dK_t = c (dS_t^T Q + dS^T Q_t)
      g.transA = 1; g.klimit = 2; g.divB = 1;
      g.A[0] = dS; g.B[0] = b.qkv; g.C = ck;
      g.At = dS_t; g.Bt = b.qkv_t; g.Ct = ck_t;
      if (grp == 1) CK(launch_gemm(g, st));
      else CK(grouped(g, SS, dh, (float*)ck, (float*)ck_t));  // grp > 1 is LLAMA: ck is the fp32 staging
    }
    }
    if (!llama) {
      if ((rc = L.bwd_dw(b.a, b.a_t, dqkv, dqkv_t, T, D, 3 * D, D, W3, o.wqkv, o.bqkv, dqkv_t, bf, group_dw ? &dw[ndw++] : nullptr))) return rc;
      if (ndw > 0) CK(launch_gemm_group(dw, ndw, st));
      if ((rc = L.bwd_dx(dqkv, dqkv_t, T, D, 3 * D, W3, o.wqkv, tmpd, tmpd_t, D, 0))) return rc;
    } else {
      CK(launch_rope(bf, rq, rq_t, RQ, dqkv, dqkv_t, nullptr, W3, T, S, H + Hkv, dh, desc.rope_theta, 1, st));
      const int64_t w3[3] = {o.wq, o.wk, o.wv};
      const int64_t offs[3] = {0, offK, offV};
      for (int i = 0; i < 3; ++i) {
        const void* dyi = cat(dqkv, offs[i]);
        const void* dyi_t = cat(dqkv_t, offs[i]);
        int64_t ldy = W3;
        const int Ni = i ? Dkv : D;
        if (i == 2 && grp > 1 && !flash) {  // dV of grouped heads lives in its own [T, Dkv] buffer
          dyi = bf ? (const void*)dvb : (const void*)rv;
          dyi_t = bf ? (const void*)dvb_t : (const void*)rv_t;
          ldy = Dkv;
        }
        if ((rc = L.bwd_dw(b.a, b.a_t, dyi, dyi_t, T, D, Ni, D, ldy, w3[i], -1, nullptr, 0))) return rc;
        if ((rc = L.bwd_dx(dyi, dyi_t, T, D, Ni, ldy, w3[i], tmpd, tmpd_t, D, 0, i ? tmpd : nullptr, i ? tmpd_t : nullptr))) return rc;
      }
    }
    CK(launch_norm_bwd(bf, rms, tmpd, tmpd_t, b.x1, b.x1_t, b.st1, L.Wp(o.n1g), v + o.n1g, T, D, 1, dx, dx_t,
                       out + o.n1g, rms ? nullptr : out + o.n1b, norm_part, st, bf ? dxb : nullptr, bf ? dxb_t : nullptr,
                       (l > 0 && loff[l - 1].bproj >= 0) ? out + loff[l - 1].bproj : nullptr));
  }
  CK(launch_embed_bwd(dx_t, tok, T, S, D, V, out + off_wte, llama ? nullptr : out + off_wpe, st));
  return HF_OK;
}

// ------------------------------------------------------------------ Lanczos ----

float* hf_ctx::cur_q() const {
  if (lz_rows_are_vectors() && lz_k < max_m) return (float*)basis + (int64_t)lz_k * ldq;
  return lz_vec[iq];
}

float* hf_ctx::prev_q() const {
  if (lz_rows_are_vectors() && lz_k >= 1) return (float*)basis + (int64_t)(lz_k - 1) * ldq;
  return lz_vec[iqp];
}

int hf_ctx::lanczos_update(float* r, double tol, double* alpha_k, double* beta_k, const int* hvp_flags, hipStream_t st) {
  hf_ctx* c = this;
  const int k = lz_k;
  const int bq = desc.basis_dtype == HF_BF16;
  const bool rows = lz_rows_are_vectors();
  float* q = cur_q();
  float* qp = prev_q();
  float* spill = nullptr;  // fp32 destination of q_{k+1} outside the basis
  if (lz_reorth == HF_REORTH_FULL) {
    // Gram-Schmidt of H q_k against q_0 .. q_k is the three-term subtraction and the
    // orthogonalisation in one.  An fp32 basis holds q_k and q_{k-1} as its rows k and k - 1; a
    // bf16 basis holds rounded copies, so those two come from the working vectors instead.
    if (!bq) CK(lz_gs_first_pass((const float*)basis, basis_bf, ldq, r, n, k + 1, scal, cvec, partials, st));
    else CK(lz_gs_first_pass_bf16((const bf16*)basis, ldq, qp, q, r, n, k, scal, cvec, partials, st));
    CK(lz_reorth_pass(basis, bq, bq ? nullptr : basis_bf, ldq, r, n, k + 1, 1, scal, cvec, partials, st));
    // q_{k+1} = r / beta_k: an fp32 basis takes it as row k + 1 and nowhere else (the rows are the
    // working vectors); a bf16 basis takes the rounded copy, which is also the operand-type copy
    // the next product multiplies with, and the fp32 vector goes over q_{k-1}.
    void* row = k + 1 < max_m ? (char*)basis + (int64_t)(k + 1) * ldq * (bq ? 2 : 4) : nullptr;
    spill = rows ? (row ? nullptr : lz_vec[iq]) : qp;
    bf16* vdst = nullptr;
    if (bf) vdst = (bq && row) ? nullptr : ((basis_bf && row) ? basis_bf + (int64_t)(k + 1) * ldq : vb);
    CK(lz_scale(r, spill, row, bq, vdst, n, scal, S_BETA, tol, hvp_flags, st));
    next_vb = bf ? ((bq && row) ? (const bf16*)row : vdst) : nullptr;
  } else {
    CK(lz3_update(r, q, qp, bf ? vb : nullptr, n, k > 0, lz_beta_prev, tol, hvp_flags, scal, partials, st));
    next_vb = bf ? vb : nullptr;
  }
  CK(hipMemcpyAsync(host_scal, scal, S_COUNT * sizeof(double), hipMemcpyDeviceToHost, st));
  CK(hipStreamSynchronize(st));
  if (hvp_flags) {  // the product's input checks; q_{k+1} was not written if any failed
    const int f0 = (int)host_scal[S_FLAG0], f1 = (int)host_scal[S_FLAG1];
    if (f0 & 1) return fail(HF_EINVAL, "token id outside [0, vocab)");
    if (f0 & 2) return fail(HF_EINVAL, "label >= number of classes");
    if (f1 == 0) return fail(HF_EINVAL, "no valid label in the batch");
  }
  const double a = host_scal[S_ALPHA], bt = host_scal[S_BETA];
  if (alpha_k) *alpha_k = a;
  if (beta_k) *beta_k = bt;
  lz_k = k + 1;
  if (!(bt >= tol) || !(bt > 0.0)) {  // also catches NaN; the kernels made the same test
    lz_done = 1;
    return HF_EBREAKDOWN;
  }
  lz_beta_prev = bt;
  if (!rows) std::swap(iq, iqp);  // q_{k+1} went over q_{k-1}
  vb_of = next_vb ? cur_q() : nullptr;
  vb_cur = next_vb;
  return HF_OK;
}
