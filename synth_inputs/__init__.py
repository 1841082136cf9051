"""Seeded synthetic inputs shared by the float64 oracle tests and the HIP path.

This module holds no arithmetic of the method (no forward pass, no Hessian, no
Lanczos).  It only produces data: the five workload descriptions, the flat
parameter vector in the canonical order, token batches, labels and Rademacher
probes.  Both the CPU oracle's tests and the GPU binding's tests draw the same
arrays from here so that they can be compared element by element.

The workloads stand in for the pretrained language models and text corpora the
paper measures on (Section "Frontier Spectra" and the random-token experiments
of Section "Understanding the Dataset Impact"), none of which are available:
random-initialised weights and uniform / Zipf token ids of the same shapes.
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------
# Workload descriptions.  Keys follow the C model descriptor field names.
# ----------------------------------------------------------------------------

def _mlp(mlp_in, hidden, out):
    return dict(arch="mlp", mlp_in=mlp_in, mlp_hidden=hidden, mlp_out=out,
                n_layer=0, d_model=0, n_head=0, d_ff=0, vocab=0, max_seq=0,
                tie_embeddings=0, norm_eps=1e-5, rope_theta=10000.0)


def _gpt(n_layer, d, h, ff, vocab, max_seq, tie=1, act="gelu_erf"):
    return dict(arch="gpt", n_layer=n_layer, d_model=d, n_head=h, d_ff=ff,
                vocab=vocab, max_seq=max_seq, tie_embeddings=tie, act=act,
                mlp_in=0, mlp_hidden=0, mlp_out=0, norm_eps=1e-5,
                rope_theta=10000.0)


def _llama(n_layer, d, h, ff, vocab, max_seq, n_kv=None):
    """n_kv: key/value heads (grouped-query attention); None = one per query head."""
    return dict(arch="llama", n_layer=n_layer, d_model=d, n_head=h, d_ff=ff,
                vocab=vocab, max_seq=max_seq, tie_embeddings=0, n_kv_head=(n_kv or h),
                mlp_in=0, mlp_hidden=0, mlp_out=0, norm_eps=1e-5,
                rope_theta=10000.0)


CONFIGS = {
    # name: (model, batch, seq, token distribution, param dtype, lanczos m,
    #        reorth, basis dtype, probes)
    "mlp_tiny": dict(model=_mlp(32, 32, 10), batch=256, seq=1, tokens=None,
                     param_dtype="f32", m=80, reorth="full", basis_dtype="f32",
                     n_probes=4),
    "gpt_2l_d128": dict(model=_gpt(2, 128, 4, 512, 512, 64), batch=8, seq=64,
                        tokens="uniform", param_dtype="f32", m=100,
                        reorth="full", basis_dtype="f32", n_probes=2),
    "gpt2_small": dict(model=_gpt(12, 768, 12, 3072, 50257, 512), batch=8,
                       seq=512, tokens="zipf", param_dtype="bf16", m=100,
                       reorth="full", basis_dtype="f32", n_probes=1),
    "gpt_1p3b": dict(model=_gpt(24, 2048, 16, 8192, 32000, 1024), batch=4,
                     seq=1024, tokens="zipf", param_dtype="bf16", m=30,
                     reorth="full", basis_dtype="bf16", n_probes=1),
    "llama_7b": dict(model=_llama(32, 4096, 32, 11008, 32000, 512), batch=1,
                     seq=512, tokens="zipf", param_dtype="bf16", m=20,
                     reorth="none", basis_dtype="none", n_probes=1),
}

SEED_PARAMS = 42
SEED_DATA = 43
SEED_PROBE0 = 44


def scaled(model, **overrides):
    """Copy of a model description with some fields replaced (reduced depth or
    width variants of a workload for tests the oracle finishes in seconds)."""
    m = dict(model)
    m.update(overrides)
    return m


# ----------------------------------------------------------------------------
# Canonical flat parameter order.  Matrices are row-major [in, out].
# init kinds: ("normal", std) | ("zeros",) | ("ones",)
# ----------------------------------------------------------------------------

def param_spec(model):
    """List of (name, shape, init) in the canonical flat order."""
    a = model["arch"]
    out = []
    if a == "mlp":
        i, h, o = model["mlp_in"], model["mlp_hidden"], model["mlp_out"]
        s1, s2 = (1.0 / i) ** 0.5, (1.0 / h) ** 0.5
        out += [("W1", (i, h), ("normal", s1)), ("b1", (h,), ("normal", s1)),
                ("W2", (h, o), ("normal", s2)), ("b2", (o,), ("normal", s2))]
        return out
    L, d, ff, V = model["n_layer"], model["d_model"], model["d_ff"], model["vocab"]
    N = ("normal", 0.02)
    Z, O = ("zeros",), ("ones",)
    if a == "gpt":
        out += [("wte", (V, d), N), ("wpe", (model["max_seq"], d), N)]
        for l in range(L):
            p = f"h{l}."
            out += [(p + "ln1.g", (d,), O), (p + "ln1.b", (d,), Z),
                    (p + "Wqkv", (d, 3 * d), N), (p + "bqkv", (3 * d,), Z),
                    (p + "Wo", (d, d), N), (p + "bo", (d,), Z),
                    (p + "ln2.g", (d,), O), (p + "ln2.b", (d,), Z),
                    (p + "Wfc", (d, ff), N), (p + "bfc", (ff,), Z),
                    (p + "Wproj", (ff, d), N), (p + "bproj", (d,), Z)]
        out += [("lnf.g", (d,), O), ("lnf.b", (d,), Z)]
        if not model["tie_embeddings"]:
            out += [("lm_head", (d, V), N)]
        return out
    if a == "llama":
        dkv = d // model["n_head"] * model.get("n_kv_head", model["n_head"])
        out += [("wte", (V, d), N)]
        for l in range(L):
            p = f"h{l}."
            out += [(p + "rms1.g", (d,), O),
                    (p + "Wq", (d, d), N), (p + "Wk", (d, dkv), N),
                    (p + "Wv", (d, dkv), N), (p + "Wo", (d, d), N),
                    (p + "rms2.g", (d,), O),
                    (p + "Wgate", (d, ff), N), (p + "Wup", (d, ff), N),
                    (p + "Wdown", (ff, d), N)]
        out += [("rmsf.g", (d,), O), ("lm_head", (d, V), N)]
        return out
    raise ValueError(a)


def num_params(model):
    return int(sum(int(np.prod(s)) for _, s, _ in param_spec(model)))


# ----------------------------------------------------------------------------
# bf16 storage helpers (data format only: round-to-nearest-even truncation of
# the fp32 bit pattern, and the exact widening back).
# ----------------------------------------------------------------------------

def f32_to_bf16_bits(x):
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (b.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# Generators
# ----------------------------------------------------------------------------

def make_params(model, seed=SEED_PARAMS, param_dtype="f32", perturb=0.0):
    """Flat fp32 parameter vector in canonical order.

    param_dtype "bf16": every value is rounded to bf16 and widened back, so the
    returned fp32 array holds exactly the values a bf16 buffer stores.
    perturb > 0 adds N(0, perturb) noise to the norm gains / biases (which are
    otherwise exactly 1 / 0) so that tests exercise generic values there.
    """
    rng = np.random.default_rng(seed)
    n = num_params(model)
    flat = np.empty(n, dtype=np.float32)
    off = 0
    for _, shape, init in param_spec(model):
        cnt = int(np.prod(shape))
        if init[0] == "normal":
            flat[off:off + cnt] = rng.standard_normal(cnt, dtype=np.float32) * np.float32(init[1])
        else:
            base = 1.0 if init[0] == "ones" else 0.0
            if perturb > 0.0:
                flat[off:off + cnt] = base + rng.standard_normal(cnt, dtype=np.float32) * np.float32(perturb)
            else:
                flat[off:off + cnt] = base
        off += cnt
    if param_dtype == "bf16":
        flat = bf16_bits_to_f32(f32_to_bf16_bits(flat))
    return flat


def make_tokens(vocab, batch, seq, dist, seed=SEED_DATA):
    """int32 [batch, seq] token ids: 'uniform', or 'zipf' = truncated Zipf with
    exponent 1.1 over ranks 1..vocab (id = rank-1), i.i.d. by inverse CDF."""
    rng = np.random.default_rng(seed)
    if dist == "uniform":
        return rng.integers(0, vocab, size=(batch, seq), dtype=np.int64).astype(np.int32)
    if dist == "zipf":
        w = np.arange(1, vocab + 1, dtype=np.float64) ** -1.1
        cdf = np.cumsum(w)
        cdf /= cdf[-1]
        u = rng.random(size=(batch, seq))
        ids = np.searchsorted(cdf, u, side="left")
        return np.minimum(ids, vocab - 1).astype(np.int32)
    raise ValueError(dist)


def next_token_labels(tokens):
    """labels[b, s] = tokens[b, s+1]; the last position is ignored (-1)."""
    lab = np.full_like(tokens, -1)
    lab[:, :-1] = tokens[:, 1:]
    return lab


def make_batch(cfg, seed=SEED_DATA, batch=None, seq=None):
    """(inputs, labels) for a workload: MLP -> fp32 x[B, in] ~ N(0,1) and
    uniform class labels; LMs -> int32 tokens[B,S] and next-token labels."""
    model = cfg["model"]
    B = batch or cfg["batch"]
    if model["arch"] == "mlp":
        rng = np.random.default_rng(seed)
        x = rng.standard_normal((B, model["mlp_in"]), dtype=np.float32)
        y = rng.integers(0, model["mlp_out"], size=B, dtype=np.int64).astype(np.int32)
        return x, y
    S = seq or cfg["seq"]
    tok = make_tokens(model["vocab"], B, S, cfg["tokens"], seed)
    return tok, next_token_labels(tok)


def make_probe(n, index=0, seed0=SEED_PROBE0):
    """Rademacher +-1 probe of length n as fp32 (unnormalised)."""
    rng = np.random.default_rng(seed0 + index)
    return (rng.integers(0, 2, size=n, dtype=np.int8).astype(np.float32) * 2.0 - 1.0)


def make_direction(n, seed):
    """Dense Gaussian direction (fp32) for HVP parity tests."""
    rng = np.random.default_rng(seed)
    return rng.standard_normal(n, dtype=np.float32)
