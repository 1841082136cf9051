"""Float64 loss, gradient and Hessian-vector product of the three model families.

TEST INFRASTRUCTURE ONLY (see oracle/ops.py).  `loss_grad_hvp` returns what one
batch iteration of the paper's Algorithm 1 produces: the mean cross-entropy
loss L, g = dL/dp and u = d<g, v>/dp = H v, for the flat parameter vector p in
the canonical order.  It is computed forward-over-reverse from the operator
definitions in oracle/ops.py; the result is the same vector Algorithm 1's
double backward yields (v is constant), which tests/test_oracle_pins.py
verifies against PyTorch's autograd run exactly as Algorithm 1 is written.

Architectures (the paper only says "HuggingFace causal LM .loss"; these are the
standard definitions of the shapes the workloads name):
  mlp   : h = tanh(x W1 + b1); z = h W2 + b2
  gpt   : pre-LayerNorm decoder, learned positions, erf-GELU (model["act"] ==
          "gelu_tanh": the tanh form), optional tied head
  llama : RMSNorm, rotary positions (half-split pairs), SwiGLU, no biases;
          model["n_kv_head"] < n_head: grouped-query attention
Loss: mean softmax cross-entropy over positions with label >= 0 (next-token
prediction); MLP: mean over the samples.
"""
from __future__ import annotations

import numpy as np

from . import ops

# ---------------------------------------------------------------- layout ----


def layout(model):
    """Canonical flat order: list of (name, offset, shape).  Row-major, matrices
    stored [in, out]."""
    names = []
    a = model["arch"]
    if a == "mlp":
        i, h, o = model["mlp_in"], model["mlp_hidden"], model["mlp_out"]
        names = [("W1", (i, h)), ("b1", (h,)), ("W2", (h, o)), ("b2", (o,))]
    else:
        L, d, ff, V = model["n_layer"], model["d_model"], model["d_ff"], model["vocab"]
        if a == "gpt":
            names = [("wte", (V, d)), ("wpe", (model["max_seq"], d))]
            for l in range(L):
                names += [(f"h{l}.ln1.g", (d,)), (f"h{l}.ln1.b", (d,)),
                          (f"h{l}.Wqkv", (d, 3 * d)), (f"h{l}.bqkv", (3 * d,)),
                          (f"h{l}.Wo", (d, d)), (f"h{l}.bo", (d,)),
                          (f"h{l}.ln2.g", (d,)), (f"h{l}.ln2.b", (d,)),
                          (f"h{l}.Wfc", (d, ff)), (f"h{l}.bfc", (ff,)),
                          (f"h{l}.Wproj", (ff, d)), (f"h{l}.bproj", (d,))]
            names += [("lnf.g", (d,)), ("lnf.b", (d,))]
            if not model["tie_embeddings"]:
                names += [("lm_head", (d, V))]
        elif a == "llama":
            dkv = d // model["n_head"] * model.get("n_kv_head", model["n_head"])
            names = [("wte", (V, d))]
            for l in range(L):
                names += [(f"h{l}.rms1.g", (d,)), (f"h{l}.Wq", (d, d)),
                          (f"h{l}.Wk", (d, dkv)), (f"h{l}.Wv", (d, dkv)),
                          (f"h{l}.Wo", (d, d)), (f"h{l}.rms2.g", (d,)),
                          (f"h{l}.Wgate", (d, ff)), (f"h{l}.Wup", (d, ff)),
                          (f"h{l}.Wdown", (ff, d))]
            names += [("rmsf.g", (d,)), ("lm_head", (d, V))]
        else:
            raise ValueError(a)
    out, off = [], 0
    for nm, sh in names:
        out.append((nm, off, sh))
        off += int(np.prod(sh))
    return out


def num_params(model):
    nm, off, sh = layout(model)[-1]
    return off + int(np.prod(sh))


def unflatten(model, flat):
    flat = np.asarray(flat, dtype=np.float64)
    return {nm: flat[off:off + int(np.prod(sh))].reshape(sh) for nm, off, sh in layout(model)}


def flatten(model, d):
    out = np.empty(num_params(model), dtype=np.float64)
    for nm, off, sh in layout(model):
        out[off:off + int(np.prod(sh))] = np.asarray(d[nm], dtype=np.float64).reshape(-1)
    return out


# ---------------------------------------------------------------- helpers ----


def _heads(x, B, S, H):
    """[T, d] -> [B, H, S, dh]"""
    return x.reshape(B, S, H, -1).transpose(0, 2, 1, 3)


def _unheads(x):
    """[B, H, S, dh] -> [T, d]"""
    B, H, S, dh = x.shape
    return x.transpose(0, 2, 1, 3).reshape(B * S, H * dh)


# -------------------------------------------------------------------- MLP ----


def _mlp(model, P, V, x, labels):
    x = np.asarray(x, dtype=np.float64)
    G, U = {}, {}
    a, a_t, c1 = ops.linear_fwd(x, np.zeros_like(x), P["W1"], V["W1"], P["b1"], V["b1"])
    h, h_t, c2 = ops.tanh_fwd(a, a_t)
    z, z_t, c3 = ops.linear_fwd(h, h_t, P["W2"], V["W2"], P["b2"], V["b2"])
    loss, loss_t, dz, dz_t = ops.cross_entropy_fwd(z, z_t, np.asarray(labels).reshape(-1))
    dh, dh_t, G["W2"], U["W2"], G["b2"], U["b2"] = ops.linear_bwd(dz, dz_t, c3)
    da, da_t = ops.tanh_bwd(dh, dh_t, c2)
    _, _, G["W1"], U["W1"], G["b1"], U["b1"] = ops.linear_bwd(da, da_t, c1)
    return loss, loss_t, G, U


# -------------------------------------------------------------------- GPT ----


def _gpt(model, P, V, tokens, labels):
    B, S = tokens.shape
    H, d, L = model["n_head"], model["d_model"], model["n_layer"]
    eps = model["norm_eps"]
    tok = tokens.reshape(-1)
    pos = np.tile(np.arange(S), B)
    x = P["wte"][tok] + P["wpe"][pos]
    x_t = V["wte"][tok] + V["wpe"][pos]
    caches = []
    for l in range(L):
        p = f"h{l}."
        a, a_t, c_ln1 = ops.layernorm_fwd(x, x_t, P[p + "ln1.g"], V[p + "ln1.g"], P[p + "ln1.b"], V[p + "ln1.b"], eps)
        qkv, qkv_t, c_qkv = ops.linear_fwd(a, a_t, P[p + "Wqkv"], V[p + "Wqkv"], P[p + "bqkv"], V[p + "bqkv"])
        q, k, v = (_heads(qkv[:, i * d:(i + 1) * d], B, S, H) for i in range(3))
        q_t, k_t, v_t = (_heads(qkv_t[:, i * d:(i + 1) * d], B, S, H) for i in range(3))
        o, o_t, c_att = ops.attention_fwd(q, q_t, k, k_t, v, v_t)
        y, y_t, c_o = ops.linear_fwd(_unheads(o), _unheads(o_t), P[p + "Wo"], V[p + "Wo"], P[p + "bo"], V[p + "bo"])
        x, x_t = x + y, x_t + y_t
        m, m_t, c_ln2 = ops.layernorm_fwd(x, x_t, P[p + "ln2.g"], V[p + "ln2.g"], P[p + "ln2.b"], V[p + "ln2.b"], eps)
        f, f_t, c_fc = ops.linear_fwd(m, m_t, P[p + "Wfc"], V[p + "Wfc"], P[p + "bfc"], V[p + "bfc"])
        tanh_form = model.get("act", "gelu_erf") == "gelu_tanh"
        g, g_t, c_act = (ops.gelu_tanh_fwd if tanh_form else ops.gelu_fwd)(f, f_t)
        y, y_t, c_pr = ops.linear_fwd(g, g_t, P[p + "Wproj"], V[p + "Wproj"], P[p + "bproj"], V[p + "bproj"])
        x, x_t = x + y, x_t + y_t
        caches.append((c_ln1, c_qkv, c_att, c_o, c_ln2, c_fc, c_act, c_pr))
    xf, xf_t, c_lnf = ops.layernorm_fwd(x, x_t, P["lnf.g"], V["lnf.g"], P["lnf.b"], V["lnf.b"], eps)
    tied = bool(model["tie_embeddings"])
    Wh, Wh_t = (P["wte"].T, V["wte"].T) if tied else (P["lm_head"], V["lm_head"])
    z, z_t, c_head = ops.linear_fwd(xf, xf_t, Wh, Wh_t)
    loss, loss_t, dz, dz_t = ops.cross_entropy_fwd(z, z_t, labels.reshape(-1))

    G = {nm: None for nm in P}
    U = {nm: None for nm in P}
    dxf, dxf_t, dWh, dWh_t = ops.linear_bwd(dz, dz_t, c_head)
    dx, dx_t, G["lnf.g"], U["lnf.g"], G["lnf.b"], U["lnf.b"] = ops.layernorm_bwd(dxf, dxf_t, c_lnf)
    for l in reversed(range(L)):
        p = f"h{l}."
        c_ln1, c_qkv, c_att, c_o, c_ln2, c_fc, c_act, c_pr = caches[l]
        dg, dg_t, G[p + "Wproj"], U[p + "Wproj"], G[p + "bproj"], U[p + "bproj"] = ops.linear_bwd(dx, dx_t, c_pr)
        df, df_t = (ops.gelu_tanh_bwd if model.get("act", "gelu_erf") == "gelu_tanh" else ops.gelu_bwd)(dg, dg_t, c_act)
        dm, dm_t, G[p + "Wfc"], U[p + "Wfc"], G[p + "bfc"], U[p + "bfc"] = ops.linear_bwd(df, df_t, c_fc)
        r, r_t, G[p + "ln2.g"], U[p + "ln2.g"], G[p + "ln2.b"], U[p + "ln2.b"] = ops.layernorm_bwd(dm, dm_t, c_ln2)
        dx, dx_t = dx + r, dx_t + r_t
        do, do_t, G[p + "Wo"], U[p + "Wo"], G[p + "bo"], U[p + "bo"] = ops.linear_bwd(dx, dx_t, c_o)
        dq, dq_t, dk, dk_t, dv, dv_t = ops.attention_bwd(_heads(do, B, S, H), _heads(do_t, B, S, H), c_att)
        dqkv = np.concatenate([_unheads(dq), _unheads(dk), _unheads(dv)], axis=1)
        dqkv_t = np.concatenate([_unheads(dq_t), _unheads(dk_t), _unheads(dv_t)], axis=1)
        da, da_t, G[p + "Wqkv"], U[p + "Wqkv"], G[p + "bqkv"], U[p + "bqkv"] = ops.linear_bwd(dqkv, dqkv_t, c_qkv)
        r, r_t, G[p + "ln1.g"], U[p + "ln1.g"], G[p + "ln1.b"], U[p + "ln1.b"] = ops.layernorm_bwd(da, da_t, c_ln1)
        dx, dx_t = dx + r, dx_t + r_t
    # embeddings: scatter-add of the residual-stream adjoint
    Vv, ms = model["vocab"], model["max_seq"]
    G["wte"], U["wte"] = np.zeros((Vv, d)), np.zeros((Vv, d))
    np.add.at(G["wte"], tok, dx)
    np.add.at(U["wte"], tok, dx_t)
    G["wpe"], U["wpe"] = np.zeros((ms, d)), np.zeros((ms, d))
    np.add.at(G["wpe"], pos, dx)
    np.add.at(U["wpe"], pos, dx_t)
    if tied:
        G["wte"] += dWh.T
        U["wte"] += dWh_t.T
    else:
        G["lm_head"], U["lm_head"] = dWh, dWh_t
    return loss, loss_t, G, U


# ------------------------------------------------------------------ Llama ----


def _llama(model, P, V, tokens, labels):
    B, S = tokens.shape
    H, d, L = model["n_head"], model["d_model"], model["n_layer"]
    Hkv = model.get("n_kv_head", H)   # grouped-query attention: query head h reads key/value head h // grp
    grp = H // Hkv
    eps = model["norm_eps"]
    cos, sin = ops.rope_tables(S, d // H, model["rope_theta"])

    def spread(t):   # [B, Hkv, S, dh] -> [B, H, S, dh], each key/value head repeated for its group
        return np.repeat(t, grp, axis=1)

    def gather(t):   # adjoint of spread: sum over the query heads of each group
        return t.reshape(B, Hkv, grp, S, -1).sum(axis=2)
    tok = tokens.reshape(-1)
    x, x_t = P["wte"][tok], V["wte"][tok]
    caches = []
    for l in range(L):
        p = f"h{l}."
        a, a_t, c_n1 = ops.rmsnorm_fwd(x, x_t, P[p + "rms1.g"], V[p + "rms1.g"], eps)
        q, q_t, c_q = ops.linear_fwd(a, a_t, P[p + "Wq"], V[p + "Wq"])
        k, k_t, c_k = ops.linear_fwd(a, a_t, P[p + "Wk"], V[p + "Wk"])
        v, v_t, c_v = ops.linear_fwd(a, a_t, P[p + "Wv"], V[p + "Wv"])
        qr, qr_t = ops.rope_apply(_heads(q, B, S, H), cos, sin), ops.rope_apply(_heads(q_t, B, S, H), cos, sin)
        kr, kr_t = ops.rope_apply(_heads(k, B, S, Hkv), cos, sin), ops.rope_apply(_heads(k_t, B, S, Hkv), cos, sin)
        o, o_t, c_att = ops.attention_fwd(qr, qr_t, spread(kr), spread(kr_t), spread(_heads(v, B, S, Hkv)),
                                          spread(_heads(v_t, B, S, Hkv)))
        y, y_t, c_o = ops.linear_fwd(_unheads(o), _unheads(o_t), P[p + "Wo"], V[p + "Wo"])
        x, x_t = x + y, x_t + y_t
        u, u_t, c_n2 = ops.rmsnorm_fwd(x, x_t, P[p + "rms2.g"], V[p + "rms2.g"], eps)
        g, g_t, c_g = ops.linear_fwd(u, u_t, P[p + "Wgate"], V[p + "Wgate"])
        w, w_t, c_u = ops.linear_fwd(u, u_t, P[p + "Wup"], V[p + "Wup"])
        s, s_t, c_act = ops.swiglu_fwd(g, g_t, w, w_t)
        y, y_t, c_d = ops.linear_fwd(s, s_t, P[p + "Wdown"], V[p + "Wdown"])
        x, x_t = x + y, x_t + y_t
        caches.append((c_n1, c_q, c_k, c_v, c_att, c_o, c_n2, c_g, c_u, c_act, c_d))
    xf, xf_t, c_nf = ops.rmsnorm_fwd(x, x_t, P["rmsf.g"], V["rmsf.g"], eps)
    z, z_t, c_head = ops.linear_fwd(xf, xf_t, P["lm_head"], V["lm_head"])
    loss, loss_t, dz, dz_t = ops.cross_entropy_fwd(z, z_t, labels.reshape(-1))

    G, U = {}, {}
    dxf, dxf_t, G["lm_head"], U["lm_head"] = ops.linear_bwd(dz, dz_t, c_head)
    dx, dx_t, G["rmsf.g"], U["rmsf.g"] = ops.rmsnorm_bwd(dxf, dxf_t, c_nf)
    for l in reversed(range(L)):
        p = f"h{l}."
        c_n1, c_q, c_k, c_v, c_att, c_o, c_n2, c_g, c_u, c_act, c_d = caches[l]
        ds, ds_t, G[p + "Wdown"], U[p + "Wdown"] = ops.linear_bwd(dx, dx_t, c_d)
        dg, dg_t, dw, dw_t = ops.swiglu_bwd(ds, ds_t, c_act)
        du1, du1_t, G[p + "Wgate"], U[p + "Wgate"] = ops.linear_bwd(dg, dg_t, c_g)
        du2, du2_t, G[p + "Wup"], U[p + "Wup"] = ops.linear_bwd(dw, dw_t, c_u)
        r, r_t, G[p + "rms2.g"], U[p + "rms2.g"] = ops.rmsnorm_bwd(du1 + du2, du1_t + du2_t, c_n2)
        dx, dx_t = dx + r, dx_t + r_t
        do, do_t, G[p + "Wo"], U[p + "Wo"] = ops.linear_bwd(dx, dx_t, c_o)
        dq, dq_t, dk, dk_t, dv, dv_t = ops.attention_bwd(_heads(do, B, S, H), _heads(do_t, B, S, H), c_att)
        dk, dk_t, dv, dv_t = gather(dk), gather(dk_t), gather(dv), gather(dv_t)
        dq, dq_t = ops.rope_apply(dq, cos, sin, True), ops.rope_apply(dq_t, cos, sin, True)
        dk, dk_t = ops.rope_apply(dk, cos, sin, True), ops.rope_apply(dk_t, cos, sin, True)
        da1, da1_t, G[p + "Wq"], U[p + "Wq"] = ops.linear_bwd(_unheads(dq), _unheads(dq_t), c_q)
        da2, da2_t, G[p + "Wk"], U[p + "Wk"] = ops.linear_bwd(_unheads(dk), _unheads(dk_t), c_k)
        da3, da3_t, G[p + "Wv"], U[p + "Wv"] = ops.linear_bwd(_unheads(dv), _unheads(dv_t), c_v)
        r, r_t, G[p + "rms1.g"], U[p + "rms1.g"] = ops.rmsnorm_bwd(da1 + da2 + da3, da1_t + da2_t + da3_t, c_n1)
        dx, dx_t = dx + r, dx_t + r_t
    G["wte"], U["wte"] = np.zeros_like(P["wte"]), np.zeros_like(P["wte"])
    np.add.at(G["wte"], tok, dx)
    np.add.at(U["wte"], tok, dx_t)
    return loss, loss_t, G, U


# ------------------------------------------------------------------- API ----

_ARCH = {"mlp": _mlp, "gpt": _gpt, "llama": _llama}


def loss_grad_hvp(model, params, inputs, labels, v=None):
    """Returns (loss, grad[n], Hv[n], dloss_along_v) in float64.

    params, v: flat arrays in canonical order (v None -> zeros, Hv = 0)."""
    P = unflatten(model, params)
    V = unflatten(model, np.zeros(num_params(model)) if v is None else v)
    loss, loss_t, G, U = _ARCH[model["arch"]](model, P, V, np.asarray(inputs), np.asarray(labels))
    return float(loss), flatten(model, G), flatten(model, U), float(loss_t)


def loss_only(model, params, inputs, labels):
    return loss_grad_hvp(model, params, inputs, labels)[0]


def hvp(model, params, inputs, labels, v):
    return loss_grad_hvp(model, params, inputs, labels, v)[2]


def dense_hessian(model, params, inputs, labels):
    """Column j = hvp(e_j).  Only for tiny models."""
    n = num_params(model)
    Hm = np.empty((n, n))
    e = np.zeros(n)
    for j in range(n):
        e[j] = 1.0
        Hm[:, j] = hvp(model, params, inputs, labels, e)
        e[j] = 0.0
    return Hm
