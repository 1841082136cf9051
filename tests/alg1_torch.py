"""Algorithm 1 of the paper run literally with PyTorch CPU autograd in float64:
L = model(batch).loss; g = dL/dp with create_graph; d = sum(g * v); u = dd/dp.

The model forward here is written with PyTorch's own library operators
(layer_norm, scaled_dot_product_attention, gelu, cross_entropy) and is an
independent derivation used to pin the hand-written numpy oracle; it shares no
code with it.  Parameters come in as a dict name -> array in the canonical
shapes (matrices [in, out]).
"""
import math

import numpy as np
import torch
import torch.nn.functional as F


def _rope(x, theta):
    # x: [B, H, S, dh]; rotate pairs (i, i+dh/2) by pos * theta^(-2i/dh),
    # written with complex multiplication.
    B, H, S, dh = x.shape
    half = dh // 2
    inv = theta ** (-2.0 * torch.arange(half, dtype=torch.float64) / dh)
    ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)
    xc = torch.complex(x[..., :half], x[..., half:]) * rot
    return torch.cat([xc.real, xc.imag], dim=-1)


def _attn(q, k, v, B, S, H):
    def heads(t):
        return t.reshape(B, S, H, -1).transpose(1, 2)
    return heads(q), heads(k), heads(v)


def forward_loss(model, P, inputs, labels):
    a = model["arch"]
    if a == "mlp":
        x = torch.as_tensor(np.asarray(inputs), dtype=torch.float64)
        h = torch.tanh(x @ P["W1"] + P["b1"])
        z = h @ P["W2"] + P["b2"]
        return F.cross_entropy(z, torch.as_tensor(np.asarray(labels), dtype=torch.long))
    tok = torch.as_tensor(np.asarray(inputs), dtype=torch.long)
    lab = torch.as_tensor(np.asarray(labels), dtype=torch.long)
    B, S = tok.shape
    H, d, L, eps = model["n_head"], model["d_model"], model["n_layer"], model["norm_eps"]
    if a == "gpt":
        x = P["wte"][tok] + P["wpe"][torch.arange(S)][None]
        for l in range(L):
            p = f"h{l}."
            y = F.layer_norm(x, (d,), P[p + "ln1.g"], P[p + "ln1.b"], eps)
            qkv = y @ P[p + "Wqkv"] + P[p + "bqkv"]
            q, k, v = _attn(*qkv.split(d, dim=-1), B, S, H)
            o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
            x = x + o.transpose(1, 2).reshape(B, S, d) @ P[p + "Wo"] + P[p + "bo"]
            y = F.layer_norm(x, (d,), P[p + "ln2.g"], P[p + "ln2.b"], eps)
            approx = "tanh" if model.get("act", "gelu_erf") == "gelu_tanh" else "none"
            x = x + F.gelu(y @ P[p + "Wfc"] + P[p + "bfc"], approximate=approx) @ P[p + "Wproj"] + P[p + "bproj"]
        x = F.layer_norm(x, (d,), P["lnf.g"], P["lnf.b"], eps)
        z = x @ (P["wte"].T if model["tie_embeddings"] else P["lm_head"])
    else:
        def rms(t, g):
            return t * torch.rsqrt(t.pow(2).mean(-1, keepdim=True) + eps) * g
        x = P["wte"][tok]
        for l in range(L):
            p = f"h{l}."
            y = rms(x, P[p + "rms1.g"])
            Hkv = model.get("n_kv_head", H)
            q = _attn(y @ P[p + "Wq"], y @ P[p + "Wq"], y @ P[p + "Wq"], B, S, H)[0]
            k, v = _attn(y @ P[p + "Wk"], y @ P[p + "Wk"], y @ P[p + "Wv"], B, S, Hkv)[1:]
            q, k = _rope(q, model["rope_theta"]), _rope(k, model["rope_theta"])
            k, v = k.repeat_interleave(H // Hkv, dim=1), v.repeat_interleave(H // Hkv, dim=1)
            o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
            x = x + o.transpose(1, 2).reshape(B, S, d) @ P[p + "Wo"]
            y = rms(x, P[p + "rms2.g"])
            x = x + (F.silu(y @ P[p + "Wgate"]) * (y @ P[p + "Wup"])) @ P[p + "Wdown"]
        z = rms(x, P["rmsf.g"]) @ P["lm_head"]
    return F.cross_entropy(z.reshape(B * S, -1), lab.reshape(-1), ignore_index=-1)


def alg1_hvp(model, named_params, named_v, inputs, labels):
    """named_params / named_v: list of (name, ndarray) in canonical order.
    Returns (loss, flat grad, flat Hv) as float64 numpy."""
    P = {nm: torch.tensor(np.asarray(a, dtype=np.float64), requires_grad=True) for nm, a in named_params}
    vs = [torch.tensor(np.asarray(a, dtype=np.float64)) for _, a in named_v]
    plist = [P[nm] for nm, _ in named_params]
    with torch.nn.attention.sdpa_kernel(torch.nn.attention.SDPBackend.MATH):
        loss = forward_loss(model, P, inputs, labels)
        g = torch.autograd.grad(loss, plist, create_graph=True)
        d = sum((gi * vi).sum() for gi, vi in zip(g, vs))
    u = torch.autograd.grad(d, plist)
    flat = lambda ts: np.concatenate([t.detach().numpy().reshape(-1) for t in ts])
    return float(loss.detach()), flat(g), flat(u)
