"""Helpers for the GPU parity tests: move seeded inputs to the device and call
the C ABI through the ctypes binding."""
import numpy as np
import torch

import paper_2505_11564_amd as hf
import synth_inputs as si


def to_dev_params(flat_f32, param_dtype):
    t = torch.from_numpy(np.ascontiguousarray(flat_f32)).cuda()
    if param_dtype == "bf16":
        return t.to(torch.bfloat16).contiguous()   # values are already bf16-exact
    return t


def gpu_hvp(model, params_f32, inputs, labels, v, param_dtype="f32", ctx=None, max_batch=None):
    """Returns (Hv as float64 numpy, loss)."""
    B = inputs.shape[0]
    S = inputs.shape[1] if model["arch"] != "mlp" else 1
    own = ctx is None
    if own:
        ctx = hf.Context(model, max_batch or B, 0, param_dtype)
    p = to_dev_params(params_f32, param_dtype)
    x = torch.from_numpy(np.ascontiguousarray(inputs)).cuda()
    y = torch.from_numpy(np.ascontiguousarray(labels.astype(np.int32))).cuda()
    vd = torch.from_numpy(np.ascontiguousarray(v.astype(np.float32))).cuda()
    # NaN-filled result buffer: every element must be written (or cleared) by the library itself
    out = torch.full((ctx.n,), float("nan"), dtype=torch.float32, device="cuda")
    loss = ctx.hf_hvp(p, x, y, B, S, vd, out)
    res = out.cpu().numpy().astype(np.float64)
    if own:
        ctx.close()
    return res, loss


def rel_l2(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def block_errors(model, got, want, lay):
    """Per-tensor relative errors (for diagnostics on failure)."""
    rows = []
    for nm, off, sh in lay:
        cnt = int(np.prod(sh))
        w = want[off:off + cnt]
        g = got[off:off + cnt]
        den = np.linalg.norm(w)
        rows.append((nm, float(np.linalg.norm(g - w) / den) if den > 0 else float(np.linalg.norm(g - w)), float(den)))
    return rows


def device_params(model, param_dtype, seed=42):
    """Random-init parameters generated directly on the GPU (std 0.02 matrices
    and embeddings, gains 1, biases 0), for full-size invariant tests where no
    host copy is needed.  Returns a flat tensor in the storage dtype."""
    gen = torch.Generator(device="cuda").manual_seed(seed)
    n = si.num_params(model)
    dt = torch.bfloat16 if param_dtype == "bf16" else torch.float32
    flat = torch.empty(n, dtype=dt, device="cuda")
    off = 0
    for _, shape, init in si.param_spec(model):
        cnt = int(np.prod(shape))
        if init[0] == "normal":
            step = 1 << 28
            for a in range(0, cnt, step):
                b = min(cnt, a + step)
                flat[off + a:off + b] = (torch.randn(b - a, generator=gen, device="cuda") * init[1]).to(dt)
        else:
            flat[off:off + cnt] = 1.0 if init[0] == "ones" else 0.0
        off += cnt
    return flat


def device_randn(n, seed):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    step = 1 << 28
    for a in range(0, n, step):
        b = min(n, a + step)
        out[a:b] = torch.randn(b - a, generator=gen, device="cuda")
    return out
