#!/usr/bin/env python3
"""Benchmark of the HessFormer hot path on one MI355X.

A "step" is one Lanczos iteration of Algorithm 2 on a synthetic workload: one
exact Hessian-vector product (Algorithm 1, forward-over-reverse) followed by
the vector update (three-term recurrence, full re-orthogonalisation against
the stored basis where the workload asks for it, normalisation, basis append).
Inputs are resident in HBM before the timed region starts.

The cost of a step grows with the basis depth k (the orthogonalisation reads
k + 1 stored vectors twice), so the K timed steps are the iterations
k0 .. k0 + K - 1 with k0 = (m - K) / 2 of one m-step run: their mean depth is
that of the whole run, whatever K is.  The iterations before k0 run untimed.

Prints ONE JSON line: steps/s (the metric) on the GPT-2-small workload, HVPs/s,
the MFMA roofline of the HVP, the HBM roofline of the Lanczos vector kernels,
the same figures at the 1.3B shape and the vector-kernel roofline at the
Llama-7B parameter count under extra keys, and the float64 CPU oracle timed on
a bounded sample of the headline workload on this host's cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_F32_TFLOPS = 157.3     # fp32 vector/matrix
PEAK_HBM_GBS = 8000.0       # HBM3E


def hvp_flops(model, batch, seq):
    """Algorithmic flops of one HVP: 8 products of 2*T*d_in*d_out per linear
    layer (forward 1, tangent-forward 2, adjoint 1, tangent-adjoint 2, H v
    block 2; the plain weight gradient is not formed) plus 18 products of
    2*S^2*dh per head and layer for attention, halved for causality."""
    if model["arch"] == "mlp":
        pm = model["mlp_in"] * model["mlp_hidden"] + model["mlp_hidden"] * model["mlp_out"]
        return 16.0 * batch * pm
    d, ff, L, V = model["d_model"], model["d_ff"], model["n_layer"], model["vocab"]
    per_layer = 4 * d * d + (3 if model["arch"] == "llama" else 2) * d * ff
    pm = L * per_layer + V * d
    T = batch * seq
    return 16.0 * T * pm + 18.0 * batch * L * seq * seq * d


def hvp_algorithmic_bytes(model, batch, seq):
    """HBM bytes one HVP has to move if every product fused its primal and
    tangent pass and attention and the loss kept their S x S and T x V
    intermediates on chip.  Per matrix parameter: W and the bf16 direction read
    once in the forward and once in the backward sweep (2 + 2 + 2 + 2 bytes),
    the H v block written once in fp32 (4).  Per layer and token: the
    activations the backward sweep needs (norm outputs, q|k|v, attention
    output, the feed-forward pre-activation(s) and activation), each with its
    tangent, written once and read once in bf16 (8 bytes per element), and the
    fp32 residual stream with its tangent at the two norm inputs, written and
    read once (32 bytes per element of d_model)."""
    if model["arch"] == "mlp":
        pm = model["mlp_in"] * model["mlp_hidden"] + model["mlp_hidden"] * model["mlp_out"]
        return 12.0 * pm
    d, ff, L, V = model["d_model"], model["d_ff"], model["n_layer"], model["vocab"]
    llama = model["arch"] == "llama"
    per_layer = 4 * d * d + (3 if llama else 2) * d * ff
    pm = L * per_layer + V * d
    T = batch * seq
    saved = 6 * d + (3 if llama else 2) * ff
    return 12.0 * pm + L * T * (8.0 * saved + 32.0 * d)


def lanczos_bytes(n, k, reorth, basis_bytes, bf16_operands=False):
    """Algorithmic HBM bytes of the vector update of iteration k.  Without a
    basis: 9 fp32 words per element (3R+1W, 2R+1W, normalisation 1R+1W) as
    Algorithm 2 is written with fused passes.  With full re-orthogonalisation
    the Gram-Schmidt pass is applied to H q_k itself and subsumes the
    three-term part: it reads q_0..q_k twice (an fp32 basis holds them all;
    with a bf16 basis q_k and q_{k-1} are read from the fp32 working vectors
    and the k-1 older ones from the basis) and r three times (2R+1W); then
    normalisation (1R+1W) and the appended basis vector.  With bf16 operands
    the normalisation also leaves the bf16 copy of q_{k+1} that the next
    Hessian-vector product multiplies with."""
    vb = 2.0 * n if bf16_operands else 0.0
    if reorth != "full":
        return 36.0 * n + vb
    if basis_bytes == 4:
        rows = (k + 1) * 4.0 * n
    else:
        rows = max(0, k - 1) * 2.0 * n + min(k + 1, 2) * 4.0 * n
    return 8.0 * n + vb + 2.0 * rows + 12.0 * n + basis_bytes * n


def measured_traffic(workload):
    """HBM bytes per Hessian-vector product from the committed rocprofv3 --pmc
    summary of this workload (FETCH_SIZE and WRITE_SIZE summed over the
    kernels of one product, scaled by a copy kernel of known size); None when
    no summary has been committed for it."""
    path = os.path.join(ROOT, "profiles", f"hvp_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_hvp:"):
                    return float(line.split(":")[1])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, params, seq_sample, budget_note):
    """The float64 oracle, as it stands, on a sample of the workload's batch:
    one Lanczos iteration (one oracle HVP plus the vector update)."""
    from oracle import lanczos as olz
    from oracle import models as om
    import synth_inputs as si
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count()
    model = cfg["model"]
    x, y = si.make_batch(cfg, batch=seq_sample)
    p64 = params.astype(np.float64)
    z = si.make_probe(len(params), 0).astype(np.float64)
    t0 = time.perf_counter()
    olz.lanczos(lambda q: om.hvp(model, p64, x, y, q), z, 1, cfg["reorth"])
    dt = time.perf_counter() - t0
    scale = cfg["batch"] / seq_sample
    return {"value": 1.0 / (dt * scale), "unit": "lanczos_steps/s", "cores": int(cores), "kind": "oracle",
            "sample": f"one float64 oracle Lanczos iteration (one HVP) on {seq_sample} of {cfg['batch']} "
                      f"sequences ({dt:.1f} s), scaled by {scale:g} to the full batch; {budget_note}"}


def device_params(model, dtype):
    """Random-init parameters made on the device (std 0.02 matrices and embeddings, gains 1, biases 0)."""
    import torch
    import synth_inputs as si
    gen = torch.Generator(device="cuda").manual_seed(si.SEED_PARAMS)
    n = si.num_params(model)
    flat = torch.empty(n, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda")
    off = 0
    for _, shape, init in si.param_spec(model):
        cnt = int(np.prod(shape))
        if init[0] == "normal":
            for a in range(0, cnt, 1 << 28):
                b = min(cnt, a + (1 << 28))
                flat[off + a:off + b] = (torch.randn(b - a, generator=gen, device="cuda") * init[1]).to(flat.dtype)
        else:
            flat[off:off + cnt] = 1.0 if init[0] == "ones" else 0.0
        off += cnt
    return flat


def time_update_only(ctx, cfg, n, k_first, k_last, dtype, stream, probe=None, q=None, r=None):
    """The vector update alone over the iterations k_first .. k_last of one run, driven by a seeded
    diagonal operator (r = d * q_k) so that the recurrence is a genuine Lanczos run and the kernels
    see the same sequence of calls as in a real iteration.  HIP events on the library's stream.
    probe / q / r: n-vectors the caller already holds (the 7B-size vectors are 27 GB each)."""
    import torch
    basis = cfg["basis_dtype"]
    gen = torch.Generator(device="cuda").manual_seed(1)
    dvec = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1.0, 1.0, generator=gen)
    zd = probe if probe is not None else torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1.0, 1.0, generator=gen).sign_()
    q = q if q is not None else torch.empty(n, dtype=torch.float32, device="cuda")
    r = r if r is not None else torch.empty(n, dtype=torch.float32, device="cuda")
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ctx.hf_lanczos_init(zd, cfg["reorth"])
    del zd
    ms, nbytes = [], []
    for k in range(k_last + 1):
        ctx.hf_lanczos_get_vector(0, q)
        torch.mul(dvec, q, out=r)
        torch.cuda.synchronize()
        e0.record(stream)
        ctx.hf_lanczos_update(r)
        e1.record(stream)
        torch.cuda.synchronize()
        if k >= k_first:
            ms.append(e0.elapsed_time(e1))
            nbytes.append(lanczos_bytes(n, k, cfg["reorth"], {"bf16": 2, "f32": 4, "none": 0}[basis], dtype == "bf16"))
    gbs = sum(nbytes) / (sum(ms) * 1e-3) / 1e9
    return {"kernel": "hf_lanczos_update (vector kernels of one iteration)", "bound": "hbm", "achieved": gbs,
            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "depth_range": [k_first, k_last],
            "ms": sum(ms) / len(ms), "algorithmic_bytes": sum(nbytes) / len(nbytes), "traffic": None}


def measure(name, K, W, hvp_reps, pd=None, params_host=None):
    """HVP timing, K depth-centred Lanczos steps and the update-only roofline of one workload."""
    import torch
    import paper_2505_11564_amd as hf
    import synth_inputs as si
    cfg = si.CONFIGS[name]
    model, B, S, m = cfg["model"], cfg["batch"], cfg["seq"], cfg["m"]
    dtype, basis = cfg["param_dtype"], cfg["basis_dtype"]
    Sarg = S if model["arch"] != "mlp" else 1
    K = min(K, m) if K is not None else m
    stream = torch.cuda.current_stream()
    n = si.num_params(model)
    x, y = si.make_batch(cfg)
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    yd = torch.from_numpy(np.ascontiguousarray(y.astype(np.int32))).cuda()
    zd = torch.from_numpy(si.make_probe(n, 0)).cuda()
    ctx = hf.Context(model, B, m, dtype, basis)

    # ---- HVP alone (MFMA roofline): HIP events on the stream the library launches on
    vd = (zd / float(np.sqrt(n))).contiguous()
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    for _ in range(2):
        ctx.hf_hvp(pd, xd, yd, B, Sarg, vd, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(hvp_reps):
        ctx.hf_hvp(pd, xd, yd, B, Sarg, vd, out, want_loss=False)
    e1.record(stream)
    torch.cuda.synchronize()
    hvp_ms = e0.elapsed_time(e1) / hvp_reps
    flops = hvp_flops(model, B, Sarg)
    hvp_tflops = flops / (hvp_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_TFLOPS
    alg_bytes = hvp_algorithmic_bytes(model, B, Sarg)
    traffic = measured_traffic(name)

    # ---- Lanczos steps (the metric): W warm-up steps, then one run whose iterations k0 .. k0+K-1 are timed
    def steps(count):
        for _ in range(count):
            ctx.hf_lanczos_step(pd, xd, yd, B, Sarg)

    ctx.hf_lanczos_init(zd, cfg["reorth"])
    steps(min(W, m))
    k0 = (m - K) // 2
    ctx.hf_lanczos_init(zd, cfg["reorth"])
    steps(k0)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    steps(K)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    lz = time_update_only(ctx, cfg, n, k0, k0 + K - 1, dtype, stream, probe=zd, q=out, r=vd)
    vd.copy_(zd).div_(float(np.sqrt(n)))  # (r was scratch: the direction again, for the legs that follow)
    res = {
        "steps_per_s": K / elapsed, "ms_per_step": 1e3 * elapsed / K, "depth_range": [k0, k0 + K - 1],
        "hvps_per_s": 1e3 / hvp_ms, "hvp_ms": hvp_ms,
        "roofline": {"kernel": "hf_hvp (all kernels of one Hessian-vector product)", "bound": "mfma",
                     "achieved": hvp_tflops, "peak": peak, "unit": "TFLOP/s", "frac": hvp_tflops / peak,
                     "flops_per_launch": flops, "algorithmic_bytes": alg_bytes, "traffic": traffic,
                     "traffic_over_algorithmic": (traffic / alg_bytes) if traffic else None},
        "roofline_lanczos": lz,
    }
    return res, ctx, (xd, yd, vd, out, Sarg, flops, n)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2_small")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="skip the 1.3B and Llama-7B-size legs")
    ap.add_argument("--hvp-reps", type=int, default=10)
    ap.add_argument("--attention", default="auto", choices=["auto", "streamed", "stored"],
                    help="how attention is evaluated (hf_model_desc.attention); auto = the library's choice")
    ap.add_argument("--hvp-only", type=int, default=0, metavar="N",
                    help="profiling aid: run N Hessian-vector products, then one elementwise pass over a "
                         "1 GiB fp32 tensor (a kernel of known HBM traffic that calibrates the byte counters), and exit")
    ap.add_argument("--update-only", type=int, default=0, metavar="N",
                    help="profiling aid: run the first N vector updates of the workload (diagonal operator), "
                         "then the same calibration pass, and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_11564_amd as hf
    import synth_inputs as si

    if args.attention != "auto":
        for c in si.CONFIGS.values():
            c["model"] = dict(c["model"], attention=args.attention)
    cfg = si.CONFIGS[args.workload]
    model, B, S, m = cfg["model"], cfg["batch"], cfg["seq"], cfg["m"]
    dtype, basis = cfg["param_dtype"], cfg["basis_dtype"]
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()
    big = si.num_params(model) > 500_000_000  # parameters made on the device; no CPU baseline leg

    def calibrate():
        cal = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        cal2 = torch.empty_like(cal)
        torch.cuda.synchronize()
        torch.mul(cal, 2.0, out=cal2)  # last dispatch of the run: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()

    if args.update_only > 0:
        ctx = hf.Context(model, 1, m, dtype, basis)
        lz = time_update_only(ctx, cfg, ctx.n, 0, min(m, args.update_only) - 1, dtype, stream)
        calibrate()
        print(json.dumps({"workload": args.workload, "updates": args.update_only, "roofline_lanczos": lz,
                          "calibration_read_bytes": 4 << 28, "calibration_write_bytes": 4 << 28}))
        ctx.close()
        return

    params = None
    if big:
        pd = device_params(model, dtype)
    else:
        params = si.make_params(model, param_dtype=dtype)
        pd = torch.from_numpy(params).cuda()
        if dtype == "bf16":
            pd = pd.to(torch.bfloat16).contiguous()

    if args.hvp_only > 0:
        n = si.num_params(model)
        x, y = si.make_batch(cfg)
        xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
        yd = torch.from_numpy(np.ascontiguousarray(y.astype(np.int32))).cuda()
        vd = (torch.from_numpy(si.make_probe(n, 0)).cuda() / float(np.sqrt(n))).contiguous()
        out = torch.empty(n, dtype=torch.float32, device="cuda")
        ctx = hf.Context(model, B, 0, dtype, basis)
        for _ in range(args.hvp_only):
            ctx.hf_hvp(pd, xd, yd, B, S if model["arch"] != "mlp" else 1, vd, out, want_loss=False)
        torch.cuda.synchronize()
        calibrate()
        print(json.dumps({"workload": args.workload, "hvps": args.hvp_only, "calibration_read_bytes": 4 << 28,
                          "calibration_write_bytes": 4 << 28}))
        ctx.close()
        return

    K, W = args.steps, args.warmup
    head, ctx, (xd, yd, vd, out, Sarg, flops, n) = measure(args.workload, K, W, args.hvp_reps, pd, params)
    Kt = head["depth_range"][1] - head["depth_range"][0] + 1
    res = {
        "metric": "lanczos_steps_per_s", "value": head["steps_per_s"], "unit": "steps/s", "n_gpus": 1, "steps": Kt,
        "warmup": W, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_params": n, "batch": B, "seq": Sarg, "lanczos_m": m,
                   "reorth": cfg["reorth"], "basis_dtype": basis, "tokens": cfg["tokens"], "attention": args.attention,
                   "primal": "auto (GPT: single bf16 numbers, Llama: bf16 pairs)",
                   "depth_range": head["depth_range"],
                   "depth_note": "timed steps are iterations depth_range[0]..depth_range[1] of one m-step run "
                                 "(mean basis depth = that of the whole run); earlier iterations run untimed"},
        "hvps_per_s": head["hvps_per_s"], "hvp_ms": head["hvp_ms"],
        "roofline": head["roofline"], "roofline_lanczos": head["roofline_lanczos"],
    }
    # ---- widened rows: Hessian-column statistics (two streaming passes over an
    # n-vector, 8 n bytes) and the batch loop of Algorithm 1 over two half batches
    thr = 10.0 ** np.arange(-12, 0, dtype=np.float64)
    ctx.hf_column_stats(out, n, thr, 50)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        ctx.hf_column_stats(out, n, thr, 50)
    cs_ms = (time.perf_counter() - t0) / 3 * 1e3
    res["next_rows"] = {"column_stats": {"bound": "hbm", "bytes": 8.0 * n, "ms": cs_ms,
                                         "achieved": 8.0 * n / (cs_ms * 1e-3) / 1e9, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                         "frac": 8.0 * n / (cs_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                                         "note": "wall clock of hf_column_stats incl. its host synchronisation"}}
    if B >= 2:
        half = B // 2
        ctx.hf_hvp_accumulate(pd, xd, yd, B, half, Sarg, vd, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            ctx.hf_hvp_accumulate(pd, xd, yd, B, half, Sarg, vd, out)
        acc_ms = (time.perf_counter() - t0) / 3 * 1e3
        res["next_rows"]["hvp_accumulate"] = {"samples": B, "micro_batch": half, "ms": acc_ms,
                                              "tflops": flops / (acc_ms * 1e-3) / 1e12}
    ctx.close()
    del ctx, pd, out, xd, yd, vd
    torch.cuda.empty_cache()

    # ---- the other shapes the metric names: the 1.3B workload (whole m-step run) and the vector
    # kernels at the Llama-7B parameter count (three-term recurrence, no basis)
    if not args.no_extra and args.workload == "gpt2_small":
        c4 = si.CONFIGS["gpt_1p3b"]
        pd4 = device_params(c4["model"], c4["param_dtype"])
        r4, ctx4, keep = measure("gpt_1p3b", None, 1, 5, pd4)
        ctx4.close()
        del ctx4, pd4, keep
        torch.cuda.empty_cache()
        res["gpt_1p3b"] = r4
        c5 = si.CONFIGS["llama_7b"]
        ctx5 = hf.Context(c5["model"], 1, c5["m"], c5["param_dtype"], c5["basis_dtype"])
        res["llama_7b"] = {"n_params": ctx5.n,
                           "roofline_lanczos": time_update_only(ctx5, c5, ctx5.n, 2, c5["m"] - 1, c5["param_dtype"], stream)}
        ctx5.close()
        del ctx5
        torch.cuda.empty_cache()

    if not args.no_cpu_baseline and params is not None:
        # sample sized for roughly 15 s of oracle work (the oracle sustains about 3e11 flop/s on 16 cores)
        per_seq_s = flops / B / 3e11
        sample = int(max(1, min(B, round(15.0 / max(per_seq_s, 1e-9)))))
        res["cpu_baseline"] = cpu_baseline(cfg, params, sample, "the HVP dominates; the vector update is included")
    print(json.dumps(res))


if __name__ == "__main__":
    main()
