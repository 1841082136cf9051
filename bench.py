#!/usr/bin/env python3
"""Benchmark of the HessFormer hot path on one MI355X.

A "step" is one Lanczos iteration of Algorithm 2 on a synthetic workload: one
exact Hessian-vector product (Algorithm 1, forward-over-reverse) followed by
the vector update (three-term recurrence, full re-orthogonalisation against
the stored basis where the workload asks for it, normalisation, basis append).
Inputs are resident in HBM before the timed region starts.

Prints ONE JSON line: steps/s (the metric), HVPs/s, the MFMA roofline of the
HVP, the HBM roofline of the Lanczos vector kernels, and the float64 CPU oracle
timed on a bounded sample of the same workload on this host's cores.
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


def lanczos_bytes(n, k, reorth, basis_bytes, bf16_operands=False):
    """Algorithmic HBM bytes of the vector update of iteration k.  Without a
    basis: 9 fp32 words per element (3R+1W, 2R+1W, normalisation 1R+1W).  With
    full re-orthogonalisation the Gram-Schmidt pass is applied to H q_k itself
    and subsumes the three-term part: it reads q_0..q_k twice (an fp32 basis
    holds them all; with a bf16 basis q_k and q_{k-1} are read from the fp32
    working vectors and the k-1 older ones from the basis) and r three times
    (2R+1W); then normalisation (1R+1W) and the appended basis vector.  With
    bf16 operands the normalisation also writes the bf16 copy of q_{k+1} that
    the next Hessian-vector product multiplies with."""
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
    """The float64 oracle, as it stands, on one sequence of the workload's
    batch: one Lanczos iteration (one oracle HVP plus the vector update)."""
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="gpt2_small")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--hvp-reps", type=int, default=10)
    ap.add_argument("--hvp-only", type=int, default=0, metavar="N",
                    help="profiling aid: run N Hessian-vector products, then one elementwise pass over a "
                         "1 GiB fp32 tensor (a kernel of known HBM traffic that calibrates the byte counters), and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2505_11564_amd as hf
    import synth_inputs as si

    cfg = si.CONFIGS[args.workload]
    model, B, S, m = cfg["model"], cfg["batch"], cfg["seq"], cfg["m"]
    K = args.steps if args.steps is not None else m
    W = args.warmup
    dtype, basis = cfg["param_dtype"], cfg["basis_dtype"]
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    params = si.make_params(model, param_dtype=dtype)
    n = len(params)
    x, y = si.make_batch(cfg)
    pd = torch.from_numpy(params).cuda()
    if dtype == "bf16":
        pd = pd.to(torch.bfloat16).contiguous()
    xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    yd = torch.from_numpy(np.ascontiguousarray(y.astype(np.int32))).cuda()
    zd = torch.from_numpy(si.make_probe(n, 0)).cuda()
    Sarg = S if model["arch"] != "mlp" else 1
    ctx = hf.Context(model, B, m, dtype, basis)

    # ---- HVP alone (MFMA roofline) ------------------------------------------
    vd = (zd / float(np.sqrt(n))).contiguous()
    out = torch.empty(n, dtype=torch.float32, device="cuda")
    if args.hvp_only > 0:
        for _ in range(args.hvp_only):
            ctx.hf_hvp(pd, xd, yd, B, Sarg, vd, out, want_loss=False)
        torch.cuda.synchronize()
        cal = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        cal2 = torch.empty_like(cal)
        torch.cuda.synchronize()
        torch.mul(cal, 2.0, out=cal2)  # last dispatch of the run: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        print(json.dumps({"workload": args.workload, "hvps": args.hvp_only, "calibration_read_bytes": 4 << 28,
                          "calibration_write_bytes": 4 << 28}))
        ctx.close()
        return
    for _ in range(2):
        ctx.hf_hvp(pd, xd, yd, B, Sarg, vd, out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record(stream)
    for _ in range(args.hvp_reps):
        ctx.hf_hvp(pd, xd, yd, B, Sarg, vd, out, want_loss=False)
    e1.record(stream)
    torch.cuda.synchronize()
    hvp_ms = e0.elapsed_time(e1) / args.hvp_reps
    flops = hvp_flops(model, B, Sarg)
    hvp_tflops = flops / (hvp_ms * 1e-3) / 1e12
    peak = PEAK_BF16_TFLOPS if dtype == "bf16" else PEAK_F32_TFLOPS

    # ---- Lanczos steps (the metric) ------------------------------------------
    def run_steps(count):
        done = 0
        while done < count:
            ctx.hf_lanczos_init(zd, cfg["reorth"])
            for _ in range(min(m, count - done)):
                ctx.hf_lanczos_step(pd, xd, yd, B, Sarg)
                done += 1

    run_steps(W)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run_steps(K)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- Lanczos vector update alone (HBM roofline), at the mean basis depth --
    # A seeded diagonal operator stands in for H (r = d * q_k), so the
    # recurrence is a genuine Lanczos run and the vector kernels see the same
    # sequence of calls as in a real iteration.
    ctx.hf_lanczos_init(zd, cfg["reorth"])
    depth = min(m, max(1, K)) // 2
    gen = torch.Generator(device="cuda").manual_seed(1)
    dvec = torch.empty(n, dtype=torch.float32, device="cuda").uniform_(-1.0, 1.0, generator=gen)
    r = torch.empty(n, dtype=torch.float32, device="cuda")
    upd_ms, upd_bytes = [], []
    for k in range(depth + 1):
        ctx.hf_lanczos_get_vector(0, out)
        torch.mul(dvec, out, out=r)
        torch.cuda.synchronize()
        e0.record(stream)
        ctx.hf_lanczos_update(r)
        e1.record(stream)
        torch.cuda.synchronize()
        if k >= max(0, depth - 4):
            upd_ms.append(e0.elapsed_time(e1))
            upd_bytes.append(lanczos_bytes(n, k, cfg["reorth"], {"bf16": 2, "f32": 4, "none": 0}[basis], dtype == "bf16"))
    lz_gbs = sum(upd_bytes) / (sum(upd_ms) * 1e-3) / 1e9

    res = {
        "metric": "lanczos_steps_per_s", "value": K / elapsed, "unit": "steps/s", "n_gpus": 1, "steps": K,
        "warmup": W, "ms_per_step": 1e3 * elapsed / K, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": args.workload, "n_params": n, "batch": B, "seq": Sarg, "lanczos_m": m,
                   "reorth": cfg["reorth"], "basis_dtype": basis, "tokens": cfg["tokens"]},
        "hvps_per_s": 1e3 / hvp_ms, "hvp_ms": hvp_ms,
        "roofline": {"kernel": "hf_hvp (all kernels of one Hessian-vector product)", "bound": "mfma",
                     "achieved": hvp_tflops, "peak": peak, "unit": "TFLOP/s", "frac": hvp_tflops / peak,
                     "flops_per_launch": flops, "traffic": measured_traffic(args.workload)},
        "roofline_lanczos": {"kernel": "hf_lanczos_update (vector kernels of one iteration)", "bound": "hbm",
                             "achieved": lz_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": lz_gbs / PEAK_HBM_GBS,
                             "basis_depth": depth, "ms": sum(upd_ms) / len(upd_ms), "traffic": None},
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
                                         "note": "wall clock of hf_column_stats incl. its two host synchronisations"}}
    if B >= 2:
        half = B // 2
        ctx.hf_hvp_accumulate(pd, xd, yd, B, half, Sarg, vd, out)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.hf_hvp_accumulate(pd, xd, yd, B, half, Sarg, vd, out)
        acc_ms = (time.perf_counter() - t0) * 1e3
        res["next_rows"]["hvp_accumulate"] = {"samples": B, "micro_batch": half, "ms": acc_ms,
                                              "tflops": flops / (acc_ms * 1e-3) / 1e12}
    ctx.close()
    if not args.no_cpu_baseline:
        del pd, out, r, dvec
        torch.cuda.empty_cache()
        # sample sized for roughly 15 s of oracle work (the oracle sustains about 3e11 flop/s here)
        per_seq_s = flops / B / 3e11
        sample = int(max(1, min(B, round(15.0 / max(per_seq_s, 1e-9)))))
        res["cpu_baseline"] = cpu_baseline(cfg, params, sample, "the HVP dominates; the vector update is included")
    print(json.dumps(res))


if __name__ == "__main__":
    main()
