"""Parity of the HIP Hessian-vector product (hf_hvp, through the C ABI) with
the float64 oracle on the same seeded inputs.  Tolerances: relative L2 error
<= 1e-4 with fp32 parameters, <= 2e-2 with bf16 parameters."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import models as om

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}

SHAPES = {
    # tiny, ragged: nothing is a multiple of a tile
    "mlp_ragged": dict(model=si._mlp(13, 21, 7), batch=37, seq=1, tokens=None),
    "gpt_tiny": dict(model=si._gpt(2, 16, 2, 40, 23, 9), batch=3, seq=7, tokens="uniform"),
    "gpt_untied": dict(model=si._gpt(1, 24, 3, 32, 19, 6, tie=0), batch=2, seq=6, tokens="zipf"),
    "llama_tiny": dict(model=si._llama(2, 16, 2, 24, 21, 8), batch=2, seq=8, tokens="zipf"),
    # several 128-wide tiles with ragged tails in every dimension
    "gpt_mid": dict(model=si._gpt(2, 192, 3, 328, 1003, 160), batch=3, seq=150, tokens="zipf"),
    "llama_mid": dict(model=si._llama(2, 256, 4, 344, 777, 136), batch=2, seq=136, tokens="zipf"),
    # sequence length a multiple of 8 and head width of 32: in bf16 mode the scores take the fused
    # attention epilogues (two column tiles, the second one ragged)
    # grouped-query attention: 6 / 8 query heads on 2 key-value heads
    "llama_gqa_tiny": dict(model=si._llama(2, 24, 6, 24, 21, 8, n_kv=2), batch=2, seq=8, tokens="zipf"),
    "llama_gqa_mid": dict(model=si._llama(2, 256, 8, 344, 777, 136, n_kv=2), batch=2, seq=136, tokens="zipf"),
    "gpt_gelu_tanh": dict(model=si._gpt(2, 64, 2, 136, 301, 40, act="gelu_tanh"), batch=2, seq=40, tokens="zipf"),
    "gpt_fused": dict(model=si._gpt(2, 128, 4, 264, 517, 200), batch=2, seq=200, tokens="zipf"),
    # few output tiles and a contraction over more than 1024: in bf16 mode the dual-output products
    # of the feed-forward layers split k over blocks and are summed by a second kernel (ragged k)
    "gpt_long_k": dict(model=si._gpt(1, 64, 2, 1048, 301, 50), batch=3, seq=50, tokens="zipf"),
    # 8 heads and 4 x 4 score tiles: the fused attention kernels deal whole heads to the XCDs
    "gpt_heads8": dict(model=si._gpt(1, 256, 8, 72, 97, 400), batch=1, seq=400, tokens="zipf"),
    "llama_long_k": dict(model=si._llama(1, 64, 2, 1544, 257, 40), batch=2, seq=40, tokens="zipf"),
    # 2000 x 4088 products with k = 264: several hundred tiles with a ragged last tile in every
    # dimension
    "gpt_wide_ffn": dict(model=si._gpt(1, 264, 4, 4088, 97, 500), batch=4, seq=500, tokens="zipf"),
    # more than two layers (per-layer buffers, layer >= 2 of each family's schedule), with and
    # without grouped key/value heads
    "gpt_deep": dict(model=si._gpt(6, 64, 2, 136, 211, 40), batch=2, seq=40, tokens="zipf"),
    "llama_deep": dict(model=si._llama(6, 64, 2, 96, 211, 40), batch=2, seq=40, tokens="zipf"),
    "llama_gqa_deep": dict(model=si._llama(5, 128, 4, 176, 211, 40, n_kv=2), batch=2, seq=40, tokens="zipf"),
    # head widths 64 and 128 (bf16: the streamed attention kernels), several query blocks of 128 with a
    # ragged last one, grouped key/value heads at width 128
    "gpt_dh64_long": dict(model=si._gpt(1, 128, 2, 136, 301, 300), batch=1, seq=300, tokens="zipf"),
    "gpt_dh128": dict(model=si._gpt(2, 256, 2, 264, 301, 200), batch=2, seq=200, tokens="zipf"),
    "llama_gqa_dh128": dict(model=si._llama(2, 512, 4, 344, 301, 136, n_kv=2), batch=2, seq=136, tokens="zipf"),
}
# (attention modes only) 45 (batch, head) pairs of 6 query tiles each: 36 blocks per XCD, i.e. more
# than its 32 CUs and at most two per CU, which is where the streamed kernels pair long and short
# tiles on a CU; 45 is not a multiple of 8, so three of the 48 head slots of a launch are empty
ATTN_SHAPES = dict(SHAPES, gpt_many_heads=dict(model=si._gpt(1, 288, 9, 136, 97, 700), batch=5, seq=700, tokens="zipf"))


def run_case(cfg, dtype, seed=0, short_seq=None):
    from gpu_util import gpu_hvp, rel_l2, block_errors
    model = cfg["model"]
    p = si.make_params(model, seed=42 + seed, param_dtype=dtype, perturb=0.1)
    if dtype == "bf16":
        p = si.bf16_bits_to_f32(si.f32_to_bf16_bits(p))
    x, y = si.make_batch(cfg, seed=43 + seed, seq=short_seq)
    n = om.num_params(model)
    v = si.make_direction(n, 7 + seed)
    want_loss, _, want, _ = om.loss_grad_hvp(model, p.astype(np.float64), x, y, v.astype(np.float64))
    got, loss = gpu_hvp(model, p, x, y, v, dtype, max_batch=cfg["batch"])
    err = rel_l2(got, want)
    rows = sorted(block_errors(model, got, want, om.layout(model)), key=lambda r: -r[1])
    if not err <= TOL[dtype]:
        raise AssertionError(f"rel L2 {err:.3e} > {TOL[dtype]}; worst blocks: {rows[:12]}")
    # the same bar for every parameter tensor's block of H v on its own, so that a mistake confined
    # to a small block (a bias, a gain) cannot hide in the norm of the whole vector
    total = float(np.linalg.norm(want))
    bad = [r for r in rows if r[2] > 1e-6 * total and not r[1] <= TOL[dtype]]
    assert not bad, f"blocks above {TOL[dtype]}: {bad[:12]}"
    assert abs(loss - want_loss) <= (1e-5 if dtype == "f32" else 2e-2) * max(1.0, abs(want_loss))
    return err


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("name", list(SHAPES))
def test_hvp_parity_small(name, dtype):
    run_case(SHAPES[name], dtype)


@pytest.mark.parametrize("mode", ["streamed", "stored"])
@pytest.mark.parametrize("name", ["gpt_fused", "gpt_heads8", "llama_gqa_mid", "gpt_mid", "gpt_dh64_long", "gpt_dh128",
                                  "llama_gqa_dh128", "llama_gqa_deep", "gpt_many_heads"])
def test_hvp_attention_modes(name, mode):
    # both evaluations of attention at every head width the streamed kernels take (32, 64, 128),
    # whichever of them the library would choose by itself
    cfg = ATTN_SHAPES[name]
    run_case(dict(cfg, model=dict(cfg["model"], attention=mode)), "bf16", seed=3)


@pytest.mark.parametrize("primal", ["pairs", "single"])
@pytest.mark.parametrize("mode", ["streamed", "stored"])
@pytest.mark.parametrize("name", ["gpt_fused", "gpt_dh64_long", "gpt_dh128", "gpt_deep", "llama_gqa_mid", "llama_gqa_dh128"])
def test_hvp_primal_pairs_and_single(name, mode, primal):
    # bf16 parameters with the primal activations carried as (value, remainder) pairs or as single
    # bf16 numbers, whichever of the two the library would choose for the family, on both
    # evaluations of attention and at every head width of the streamed kernels
    cfg = SHAPES[name]
    run_case(dict(cfg, model=dict(cfg["model"], attention=mode, primal=primal)), "bf16", seed=5)


def test_hvp_streamed_attention_needs_a_supported_head_width():
    import paper_2505_11564_amd as hf
    model = dict(si._gpt(1, 48, 2, 64, 97, 16), attention="streamed")   # head width 24
    with pytest.raises(hf.HessformerError) as e:
        hf.Context(model, 1, 0, "bf16")
    assert e.value.code == hf.binding.HF_ESHAPE
    with pytest.raises(hf.HessformerError):
        hf.Context(dict(SHAPES["gpt_fused"]["model"], attention="streamed"), 1, 0, "f32")   # fp32 parameters


def test_hvp_parity_many_whole_tiles():
    # 2048 x 4096 products with k = 256: 512 tiles of 128 x 128 without any ragged edge
    run_case(dict(model=si._gpt(1, 256, 4, 4096, 97, 512), batch=4, seq=512, tokens="zipf"), "bf16")


def test_hvp_shorter_sequence_than_max():
    run_case(SHAPES["gpt_mid"], "f32", seed=1, short_seq=77)


def test_hvp_bf16_sequence_length_changes_on_one_context():
    # The fused attention kernels write only the score tiles on and below the diagonal and rely on
    # the rest having been cleared for the current [batch, seq] layout: alternate layouts on one
    # context and check every product against the oracle.  Sequence length 77 is not a multiple of
    # 8 and takes the unfused kernels, which write whole score matrices in another layout.
    import paper_2505_11564_amd as hf
    from gpu_util import gpu_hvp, rel_l2
    cfg = SHAPES["gpt_fused"]
    model = cfg["model"]
    p = si.bf16_bits_to_f32(si.f32_to_bf16_bits(si.make_params(model, param_dtype="bf16", perturb=0.1)))
    n = om.num_params(model)
    ctx = hf.Context(model, cfg["batch"], 0, "bf16")
    for k, (batch, seq) in enumerate([(2, 200), (2, 136), (1, 200), (2, 72), (2, 200), (2, 77), (2, 200)]):
        x, y = si.make_batch(cfg, seed=50 + k, batch=batch, seq=seq)
        v = si.make_direction(n, 60 + k)
        want = om.hvp(model, p.astype(np.float64), x, y, v.astype(np.float64))
        got, _ = gpu_hvp(model, p, x, y, v, "bf16", ctx=ctx)
        assert rel_l2(got, want) <= TOL["bf16"], (batch, seq)
    ctx.close()


def test_hvp_ignored_labels_and_single_valid():
    from gpu_util import gpu_hvp, rel_l2
    cfg = SHAPES["gpt_tiny"]
    model = cfg["model"]
    p = si.make_params(model, perturb=0.1)
    x, y = si.make_batch(cfg)
    y[:] = -1
    y[1, 3] = 5
    v = si.make_direction(om.num_params(model), 3)
    want = om.hvp(model, p.astype(np.float64), x, y, v.astype(np.float64))
    got, _ = gpu_hvp(model, p, x, y, v)
    assert rel_l2(got, want) <= 1e-4


@pytest.mark.parametrize("name", ["mlp_tiny", "gpt_2l_d128"])
def test_hvp_parity_workloads_1_and_2(name):
    cfg = si.CONFIGS[name]
    run_case(dict(model=cfg["model"], batch=cfg["batch"], seq=cfg["seq"], tokens=cfg["tokens"]), "f32")


def test_hvp_symmetry_on_gpu():
    from gpu_util import gpu_hvp
    cfg = si.CONFIGS["gpt_2l_d128"]
    model = cfg["model"]
    p = si.make_params(model)
    x, y = si.make_batch(cfg)
    n = om.num_params(model)
    v, w = si.make_direction(n, 1), si.make_direction(n, 2)
    hv, _ = gpu_hvp(model, p, x, y, v)
    hw, _ = gpu_hvp(model, p, x, y, w)
    a, b = float(w.astype(np.float64) @ hv), float(v.astype(np.float64) @ hw)
    assert abs(a - b) <= 1e-4 * max(abs(a), abs(b))


def test_hvp_input_errors():
    import paper_2505_11564_amd as hf
    import torch
    cfg = SHAPES["gpt_tiny"]
    model = cfg["model"]
    ctx = hf.Context(model, cfg["batch"], 0)
    p = torch.from_numpy(si.make_params(model)).cuda()
    x, y = si.make_batch(cfg)
    v = torch.ones(ctx.n, device="cuda")
    out = torch.empty(ctx.n, device="cuda")
    xd, yd = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_hvp(p, xd, yd, cfg["batch"] + 1, cfg["seq"], v, out)
    assert e.value.code == hf.binding.HF_ESHAPE
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_hvp(p, xd, yd, cfg["batch"], cfg["seq"], v, v)
    assert e.value.code == hf.binding.HF_EINVAL
    bad = x.copy(); bad[0, 0] = model["vocab"]
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_hvp(p, torch.from_numpy(bad).cuda(), yd, cfg["batch"], cfg["seq"], v, out)
    assert e.value.code == hf.binding.HF_EINVAL
    ybad = y.copy(); ybad[0, 0] = model["vocab"] + 3
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_hvp(p, xd, torch.from_numpy(ybad).cuda(), cfg["batch"], cfg["seq"], v, out)
    assert e.value.code == hf.binding.HF_EINVAL
    # and the context still works afterwards
    ctx.hf_hvp(p, xd, yd, cfg["batch"], cfg["seq"], v, out)
    ctx.close()
