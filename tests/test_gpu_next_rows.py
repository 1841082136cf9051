"""GPU parity of the widened rows, through the C ABI: the dataset-averaged
Hessian-vector product (batch loop of Algorithm 1), a Hessian column, and the
column statistics of the section "Banded Hessians".

Tolerances: products as in test_gpu_hvp.py (relative L2 <= 1e-4 with fp32
parameters, <= 2e-2 with bf16); the statistics are integer counts decided in
float32 on both sides and must agree exactly when both sides see the same
float32 vector."""
import numpy as np
import pytest
import torch

import paper_2505_11564_amd as hf
import synth_inputs as si
from oracle import column_probe, dataset_hvp, models as om

from gpu_util import rel_l2, to_dev_params

pytestmark = pytest.mark.gpu

THRESHOLDS = 10.0 ** np.arange(-12, 0, dtype=np.float64)   # 1e-12 .. 1e-1, the paper's table


def _dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return t.cuda() if dtype is None else t.to(dtype).cuda()


def _accumulate(cfg, n_samples, micro, param_dtype, seed=0):
    model = cfg["model"]
    p = si.make_params(model, seed=42 + seed, param_dtype=param_dtype)
    x, y = si.make_batch(cfg, seed=43 + seed, batch=n_samples)
    v = si.make_direction(len(p), 9 + seed)
    if param_dtype == "bf16":
        v = si.bf16_bits_to_f32(si.f32_to_bf16_bits(v))
    S = x.shape[1] if model["arch"] != "mlp" else 1
    ctx = hf.Context(model, micro, 0, param_dtype)
    out = torch.full((ctx.n,), float("nan"), dtype=torch.float32, device="cuda")  # must be overwritten, not added to
    loss = ctx.hf_hvp_accumulate(to_dev_params(p, param_dtype), _dev(x), _dev(y.astype(np.int32)), n_samples, micro, S,
                                 _dev(v), out)
    got = out.cpu().numpy().astype(np.float64)
    # a second call on the same context must not depend on what the first left behind
    out.fill_(7.0)
    ctx.hf_hvp_accumulate(to_dev_params(p, param_dtype), _dev(x), _dev(y.astype(np.int32)), n_samples, micro, S, _dev(v), out)
    again = out.cpu().numpy().astype(np.float64)
    ctx.close()
    want, want_loss = dataset_hvp.hvp_dataset(model, p.astype(np.float64), dataset_hvp.split_batches(x, y, micro),
                                              v.astype(np.float64))
    return got, again, loss, want, want_loss


def test_accumulate_mlp_ragged_last_batch():
    got, again, loss, want, want_loss = _accumulate(si.CONFIGS["mlp_tiny"], 256, 100, "f32")   # 100, 100, 56
    assert rel_l2(got, want) <= 1e-4
    assert rel_l2(again, got) <= 1e-6   # atomics make the product's rounding order vary run to run
    assert abs(loss - want_loss) <= 1e-5 * abs(want_loss)


def test_accumulate_gpt_fp32():
    got, again, loss, want, want_loss = _accumulate(si.CONFIGS["gpt_2l_d128"], 11, 4, "f32")   # 4, 4, 3
    assert rel_l2(got, want) <= 1e-4
    assert rel_l2(again, got) <= 1e-6   # atomics make the product's rounding order vary run to run
    assert abs(loss - want_loss) <= 1e-5 * abs(want_loss)


def test_accumulate_gpt_bf16_single_sample_batches():
    got, _, loss, want, want_loss = _accumulate(si.CONFIGS["gpt_2l_d128"], 3, 1, "bf16", seed=1)
    assert rel_l2(got, want) <= 2e-2
    assert abs(loss - want_loss) <= 1e-3 * abs(want_loss)


def test_accumulate_one_batch_equals_hvp():
    cfg = si.CONFIGS["gpt_2l_d128"]
    model = cfg["model"]
    p = si.make_params(model)
    x, y = si.make_batch(cfg)
    v = si.make_direction(len(p), 5)
    ctx = hf.Context(model, cfg["batch"], 0, "f32")
    pd, xd, yd, vd = _dev(p), _dev(x), _dev(y.astype(np.int32)), _dev(v)
    a = torch.empty(ctx.n, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    ctx.hf_hvp(pd, xd, yd, cfg["batch"], cfg["seq"], vd, a)
    ctx.hf_hvp_accumulate(pd, xd, yd, cfg["batch"], cfg["batch"], cfg["seq"], vd, b)
    assert rel_l2(b.cpu().numpy().astype(np.float64), a.cpu().numpy().astype(np.float64)) <= 1e-6
    with pytest.raises(hf.HessformerError):
        ctx.hf_hvp_accumulate(pd, xd, yd, cfg["batch"], cfg["batch"] + 1, cfg["seq"], vd, b)
    with pytest.raises(hf.HessformerError):
        ctx.hf_hvp_accumulate(pd, xd, yd, 0, 4, cfg["seq"], vd, b)
    ctx.close()


@pytest.mark.parametrize("name,index", [("mlp_tiny", 37), ("gpt_2l_d128", 70001), ("gpt_2l_d128", 470527)])
def test_hessian_column_and_its_statistics(name, index):
    cfg = si.CONFIGS[name]
    model = cfg["model"]
    p = si.make_params(model)
    x, y = si.make_batch(cfg)
    S = x.shape[1] if model["arch"] != "mlp" else 1
    ctx = hf.Context(model, cfg["batch"], 0, "f32")
    col = torch.empty(ctx.n, dtype=torch.float32, device="cuda")
    ctx.hf_hessian_column(_dev(p), _dev(x), _dev(y.astype(np.int32)), cfg["batch"], S, index, col)
    got = col.cpu().numpy()
    want = column_probe.hessian_column(model, p.astype(np.float64), x, y, index)
    assert rel_l2(got.astype(np.float64), want) <= 1e-4
    # the statistics of the column the GPU produced, against the oracle's on the same float32 values
    below, mx, hist = ctx.hf_column_stats(col, ctx.n, THRESHOLDS, 50)
    o_below, o_mx, o_hist = column_probe.column_stats(got, THRESHOLDS, 50)
    np.testing.assert_array_equal(below, o_below)
    assert mx == o_mx
    np.testing.assert_array_equal(hist, o_hist)
    assert hist.sum() == ctx.n
    with pytest.raises(hf.HessformerError):
        ctx.hf_hessian_column(_dev(p), _dev(x), _dev(y.astype(np.int32)), cfg["batch"], S, ctx.n, col)
    ctx.close()


@pytest.mark.parametrize("n,offset", [(0, 0), (1, 0), (3, 1), (4097, 0), (1_000_003, 3), (20_000_001, 2)])
def test_column_stats_synthetic_vectors(n, offset):
    # magnitudes spread over the decades of the paper's thresholds, exact zeros, a NaN, ragged
    # lengths and start addresses that are not 16-byte aligned
    rng = np.random.default_rng(n + offset)
    h = (rng.standard_normal(n) * 10.0 ** rng.uniform(-14, 0, n)).astype(np.float32)
    if n > 10:
        h[::7] = 0.0
        h[5] = np.nan
    buf = torch.zeros(n + 8, dtype=torch.float32, device="cuda")
    buf[offset:offset + n] = _dev(h)
    view = buf[offset:offset + n]
    model = si.CONFIGS["mlp_tiny"]["model"]
    ctx = hf.Context(model, 4, 0, "f32")
    for n_bins in (50, 1, 256):
        below, mx, hist = ctx.hf_column_stats(view.data_ptr(), n, THRESHOLDS, n_bins)
        o_below, o_mx, o_hist = column_probe.column_stats(h, THRESHOLDS, n_bins)
        np.testing.assert_array_equal(below, o_below)
        assert mx == o_mx
        np.testing.assert_array_equal(hist, o_hist)
    ctx.close()


def test_column_stats_infinite_entries():
    # an infinite maximum: finite entries in the first bin, infinite ones in the last, NaN nowhere
    rng = np.random.default_rng(8)
    n = 300_007
    h = (rng.standard_normal(n) * 10.0 ** rng.uniform(-14, 0, n)).astype(np.float32)
    h[[2, 4099, n - 1]] = [np.inf, -np.inf, np.inf]
    h[9] = np.nan
    model = si.CONFIGS["mlp_tiny"]["model"]
    ctx = hf.Context(model, 4, 0, "f32")
    below, mx, hist = ctx.hf_column_stats(_dev(h), n, THRESHOLDS, 50)
    o_below, o_mx, o_hist = column_probe.column_stats(h, THRESHOLDS, 50)
    np.testing.assert_array_equal(below, o_below)
    assert mx == o_mx == np.float32(np.inf)
    np.testing.assert_array_equal(hist, o_hist)
    assert hist[0] == n - 4 and hist[-1] == 3
    ctx.close()


def test_column_stats_zero_vector_and_bad_arguments():
    model = si.CONFIGS["mlp_tiny"]["model"]
    ctx = hf.Context(model, 4, 0, "f32")
    z = torch.zeros(1000, dtype=torch.float32, device="cuda")
    below, mx, hist = ctx.hf_column_stats(z, 1000, [1e-12, 1.0], 50)
    assert list(below) == [1000, 1000] and mx == 0 and hist[0] == 1000 and hist.sum() == 1000
    with pytest.raises(hf.HessformerError):
        ctx.hf_column_stats(z, 1000, np.ones(17), 50)
    with pytest.raises(hf.HessformerError):
        ctx.hf_column_stats(z, 1000, [1.0], 257)
    with pytest.raises(hf.HessformerError):
        ctx.hf_column_stats(z, -1, [1.0], 50)
    ctx.close()
