"""The column statistics through the entry point that allocates nothing
(hf_column_stats_noalloc, counters in a static device array of the library)
against the context-based entry point, bit for bit, on two calls in a row, the
second on a smaller vector."""
import numpy as np
import pytest
import torch

import paper_2505_11564_amd as hf
import synth_inputs as si

pytestmark = pytest.mark.gpu

THRESHOLDS = 10.0 ** np.arange(-12, 0, dtype=np.float64)


def _vec(n, seed):
    rng = np.random.default_rng(seed)
    h = (rng.standard_normal(n) * 10.0 ** rng.uniform(-14, 0, n)).astype(np.float32)
    h[::7] = 0.0
    h[5] = np.nan
    return h


def test_noalloc_entry_point_matches_context_entry_point_twice():
    model = si.CONFIGS["mlp_tiny"]["model"]
    ctx = hf.Context(model, 4, 0, "f32")
    for n, seed, n_bins in ((3_000_017, 1, 50), (40_001, 2, 256)):   # the second call on a smaller vector
        h = torch.from_numpy(_vec(n, seed)).cuda()
        before = torch.cuda.memory_allocated()
        below, mx, hist = hf.hf_column_stats_noalloc(h, n, THRESHOLDS, n_bins)
        assert torch.cuda.memory_allocated() == before
        w_below, w_mx, w_hist = ctx.hf_column_stats(h, n, THRESHOLDS, n_bins)
        np.testing.assert_array_equal(below, w_below)
        assert mx == w_mx
        np.testing.assert_array_equal(hist, w_hist)
        assert hist.sum() == n - 1                                   # every entry but the NaN
    ctx.close()


def test_noalloc_entry_point_rejects_sizes_beyond_its_limits():
    h = torch.zeros(16, device="cuda")
    for args in ((h, 16, np.ones(17), 50), (h, 16, [1.0], 257), (h, 16, [1.0], 0), (h, 1 << 40, [1.0], 50), (h, -1, [1.0], 50)):
        with pytest.raises(hf.HessformerError) as e:
            hf.hf_column_stats_noalloc(*args)
        assert e.value.code in (hf.binding.HF_EINVAL, hf.binding.HF_ESHAPE) and "hf_column_stats_noalloc" in str(e.value)
    # and still works afterwards, including the empty vector
    below, mx, hist = hf.hf_column_stats_noalloc(h, 16, [1.0], 4)
    assert list(below) == [16] and mx == 0 and list(hist) == [16, 0, 0, 0]
    below, mx, hist = hf.hf_column_stats_noalloc(h, 0, [1.0], 4)
    assert list(below) == [0] and hist.sum() == 0
