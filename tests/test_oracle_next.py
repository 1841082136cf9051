"""Pins for the oracle functions of the widened rows (dataset-averaged HVP,
Hessian-column probe, smoothed density).  Each is checked against something
other than itself: PyTorch autograd run as Algorithm 1 is written, brute-force
loops, numpy's own histogram on exactly representable data, closed forms."""
import itertools

import numpy as np

import synth_inputs as si
from oracle import column_probe, dataset_hvp, density, lanczos as olz, models as om
import alg1_torch


def _named(model, flat):
    return [(nm, np.asarray(flat[off:off + int(np.prod(shp))]).reshape(shp)) for nm, off, shp in om.layout(model)]


def test_dataset_hvp_equals_alg1_loop_with_autograd():
    # Algorithm 1's batch loop with PyTorch autograd per batch: h += u*|B|; N += |B|; h/N
    cfg = dict(model=si._gpt(2, 32, 2, 64, 50, 12), batch=7, seq=12, tokens="uniform")
    model = cfg["model"]
    p = si.make_params(model, seed=3).astype(np.float64)
    v = si.make_direction(len(p), seed=4).astype(np.float64)
    x, y = si.make_batch(cfg, seed=5, batch=7, seq=12)
    batches = dataset_hvp.split_batches(x, y, 3)  # sizes 3, 3, 1
    assert [b[0].shape[0] for b in batches] == [3, 3, 1]
    h, loss = dataset_hvp.hvp_dataset(model, p, batches, v)
    acc, N, lacc = 0.0, 0, 0.0
    for xb, yb in batches:
        Lb, _, ub = alg1_torch.alg1_hvp(model, _named(model, p), _named(model, v), xb, yb)
        acc = acc + ub * xb.shape[0]
        lacc += Lb * xb.shape[0]
        N += xb.shape[0]
    np.testing.assert_allclose(h, acc / N, rtol=1e-9, atol=1e-12)
    assert abs(loss - lacc / N) < 1e-12


def test_dataset_hvp_equal_batches_is_hvp_of_the_whole_set():
    # equal batch sizes and equal numbers of valid labels: the weighted mean of the
    # batch losses is the mean loss over the whole set, so the products agree
    cfg = si.CONFIGS["mlp_tiny"]
    model = cfg["model"]
    p = si.make_params(model).astype(np.float64)
    v = si.make_direction(len(p), 7).astype(np.float64)
    x, y = si.make_batch(cfg, batch=60)
    h, loss = dataset_hvp.hvp_dataset(model, p, dataset_hvp.split_batches(x, y, 20), v)
    np.testing.assert_allclose(h, om.hvp(model, p, x, y, v), rtol=1e-10, atol=1e-13)
    assert abs(loss - om.loss_only(model, p, x, y)) < 1e-12


def test_dataset_hvp_weights_by_samples_not_tokens():
    # a batch with fewer valid labels still weighs by its number of sequences
    cfg = dict(model=si._gpt(2, 16, 2, 32, 20, 8), batch=4, seq=8, tokens="uniform")
    model = cfg["model"]
    p = si.make_params(model, seed=1).astype(np.float64)
    v = si.make_direction(len(p), seed=2).astype(np.float64)
    x, y = si.make_batch(cfg, seed=3, batch=4, seq=8)
    y = y.copy(); y[0, :5] = -1
    (xa, ya), (xb, yb) = dataset_hvp.split_batches(x, y, 3)
    h, _ = dataset_hvp.hvp_dataset(model, p, [(xa, ya), (xb, yb)], v)
    np.testing.assert_allclose(h, (3 * om.hvp(model, p, xa, ya, v) + 1 * om.hvp(model, p, xb, yb, v)) / 4, rtol=1e-12)
    assert np.linalg.norm(h - om.hvp(model, p, x, y, v)) > 1e-6 * np.linalg.norm(h)


def test_hessian_column_is_a_column_of_the_dense_hessian():
    cfg = si.CONFIGS["mlp_tiny"]
    model = cfg["model"]
    p = si.make_params(model).astype(np.float64)
    x, y = si.make_batch(cfg, batch=16)
    # finite differences of the gradient along e_j, and symmetry H[i, j] = H[j, i]
    j, i = 37, 1200
    col_j = column_probe.hessian_column(model, p, x, y, j)
    col_i = column_probe.hessian_column(model, p, x, y, i)
    eps = 1e-5
    e = np.zeros(len(p)); e[j] = eps
    g1 = om.loss_grad_hvp(model, p + e, x, y)[1]
    g0 = om.loss_grad_hvp(model, p - e, x, y)[1]
    np.testing.assert_allclose(col_j, (g1 - g0) / (2 * eps), rtol=1e-5, atol=1e-9)
    assert abs(col_j[i] - col_i[j]) < 1e-12


def test_column_stats_brute_force_and_numpy_histogram():
    rng = np.random.default_rng(0)
    # integers 0..100 as float32: every quantity below is exactly representable
    h = rng.integers(-100, 101, size=5000).astype(np.float32)
    h[17] = 100.0
    thr = np.array([0.5, 1.0, 10.0, 50.5, 1000.0], dtype=np.float32)
    below, mx, hist = column_probe.column_stats(h, thr, 50)
    assert mx == np.float32(100.0)
    for t, b in zip(thr, below):
        assert b == sum(1 for val in h if abs(float(val)) < float(t))
    ref, _ = np.histogram(np.abs(h), bins=50, range=(0.0, 100.0))
    np.testing.assert_array_equal(hist, ref)
    assert hist.sum() == len(h) and hist[-1] >= 1
    # bin of each entry by the plain definition [i w, (i+1) w), last bin closed
    w = 2.0
    manual = np.zeros(50, dtype=np.int64)
    for val in np.abs(h):
        manual[min(int(val // w), 49)] += 1
    np.testing.assert_array_equal(hist, manual)


def test_column_stats_degenerate():
    below, mx, hist = column_probe.column_stats(np.zeros(9, np.float32), [1e-12, 1.0], 50)
    assert list(below) == [9, 9] and mx == 0 and hist[0] == 9 and hist.sum() == 9
    below, mx, hist = column_probe.column_stats(np.zeros(0, np.float32), [1.0], 4)
    assert list(below) == [0] and mx == 0 and hist.sum() == 0
    h = np.array([np.nan, 1.0, -4.0], np.float32)
    below, mx, hist = column_probe.column_stats(h, [2.0], 4)
    assert list(below) == [1] and mx == 4 and list(hist) == [0, 1, 0, 1]
    # thresholds spanning the paper's table: monotone counts
    rng = np.random.default_rng(1)
    h = (rng.standard_normal(10000) * 10.0 ** rng.uniform(-13, 0, 10000)).astype(np.float32)
    thr = 10.0 ** np.arange(-12, 0, dtype=np.float64)
    below, _, _ = column_probe.column_stats(h, thr, 50)
    assert np.all(np.diff(below) >= 0) and below[-1] <= len(h)


def test_column_stats_infinite_entries():
    # Section "Banded Hessians" histograms |H_ij| over [0, max].  With an infinite maximum every bin
    # is infinitely wide: each finite entry lies in the first bin and the maximum itself (every
    # infinite entry, of either sign) belongs to the last one; an infinite entry is below no finite
    # threshold and NaN entries are counted nowhere.  Expected values written out by hand.
    inf, nan = np.inf, np.nan
    h = np.array([0.5, -inf, 2.0, inf, nan, 0.0, -1e-3, inf, 7e30], np.float32)
    below, mx, hist = column_probe.column_stats(h, [1e-2, 1.0, 3.0e38], 4)
    assert list(below) == [2, 3, 5]          # {0, -1e-3}; + 0.5; + 2.0 and 7e30
    assert mx == np.float32(inf)
    assert list(hist) == [5, 0, 0, 3]        # five finite entries, three infinite ones, the NaN nowhere
    # the same by a plain loop over the entries, for a seeded vector with planted infinities
    rng = np.random.default_rng(3)
    h = rng.standard_normal(2000).astype(np.float32)
    planted = [3, 777, 1999]
    h[planted[0]], h[planted[1]], h[planted[2]] = inf, -inf, inf
    h[11] = nan
    thr = [0.1, 1.0, 2.5]
    below, mx, hist = column_probe.column_stats(h, thr, 50)
    want_below = [0] * len(thr)
    want_hist = [0] * 50
    for val in h.tolist():
        if val != val:
            continue
        for j, t in enumerate(thr):
            if abs(val) < float(np.float32(t)):
                want_below[j] += 1
        want_hist[49 if abs(val) == inf else 0] += 1
    assert list(below) == want_below and list(hist) == want_hist and mx == np.float32(inf)
    assert hist[0] == 2000 - 4 and hist[-1] == 3


def test_density_closed_forms():
    ritz = np.array([[-1.0, 0.5, 2.0, 0.0], [0.25, 3.0, 0.0, 0.0]])
    w = np.array([[0.2, 0.3, 0.5, 0.0], [0.6, 0.4, 0.0, 0.0]])
    m_eff = [3, 2]
    grid = np.linspace(-12.0, 14.0, 26001)
    rho = density.smoothed_density(ritz, w, m_eff, 0.3, grid)
    dt = grid[1] - grid[0]
    assert abs(rho.sum() * dt - 1.0) < 1e-9                       # unit mass
    mean = 0.5 * (0.2 * -1 + 0.3 * 0.5 + 0.5 * 2.0) + 0.5 * (0.6 * 0.25 + 0.4 * 3.0)
    assert abs((rho * grid).sum() * dt - mean) < 1e-8             # first moment is kept
    second = 0.5 * (0.2 * 1 + 0.3 * 0.25 + 0.5 * 4.0) + 0.5 * (0.6 * 0.0625 + 0.4 * 9.0)
    assert abs((rho * grid * grid).sum() * dt - (second + 0.3 ** 2)) < 1e-7   # variance grows by sigma^2
    # a single node: the normal density itself
    one = density.smoothed_density([[1.5]], [[1.0]], [1], 0.7, np.array([1.5, 2.2]))
    np.testing.assert_allclose(one, [1 / (0.7 * np.sqrt(2 * np.pi)), np.exp(-0.5) / (0.7 * np.sqrt(2 * np.pi))], rtol=1e-14)
    mu = density.moments(ritz, w, m_eff, 3)
    np.testing.assert_allclose(mu, [1.0, mean, second], rtol=1e-14)


def test_moments_from_all_rademacher_probes_give_the_trace():
    # n = 4: the 16 sign vectors; mean of q^T A^p q over all of them is tr(A^p)/n for p <= 1,
    # and full-length Lanczos reproduces q^T A^p q for every p
    rng = np.random.default_rng(5)
    A = rng.standard_normal((4, 4)); A = A + A.T
    ritz, w = [], []
    for signs in itertools.product([-1.0, 1.0], repeat=4):
        al, be, _ = olz.lanczos(lambda q: A @ q, np.array(signs), 4, "full")
        th, ww = olz.slq_readout(al, be)
        ritz.append(th); w.append(ww)
    mu = density.moments(np.array(ritz), np.array(w), [4] * 16, 3)
    assert abs(mu[0] - 1.0) < 1e-12
    assert abs(mu[1] - np.trace(A) / 4) < 1e-12
    # E[z^T A^2 z] = tr(A^2) for Rademacher z (diagonal of A^2 only)
    assert abs(mu[2] - np.trace(A @ A) / 4) < 1e-10
