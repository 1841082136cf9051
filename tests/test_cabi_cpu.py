"""CPU-only checks of the C ABI library: it loads, exports every symbol the
header declares, and its host-side logic (canonical layout, parameter counts,
tridiagonal read-out, argument validation) is right.  No compute calls."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2505_11564_amd as hf
from paper_2505_11564_amd import binding
import synth_inputs as si
from oracle import lanczos as olz
from oracle import models as om

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "hessformer.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(hf_[a-z0-9_]+)\s*\(", hdr))
    assert declared, "no declarations parsed"
    L = hf.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert declared == set(hf.EXPORTS)
    assert "gfx950" in hf.hf_version()


@pytest.mark.parametrize("name", list(si.CONFIGS))
def test_layout_matches_oracle_and_generator(name):
    cfg = si.CONFIGS[name]
    d = hf.make_desc(cfg["model"], cfg["param_dtype"], cfg["basis_dtype"])
    lay = hf.hf_layout(d)
    assert [(a, o, tuple(s)) for a, o, s in lay] == [(a, o, tuple(s)) for a, o, s in om.layout(cfg["model"])]
    assert [(a, tuple(s)) for a, _, s in lay] == [(a, tuple(s)) for a, s, _ in si.param_spec(cfg["model"])]
    assert hf.hf_desc_num_params(d) == om.num_params(cfg["model"])


def test_layout_grouped_query_llama():
    model = si._llama(3, 64, 8, 96, 101, 16, n_kv=2)
    d = hf.make_desc(model)
    lay = hf.hf_layout(d)
    assert [(a, o, tuple(s)) for a, o, s in lay] == [(a, o, tuple(s)) for a, o, s in om.layout(model)]
    assert dict((a, tuple(s)) for a, _, s in lay)["h0.Wk"] == (64, 16)
    assert hf.hf_desc_num_params(d) == om.num_params(model) == si.num_params(model)
    bad = hf.make_desc(si._llama(1, 64, 8, 96, 101, 16, n_kv=3))      # 3 does not divide 8
    assert hf.hf_desc_num_params(bad) < 0
    gpt = hf.make_desc(si._gpt(1, 64, 8, 96, 101, 16))
    gpt.n_kv_head = 2                                                   # a LLAMA option only
    assert hf.hf_desc_num_params(gpt) < 0


def test_layout_untied_gpt_and_errors():
    m = si._gpt(1, 24, 3, 32, 19, 6, tie=0)
    lay = hf.hf_layout(hf.make_desc(m))
    assert lay[-1][0] == "lm_head" and lay[-1][2] == (24, 19)
    bad = si._gpt(1, 25, 3, 32, 19, 6)            # d_model not a multiple of n_head
    assert hf.hf_desc_num_params(hf.make_desc(bad)) == binding.HF_EINVAL
    odd = si._llama(1, 6, 2, 8, 11, 4)            # head width 3: no rotary pairs
    assert hf.hf_desc_num_params(hf.make_desc(odd)) == binding.HF_EINVAL
    d = hf.make_desc(m)
    d.param_dtype = 7
    assert hf.hf_desc_num_params(d) == binding.HF_EINVAL
    assert hf.lib().hf_desc_num_params(None) == binding.HF_EINVAL


@pytest.mark.parametrize("k", [1, 2, 3, 10, 37, 100])
def test_tridiag_readout_vs_eigh(k):
    rng = np.random.default_rng(k)
    a = rng.standard_normal(k) * 3
    b = np.abs(rng.standard_normal(k)) + 0.05
    ritz, w, last = hf.hf_tridiag_readout(a, b, want_last_row=True)
    T = olz.tridiagonal(a, b)
    lam, Y = np.linalg.eigh(T)
    np.testing.assert_allclose(ritz, lam, rtol=0, atol=1e-12 * max(1, np.abs(lam).max()))
    np.testing.assert_allclose(w, Y[0] ** 2, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.abs(last), np.abs(Y[-1]), rtol=0, atol=1e-10)
    assert abs(w.sum() - 1) < 1e-12 and np.all(np.diff(ritz) >= 0) and np.all(w >= 0)
    # quadrature identity: sum w theta = alpha_0
    assert abs((w * ritz).sum() - a[0]) < 1e-11 * max(1, abs(a[0]))


def test_tridiag_readout_graded_and_degenerate():
    # strongly graded entries (as in the paper's Table 2: Ritz values from 1e-6 to 8e4)
    a = np.array([1e-6, 3.0, -8e4, 2e4, 0.5, -7e3])
    b = np.array([1e-3, 2.0, 5e2, 1e1, 3e-2, 0.0])
    ritz, w = hf.hf_tridiag_readout(a, b)
    lam, Y = np.linalg.eigh(olz.tridiagonal(a, b))
    np.testing.assert_allclose(ritz, lam, rtol=1e-12, atol=1e-9)
    # zero off-diagonals: T is already diagonal
    ritz, w = hf.hf_tridiag_readout([3.0, 1.0, 2.0], [0.0, 0.0, 0.0])
    np.testing.assert_allclose(ritz, [1.0, 2.0, 3.0])
    np.testing.assert_allclose(w, [0.0, 0.0, 1.0])


def test_readout_and_create_argument_errors():
    L = hf.lib()
    dp = C.POINTER(C.c_double)
    buf = (C.c_double * 4)()
    assert L.hf_tridiag_readout(None, buf, 2, buf, buf, None) == binding.HF_EINVAL
    assert L.hf_tridiag_readout(buf, buf, 0, buf, buf, None) == binding.HF_EINVAL
    h = C.c_void_p()
    d = hf.make_desc(si.CONFIGS["mlp_tiny"]["model"])
    assert L.hf_create(None, 0, 1, 0, C.byref(h)) == binding.HF_EINVAL
    assert L.hf_create(C.byref(d), 0, 0, 0, C.byref(h)) == binding.HF_EINVAL
    assert L.hf_create(C.byref(d), 0, 4, -1, C.byref(h)) == binding.HF_EINVAL
    d.mlp_out = 1
    assert L.hf_create(C.byref(d), 0, 4, 0, C.byref(h)) == binding.HF_EINVAL
    assert b"MLP" in L.hf_last_error(None)
    # NULL handles are rejected, not dereferenced
    assert L.hf_num_params(None) == binding.HF_EINVAL
    assert L.hf_lanczos_iterations(None) == binding.HF_EINVAL
    assert L.hf_hvp(None, None, None, None, 1, 1, None, None, None, None) == binding.HF_EINVAL
    L.hf_destroy(None)


def test_density_and_moments_match_oracle():
    from oracle import density
    rng = np.random.default_rng(3)
    P, m = 3, 7
    ritz = np.sort(rng.standard_normal((P, m)) * 2.0, axis=1)
    w = rng.random((P, m))
    m_eff = np.array([7, 5, 1], dtype=np.int32)
    for p in range(P):
        w[p, :m_eff[p]] /= w[p, :m_eff[p]].sum()
    grid = np.linspace(-8.0, 8.0, 401)
    got = hf.hf_slq_density(ritz, w, m_eff, 0.25, grid)
    np.testing.assert_allclose(got, density.smoothed_density(ritz, w, m_eff, 0.25, grid), rtol=1e-12, atol=1e-300)
    got = hf.hf_slq_moments(ritz, w, m_eff, 4)
    np.testing.assert_allclose(got, density.moments(ritz, w, m_eff, 4), rtol=1e-12)
    with pytest.raises(hf.HessformerError):
        hf.hf_slq_density(ritz, w, m_eff, 0.0, grid)
    with pytest.raises(hf.HessformerError):
        hf.hf_slq_moments(ritz, w, np.array([8, 1, 1], dtype=np.int32), 2)
