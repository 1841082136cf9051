"""Parity of the HIP Lanczos iteration and SLQ read-out (hf_lanczos_*, hf_slq,
through the C ABI) with the float64 oracle of Algorithm 2.

The fp32 trajectory of late alpha_k, beta_k legitimately departs from the
float64 one, so the comparison is: early coefficients tightly, converged
extreme Ritz values within relative 1e-3, and the invariants of the read-out
(weights >= 0 summing to 1, ascending Ritz values)."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import lanczos as olz
from oracle import models as om

pytestmark = pytest.mark.gpu


def _dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run_update_only(ctx, dvec, z, m, reorth, tol=0.0):
    """Algorithm 2 on the GPU with a synthetic diagonal operator standing in
    for the Hessian-vector product."""
    import torch
    n = ctx.n
    d_dev, q = _dev(dvec.astype(np.float32)), torch.empty(n, device="cuda")
    ctx.hf_lanczos_init(_dev(z.astype(np.float32)), reorth)
    al, be = [], []
    for k in range(m):
        ctx.hf_lanczos_get_vector(0, q)
        r = (d_dev * q).contiguous()
        a, b, rc = ctx.hf_lanczos_update(r, tol)
        al.append(a); be.append(b)
        if rc == 1:
            break
    return np.array(al), np.array(be)


# only the models' parameter counts matter here: a multiple of 4, and one that leaves a tail of one
# element after the 16-byte groups
UPDATE_MODELS = {"n54032": si._gpt(1, 40, 2, 72, 1001, 33), "n56981_ragged": si._gpt(1, 42, 2, 71, 1001, 33)}


# (parameter type, basis type): with bf16 parameters and an fp32 basis the subtraction pass reads
# the old rows from bf16 copies, which must leave the coefficients at fp32 level
@pytest.mark.parametrize("dtype,basis", [("f32", "f32"), ("f32", "bf16"), ("bf16", "f32")])
@pytest.mark.parametrize("reorth", ["none", "full"])
@pytest.mark.parametrize("size", list(UPDATE_MODELS))
def test_update_kernels_diagonal_operator(size, reorth, basis, dtype):
    import paper_2505_11564_amd as hf
    model = UPDATE_MODELS[size]
    ctx = hf.Context(model, 1, 48, dtype, basis)
    n = ctx.n
    assert (n % 4 != 0) == size.endswith("ragged")
    rng = np.random.default_rng(5)
    dvec = np.concatenate([rng.uniform(-1, 1, n - 3), [-7.0, 9.0, 12.0]]).astype(np.float32)
    z = si.make_probe(n, 0)
    m = 40
    a, b = run_update_only(ctx, dvec, z, m, reorth)
    ao, bo, _ = olz.lanczos(lambda q: dvec.astype(np.float64) * q, z.astype(np.float64), m, reorth)
    # A bf16 basis perturbs r by the rounding of the stored vectors (2^-9
    # relative per element) in every orthogonalisation pass, so only the first
    # two iterations (whose pass is against q_0, q_1 only) stay at fp32 level.
    tol = (2e-5, 2e-6) if (basis == "f32" or reorth == "none") else (2e-2, 2e-2 * 12.0)
    np.testing.assert_allclose(a[:2], ao[:2], rtol=2e-5, atol=2e-6)
    np.testing.assert_allclose(a[:6], ao[:6], rtol=tol[0], atol=tol[1])
    np.testing.assert_allclose(b[:6], bo[:6], rtol=tol[0], atol=tol[1])
    th, w = hf.hf_tridiag_readout(a, b)
    tho, wo = olz.slq_readout(ao, bo)
    assert abs(th[-1] - 12.0) <= 1e-3 * 12.0 and abs(th[0] + 7.0) <= 1e-3 * 7.0
    assert abs(th[-1] - tho[-1]) <= 1e-3 * abs(tho[-1]) and abs(th[0] - tho[0]) <= 1e-3 * abs(tho[0])
    assert abs(w.sum() - 1) < 1e-12 and np.all(w >= 0)
    if reorth == "full":
        # stored basis is orthonormal to fp32 (bf16: to its rounding) level
        import torch
        Q = torch.empty(10, n, device="cuda")
        for j in range(10):
            ctx.hf_lanczos_get_vector(16 + j, Q[j])
        G = (Q.double() @ Q.double().T).cpu().numpy()
        # (bf16: every stored entry carries a relative rounding error of up to 2^-9, which does not
        # average out where it is systematic: the equal-magnitude entries of the normalised
        # Rademacher probe q_0 all round the same way, and the later vectors concentrate on the
        # three planted coordinates, so <q_i, q_j> of the stored copies is off by up to about 2^-7)
        dev = np.abs(G - np.eye(10))
        assert dev.max() <= (1e-5 if basis == "f32" else 2.0 ** -7)
        # the newest row is the working vector q_m itself (fp32) or its rounding to nearest even
        # (bf16), to the last element of a ragged length
        qm, row = torch.empty(n, device="cuda"), torch.empty(n, device="cuda")
        ctx.hf_lanczos_get_vector(0, qm)
        ctx.hf_lanczos_get_vector(16 + m, row)
        assert torch.equal(row, qm if basis == "f32" else qm.bfloat16().float())
        # no ghost copies of the converged top eigenvalue
        assert int(np.sum(np.abs(th - 12.0) <= 1e-3 * 12.0)) == 1
    ctx.close()


def test_update_is_bitwise_reproducible_and_breaks_down():
    import paper_2505_11564_amd as hf
    model = si._gpt(1, 16, 2, 24, 37, 9)
    ctx = hf.Context(model, 1, 12, "f32", "f32")
    n = ctx.n
    rng = np.random.default_rng(1)
    dvec = rng.uniform(-2, 2, n)
    z = si.make_probe(n, 3)
    r1 = run_update_only(ctx, dvec, z, 10, "full")
    r2 = run_update_only(ctx, dvec, z, 10, "full")
    assert np.array_equal(r1[0], r2[0]) and np.array_equal(r1[1], r2[1])
    # three distinct eigenvalues: the Krylov space is exhausted after 3 steps
    d3 = np.resize([1.0, 2.0, 4.0], n)
    a, b = run_update_only(ctx, d3, np.ones(n), 10, "none", tol=1e-4)
    assert len(a) == 3
    th, _ = hf.hf_tridiag_readout(a, b)
    np.testing.assert_allclose(th, [1.0, 2.0, 4.0], rtol=1e-5)
    with pytest.raises(hf.HessformerError) as e:          # iteration has ended
        ctx.hf_lanczos_update(_dev(np.ones(n, dtype=np.float32)))
    assert e.value.code == hf.binding.HF_ESTATE
    ctx.close()


def _slq_case(cfg, m, n_probes, reorth, n_early, dtype="f32", basis="f32", rtol_early=1e-4):
    import paper_2505_11564_amd as hf
    from gpu_util import to_dev_params
    model = cfg["model"]
    p = si.make_params(model, param_dtype=dtype)
    x, y = si.make_batch(cfg)
    n = om.num_params(model)
    probes = np.stack([si.make_probe(n, i) for i in range(n_probes)])
    B = x.shape[0]
    S = x.shape[1] if model["arch"] != "mlp" else 1
    ctx = hf.Context(model, B, m, dtype, basis)
    res = ctx.hf_slq(to_dev_params(p, dtype), _dev(x), _dev(y.astype(np.int32)), B, S, _dev(probes), n_probes, m, reorth)
    ctx.close()
    p64 = p.astype(np.float64)
    ora = olz.slq(lambda q: om.hvp(model, p64, x, y, q), probes.astype(np.float64), m, reorth)
    for i in range(n_probes):
        ao, bo, tho, wo, meo = ora[i]
        assert res["m_eff"][i] == m == meo
        a, b, th, w = res["alpha"][i], res["beta"][i], res["ritz"][i], res["weights"][i]
        scale = max(np.abs(tho).max(), 1e-30)
        np.testing.assert_allclose(a[:n_early], ao[:n_early], rtol=rtol_early, atol=rtol_early * scale)
        np.testing.assert_allclose(b[:n_early], bo[:n_early], rtol=rtol_early, atol=rtol_early * scale)
        assert np.all(np.diff(th) >= 0) and np.all(w >= 0) and abs(w.sum() - 1) < 1e-10
    return res, ora


def test_slq_workload_1_mlp_full_reorth_vs_dense_hessian():
    cfg = si.CONFIGS["mlp_tiny"]
    res, ora = _slq_case(cfg, cfg["m"], cfg["n_probes"], "full", n_early=5)
    model = cfg["model"]
    p = si.make_params(model).astype(np.float64)
    x, y = si.make_batch(cfg)
    lam = np.linalg.eigvalsh(om.dense_hessian(model, p, x, y))
    for i in range(cfg["n_probes"]):
        th, tho = res["ritz"][i], ora[i][2]
        for j in (0, -1):                                  # extreme Ritz values: 1e-3 relative
            assert abs(th[j] - tho[j]) <= 1e-3 * abs(tho[j]), (i, j, th[j], tho[j])
        assert abs(th[-1] - lam[-1]) <= 1e-3 * abs(lam[-1])
        assert th[0] >= lam[0] - 1e-3 * abs(lam[-1]) and th[-1] <= lam[-1] * (1 + 1e-3)
        # no ghosts of the top eigenvalue with the stored basis
        assert int(np.sum(np.abs(th - lam[-1]) <= 1e-3 * lam[-1])) == int(np.sum(np.abs(lam - lam[-1]) <= 1e-3 * lam[-1]))


def test_slq_workload_2_gpt_full_reorth():
    cfg = si.CONFIGS["gpt_2l_d128"]
    res, ora = _slq_case(cfg, cfg["m"], cfg["n_probes"], "full", n_early=4)
    for i in range(cfg["n_probes"]):
        th, tho = res["ritz"][i], ora[i][2]
        for j in (0, -1):
            assert abs(th[j] - tho[j]) <= 1e-3 * abs(tho[j]), (i, j, th[j], tho[j])


def test_slq_llama_three_term_recurrence():
    cfg = dict(model=si._llama(2, 32, 2, 48, 61, 12), batch=2, seq=12, tokens="zipf")
    _slq_case(cfg, 20, 1, "none", n_early=6)


def test_slq_bf16_parameters_and_bf16_basis():
    cfg = dict(model=si._gpt(2, 64, 2, 128, 211, 24), batch=2, seq=24, tokens="zipf")
    _slq_case(cfg, 30, 1, "full", n_early=2, dtype="bf16", basis="bf16", rtol_early=3e-2)


def test_lanczos_step_matches_slq_and_state_errors():
    import paper_2505_11564_amd as hf
    cfg = si.CONFIGS["mlp_tiny"]
    model = cfg["model"]
    p, (x, y) = si.make_params(model), si.make_batch(cfg)
    n = om.num_params(model)
    ctx = hf.Context(model, 256, 8)
    pd, xd, yd, z = _dev(p), _dev(x), _dev(y), _dev(si.make_probe(n, 0))
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_lanczos_step(pd, xd, yd, 256, 1)
    assert e.value.code == hf.binding.HF_ESTATE
    ctx.hf_lanczos_init(z, "full")
    steps = [ctx.hf_lanczos_step(pd, xd, yd, 256, 1)[:2] for _ in range(8)]
    assert ctx.hf_lanczos_iterations() == 8
    with pytest.raises(hf.HessformerError) as e:           # basis is full
        ctx.hf_lanczos_step(pd, xd, yd, 256, 1)
    assert e.value.code == hf.binding.HF_ESHAPE
    res = ctx.hf_slq(pd, xd, yd, 256, 1, z, 1, 8, "full")
    np.testing.assert_allclose(res["alpha"][0], [s[0] for s in steps], rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose(res["beta"][0], [s[1] for s in steps], rtol=1e-5, atol=1e-7)
    with pytest.raises(hf.HessformerError) as e:
        ctx.hf_slq(pd, xd, yd, 256, 1, z, 1, 9, "full")
    assert e.value.code == hf.binding.HF_ESHAPE
    ctx.close()


def _continue_update_only(ctx, d_dev, steps):
    import torch
    q = torch.empty(ctx.n, device="cuda")
    al, be = [], []
    for _ in range(steps):
        ctx.hf_lanczos_get_vector(0, q)
        r = (d_dev * q).contiguous()
        a, b, _ = ctx.hf_lanczos_update(r, 0.0)
        al.append(a); be.append(b)
    return al, be


@pytest.mark.parametrize("reorth,basis,dtype", [("none", "none", "f32"), ("full", "f32", "f32"), ("full", "bf16", "f32"),
                                                 ("full", "f32", "bf16")])
def test_state_export_import_continues_the_same_iteration(reorth, basis, dtype):
    # A run interrupted after 7 iterations, moved through the state image into a
    # fresh context and continued, yields the coefficients of the uninterrupted
    # run bit for bit (the vector kernels are deterministic).  A context with bf16 parameters
    # keeps bf16 copies of the rows of an fp32 basis, which the image does not hold: the import
    # rebuilds them.
    import torch
    import paper_2505_11564_amd as hf
    model = si._gpt(1, 40, 2, 72, 1001, 33)
    a_ctx = hf.Context(model, 1, 20, dtype, basis)
    n = a_ctx.n
    rng = np.random.default_rng(9)
    d_dev = _dev(rng.uniform(-2, 3, n).astype(np.float32))
    a_ctx.hf_lanczos_init(_dev(si.make_probe(n, 1)), reorth)
    first = _continue_update_only(a_ctx, d_dev, 7)
    nbytes = a_ctx.hf_lanczos_state_bytes()
    image = torch.empty(nbytes + 256, dtype=torch.uint8, device="cuda")
    a_ctx.hf_lanczos_export(image, nbytes)
    rest = _continue_update_only(a_ctx, d_dev, 9)
    a_ctx.close()
    b_ctx = hf.Context(model, 1, 20, dtype, basis)
    host_copy = image.cpu()                       # the image is plain memory: through the host and back
    image2 = host_copy.cuda()
    b_ctx.hf_lanczos_import(image2, nbytes)
    assert b_ctx.hf_lanczos_iterations() == 7
    resumed = _continue_update_only(b_ctx, d_dev, 9)
    assert resumed[0] == rest[0] and resumed[1] == rest[1]
    # against the oracle's uninterrupted run, first coefficients
    dv = d_dev.cpu().numpy().astype(np.float64)
    ao, bo, _ = olz.lanczos(lambda q: dv * q, si.make_probe(n, 1).astype(np.float64), 16, reorth)
    got_a = np.array(first[0] + resumed[0])
    tol = 2e-2 if basis == "bf16" else 1e-4
    np.testing.assert_allclose(got_a[:4], ao[:4], rtol=tol, atol=tol)
    b_ctx.close()


def test_state_image_errors():
    import torch
    import paper_2505_11564_amd as hf
    model = si._gpt(1, 40, 2, 72, 1001, 33)
    ctx = hf.Context(model, 1, 8, "f32", "f32")
    with pytest.raises(hf.HessformerError):
        ctx.hf_lanczos_state_bytes()              # nothing in progress
    ctx.hf_lanczos_init(_dev(si.make_probe(ctx.n, 0)), "full")
    nbytes = ctx.hf_lanczos_state_bytes()
    image = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(hf.HessformerError):
        ctx.hf_lanczos_export(image, nbytes - 1)  # too small
    ctx.hf_lanczos_export(image, nbytes)
    with pytest.raises(hf.HessformerError):
        ctx.hf_lanczos_import(image, 100)         # truncated
    other = hf.Context(si._gpt(1, 48, 2, 72, 1001, 33), 1, 8, "f32", "f32")
    with pytest.raises(hf.HessformerError):
        other.hf_lanczos_import(image, nbytes)    # another parameter count
    nobasis = hf.Context(model, 1, 8, "f32", "none")
    with pytest.raises(hf.HessformerError):
        nobasis.hf_lanczos_import(image, nbytes)  # the image holds a basis
    junk = torch.zeros(nbytes, dtype=torch.uint8, device="cuda")
    with pytest.raises(hf.HessformerError):
        ctx.hf_lanczos_import(junk, nbytes)       # not an image
    for c in (ctx, other, nobasis):
        c.close()
