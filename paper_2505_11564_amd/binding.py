"""ctypes binding of libhessformer_hip.so: same names as include/hessformer.h,
argument marshalling only.  Device buffers are torch tensors (PyTorch-ROCm is
used for device memory and streams, nothing else) or raw integer addresses.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libhessformer_hip.so")

HF_OK, HF_EBREAKDOWN = 0, 1
HF_EINVAL, HF_ENOMEM, HF_EDEVICE, HF_ESHAPE, HF_ESTATE = -1, -2, -3, -4, -5
HF_ARCH = {"mlp": 0, "gpt": 1, "llama": 2}
HF_DTYPE = {"f32": 0, "bf16": 1, "none": 2}
HF_REORTH = {"none": 0, "full": 1}
HF_ACT = {"gelu_erf": 0, "gelu_tanh": 1}
HF_ATTN = {"auto": 0, "streamed": 1, "stored": 2}
HF_PRIMAL = {"auto": 0, "pairs": 1, "single": 2}

EXPORTS = [
    "hf_desc_num_params", "hf_layout_count", "hf_layout_entry", "hf_tridiag_readout", "hf_version",
    "hf_create", "hf_destroy", "hf_num_params", "hf_workspace_bytes", "hf_last_error",
    "hf_hvp", "hf_lanczos_init", "hf_lanczos_step", "hf_lanczos_iterations", "hf_lanczos_get_vector",
    "hf_slq", "hf_lanczos_update",
    "hf_hvp_accumulate", "hf_hessian_column", "hf_column_stats", "hf_slq_density", "hf_slq_moments",
    "hf_lanczos_state_bytes", "hf_lanczos_export", "hf_lanczos_import", "hf_column_stats_noalloc",
]


class hf_model_desc(C.Structure):
    _fields_ = [("arch", C.c_int32), ("n_layer", C.c_int32), ("d_model", C.c_int32), ("n_head", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("max_seq", C.c_int32), ("mlp_in", C.c_int32),
                ("mlp_hidden", C.c_int32), ("mlp_out", C.c_int32), ("tie_embeddings", C.c_int32),
                ("norm_eps", C.c_float), ("rope_theta", C.c_float), ("param_dtype", C.c_int32),
                ("basis_dtype", C.c_int32), ("activation", C.c_int32), ("n_kv_head", C.c_int32),
                ("attention", C.c_int32), ("primal", C.c_int32)]


class HessformerError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"hessformer status {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Loads the shared library; raises if it has not been built (there is no
    fallback path: every step of the hot path runs in the HIP kernels)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2505_11564_amd.build` "
                          "(or __graft_entry__.build()) first")
    # PyTorch-ROCm bundles its own HIP runtime under the same soname as the
    # system one.  Import torch first so that the library binds to the runtime
    # that owns the tensors and streams it is handed; loading it first would
    # put two HIP runtimes in one process.
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, dp = C.c_void_p, C.c_int32, C.c_int64, C.POINTER(C.c_double)
    descp = C.POINTER(hf_model_desc)
    L.hf_desc_num_params.argtypes, L.hf_desc_num_params.restype = [descp], i64
    L.hf_layout_count.argtypes, L.hf_layout_count.restype = [descp], i32
    L.hf_layout_entry.argtypes = [descp, i32, C.c_char_p, i32, C.POINTER(i64), C.POINTER(i64)]
    L.hf_layout_entry.restype = i32
    L.hf_tridiag_readout.argtypes, L.hf_tridiag_readout.restype = [dp, dp, i32, dp, dp, dp], i32
    L.hf_version.argtypes, L.hf_version.restype = [], C.c_char_p
    L.hf_create.argtypes, L.hf_create.restype = [descp, i32, i32, i32, C.POINTER(vp)], i32
    L.hf_destroy.argtypes, L.hf_destroy.restype = [vp], None
    L.hf_num_params.argtypes, L.hf_num_params.restype = [vp], i64
    L.hf_workspace_bytes.argtypes, L.hf_workspace_bytes.restype = [vp], i64
    L.hf_last_error.argtypes, L.hf_last_error.restype = [vp], C.c_char_p
    L.hf_hvp.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, dp, vp]
    L.hf_hvp.restype = i32
    L.hf_lanczos_init.argtypes, L.hf_lanczos_init.restype = [vp, vp, i32, vp], i32
    L.hf_lanczos_step.argtypes = [vp, vp, vp, vp, i32, i32, C.c_double, dp, dp, vp]
    L.hf_lanczos_step.restype = i32
    L.hf_lanczos_iterations.argtypes, L.hf_lanczos_iterations.restype = [vp], i32
    L.hf_lanczos_get_vector.argtypes, L.hf_lanczos_get_vector.restype = [vp, i32, vp, vp], i32
    L.hf_slq.argtypes = [vp, vp, vp, vp, i32, i32, vp, i32, i32, i32, C.c_double, dp, dp, dp, dp,
                         C.POINTER(i32), vp]
    L.hf_slq.restype = i32
    L.hf_lanczos_update.argtypes = [vp, vp, C.c_double, dp, dp, vp]
    L.hf_lanczos_update.restype = i32
    L.hf_hvp_accumulate.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, dp, vp]
    L.hf_hvp_accumulate.restype = i32
    L.hf_hessian_column.argtypes = [vp, vp, vp, vp, i32, i32, i64, vp, dp, vp]
    L.hf_hessian_column.restype = i32
    L.hf_column_stats.argtypes = [vp, vp, i64, C.POINTER(C.c_float), i32, i32, C.POINTER(i64), C.POINTER(C.c_float),
                                  C.POINTER(i64), vp]
    L.hf_column_stats.restype = i32
    L.hf_column_stats_noalloc.argtypes = [vp, i64, C.POINTER(C.c_float), i32, i32, C.POINTER(i64), C.POINTER(C.c_float),
                                          C.POINTER(i64), vp]
    L.hf_column_stats_noalloc.restype = i32
    L.hf_slq_density.argtypes = [dp, dp, C.POINTER(i32), i32, i32, C.c_double, dp, i32, dp]
    L.hf_slq_density.restype = i32
    L.hf_slq_moments.argtypes = [dp, dp, C.POINTER(i32), i32, i32, i32, dp]
    L.hf_slq_moments.restype = i32
    L.hf_lanczos_state_bytes.argtypes, L.hf_lanczos_state_bytes.restype = [vp], i64
    L.hf_lanczos_export.argtypes, L.hf_lanczos_export.restype = [vp, vp, i64, vp], i32
    L.hf_lanczos_import.argtypes, L.hf_lanczos_import.restype = [vp, vp, i64, vp], i32
    _lib = L
    return L


def make_desc(model, param_dtype="f32", basis_dtype="f32"):
    d = hf_model_desc()
    d.arch = HF_ARCH[model["arch"]]
    for k in ("n_layer", "d_model", "n_head", "d_ff", "vocab", "max_seq", "mlp_in", "mlp_hidden", "mlp_out",
              "tie_embeddings"):
        setattr(d, k, int(model[k]))
    d.norm_eps = float(model["norm_eps"])
    d.rope_theta = float(model["rope_theta"])
    d.param_dtype = HF_DTYPE[param_dtype]
    d.basis_dtype = HF_DTYPE[basis_dtype]
    d.activation = HF_ACT[model.get("act", "gelu_erf")]
    d.n_kv_head = int(model.get("n_kv_head", 0) or 0) if model["arch"] == "llama" else 0
    d.attention = HF_ATTN[model.get("attention", "auto")]
    d.primal = HF_PRIMAL[model.get("primal", "auto")]
    return d


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


# ---- host-only helpers ------------------------------------------------------

def hf_version():
    return lib().hf_version().decode()


def hf_desc_num_params(desc):
    return int(lib().hf_desc_num_params(C.byref(desc)))


def hf_layout(desc):
    """[(name, offset, shape)] from hf_layout_count / hf_layout_entry."""
    L = lib()
    cnt = L.hf_layout_count(C.byref(desc))
    if cnt < 0:
        raise HessformerError(cnt, "invalid model description")
    out = []
    name = C.create_string_buffer(64)
    off = C.c_int64()
    shape = (C.c_int64 * 2)()
    for i in range(cnt):
        rc = L.hf_layout_entry(C.byref(desc), i, name, 64, C.byref(off), shape)
        if rc != HF_OK:
            raise HessformerError(rc, "hf_layout_entry")
        shp = (int(shape[0]),) if shape[1] == 0 else (int(shape[0]), int(shape[1]))
        out.append((name.value.decode(), int(off.value), shp))
    return out


def hf_tridiag_readout(alpha, beta, want_last_row=False):
    a = np.ascontiguousarray(alpha, dtype=np.float64)
    b = np.ascontiguousarray(beta, dtype=np.float64)
    k = len(a)
    if k > 1 and len(b) < k - 1:
        raise ValueError("beta needs at least k-1 entries")
    if len(b) == 0:
        b = np.zeros(1)
    ritz, w, last = np.empty(k), np.empty(k), np.empty(k)
    dp = C.POINTER(C.c_double)
    rc = lib().hf_tridiag_readout(a.ctypes.data_as(dp), b.ctypes.data_as(dp), k, ritz.ctypes.data_as(dp),
                                  w.ctypes.data_as(dp), last.ctypes.data_as(dp))
    if rc != HF_OK:
        raise HessformerError(rc, "hf_tridiag_readout")
    return (ritz, w, last) if want_last_row else (ritz, w)


def _slq_arrays(ritz, weights, m_eff):
    r = np.ascontiguousarray(np.atleast_2d(ritz), dtype=np.float64)
    w = np.ascontiguousarray(np.atleast_2d(weights), dtype=np.float64)
    if r.shape != w.shape:
        raise ValueError("ritz and weights must have the same shape")
    me = np.ascontiguousarray(m_eff, dtype=np.int32)
    if me.shape != (r.shape[0],):
        raise ValueError("m_eff needs one entry per probe")
    return r, w, me


def hf_slq_density(ritz, weights, m_eff, sigma, grid):
    r, w, me = _slq_arrays(ritz, weights, m_eff)
    g = np.ascontiguousarray(grid, dtype=np.float64)
    out = np.empty_like(g)
    dp = C.POINTER(C.c_double)
    rc = lib().hf_slq_density(r.ctypes.data_as(dp), w.ctypes.data_as(dp), me.ctypes.data_as(C.POINTER(C.c_int32)),
                              r.shape[0], r.shape[1], float(sigma), g.ctypes.data_as(dp), len(g), out.ctypes.data_as(dp))
    if rc != HF_OK:
        raise HessformerError(rc, "hf_slq_density")
    return out


def hf_slq_moments(ritz, weights, m_eff, n_moments):
    r, w, me = _slq_arrays(ritz, weights, m_eff)
    out = np.empty(n_moments)
    dp = C.POINTER(C.c_double)
    rc = lib().hf_slq_moments(r.ctypes.data_as(dp), w.ctypes.data_as(dp), me.ctypes.data_as(C.POINTER(C.c_int32)),
                              r.shape[0], r.shape[1], n_moments, out.ctypes.data_as(dp))
    if rc != HF_OK:
        raise HessformerError(rc, "hf_slq_moments")
    return out


def hf_column_stats_noalloc(h, n, thresholds, n_bins, stream=None):
    """Context-free column statistics on the library's static counters."""
    thr = np.ascontiguousarray(thresholds, dtype=np.float32)
    below = np.zeros(max(len(thr), 1), dtype=np.int64)
    hist = np.zeros(max(n_bins, 1), dtype=np.int64)
    mx = C.c_float(0.0)
    i64p = C.POINTER(C.c_int64)
    rc = lib().hf_column_stats_noalloc(_ptr(h), int(n), thr.ctypes.data_as(C.POINTER(C.c_float)), len(thr), n_bins,
                                       below.ctypes.data_as(i64p), C.byref(mx), hist.ctypes.data_as(i64p), _stream(stream))
    if rc != HF_OK:
        raise HessformerError(rc, lib().hf_last_error(None).decode())
    return below[:len(thr)], np.float32(mx.value), hist[:n_bins]


# ---- context ----------------------------------------------------------------

class Context:
    """Owns an hf_ctx*.  Methods mirror the C entry points one to one."""

    def __init__(self, model, max_batch, max_m=0, param_dtype="f32", basis_dtype="f32", device=0):
        self.L = lib()
        self.desc = make_desc(model, param_dtype, basis_dtype)
        self.h = C.c_void_p()
        rc = self.L.hf_create(C.byref(self.desc), device, max_batch, max_m, C.byref(self.h))
        if rc != HF_OK:
            self.h = C.c_void_p()
            raise HessformerError(rc, self.L.hf_last_error(None).decode())
        self.n = int(self.L.hf_num_params(self.h))
        self.max_m = max_m

    def close(self):
        h = getattr(self, "h", None)
        if h:
            self.h = None
            self.L.hf_destroy(h)

    __del__ = close

    def _check(self, rc, ok=(HF_OK,)):
        if rc not in ok:
            raise HessformerError(rc, self.L.hf_last_error(self.h).decode())
        return rc

    def workspace_bytes(self):
        return int(self.L.hf_workspace_bytes(self.h))

    def hf_hvp(self, params, inputs, labels, batch, seq, v, out, want_loss=True, stream=None):
        loss = C.c_double(float("nan"))
        rc = self.L.hf_hvp(self.h, _ptr(params), _ptr(inputs), _ptr(labels), batch, seq, _ptr(v), _ptr(out),
                           C.byref(loss) if want_loss else None, _stream(stream))
        self._check(rc)
        return loss.value

    def hf_hvp_accumulate(self, params, inputs, labels, n_samples, micro_batch, seq, v, out, stream=None):
        loss = C.c_double(float("nan"))
        self._check(self.L.hf_hvp_accumulate(self.h, _ptr(params), _ptr(inputs), _ptr(labels), n_samples, micro_batch,
                                             seq, _ptr(v), _ptr(out), C.byref(loss), _stream(stream)))
        return loss.value

    def hf_hessian_column(self, params, inputs, labels, batch, seq, index, column, stream=None):
        loss = C.c_double(float("nan"))
        self._check(self.L.hf_hessian_column(self.h, _ptr(params), _ptr(inputs), _ptr(labels), batch, seq, int(index),
                                             _ptr(column), C.byref(loss), _stream(stream)))
        return loss.value

    def hf_column_stats(self, h, n, thresholds, n_bins, stream=None):
        thr = np.ascontiguousarray(thresholds, dtype=np.float32)
        below = np.zeros(max(len(thr), 1), dtype=np.int64)
        hist = np.zeros(max(n_bins, 1), dtype=np.int64)
        mx = C.c_float(0.0)
        i64p = C.POINTER(C.c_int64)
        self._check(self.L.hf_column_stats(self.h, _ptr(h), int(n), thr.ctypes.data_as(C.POINTER(C.c_float)), len(thr),
                                           n_bins, below.ctypes.data_as(i64p), C.byref(mx), hist.ctypes.data_as(i64p),
                                           _stream(stream)))
        return below[:len(thr)], np.float32(mx.value), hist[:n_bins]

    def hf_lanczos_init(self, q0, reorth="none", stream=None):
        self._check(self.L.hf_lanczos_init(self.h, _ptr(q0), HF_REORTH[reorth], _stream(stream)))

    def hf_lanczos_step(self, params, inputs, labels, batch, seq, tol=0.0, stream=None):
        a, b = C.c_double(), C.c_double()
        rc = self.L.hf_lanczos_step(self.h, _ptr(params), _ptr(inputs), _ptr(labels), batch, seq, tol,
                                    C.byref(a), C.byref(b), _stream(stream))
        self._check(rc, (HF_OK, HF_EBREAKDOWN))
        return a.value, b.value, rc

    def hf_lanczos_update(self, r, tol=0.0, stream=None):
        a, b = C.c_double(), C.c_double()
        rc = self.L.hf_lanczos_update(self.h, _ptr(r), tol, C.byref(a), C.byref(b), _stream(stream))
        self._check(rc, (HF_OK, HF_EBREAKDOWN))
        return a.value, b.value, rc

    def hf_lanczos_state_bytes(self):
        b = int(self.L.hf_lanczos_state_bytes(self.h))
        if b < 0:
            raise HessformerError(b, "hf_lanczos_state_bytes: no iteration in progress")
        return b

    def hf_lanczos_export(self, state, capacity_bytes, stream=None):
        self._check(self.L.hf_lanczos_export(self.h, _ptr(state), int(capacity_bytes), _stream(stream)))

    def hf_lanczos_import(self, state, nbytes, stream=None):
        self._check(self.L.hf_lanczos_import(self.h, _ptr(state), int(nbytes), _stream(stream)))

    def hf_lanczos_iterations(self):
        return int(self.L.hf_lanczos_iterations(self.h))

    def hf_lanczos_get_vector(self, which, dst, stream=None):
        self._check(self.L.hf_lanczos_get_vector(self.h, which, _ptr(dst), _stream(stream)))

    def hf_slq(self, params, inputs, labels, batch, seq, probes, n_probes, m, reorth="none", tol=0.0, stream=None):
        dp = C.POINTER(C.c_double)
        alpha, beta = np.zeros((n_probes, m)), np.zeros((n_probes, m))
        ritz, w = np.zeros((n_probes, m)), np.zeros((n_probes, m))
        m_eff = np.zeros(n_probes, dtype=np.int32)
        rc = self.L.hf_slq(self.h, _ptr(params), _ptr(inputs), _ptr(labels), batch, seq, _ptr(probes), n_probes, m,
                           HF_REORTH[reorth], tol, alpha.ctypes.data_as(dp), beta.ctypes.data_as(dp),
                           ritz.ctypes.data_as(dp), w.ctypes.data_as(dp),
                           m_eff.ctypes.data_as(C.POINTER(C.c_int32)), _stream(stream))
        self._check(rc, (HF_OK, HF_EBREAKDOWN))
        return dict(alpha=alpha, beta=beta, ritz=ritz, weights=w, m_eff=m_eff, status=rc)
