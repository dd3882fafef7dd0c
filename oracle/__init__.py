"""numpy front end of the CPU oracle (test infrastructure only).

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import
this package.  It loads oracle/libflashoptim_oracle.so (built by oracle/build.py
from flashoptim_oracle.cpp) and does nothing but marshal numpy arrays into it.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        # FLASHOPTIM_ORACLE_LIB: an alternative build to load instead (the mutant test plants mistakes
        # in copies of the source and checks that the pins notice)
        path = os.environ.get("FLASHOPTIM_ORACLE_LIB") or _build.build(force=False)
        _lib = C.CDLL(path)
        _declare(_lib)
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _declare(L):
    i64, f32, vp, i32 = C.c_int64, C.c_float, C.c_void_p, C.c_int
    L.fo_oracle_bf16_rne.restype = C.c_uint16
    L.fo_oracle_bf16_rne.argtypes = [f32]
    L.fo_oracle_bf16_to_f32.restype = f32
    L.fo_oracle_bf16_to_f32.argtypes = [C.c_uint16]
    L.fo_oracle_fp16_rne.restype = C.c_uint16
    L.fo_oracle_fp16_rne.argtypes = [f32]
    L.fo_oracle_fp16_to_f32.restype = f32
    L.fo_oracle_fp16_to_f32.argtypes = [C.c_uint16]
    L.fo_oracle_half_ulp_log2.restype = i32
    L.fo_oracle_half_ulp_log2.argtypes = [C.c_uint16]
    for name in ("fo_oracle_bf16_rne_array", "fo_oracle_fp16_rne_array", "fo_oracle_fp16_to_f32_array"):
        getattr(L, name).restype = None
        getattr(L, name).argtypes = [vp, vp, i64]
    L.fo_oracle_split.restype = None
    L.fo_oracle_split.argtypes = [vp, vp, vp, i64, i32]
    L.fo_oracle_reconstruct.restype = None
    L.fo_oracle_reconstruct.argtypes = [vp, vp, vp, i64, i32]
    L.fo_oracle_split_directional.restype = None
    L.fo_oracle_split_directional.argtypes = [vp, vp, vp, i64, i32]
    L.fo_oracle_reconstruct_directional.restype = None
    L.fo_oracle_reconstruct_directional.argtypes = [vp, vp, vp, i64, i32]
    for name in ("fo_oracle_quantize_momentum", "fo_oracle_dequantize_momentum",
                 "fo_oracle_quantize_variance", "fo_oracle_dequantize_variance",
                 "fo_oracle_quantize_momentum_linear", "fo_oracle_dequantize_momentum_linear",
                 "fo_oracle_quantize_variance_linear", "fo_oracle_dequantize_variance_linear"):
        getattr(L, name).restype = None
        getattr(L, name).argtypes = [vp, vp, vp, i64]
    L.fo_oracle_adamw_step.restype = None
    L.fo_oracle_adamw_step.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp,
                                       f32, f32, f32, f32, f32, i64, i32, i32, i32]
    L.fo_oracle_sgd_step.restype = None
    L.fo_oracle_sgd_step.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, i32, i32, i32]
    L.fo_oracle_lion_step.restype = None
    L.fo_oracle_lion_step.argtypes = [i64, vp, vp, vp, vp, vp, vp, vp, f32, f32, f32, f32, i32, i32, i32]
    L.fo_oracle_state_bytes.restype = i64
    L.fo_oracle_state_bytes.argtypes = [i64, i32]
    L.fo_oracle_checkpoint_size.restype = i64
    L.fo_oracle_checkpoint_size.argtypes = [i32, vp, i64]
    L.fo_oracle_checkpoint_pack.restype = i32
    L.fo_oracle_checkpoint_pack.argtypes = [i32, i64, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64]
    L.fo_oracle_checkpoint_unpack.restype = i32
    L.fo_oracle_checkpoint_unpack.argtypes = [i32, vp, i64, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    L.fo_oracle_split_sweep.restype = None
    L.fo_oracle_split_sweep.argtypes = [C.c_uint64, C.c_uint64, i32, vp, vp, i32]
    L.fo_oracle_split_sweep_ex.restype = None
    L.fo_oracle_split_sweep_ex.argtypes = [C.c_uint64, C.c_uint64, i32, i32, vp, vp, vp, vp, i32]
    L.fo_oracle_max_threads.restype = i32
    L.fo_oracle_max_threads.argtypes = []


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


KIND = {"adamw": 0, "sgd": 1, "lion": 2}
GROUP = 32


def n_groups(n):
    return (int(n) + GROUP - 1) // GROUP


def max_threads():
    return int(lib().fo_oracle_max_threads())


# ------------------------------------------------------------------ formats --

def bf16_rne(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().fo_oracle_bf16_rne_array(_p(x), _p(out), x.size)
    return out


def bf16_to_f32(b):
    b = _c(b, np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def fp16_rne(x):
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    lib().fo_oracle_fp16_rne_array(_p(x), _p(out), x.size)
    return out


def fp16_to_f32(h):
    h = _c(h, np.uint16)
    out = np.empty(h.shape, np.float32)
    lib().fo_oracle_fp16_to_f32_array(_p(h), _p(out), h.size)
    return out


def half_ulp_log2(thp_bits):
    return int(lib().fo_oracle_half_ulp_log2(int(thp_bits)))


# ------------------------------------------------------------------- codecs --

def split(theta, N=127, directional=False):
    """C(theta) -> (theta' as uint16 BF16 bits, rho as int8 for N=127 else int16).  directional=True: the
    alternative reading of ULP(theta') that exists for the Section 4.4 experiment only."""
    theta = _c(theta, np.float32)
    thp = np.empty(theta.shape, np.uint16)
    rho = np.empty(theta.shape, np.int16)
    fn = lib().fo_oracle_split_directional if directional else lib().fo_oracle_split
    fn(_p(theta), _p(thp), _p(rho), theta.size, int(N))
    return thp, (rho.astype(np.int8) if N == 127 else rho)


def reconstruct(thp, rho, N=127, directional=False):
    thp = _c(thp, np.uint16)
    rho16 = _c(rho, np.int16)
    out = np.empty(thp.shape, np.float32)
    fn = lib().fo_oracle_reconstruct_directional if directional else lib().fo_oracle_reconstruct
    fn(_p(thp), _p(rho16), _p(out), thp.size, int(N))
    return out


def _suffix(linear):
    return "_linear" if linear else ""


def quantize_momentum(m, linear=False):
    """Q_m (companded; linear=True: plain absmax quantisation without the compander)."""
    m = _c(m, np.float32).ravel()
    q = np.empty(m.size, np.int8)
    s = np.empty(n_groups(m.size), np.uint16)
    getattr(lib(), "fo_oracle_quantize_momentum" + _suffix(linear))(_p(m), _p(q), _p(s), m.size)
    return q, s


def dequantize_momentum(q, s, linear=False):
    q = _c(q, np.int8).ravel()
    s = _c(s, np.uint16).ravel()
    assert s.size == n_groups(q.size)
    out = np.empty(q.size, np.float32)
    getattr(lib(), "fo_oracle_dequantize_momentum" + _suffix(linear))(_p(q), _p(s), _p(out), q.size)
    return out


def quantize_variance(v, linear=False):
    v = _c(v, np.float32).ravel()
    q = np.empty(v.size, np.uint8)
    s = np.empty(n_groups(v.size), np.uint16)
    getattr(lib(), "fo_oracle_quantize_variance" + _suffix(linear))(_p(v), _p(q), _p(s), v.size)
    return q, s


def dequantize_variance(q, s, linear=False):
    q = _c(q, np.uint8).ravel()
    s = _c(s, np.uint16).ravel()
    assert s.size == n_groups(q.size)
    out = np.empty(q.size, np.float32)
    getattr(lib(), "fo_oracle_dequantize_variance" + _suffix(linear))(_p(q), _p(s), _p(out), q.size)
    return out


def nmse(x, x_hat):
    """Normalised mean squared error sum((x_hat - x)^2) / sum(x^2), in double (Section 4.5)."""
    x = np.asarray(x, np.float64).ravel()
    d = np.asarray(x_hat, np.float64).ravel() - x
    return float(np.dot(d, d) / np.dot(x, x))


# -------------------------------------------------------------------- state --

class TensorState:
    """Optimizer-side state of one flattened tensor, as the oracle holds it.

    Compressed form (the paper's layout): thp (uint16 BF16 bits), rho (int8),
    mq (int8) + ms (uint16 FP16 bits per group), and for AdamW vq (uint8) + vs.
    With split_weights=False theta32 replaces thp/rho; with quantize_states=False
    m32 (and v32) replace the code/scale arrays (the paper's two ablations).
    """

    def __init__(self, theta0, kind, split_weights=True, quantize_states=True):
        theta0 = _c(theta0, np.float32).ravel()
        n = theta0.size
        self.n, self.kind = n, kind
        self.split_weights, self.quantize_states = split_weights, quantize_states
        has_v = kind == "adamw"
        self.thp = self.rho = self.theta32 = None
        self.mq = self.ms = self.vq = self.vs = self.m32 = self.v32 = None
        if split_weights:
            self.thp, self.rho = split(theta0)          # theta'_0, rho_0 <- C(theta_0)
        else:
            self.theta32 = theta0.copy()
        if quantize_states:
            # Q_m(0), Q_v(0): all-zero codes and scales
            self.mq = np.zeros(n, np.int8)
            self.ms = np.zeros(n_groups(n), np.uint16)
            if has_v:
                self.vq = np.zeros(n, np.uint8)
                self.vs = np.zeros(n_groups(n), np.uint16)
        else:
            self.m32 = np.zeros(n, np.float32)
            if has_v:
                self.v32 = np.zeros(n, np.float32)

    def master(self):
        """FP32 master weight as the next step will see it."""
        return reconstruct(self.thp, self.rho) if self.split_weights else self.theta32.copy()

    def copy(self):
        import copy
        return copy.deepcopy(self)


def adamw_step(st, grad_bf16, lr, wd, beta1, beta2, eps, t, nthreads=0):
    g = _c(grad_bf16, np.uint16).ravel()
    assert g.size == st.n and st.kind == "adamw" and t >= 1
    lib().fo_oracle_adamw_step(st.n, _p(st.thp), _p(st.rho), _p(st.theta32), _p(g),
                               _p(st.mq), _p(st.ms), _p(st.vq), _p(st.vs), _p(st.m32), _p(st.v32),
                               lr, wd, beta1, beta2, eps, int(t),
                               int(st.split_weights), int(st.quantize_states), int(nthreads))


def sgd_step(st, grad_bf16, lr, wd, momentum, nthreads=0):
    g = _c(grad_bf16, np.uint16).ravel()
    assert g.size == st.n and st.kind == "sgd"
    lib().fo_oracle_sgd_step(st.n, _p(st.thp), _p(st.rho), _p(st.theta32), _p(g),
                             _p(st.mq), _p(st.ms), _p(st.m32), lr, wd, momentum,
                             int(st.split_weights), int(st.quantize_states), int(nthreads))


def lion_step(st, grad_bf16, lr, wd, beta1, beta2, nthreads=0):
    g = _c(grad_bf16, np.uint16).ravel()
    assert g.size == st.n and st.kind == "lion"
    lib().fo_oracle_lion_step(st.n, _p(st.thp), _p(st.rho), _p(st.theta32), _p(g),
                              _p(st.mq), _p(st.ms), _p(st.m32), lr, wd, beta1, beta2,
                              int(st.split_weights), int(st.quantize_states), int(nthreads))


# --------------------------------------------------------------- checkpoint --

def state_bytes(n, has_variance):
    return int(lib().fo_oracle_state_bytes(int(n), int(bool(has_variance))))


def checkpoint_size(kind, numels):
    nm = np.asarray(numels, np.int64)
    return int(lib().fo_oracle_checkpoint_size(KIND[kind], _p(nm), nm.size))


def _ptr_array(arrs):
    out = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        out[i] = None if a is None else a.ctypes.data
    return out


def checkpoint_pack(kind, states, step):
    nm = np.asarray([s.n for s in states], np.int64)
    total = checkpoint_size(kind, nm)
    blob = np.empty(total, np.uint8)
    rc = lib().fo_oracle_checkpoint_pack(
        KIND[kind], nm.size, _p(nm),
        _ptr_array([s.thp for s in states]), _ptr_array([s.rho for s in states]),
        _ptr_array([s.mq for s in states]), _ptr_array([s.ms for s in states]),
        _ptr_array([s.vq for s in states]), _ptr_array([s.vs for s in states]),
        int(step), _p(blob), total)
    if rc != 0:
        raise ValueError("oracle checkpoint_pack failed")
    return blob


def checkpoint_unpack(kind, blob, states):
    """Fill the (pre-shaped) states from blob; returns the stored step."""
    blob = _c(blob, np.uint8)
    nm = np.asarray([s.n for s in states], np.int64)
    step = C.c_int64(0)
    rc = lib().fo_oracle_checkpoint_unpack(
        KIND[kind], _p(blob), blob.size, nm.size, _p(nm),
        _ptr_array([s.thp for s in states]), _ptr_array([s.rho for s in states]),
        _ptr_array([s.mq for s in states]), _ptr_array([s.ms for s in states]),
        _ptr_array([s.vq for s in states]), _ptr_array([s.vs for s in states]),
        C.addressof(step))
    if rc != 0:
        raise ValueError("oracle checkpoint_unpack rejected the blob")
    return int(step.value)


# -------------------------------------------------------------------- sweep --

def split_sweep(first=0, stride=1, N=127, nthreads=0, directional=False):
    out = np.zeros(9, np.float64)
    mean_rel = np.zeros(256, np.float64)
    exact_by = np.zeros(256, np.float64)
    count_by = np.zeros(256, np.float64)
    lib().fo_oracle_split_sweep_ex(int(first), int(stride), int(N), int(bool(directional)), _p(out), _p(mean_rel),
                                   _p(exact_by), _p(count_by), int(nthreads))
    keys = ["measured", "skipped", "interval_violations", "max_err_over_bound", "max_rel_err",
            "bit_exact", "rho_out_of_range", "tie_rule_differs", "not_nearest"]
    d = {k: float(v) for k, v in zip(keys, out)}
    d["mean_rel_by_exponent"] = mean_rel
    d["bit_exact_by_exponent"] = exact_by
    d["count_by_exponent"] = count_by
    return d
