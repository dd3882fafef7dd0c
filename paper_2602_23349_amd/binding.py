"""ctypes binding of include/flashoptim.h: argument marshalling only.

Every function here has the name of the C entry point it calls (without the
`flashoptim_` prefix) and does nothing but turn torch tensors into device pointers.
torch is used for device memory and streams only.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libflashoptim.so")
_lib = None

KIND = {"adamw": 0, "sgd": 1, "lion": 2}

EXPORTED_SYMBOLS = [
    "flashoptim_adamw_step", "flashoptim_adamw_step_exact", "flashoptim_sgd_step", "flashoptim_lion_step",
    "flashoptim_split_weights", "flashoptim_reconstruct_weights",
    "flashoptim_quantize_momentum", "flashoptim_dequantize_momentum",
    "flashoptim_quantize_variance", "flashoptim_dequantize_variance",
    "flashoptim_checkpoint_size", "flashoptim_checkpoint_pack", "flashoptim_checkpoint_unpack",
    "flashoptim_strerror", "flashoptim_last_hip_error", "flashoptim_release_cache", "flashoptim_version",
    "flashoptim_faithful_rounding_stats", "flashoptim_short_sqrt_state", "flashoptim_clock_monitor",
    "flashoptim_step_launch_count",
    "flashoptim_selftest", "flashoptim_split_weights_i16", "flashoptim_reconstruct_weights_i16",
    "flashoptim_reconstruction_sweep", "flashoptim_reconstruction_sweep_ex",
    "flashoptim_adamw_step_ex", "flashoptim_sgd_step_ex", "flashoptim_lion_step_ex",
    "flashoptim_quantize_state", "flashoptim_dequantize_state", "flashoptim_quantization_nmse",
    "flashoptim_compress_state", "flashoptim_decompress_state", "flashoptim_stream_probe",
    "flashoptim_adamw_step_noalloc", "flashoptim_shard_range",
]


class FlashOptimError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        msg = strerror(status)
        if status == -4:
            msg += f" (hipError_t {load_library().flashoptim_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


class _Tensor(C.Structure):
    _fields_ = [("param", C.c_void_p), ("rho", C.c_void_p), ("grad", C.c_void_p),
                ("m_q", C.c_void_p), ("m_scale", C.c_void_p), ("v_q", C.c_void_p), ("v_scale", C.c_void_p),
                ("numel", C.c_int64), ("lr", C.c_float), ("weight_decay", C.c_float)]


class _TensorEx(C.Structure):
    _fields_ = [("t", _Tensor), ("theta", C.c_void_p), ("m", C.c_void_p), ("v", C.c_void_p)]


SPLIT_WEIGHTS, QUANTIZE_STATES = 1, 2


class _AdamWHp(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float), ("step", C.c_int64)]


class _SgdHp(C.Structure):
    _fields_ = [("momentum", C.c_float)]


class _LionHp(C.Structure):
    _fields_ = [("beta1", C.c_float), ("beta2", C.c_float)]


def library_path():
    return _LIB_PATH


def load_library():
    """Loads the in-tree HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} is missing: build it with `python paper_2602_23349_amd/build.py`")
    L = C.CDLL(_LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int
    L.flashoptim_adamw_step.argtypes = [C.POINTER(_Tensor), i64, C.POINTER(_AdamWHp), vp]
    L.flashoptim_adamw_step_exact.argtypes = [C.POINTER(_Tensor), i64, C.POINTER(_AdamWHp), vp]
    L.flashoptim_adamw_step_noalloc.argtypes = [C.POINTER(_Tensor), i64, C.POINTER(_AdamWHp), vp]
    L.flashoptim_shard_range.argtypes = [i64, i64, i64, C.POINTER(i64), C.POINTER(i64)]
    L.flashoptim_sgd_step.argtypes = [C.POINTER(_Tensor), i64, C.POINTER(_SgdHp), vp]
    L.flashoptim_lion_step.argtypes = [C.POINTER(_Tensor), i64, C.POINTER(_LionHp), vp]
    L.flashoptim_adamw_step_ex.argtypes = [C.POINTER(_TensorEx), i64, C.POINTER(_AdamWHp), C.c_uint, vp]
    L.flashoptim_sgd_step_ex.argtypes = [C.POINTER(_TensorEx), i64, C.POINTER(_SgdHp), C.c_uint, vp]
    L.flashoptim_lion_step_ex.argtypes = [C.POINTER(_TensorEx), i64, C.POINTER(_LionHp), C.c_uint, vp]
    L.flashoptim_reconstruction_sweep.argtypes = [i32, C.c_uint64, C.c_uint64, C.POINTER(C.c_double), vp]
    L.flashoptim_reconstruction_sweep_ex.argtypes = [i32, i32, C.c_uint64, C.c_uint64, C.POINTER(C.c_double), vp]
    for name in ("flashoptim_split_weights", "flashoptim_reconstruct_weights", "flashoptim_split_weights_i16",
                 "flashoptim_reconstruct_weights_i16", "flashoptim_quantize_momentum",
                 "flashoptim_dequantize_momentum", "flashoptim_quantize_variance", "flashoptim_dequantize_variance"):
        getattr(L, name).argtypes = [vp, vp, vp, i64, vp]
    L.flashoptim_compress_state.argtypes = [i32, C.POINTER(_TensorEx), i64, vp]
    L.flashoptim_decompress_state.argtypes = [i32, C.POINTER(_TensorEx), i64, vp]
    L.flashoptim_stream_probe.argtypes = [i32, C.POINTER(_Tensor), i64, vp]
    L.flashoptim_quantize_state.argtypes = [i32, i32, vp, vp, vp, i64, vp]
    L.flashoptim_dequantize_state.argtypes = [i32, i32, vp, vp, vp, i64, vp]
    L.flashoptim_quantization_nmse.argtypes = [i32, i32, vp, i64, C.POINTER(C.c_double), vp]
    L.flashoptim_checkpoint_size.argtypes = [i32, C.POINTER(i64), i64]
    L.flashoptim_checkpoint_size.restype = i64
    L.flashoptim_step_launch_count.argtypes = [i32, C.POINTER(i64), i64]
    L.flashoptim_step_launch_count.restype = i64
    L.flashoptim_checkpoint_pack.argtypes = [i32, C.POINTER(_Tensor), i64, i64, vp, i64, vp]
    L.flashoptim_checkpoint_unpack.argtypes = [i32, vp, i64, C.POINTER(_Tensor), i64, C.POINTER(i64), vp]
    L.flashoptim_selftest.argtypes = [C.POINTER(i64), C.POINTER(i64), vp]
    L.flashoptim_faithful_rounding_stats.argtypes = [C.POINTER(i64), vp]
    L.flashoptim_clock_monitor.argtypes = [C.POINTER(C.c_uint64), i64, C.c_double, C.POINTER(C.c_double), vp]
    L.flashoptim_strerror.argtypes = [i32]
    L.flashoptim_strerror.restype = C.c_char_p
    for name in EXPORTED_SYMBOLS:
        if name not in ("flashoptim_checkpoint_size", "flashoptim_strerror"):
            getattr(L, name).restype = i32
    _lib = L
    return L


def _ptr(t):
    return None if t is None else t.data_ptr()


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _check(status, where):
    if status != 0:
        raise FlashOptimError(status, where)


class ParamBuffers:
    """Device buffers of one parameter (allocation only).  split_weights / quantize_states choose the
    compressed layout (default) or the FP32 arrays of the ablation variants for each half."""

    def __init__(self, numel, kind, device="cuda", with_grad=True, split_weights=True, quantize_states=True):
        ng = (numel + 31) // 32
        has_v = kind == "adamw"
        self.numel, self.kind = int(numel), kind
        self.split_weights, self.quantize_states = split_weights, quantize_states
        z = lambda n, dt: torch.zeros(n, dtype=dt, device=device)
        self.param = z(numel, torch.bfloat16) if split_weights else None
        self.rho = z(numel, torch.int8) if split_weights else None
        self.theta = None if split_weights else z(numel, torch.float32)
        self.grad = z(numel, torch.bfloat16) if with_grad else None
        self.m_q = z(numel, torch.int8) if quantize_states else None
        self.m_scale = z(ng, torch.float16) if quantize_states else None
        self.v_q = z(numel, torch.uint8) if (quantize_states and has_v) else None
        self.v_scale = z(ng, torch.float16) if (quantize_states and has_v) else None
        self.m = None if quantize_states else z(numel, torch.float32)
        self.v = z(numel, torch.float32) if (not quantize_states and has_v) else None
        self.lr, self.weight_decay = 0.0, 0.0

    @property
    def flags(self):
        return (SPLIT_WEIGHTS if self.split_weights else 0) | (QUANTIZE_STATES if self.quantize_states else 0)

    def shard(self, begin, length):
        """The same buffers restricted to elements [begin, begin + length): views (pointer offsets), no copy.
        begin must be a multiple of 256 (see flashoptim_shard_range)."""
        assert begin % 256 == 0 and 0 <= begin and begin + length <= self.numel
        out = ParamBuffers.__new__(ParamBuffers)
        out.numel, out.kind = int(length), self.kind
        out.split_weights, out.quantize_states = self.split_weights, self.quantize_states
        el = lambda t: None if t is None else t[begin:begin + length]
        gr = lambda t: None if t is None else t[begin // 32:begin // 32 + (length + 31) // 32]
        out.param, out.rho, out.theta, out.grad = el(self.param), el(self.rho), el(self.theta), el(self.grad)
        out.m_q, out.v_q, out.m, out.v = el(self.m_q), el(self.v_q), el(self.m), el(self.v)
        out.m_scale, out.v_scale = gr(self.m_scale), gr(self.v_scale)
        out.lr, out.weight_decay = self.lr, self.weight_decay
        return out


class TensorList:
    """A host array of flashoptim_tensor descriptors, built once and reused across steps."""

    def __init__(self, buffers):
        self.buffers = list(buffers)
        self.n = len(self.buffers)
        self.array = (_Tensor * max(self.n, 1))()
        for i, b in enumerate(self.buffers):
            d = self.array[i]
            d.param, d.rho, d.grad = _ptr(b.param), _ptr(b.rho), _ptr(b.grad)
            d.m_q, d.m_scale, d.v_q, d.v_scale = _ptr(b.m_q), _ptr(b.m_scale), _ptr(b.v_q), _ptr(b.v_scale)
            d.numel, d.lr, d.weight_decay = b.numel, b.lr, b.weight_decay

    def set_hyper(self, i, lr=None, weight_decay=None):
        if lr is not None:
            self.array[i].lr = lr
        if weight_decay is not None:
            self.array[i].weight_decay = weight_decay

    def set_grad(self, i, grad):
        self.array[i].grad = _ptr(grad)

    def slice(self, i):
        """A one-element list viewing tensor i (for per-tensor, gradient-release style calls)."""
        out = TensorList.__new__(TensorList)
        out.buffers, out.n = [self.buffers[i]], 1
        out.array = (_Tensor * 1)()
        C.memmove(out.array, C.byref(self.array[i]), C.sizeof(_Tensor))
        return out


class TensorListEx:
    """Host array of flashoptim_tensor_ex descriptors (ablation and conversion entry points)."""

    def __init__(self, buffers, check_flags=True):
        self.buffers = list(buffers)
        self.n = len(self.buffers)
        self.flags = self.buffers[0].flags if self.buffers else 3
        assert not check_flags or all(b.flags == self.flags for b in self.buffers)
        self.array = (_TensorEx * max(self.n, 1))()
        for i, b in enumerate(self.buffers):
            d = self.array[i]
            d.t.param, d.t.rho, d.t.grad = _ptr(b.param), _ptr(b.rho), _ptr(b.grad)
            d.t.m_q, d.t.m_scale, d.t.v_q, d.t.v_scale = _ptr(b.m_q), _ptr(b.m_scale), _ptr(b.v_q), _ptr(b.v_scale)
            d.t.numel, d.t.lr, d.t.weight_decay = b.numel, b.lr, b.weight_decay
            d.theta, d.m, d.v = _ptr(b.theta), _ptr(b.m), _ptr(b.v)


def _as_list_ex(tensors):
    return tensors if isinstance(tensors, TensorListEx) else TensorListEx(tensors)


def adamw_step_ex(tensors, beta1, beta2, eps, step, flags=None, stream=None):
    tl = _as_list_ex(tensors)
    hp = _AdamWHp(beta1, beta2, eps, int(step))
    _check(load_library().flashoptim_adamw_step_ex(tl.array, tl.n, C.byref(hp), tl.flags if flags is None else flags,
                                                   _stream(stream)), "flashoptim_adamw_step_ex")


def sgd_step_ex(tensors, momentum, flags=None, stream=None):
    tl = _as_list_ex(tensors)
    hp = _SgdHp(momentum)
    _check(load_library().flashoptim_sgd_step_ex(tl.array, tl.n, C.byref(hp), tl.flags if flags is None else flags,
                                                 _stream(stream)), "flashoptim_sgd_step_ex")


def lion_step_ex(tensors, beta1, beta2, flags=None, stream=None):
    tl = _as_list_ex(tensors)
    hp = _LionHp(beta1, beta2)
    _check(load_library().flashoptim_lion_step_ex(tl.array, tl.n, C.byref(hp), tl.flags if flags is None else flags,
                                                  _stream(stream)), "flashoptim_lion_step_ex")


def compress_state(kind, tensors, stream=None):
    tl = tensors if isinstance(tensors, TensorListEx) else TensorListEx(tensors, check_flags=False)
    _check(load_library().flashoptim_compress_state(KIND[kind], tl.array, tl.n, _stream(stream)),
           "flashoptim_compress_state")


def decompress_state(kind, tensors, stream=None):
    tl = tensors if isinstance(tensors, TensorListEx) else TensorListEx(tensors, check_flags=False)
    _check(load_library().flashoptim_decompress_state(KIND[kind], tl.array, tl.n, _stream(stream)),
           "flashoptim_decompress_state")


def _as_list(tensors):
    return tensors if isinstance(tensors, TensorList) else TensorList(tensors)


def adamw_step(tensors, beta1, beta2, eps, step, stream=None):
    tl = _as_list(tensors)
    hp = _AdamWHp(beta1, beta2, eps, int(step))
    _check(load_library().flashoptim_adamw_step(tl.array, tl.n, C.byref(hp), _stream(stream)), "flashoptim_adamw_step")


def adamw_step_exact(tensors, beta1, beta2, eps, step, stream=None):
    tl = _as_list(tensors)
    hp = _AdamWHp(beta1, beta2, eps, int(step))
    _check(load_library().flashoptim_adamw_step_exact(tl.array, tl.n, C.byref(hp), _stream(stream)),
           "flashoptim_adamw_step_exact")


def adamw_step_noalloc(tensors, beta1, beta2, eps, step, stream=None):
    tl = _as_list(tensors)
    hp = _AdamWHp(beta1, beta2, eps, int(step))
    _check(load_library().flashoptim_adamw_step_noalloc(tl.array, tl.n, C.byref(hp), _stream(stream)),
           "flashoptim_adamw_step_noalloc")


def shard_range(numel, world, rank):
    """(begin, len) of `rank`'s shard of a flat tensor cut on multiples of 256 elements."""
    begin, length = C.c_int64(0), C.c_int64(0)
    _check(load_library().flashoptim_shard_range(int(numel), int(world), int(rank), C.byref(begin), C.byref(length)),
           "flashoptim_shard_range")
    return int(begin.value), int(length.value)


def sgd_step(tensors, momentum, stream=None):
    tl = _as_list(tensors)
    hp = _SgdHp(momentum)
    _check(load_library().flashoptim_sgd_step(tl.array, tl.n, C.byref(hp), _stream(stream)), "flashoptim_sgd_step")


def lion_step(tensors, beta1, beta2, stream=None):
    tl = _as_list(tensors)
    hp = _LionHp(beta1, beta2)
    _check(load_library().flashoptim_lion_step(tl.array, tl.n, C.byref(hp), _stream(stream)), "flashoptim_lion_step")


def stream_probe(kind, tensors, stream=None):
    """Moves the bytes of one step of `kind` over the list with no arithmetic (state unchanged)."""
    tl = _as_list(tensors)
    _check(load_library().flashoptim_stream_probe(KIND[kind], tl.array, tl.n, _stream(stream)), "flashoptim_stream_probe")


def split_weights(theta, param_bf16, rho, stream=None):
    n = theta.numel()
    _check(load_library().flashoptim_split_weights(_ptr(theta), _ptr(param_bf16), _ptr(rho), n, _stream(stream)),
           "flashoptim_split_weights")


def reconstruct_weights(param_bf16, rho, theta, stream=None):
    n = param_bf16.numel()
    _check(load_library().flashoptim_reconstruct_weights(_ptr(param_bf16), _ptr(rho), _ptr(theta), n, _stream(stream)),
           "flashoptim_reconstruct_weights")


def split_weights_i16(theta, param_bf16, rho, stream=None):
    _check(load_library().flashoptim_split_weights_i16(_ptr(theta), _ptr(param_bf16), _ptr(rho), theta.numel(),
                                                       _stream(stream)), "flashoptim_split_weights_i16")


def reconstruct_weights_i16(param_bf16, rho, theta, stream=None):
    _check(load_library().flashoptim_reconstruct_weights_i16(_ptr(param_bf16), _ptr(rho), _ptr(theta),
                                                             param_bf16.numel(), _stream(stream)),
           "flashoptim_reconstruct_weights_i16")


def reconstruction_sweep(correction_bits, first=0, stride=1, stream=None):
    """Returns the 520 statistics of flashoptim_reconstruction_sweep as a list of floats."""
    stats = (C.c_double * 520)()
    _check(load_library().flashoptim_reconstruction_sweep(int(correction_bits), int(first), int(stride), stats,
                                                          _stream(stream)), "flashoptim_reconstruction_sweep")
    return list(stats)


def reconstruction_sweep_ex(correction_bits, ulp_reading, first=0, stride=1, stream=None):
    """Returns the 776 statistics of flashoptim_reconstruction_sweep_ex (ulp_reading 0 literal, 1 directional)."""
    stats = (C.c_double * 776)()
    _check(load_library().flashoptim_reconstruction_sweep_ex(int(correction_bits), int(ulp_reading), int(first),
                                                             int(stride), stats, _stream(stream)),
           "flashoptim_reconstruction_sweep_ex")
    return list(stats)


def quantize_momentum(m, q, scale, stream=None):
    _check(load_library().flashoptim_quantize_momentum(_ptr(m), _ptr(q), _ptr(scale), m.numel(), _stream(stream)),
           "flashoptim_quantize_momentum")


def dequantize_momentum(q, scale, m, stream=None):
    _check(load_library().flashoptim_dequantize_momentum(_ptr(q), _ptr(scale), _ptr(m), q.numel(), _stream(stream)),
           "flashoptim_dequantize_momentum")


def quantize_variance(v, q, scale, stream=None):
    _check(load_library().flashoptim_quantize_variance(_ptr(v), _ptr(q), _ptr(scale), v.numel(), _stream(stream)),
           "flashoptim_quantize_variance")


def dequantize_variance(q, scale, v, stream=None):
    _check(load_library().flashoptim_dequantize_variance(_ptr(q), _ptr(scale), _ptr(v), q.numel(), _stream(stream)),
           "flashoptim_dequantize_variance")


_STATE = {"momentum": 0, "variance": 1}


def quantize_state(state, linear, x, q, scale, stream=None):
    _check(load_library().flashoptim_quantize_state(_STATE[state], int(bool(linear)), _ptr(x), _ptr(q), _ptr(scale),
                                                    x.numel(), _stream(stream)), "flashoptim_quantize_state")


def dequantize_state(state, linear, q, scale, x, stream=None):
    _check(load_library().flashoptim_dequantize_state(_STATE[state], int(bool(linear)), _ptr(q), _ptr(scale), _ptr(x),
                                                      q.numel(), _stream(stream)), "flashoptim_dequantize_state")


def quantization_nmse(state, linear, x, stream=None):
    """Returns (sum of squared errors, sum of squares) of quantize -> dequantize over x."""
    sums = (C.c_double * 2)()
    _check(load_library().flashoptim_quantization_nmse(_STATE[state], int(bool(linear)), _ptr(x), x.numel(), sums,
                                                       _stream(stream)), "flashoptim_quantization_nmse")
    return float(sums[0]), float(sums[1])


def checkpoint_size(kind, numels):
    arr = (C.c_int64 * max(len(numels), 1))(*[int(x) for x in numels])
    r = load_library().flashoptim_checkpoint_size(KIND[kind], arr, len(numels))
    if r < 0:
        raise FlashOptimError(int(r), "flashoptim_checkpoint_size")
    return int(r)


def checkpoint_pack(kind, tensors, step, blob, stream=None):
    tl = _as_list(tensors)
    _check(load_library().flashoptim_checkpoint_pack(KIND[kind], tl.array, tl.n, int(step), _ptr(blob),
                                                     blob.numel() * blob.element_size(), _stream(stream)),
           "flashoptim_checkpoint_pack")


def checkpoint_unpack(kind, blob, tensors, stream=None):
    tl = _as_list(tensors)
    step = C.c_int64(0)
    _check(load_library().flashoptim_checkpoint_unpack(KIND[kind], _ptr(blob), blob.numel() * blob.element_size(),
                                                       tl.array, tl.n, C.byref(step), _stream(stream)),
           "flashoptim_checkpoint_unpack")
    return int(step.value)


def faithful_rounding_stats(stream=None):
    """(division operand pairs checked, quotients of the default AdamW step's division that are not the exactly
    rounded one)."""
    counts = (C.c_int64 * 2)()
    _check(load_library().flashoptim_faithful_rounding_stats(counts, _stream(stream)), "flashoptim_faithful_rounding_stats")
    return tuple(counts)


class ClockMonitor:
    """Samples the shader clock on a stream of its own while other work runs: start(), run the work, then
    ghz() waits for the monitor and returns one value per sample (numpy array)."""

    def __init__(self, n_samples=200, seconds_per_sample=1e-3, device="cuda"):
        self.n, self.dt = int(n_samples), float(seconds_per_sample)
        self.samples = torch.zeros(2 * self.n, dtype=torch.int64, device=device)
        self.stream = torch.cuda.Stream(device=device)
        self.tick_hz = C.c_double(0.0)

    def start(self):
        self.samples.zero_()
        torch.cuda.current_stream().synchronize()
        self.stream.wait_stream(torch.cuda.current_stream())
        _check(load_library().flashoptim_clock_monitor(C.cast(self.samples.data_ptr(), C.POINTER(C.c_uint64)), self.n,
                                                       self.dt, C.byref(self.tick_hz), _stream(self.stream)),
               "flashoptim_clock_monitor")

    def ghz(self):
        self.stream.synchronize()
        o = self.samples.cpu().numpy().reshape(self.n, 2).astype("float64")
        return o[:, 1] / o[:, 0] * self.tick_hz.value / 1e9


def short_sqrt_state():
    """0 not checked yet, 1 verified on this device, 2 not in use (check failed or switched off by the environment)."""
    return int(load_library().flashoptim_short_sqrt_state())


def selftest(stream=None):
    """Runs the device self-test; returns (status, checked[7], failed[7])."""
    checked = (C.c_int64 * 7)()
    failed = (C.c_int64 * 7)()
    status = load_library().flashoptim_selftest(checked, failed, _stream(stream))
    if status not in (0, -6):
        raise FlashOptimError(status, "flashoptim_selftest")
    return status, list(checked), list(failed)


def strerror(status):
    return load_library().flashoptim_strerror(int(status)).decode()


def step_launch_count(kind, numels):
    """Kernel launches that one step call of `kind` issues for a list with these element counts."""
    arr = (C.c_int64 * max(len(numels), 1))(*[int(n) for n in numels])
    n = int(load_library().flashoptim_step_launch_count(KIND[kind], arr, len(numels)))
    if n < 0:
        raise FlashOptimError(n, "flashoptim_step_launch_count")
    return n


def release_cache():
    _check(load_library().flashoptim_release_cache(), "flashoptim_release_cache")


def version():
    return int(load_library().flashoptim_version())
