"""ctypes binding of include/rsparse.h -- argument marshalling only; every step of the path runs
in the library's kernels.  There is no CPU fallback: a missing library is an error."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

F16, BF16, F32 = 0, 1, 2
OK, EINVAL, ENOMEM, EHIP, EBATCH, EALIGN, ESVD = range(7)
_STATUS = {1: "EINVAL", 2: "ENOMEM", 3: "EHIP", 4: "EBATCH", 5: "EALIGN", 6: "ESVD"}

EXPORTED_SYMBOLS = [
    "rsparse_prepare", "rsparse_compute_factors", "rsparse_prepare_factors", "rsparse_prepare_q4", "rsparse_linear", "rsparse_linear_static",
    "rsparse_linear_gated", "rsparse_gated_input", "rsparse_mlp_gate_up", "rsparse_dense_ref", "rsparse_linear_group", "rsparse_dense_ref_group", "rsparse_linear_group_planned", "rsparse_last_active", "rsparse_synchronize",
    "rsparse_get_factors", "rsparse_set_tau", "rsparse_set_bias", "rsparse_multiphase_bias", "rsparse_set_tuning",
    "rsparse_get_config", "rsparse_calibrate_tau", "rsparse_required_bytes", "rsparse_dense_bytes", "rsparse_io_model",
    "rsparse_recipe", "rsparse_plan_layer", "rsparse_search_recipe", "rsparse_debug_stamps", "rsparse_destroy", "rsparse_last_error",
]


class Config(C.Structure):
    _fields_ = [("d_in", C.c_int32), ("d_out", C.c_int32), ("rank", C.c_int32), ("max_batch", C.c_int32),
                ("tau", C.c_float), ("dtype", C.c_int32), ("out_dtype", C.c_int32), ("cmp_mode", C.c_int32),
                ("batch_mask_mode", C.c_int32), ("dense_rowmajor", C.c_int32), ("strip_cols", C.c_int32), ("topk", C.c_int32),
                ("lowrank_channel_major", C.c_int32)]


class Tuning(C.Structure):
    _fields_ = [("splits", C.c_int32), ("waves", C.c_int32), ("lowrank_rows", C.c_int32),
                ("dense_kernel", C.c_int32), ("nontemporal", C.c_int32), ("stages", C.c_int32),
                ("tile_map", C.c_int32), ("mfma_min_batch", C.c_int32), ("mfma_rows", C.c_int32),
                ("launches", C.c_int32), ("lowrank_wgs", C.c_int32), ("debug_wait_polls", C.c_int32), ("debug_skip_stage1", C.c_int32)]


LOSS_FN = C.CFUNCTYPE(C.c_double, C.POINTER(C.c_double), C.c_int32, C.c_void_p)


class RSparseError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"rsparse status {status} ({_STATUS.get(status, '?')}): {message}")
        self.status = status


_lib = None


def library_path() -> str:
    """The in-tree library, or the file RSPARSE_LIB names (a measurement build of the same sources)."""
    if os.environ.get("RSPARSE_LIB"):
        return os.environ["RSPARSE_LIB"]
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "librsparse.so")


def load_library():
    """Load librsparse.so (built in-tree by paper_2504_19449_amd/build.py).  Raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    path = library_path()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with `python -m paper_2504_19449_amd.build` "
                           "(there is no CPU fallback)")
    try:
        # One HIP runtime per process: PyTorch-ROCm bundles its own libamdhip64 (same SONAME as
        # the one this library links).  Loading torch first makes both share torch's copy, so
        # device pointers and streams made by torch are valid here.
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(path)
    vp, i32 = C.c_void_p, C.c_int32
    lib.rsparse_prepare.argtypes = [C.POINTER(Config), vp, C.POINTER(vp)]
    lib.rsparse_compute_factors.argtypes = [C.POINTER(Config), vp, vp, vp, vp]
    lib.rsparse_prepare_factors.argtypes = [C.POINTER(Config), vp, vp, vp, C.POINTER(vp)]
    lib.rsparse_prepare_q4.argtypes = [C.POINTER(Config), vp, vp, vp, i32, vp, vp, C.POINTER(vp)]
    lib.rsparse_linear.argtypes = [vp, vp, i32, vp, vp]
    lib.rsparse_linear_static.argtypes = [vp, vp, i32, vp, vp]
    lib.rsparse_linear_static.restype = C.c_int
    lib.rsparse_dense_ref.argtypes = [vp, vp, i32, vp, vp]
    lib.rsparse_linear_gated.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.rsparse_gated_input.argtypes = [vp, vp, vp, C.c_size_t, i32, vp]
    lib.rsparse_mlp_gate_up.argtypes = [vp, vp, vp, i32, vp, vp]
    lib.rsparse_linear_group.argtypes = [vp, i32, vp, i32, vp, vp]
    lib.rsparse_dense_ref_group.argtypes = [vp, i32, vp, i32, vp, vp]
    lib.rsparse_linear_group_planned.argtypes = [vp, i32, vp, i32, vp, vp, C.c_double, C.POINTER(i32)]
    lib.rsparse_linear_group_planned.restype = C.c_int
    lib.rsparse_last_active.argtypes = [vp, i32, vp, C.POINTER(i32)]
    lib.rsparse_synchronize.argtypes = [vp]
    lib.rsparse_get_factors.argtypes = [vp, vp, vp]
    lib.rsparse_set_tau.argtypes = [vp, C.c_float]
    lib.rsparse_set_bias.argtypes = [vp, vp]
    lib.rsparse_set_bias.restype = C.c_int
    lib.rsparse_multiphase_bias.argtypes = [vp, i32, i32, i32, vp, i32, vp, i32, vp]
    lib.rsparse_multiphase_bias.restype = C.c_int
    lib.rsparse_set_tuning.argtypes = [vp, C.POINTER(Tuning)]
    lib.rsparse_get_config.argtypes = [vp, C.POINTER(Config)]
    lib.rsparse_calibrate_tau.argtypes = [vp, i32, C.c_size_t, C.c_double, C.POINTER(C.c_float)]
    lib.rsparse_required_bytes.argtypes = [vp, i32, i32]
    lib.rsparse_required_bytes.restype = C.c_size_t
    lib.rsparse_dense_bytes.argtypes = [vp, i32]
    lib.rsparse_dense_bytes.restype = C.c_size_t
    lib.rsparse_io_model.argtypes = [C.POINTER(Config), i32, i32, i32, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t),
                                     C.POINTER(C.c_size_t)]
    lib.rsparse_io_model.restype = C.c_int
    lib.rsparse_recipe.argtypes = [i32, i32, C.c_double, C.c_double, C.POINTER(C.c_double), C.POINTER(i32),
                                   C.POINTER(C.c_double)]
    lib.rsparse_recipe.restype = C.c_int
    lib.rsparse_plan_layer.argtypes = [i32, i32, i32, C.c_double, i32, i32, C.POINTER(C.c_double), C.POINTER(C.c_double),
                                       C.POINTER(i32)]
    lib.rsparse_plan_layer.restype = C.c_int
    lib.rsparse_search_recipe.argtypes = [LOSS_FN, vp, i32, i32, i32, C.c_double, C.c_double, i32, C.c_uint64,
                                          C.c_double, C.c_double, vp, vp, vp, vp]
    lib.rsparse_search_recipe.restype = C.c_int
    lib.rsparse_debug_stamps.argtypes = [vp, i32]
    lib.rsparse_debug_stamps.restype = C.c_int
    lib.rsparse_destroy.argtypes = [vp]
    lib.rsparse_destroy.restype = None
    lib.rsparse_last_error.restype = C.c_char_p
    for name in ("rsparse_linear_group", "rsparse_dense_ref_group", "rsparse_prepare", "rsparse_compute_factors",
                 "rsparse_prepare_factors", "rsparse_linear", "rsparse_dense_ref",
                 "rsparse_last_active", "rsparse_get_factors", "rsparse_set_tau", "rsparse_set_bias", "rsparse_multiphase_bias", "rsparse_set_tuning",
                 "rsparse_get_config", "rsparse_calibrate_tau", "rsparse_synchronize", "rsparse_linear_gated", "rsparse_gated_input", "rsparse_mlp_gate_up", "rsparse_prepare_q4"):
        getattr(lib, name).restype = C.c_int
    _lib = lib
    return lib


def rsparse_last_error() -> str:
    return load_library().rsparse_last_error().decode()


def _check(st: int):
    if st != OK:
        raise RSparseError(st, rsparse_last_error())


def _host16(a, name):
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError(f"{name} must be uint16 bit patterns")
    return a


def _hp(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


class Layer:
    """Owner of an rsparse_layer handle."""

    def __init__(self, handle, cfg: Config):
        self.handle, self.cfg = handle, cfg

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "handle", None):
            rsparse_destroy(self)
            self.handle = None


def _make_config(d_in, d_out, rank, tau, dtype, max_batch=1, out_dtype=None, cmp_mode=0,
                 batch_mask_mode=0, dense_rowmajor=0, strip_cols=0, topk=0, lowrank_channel_major=0) -> Config:
    return Config(d_in, d_out, rank, max_batch, float(tau), dtype, dtype if out_dtype is None else out_dtype,
                  cmp_mode, batch_mask_mode, dense_rowmajor, strip_cols, topk, lowrank_channel_major)


def rsparse_prepare(cfg: Config, W16) -> Layer:
    W16 = _host16(W16, "W")
    if W16.shape != (cfg.d_out, cfg.d_in):
        raise ValueError("W must be [d_out, d_in]")
    h = C.c_void_p()
    _check(load_library().rsparse_prepare(C.byref(cfg), _hp(W16), C.byref(h)))
    return Layer(h, cfg)


def rsparse_compute_factors(cfg: Config, W16):
    """Host SVD only: returns (U16 [d_out, rank], SV16 [rank, d_in], sigma [rank] float64)."""
    W16 = _host16(W16, "W")
    if W16.shape != (cfg.d_out, cfg.d_in):
        raise ValueError("W must be [d_out, d_in]")
    U = np.zeros((cfg.d_out, cfg.rank), dtype=np.uint16)
    SV = np.zeros((cfg.rank, cfg.d_in), dtype=np.uint16)
    sig = np.zeros(cfg.rank, dtype=np.float64)
    _check(load_library().rsparse_compute_factors(C.byref(cfg), _hp(W16), _hp(U), _hp(SV),
                                                  sig.ctypes.data_as(C.c_void_p)))
    return U, SV, sig


def rsparse_prepare_factors(cfg: Config, W16, U16, SV16) -> Layer:
    W16, U16, SV16 = _host16(W16, "W"), _host16(U16, "U"), _host16(SV16, "SV")
    if W16.shape != (cfg.d_out, cfg.d_in):
        raise ValueError("W must be [d_out, d_in]")
    if cfg.rank > 0 and (U16 is None or SV16 is None or U16.shape != (cfg.d_out, cfg.rank)
                         or SV16.shape != (cfg.rank, cfg.d_in)):
        raise ValueError("U must be [d_out, rank] and SV [rank, d_in]")
    h = C.c_void_p()
    _check(load_library().rsparse_prepare_factors(C.byref(cfg), _hp(W16), _hp(U16), _hp(SV16), C.byref(h)))
    return Layer(h, cfg)


def rsparse_prepare_q4(cfg: Config, Q, S16, Z, group_size: int, U16=None, SV16=None) -> Layer:
    """Layer on 4-bit weights: Q [d_out, d_in] uint8 codes, S16 / Z [d_out, d_in / group_size]."""
    Q = np.ascontiguousarray(Q)
    Z = np.ascontiguousarray(Z)
    S16 = _host16(S16, "S")
    if Q.dtype != np.uint8 or Z.dtype != np.uint8:
        raise TypeError("Q and Z must be uint8")
    if group_size < 1 or cfg.d_in % group_size:
        raise ValueError("group_size must divide d_in")
    G = cfg.d_in // group_size
    if Q.shape != (cfg.d_out, cfg.d_in) or S16.shape != (cfg.d_out, G) or Z.shape != (cfg.d_out, G):
        raise ValueError("Q must be [d_out, d_in], S and Z [d_out, d_in / group_size]")
    U16, SV16 = _host16(U16, "U"), _host16(SV16, "SV")
    if cfg.rank > 0 and (U16 is None or SV16 is None or U16.shape != (cfg.d_out, cfg.rank)
                         or SV16.shape != (cfg.rank, cfg.d_in)):
        raise ValueError("U must be [d_out, rank] and SV [rank, d_in]")
    h = C.c_void_p()
    _check(load_library().rsparse_prepare_q4(C.byref(cfg), _hp(Q), _hp(S16), _hp(Z), group_size, _hp(U16), _hp(SV16),
                                             C.byref(h)))
    return Layer(h, cfg)


def rsparse_linear(layer: Layer, X_dev: int, batch: int, Y_dev: int, stream: int = 0):
    """X_dev / Y_dev / stream are raw device pointers / a hipStream_t as integers."""
    _check(load_library().rsparse_linear(layer.handle, X_dev, batch, Y_dev, stream))


def rsparse_linear_static(layer: Layer, X_dev: int, batch: int, Y_dev: int, stream: int = 0):
    """rsparse_linear with its scratch in the library's static device array (allocates nothing)."""
    _check(load_library().rsparse_linear_static(layer.handle, X_dev, batch, Y_dev, stream))


def rsparse_linear_gated(layer: Layer, G_dev: int, Up_dev: int, batch: int, Y_dev: int, stream: int = 0):
    """The layer on x = round(silu(g) * u); G_dev / Up_dev are the gate and up branches [batch][d_in]."""
    _check(load_library().rsparse_linear_gated(layer.handle, G_dev, Up_dev, batch, Y_dev, stream))


def rsparse_mlp_gate_up(gate: Layer, up: Layer, X_dev: int, batch: int, H_dev: int, stream: int = 0):
    """H = round(silu(g) * u) with g, u the R-Sparse outputs of `gate` and `up` on X (Sec. 3.1)."""
    _check(load_library().rsparse_mlp_gate_up(gate.handle, up.handle, X_dev, batch, H_dev, stream))


def rsparse_gated_input(G_dev: int, Up_dev: int, out_dev: int, n: int, dtype: int, stream: int = 0):
    _check(load_library().rsparse_gated_input(G_dev, Up_dev, out_dev, n, dtype, stream))


def rsparse_dense_ref(layer: Layer, X_dev: int, batch: int, Y_dev: int, stream: int = 0):
    _check(load_library().rsparse_dense_ref(layer.handle, X_dev, batch, Y_dev, stream))


def _group_arrays(layers, Y_devs):
    n = len(layers)
    if n != len(Y_devs):
        raise ValueError("one output pointer per layer")
    hs = (C.c_void_p * n)(*[l.handle.value for l in layers])
    ys = (C.c_void_p * n)(*[int(y) for y in Y_devs])
    return n, hs, ys


def rsparse_linear_group(layers, X_dev: int, batch: int, Y_devs, stream: int = 0):
    """Layers sharing one input (q/k/v, gate/up): one pair of launches for all of them."""
    n, hs, ys = _group_arrays(layers, Y_devs)
    _check(load_library().rsparse_linear_group(hs, n, X_dev, batch, ys, stream))


def rsparse_linear_group_planned(layers, X_dev: int, batch: int, Y_devs, keep_fraction: float, stream: int = 0) -> bool:
    """R-Sparse or dense, as rsparse_plan_layer decides for these layers at this batch; returns True if R-Sparse ran."""
    n, hs, ys = _group_arrays(layers, Y_devs)
    used = C.c_int32()
    _check(load_library().rsparse_linear_group_planned(hs, n, X_dev, batch, ys, stream, keep_fraction, C.byref(used)))
    return bool(used.value)


def rsparse_dense_ref_group(layers, X_dev: int, batch: int, Y_devs, stream: int = 0):
    n, hs, ys = _group_arrays(layers, Y_devs)
    _check(load_library().rsparse_dense_ref_group(hs, n, X_dev, batch, ys, stream))


def rsparse_synchronize(layer: Layer) -> None:
    _check(load_library().rsparse_synchronize(layer.handle))


def rsparse_last_active(layer: Layer, token: int) -> np.ndarray:
    idx = np.empty(layer.cfg.d_in, dtype=np.int32)
    n = C.c_int32(0)
    _check(load_library().rsparse_last_active(layer.handle, token, _hp(idx), C.byref(n)))
    return idx[: n.value].copy()


def rsparse_get_factors(layer: Layer):
    U = np.empty((layer.cfg.d_out, layer.cfg.rank), dtype=np.uint16)
    SV = np.empty((layer.cfg.rank, layer.cfg.d_in), dtype=np.uint16)
    _check(load_library().rsparse_get_factors(layer.handle, _hp(U), _hp(SV)))
    return U, SV


def rsparse_set_tau(layer: Layer, tau: float):
    _check(load_library().rsparse_set_tau(layer.handle, float(tau)))
    layer.cfg.tau = float(tau)


def rsparse_set_bias(layer: Layer, bias):
    """bias: float32 [d_out] on the host, or None to remove it."""
    if bias is None:
        _check(load_library().rsparse_set_bias(layer.handle, None))
        return
    b = np.ascontiguousarray(bias, dtype=np.float32)
    if b.shape != (layer.cfg.d_out,):
        raise ValueError("bias must be [d_out]")
    _check(load_library().rsparse_set_bias(layer.handle, _hp(b)))


def rsparse_multiphase_bias(W16, dtype: int, H16, T) -> np.ndarray:
    """Static bias of the multi-phase activation (Sec. 3.2) from calibration tokens H16 [n][d_in]; float32 [d_out]."""
    W16 = _host16(W16, "W")
    H16 = _host16(H16, "H")
    d_out, d_in = W16.shape
    if H16.ndim != 2 or H16.shape[1] != d_in:
        raise ValueError("H must be [n_tokens, d_in]")
    T = np.ascontiguousarray(T, dtype=np.float32)
    out = np.empty(d_out, dtype=np.float32)
    _check(load_library().rsparse_multiphase_bias(_hp(W16), dtype, d_in, d_out, _hp(H16), H16.shape[0], _hp(T), len(T), _hp(out)))
    return out


def rsparse_set_tuning(layer: Layer, **kw):
    t = Tuning()
    for k, v in kw.items():
        setattr(t, k, int(v))
    _check(load_library().rsparse_set_tuning(layer.handle, C.byref(t)))


def rsparse_get_config(layer: Layer) -> Config:
    c = Config()
    _check(load_library().rsparse_get_config(layer.handle, C.byref(c)))
    return c


def rsparse_calibrate_tau(X16, dtype: int, s: float) -> float:
    X16 = _host16(X16, "X").reshape(-1)
    tau = C.c_float(0)
    _check(load_library().rsparse_calibrate_tau(_hp(X16), dtype, X16.size, float(s), C.byref(tau)))
    return float(tau.value)


def rsparse_required_bytes(layer: Layer, batch: int, k_union: int) -> int:
    return int(load_library().rsparse_required_bytes(layer.handle, batch, k_union))


def rsparse_dense_bytes(layer: Layer, batch: int) -> int:
    return int(load_library().rsparse_dense_bytes(layer.handle, batch))


def rsparse_io_model(cfg: Config, batch: int, k_union: int, q4_group: int = 0):
    """(required, dense, required with inactive-only factor reads) bytes of Sec. 3.4's I/O model; host code."""
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check(load_library().rsparse_io_model(C.byref(cfg), q4_group, batch, k_union, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def rsparse_recipe(d_in: int, d_out: int, budget_c: float, rho: float):
    """(keep_fraction s, rank r, relative I/O) of the Sec. 3.5 recipe; r is a multiple of 8."""
    s, r, io = C.c_double(0), C.c_int32(0), C.c_double(0)
    _check(load_library().rsparse_recipe(d_in, d_out, float(budget_c), float(rho), C.byref(s), C.byref(r), C.byref(io)))
    return s.value, r.value, io.value


def rsparse_plan_layer(d_in: int, d_out: int, rank: int, keep_fraction: float, group: int = 1, batch: int = 1):
    """(estimated us with R-Sparse, estimated us dense, use R-Sparse?) for one layer at `batch` tokens; host code."""
    a, b, use = C.c_double(), C.c_double(), C.c_int32()
    _check(load_library().rsparse_plan_layer(d_in, d_out, rank, keep_fraction, group, batch, C.byref(a), C.byref(b),
                                             C.byref(use)))
    return a.value, b.value, bool(use.value)


def rsparse_debug_stamps(buf_dev: int, capacity_waves: int):
    """Stamps builds only: where the strip kernel's waves write their phase time stamps (0, 0 = off)."""
    _check(load_library().rsparse_debug_stamps(buf_dev, capacity_waves))


def rsparse_destroy(layer: Layer):
    load_library().rsparse_destroy(layer.handle)


make_config = _make_config


def rsparse_search_recipe(loss, n_layers: int, population: int = 32, generations: int = 5, p_m: float = 0.5,
                          p_c: float = 0.5, group_size: int = 28, seed: int = 0, lo: float = 0.0, hi: float = 1.0,
                          rho_start=None):
    """Sec. 3.5 recipe search; `loss` is a Python callable on a list of n_layers floats.
    Returns (rho [n_layers], best loss, history)."""
    def trampoline(rho_ptr, n, _user):
        return float(loss([rho_ptr[i] for i in range(n)]))

    cb = LOSS_FN(trampoline)
    groups = (n_layers + group_size - 1) // group_size
    rho = np.zeros(n_layers, dtype=np.float64)
    best = C.c_double(0.0)
    hist = np.zeros(1 + groups * generations, dtype=np.float64)
    start = None if rho_start is None else np.ascontiguousarray(rho_start, dtype=np.float64)
    st = load_library().rsparse_search_recipe(cb, None, n_layers, population, generations, p_m, p_c, group_size, seed,
                                              lo, hi, None if start is None else start.ctypes.data_as(C.c_void_p),
                                              rho.ctypes.data_as(C.c_void_p), C.byref(best), hist.ctypes.data_as(C.c_void_p))
    if st != OK:
        raise RSparseError(st, "rsparse_search_recipe: invalid argument" if st == EINVAL else "allocation failed")
    return rho, best.value, hist
