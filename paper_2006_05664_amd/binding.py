"""ctypes binding of libopevo.so: one Python function per C-ABI entry point, same names.

Argument marshalling only -- every step of the path (space encoding, q-random walk, the OpEvo
loop, hipRTC instantiation, launches, timing, the parity gate) runs inside the library.
Device pointers are plain integers (``tensor.data_ptr()``), the stream is the integer handle
of a HIP stream (``torch.cuda.current_stream().cuda_stream``); PyTorch is used by callers only
to own device memory and streams.

There is no fallback: if the library is missing or cannot be loaded, importing this module
raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libopevo.so")

OPEVO_OK, OPEVO_E_ARG, OPEVO_E_ILLEGAL, OPEVO_E_INVALID = 0, -1, -2, -3
OPEVO_E_HIPRTC, OPEVO_E_HIP, OPEVO_E_PARITY, OPEVO_E_TOO_LARGE, OPEVO_E_STATE = -4, -5, -6, -7, -8
OPEVO_FACTOR, OPEVO_PERMUTATION, OPEVO_DISCRETE, OPEVO_CATEGORICAL = 0, 1, 2, 3
OPEVO_MATMUL, OPEVO_BMM, OPEVO_CONV2D, OPEVO_BMM_TA = 0, 1, 2, 3
OPEVO_F32, OPEVO_BF16, OPEVO_F16 = 0, 1, 2
OPEVO_TILE2, OPEVO_TILE4, OPEVO_TILE4X, OPEVO_TILE4P, OPEVO_TILE4K, OPEVO_TILE4C, OPEVO_TILE4T, OPEVO_TILE4A, OPEVO_TILE4L = 0, 1, 2, 3, 4, 5, 6, 7, 8


class OpevoError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("%s (%d): %s" % (opevo_status_name(status), status, message))
        self.status = status
        self.message = message


class opevo_param_desc(C.Structure):
    _fields_ = [("type", C.c_int32), ("nu", C.c_int32), ("C", C.c_int64), ("n_values", C.c_int32),
                ("reserved", C.c_int32), ("values", C.POINTER(C.c_double)), ("name", C.c_char_p)]


class opevo_plan(C.Structure):
    _fields_ = [("status", C.c_int32), ("path", C.c_int32), ("grid", C.c_int32 * 3), ("block", C.c_int32),
                ("lds_bytes", C.c_int32), ("acc_per_lane", C.c_int32), ("tile", C.c_int32 * 3),
                ("wave_tile", C.c_int32 * 2), ("reason", C.c_char * 96), ("sub_tiles", C.c_int32 * 2),
                ("wave_passes", C.c_int32)]


class opevo_tune_args(C.Structure):
    _fields_ = [("a", C.c_void_p), ("b", C.c_void_p), ("c", C.c_void_p), ("ref", C.c_void_p),
                ("ref_row_index", C.c_void_p), ("n_ref_rows", C.c_int32), ("ref_row_len", C.c_int32),
                ("stream", C.c_void_p), ("trials", C.c_int32), ("lambda_", C.c_int32), ("rho", C.c_int32),
                ("q", C.c_double), ("seed", C.c_uint64), ("compile_threads", C.c_int32),
                ("warmup", C.c_int32), ("launches_per_sample", C.c_int32), ("samples", C.c_int32),
                ("warmup_ms", C.c_double), ("trial_timeout_ms", C.c_double), ("tol_max_scaled", C.c_double), ("tol_rel_fro", C.c_double),
                ("cfg_log", C.POINTER(C.c_int32)), ("fitness_log", C.POINTER(C.c_double)),
                ("status_log", C.POINTER(C.c_int32)), ("compile_ms_log", C.POINTER(C.c_double)),
                ("run_ms_log", C.POINTER(C.c_double)), ("wall_s_log", C.POINTER(C.c_double)),
                ("progress_every", C.c_int32), ("mutation", C.c_int32), ("speculate_threads", C.c_int32)]


class opevo_tune_result(C.Structure):
    _fields_ = [("n_trials", C.c_int32), ("best_trial", C.c_int32), ("best_tflops", C.c_double),
                ("best_ms", C.c_double), ("n_invalid", C.c_int32), ("n_compile_fail", C.c_int32),
                ("n_parity_fail", C.c_int32), ("wall_s", C.c_double), ("compile_s", C.c_double),
                ("run_s", C.c_double), ("n_built_ahead", C.c_int32)]


def _load() -> C.CDLL:
    # PyTorch ships its own HIP runtime.  The library must bind to that same instance (a second
    # runtime in the process cannot see the device), so torch's libraries are loaded first and
    # the dynamic linker resolves libopevo's libamdhip64 / libhiprtc dependencies to them.
    import torch  # noqa: F401
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python paper_2006_05664_amd/build.py`" % LIB_PATH)
    return C.CDLL(LIB_PATH)


lib = _load()

_i32p, _f64p, _vp = C.POINTER(C.c_int32), C.POINTER(C.c_double), C.c_void_p
_SIGNATURES = {
    "opevo_rng_create": [C.c_uint64, C.POINTER(_vp)],
    "opevo_rng_destroy": [_vp],
    "opevo_rng_next_u64": [_vp, C.POINTER(C.c_uint64)],
    "opevo_rng_next_double": [_vp, _f64p],
    "opevo_rng_next_below": [_vp, C.c_uint32, C.POINTER(C.c_uint32)],
    "opevo_space_create": [C.POINTER(opevo_param_desc), C.c_int, C.POINTER(_vp)],
    "opevo_space_destroy": [_vp],
    "opevo_space_num_params": [_vp, C.POINTER(C.c_int)],
    "opevo_space_width": [_vp, C.POINTER(C.c_int)],
    "opevo_space_param_slice": [_vp, C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int)],
    "opevo_space_param_name": [_vp, C.c_int, C.POINTER(C.c_char_p)],
    "opevo_space_param_size": [_vp, C.c_int, C.POINTER(C.c_int64)],
    "opevo_space_size": [_vp, _f64p],
    "opevo_space_is_legal": [_vp, _i32p],
    "opevo_space_enumerate": [_vp, C.c_int, _i32p, C.c_int64, C.POINTER(C.c_int64)],
    "opevo_space_neighbors": [_vp, C.c_int, _i32p, _i32p, C.c_int, C.POINTER(C.c_int)],
    "opevo_space_rank": [_vp, _i32p, C.POINTER(C.c_int64)],
    "opevo_space_unrank": [_vp, C.c_int64, _i32p],
    "opevo_space_random": [_vp, _vp, _i32p],
    "opevo_space_walk": [_vp, C.c_int, C.c_double, _vp, _i32p],
    "opevo_space_mutate": [_vp, C.c_double, _vp, _i32p],
    "opevo_qrw_exact": [_vp, C.c_int, _i32p, C.c_double, _f64p, C.c_int64],
    "opevo_recombine": [_vp, _i32p, _f64p, C.c_int, _vp, _i32p],
    "opevo_tuner_create": [_vp, C.c_int, C.c_int, C.c_double, C.c_uint64, C.POINTER(_vp)],
    "opevo_tuner_destroy": [_vp],
    "opevo_tuner_set_mutation": [_vp, C.c_int],
    "opevo_tuner_ask": [_vp, _i32p, C.c_int, C.POINTER(C.c_int)],
    "opevo_tuner_tell": [_vp, _i32p, _f64p, C.c_int],
    "opevo_tuner_num_trials": [_vp, C.POINTER(C.c_int)],
    "opevo_tuner_best": [_vp, _i32p, _f64p, C.POINTER(C.c_int)],
    "opevo_tuner_history": [_vp, _i32p, _f64p, C.c_int, C.POINTER(C.c_int)],
    "opevo_op_create": [C.c_int, C.POINTER(C.c_int64), C.c_int, C.c_int, C.POINTER(_vp)],
    "opevo_op_destroy": [_vp],
    "opevo_op_flops": [_vp, _f64p],
    "opevo_op_bytes": [_vp, _f64p],
    "opevo_op_sizes": [_vp, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int64)],
    "opevo_op_space": [_vp, C.c_int, C.POINTER(_vp)],
    "opevo_compile_pool_start": [C.c_int, C.POINTER(C.c_int)],
    "opevo_compile_pool_stop": [],
    "opevo_compile_pool_kind": [C.POINTER(C.c_int)],
    "opevo_compile_pool_deadline": [C.c_double],
    "opevo_kernel_plan": [_vp, C.c_int, _i32p, C.POINTER(opevo_plan)],
    "opevo_kernel_defines": [_vp, C.c_int, _i32p, C.c_char_p, C.c_size_t],
    "opevo_kernel_build": [_vp, C.c_int, _i32p, C.POINTER(_vp), _f64p],
    "opevo_kernel_destroy": [_vp],
    "opevo_kernel_code_size": [_vp, C.POINTER(C.c_size_t)],
    "opevo_code_cache_configure": [C.c_char_p, C.c_int64],
    "opevo_code_cache_clear": [],
    "opevo_code_cache_stats": [C.POINTER(C.c_int64)] * 5,
    "opevo_kernel_resources": [_vp, C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int), C.POINTER(C.c_int)],
    "opevo_kernel_launch": [_vp, _vp, _vp, _vp, _vp],
    "opevo_kernel_time": [_vp, _vp, _vp, _vp, _vp, C.c_int, C.c_double, C.c_int, C.c_int, C.c_double, _f64p, _f64p],
    "opevo_mfma_ceiling": [C.c_int, C.c_int, _vp, _f64p],
    "opevo_mfma_ceiling_atom": [C.c_int, C.c_int, C.c_int, _vp, _f64p],
    "opevo_compare_f32": [_vp, _vp, C.c_int64, _vp, _f64p, _f64p],
    "opevo_compare_rows_f32": [_vp, _vp, _vp, C.c_int64, C.c_int64, _vp, _f64p, _f64p],
    "opevo_compare_f32_static": [_vp, _vp, C.c_int64, _vp, _vp],
    "opevo_tune": [_vp, C.c_int, C.POINTER(opevo_tune_args), _i32p, C.POINTER(opevo_tune_result)],
}
for _name, _argtypes in _SIGNATURES.items():
    _fn = getattr(lib, _name)
    _fn.argtypes = _argtypes
    _fn.restype = C.c_int
for _name in ("opevo_last_error", "opevo_version"):
    getattr(lib, _name).restype = C.c_char_p
lib.opevo_status_name.argtypes = [C.c_int]
lib.opevo_status_name.restype = C.c_char_p

EXPORTED = sorted(list(_SIGNATURES) + ["opevo_last_error", "opevo_version", "opevo_status_name"])


def opevo_last_error() -> str:
    return lib.opevo_last_error().decode()


def opevo_version() -> str:
    return lib.opevo_version().decode()


def opevo_status_name(status: int) -> str:
    return lib.opevo_status_name(status).decode()


def _check(status: int, allow: Sequence[int] = ()) -> int:
    if status != OPEVO_OK and status not in allow:
        raise OpevoError(status, opevo_last_error())
    return status


def _cfg(cfg) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(cfg, dtype=np.int32).ravel())


def _ip(a: np.ndarray):
    return a.ctypes.data_as(_i32p)


def _dp(a: np.ndarray):
    return a.ctypes.data_as(_f64p)


# ------------------------------------------------------------------------------- rng
def opevo_rng_create(seed: int):
    h = _vp()
    _check(lib.opevo_rng_create(seed & (2 ** 64 - 1), C.byref(h)))
    return h


def opevo_rng_destroy(rng) -> None:
    _check(lib.opevo_rng_destroy(rng))


def opevo_rng_next_u64(rng) -> int:
    v = C.c_uint64()
    _check(lib.opevo_rng_next_u64(rng, C.byref(v)))
    return v.value


def opevo_rng_next_double(rng) -> float:
    v = C.c_double()
    _check(lib.opevo_rng_next_double(rng, C.byref(v)))
    return v.value


def opevo_rng_next_below(rng, n: int) -> int:
    v = C.c_uint32()
    _check(lib.opevo_rng_next_below(rng, n, C.byref(v)))
    return v.value


# ----------------------------------------------------------------------------- space
def opevo_space_create(params: Sequence[dict]):
    """params: dicts with keys type, and C/nu (FACTOR), n_values (PERMUTATION/CATEGORICAL) or
    values (DISCRETE), optional name."""
    n = len(params)
    arr = (opevo_param_desc * max(n, 1))()
    keep = []
    for i, p in enumerate(params):
        d = arr[i]
        d.type = int(p["type"])
        d.nu = int(p.get("nu", 0))
        d.C = int(p.get("C", 0))
        vals = p.get("values")
        if vals is not None:
            buf = (C.c_double * len(vals))(*[float(v) for v in vals])
            keep.append(buf)
            d.values = C.cast(buf, _f64p)
            d.n_values = len(vals)
        else:
            d.n_values = int(p.get("n_values", 0))
        name = p.get("name")
        d.name = name.encode() if name else None
    h = _vp()
    _check(lib.opevo_space_create(arr, n, C.byref(h)))
    return h


def opevo_space_destroy(space) -> None:
    _check(lib.opevo_space_destroy(space))


def opevo_space_num_params(space) -> int:
    v = C.c_int()
    _check(lib.opevo_space_num_params(space, C.byref(v)))
    return v.value


def opevo_space_width(space) -> int:
    v = C.c_int()
    _check(lib.opevo_space_width(space, C.byref(v)))
    return v.value


def opevo_space_param_slice(space, param: int) -> Tuple[int, int]:
    o, w = C.c_int(), C.c_int()
    _check(lib.opevo_space_param_slice(space, param, C.byref(o), C.byref(w)))
    return o.value, w.value


def opevo_space_param_name(space, param: int) -> str:
    s = C.c_char_p()
    _check(lib.opevo_space_param_name(space, param, C.byref(s)))
    return s.value.decode()


def opevo_space_param_size(space, param: int) -> int:
    v = C.c_int64()
    _check(lib.opevo_space_param_size(space, param, C.byref(v)))
    return v.value


def opevo_space_size(space) -> float:
    v = C.c_double()
    _check(lib.opevo_space_size(space, C.byref(v)))
    return v.value


def opevo_space_is_legal(space, cfg) -> bool:
    cfg = _cfg(cfg)
    if cfg.size != opevo_space_width(space):
        return False
    return _check(lib.opevo_space_is_legal(space, _ip(cfg)), allow=(OPEVO_E_ILLEGAL,)) == OPEVO_OK


def opevo_space_enumerate(space, param: int) -> np.ndarray:
    n = opevo_space_param_size(space, param)
    _, w = opevo_space_param_slice(space, param)
    out = np.empty((n, w), dtype=np.int32)
    got = C.c_int64()
    _check(lib.opevo_space_enumerate(space, param, _ip(out), n, C.byref(got)))
    return out


def opevo_space_neighbors(space, param: int, v) -> np.ndarray:
    v = _cfg(v)
    _, w = opevo_space_param_slice(space, param)
    assert v.size == w
    cap = 4096
    out = np.empty((cap, w), dtype=np.int32)
    n = C.c_int()
    _check(lib.opevo_space_neighbors(space, param, _ip(v), _ip(out), cap, C.byref(n)))
    return out[:n.value].copy()


def opevo_space_rank(space, cfg) -> int:
    cfg = _cfg(cfg)
    assert cfg.size == opevo_space_width(space)
    r = C.c_int64()
    _check(lib.opevo_space_rank(space, _ip(cfg), C.byref(r)))
    return r.value


def opevo_space_unrank(space, rank: int) -> np.ndarray:
    out = np.empty(opevo_space_width(space), dtype=np.int32)
    _check(lib.opevo_space_unrank(space, rank, _ip(out)))
    return out


def opevo_space_random(space, rng) -> np.ndarray:
    out = np.empty(opevo_space_width(space), dtype=np.int32)
    _check(lib.opevo_space_random(space, rng, _ip(out)))
    return out


def opevo_space_walk(space, param: int, q: float, rng, v) -> np.ndarray:
    v = _cfg(v).copy()
    _, w = opevo_space_param_slice(space, param)
    assert v.size == w
    _check(lib.opevo_space_walk(space, param, q, rng, _ip(v)))
    return v


def opevo_space_mutate(space, q: float, rng, cfg) -> np.ndarray:
    cfg = _cfg(cfg).copy()
    assert cfg.size == opevo_space_width(space)
    _check(lib.opevo_space_mutate(space, q, rng, _ip(cfg)))
    return cfg


def opevo_qrw_exact(space, param: int, start, q: float) -> np.ndarray:
    start = _cfg(start)
    n = opevo_space_param_size(space, param)
    out = np.empty(n, dtype=np.float64)
    _check(lib.opevo_qrw_exact(space, param, _ip(start), q, _dp(out), n))
    return out


# ----------------------------------------------------------------------------- tuner
def opevo_recombine(space, parents, fitness, rng) -> np.ndarray:
    parents = np.ascontiguousarray(np.asarray(parents, dtype=np.int32))
    fitness = np.ascontiguousarray(np.asarray(fitness, dtype=np.float64))
    w = opevo_space_width(space)
    assert parents.ndim == 2 and parents.shape == (fitness.size, w)
    out = np.empty(w, dtype=np.int32)
    _check(lib.opevo_recombine(space, _ip(parents), _dp(fitness), fitness.size, rng, _ip(out)))
    return out


def opevo_tuner_create(space, lambda_: int, rho: int, q: float, seed: int):
    h = _vp()
    _check(lib.opevo_tuner_create(space, lambda_, rho, q, seed & (2 ** 64 - 1), C.byref(h)))
    h._cap = max(lambda_, rho)
    h._width = opevo_space_width(space)
    return h


def opevo_tuner_destroy(tuner) -> None:
    _check(lib.opevo_tuner_destroy(tuner))


def opevo_tuner_set_mutation(tuner, kind: int) -> None:
    _check(lib.opevo_tuner_set_mutation(tuner, kind))


def opevo_tuner_ask(tuner, max_n: int = 0) -> np.ndarray:
    out = np.empty((tuner._cap, tuner._width), dtype=np.int32)
    n = C.c_int()
    _check(lib.opevo_tuner_ask(tuner, _ip(out), max_n, C.byref(n)))
    return out[:n.value].copy()


def opevo_tuner_tell(tuner, cfgs, fitness) -> None:
    cfgs = np.ascontiguousarray(np.asarray(cfgs, dtype=np.int32)).reshape(-1, tuner._width)
    fitness = np.ascontiguousarray(np.asarray(fitness, dtype=np.float64).ravel())
    assert cfgs.shape[0] == fitness.size
    _check(lib.opevo_tuner_tell(tuner, _ip(cfgs), _dp(fitness), fitness.size))


def opevo_tuner_num_trials(tuner) -> int:
    n = C.c_int()
    _check(lib.opevo_tuner_num_trials(tuner, C.byref(n)))
    return n.value


def opevo_tuner_best(tuner) -> Tuple[np.ndarray, float, int]:
    cfg = np.empty(tuner._width, dtype=np.int32)
    f, t = C.c_double(), C.c_int()
    _check(lib.opevo_tuner_best(tuner, _ip(cfg), C.byref(f), C.byref(t)))
    return cfg, f.value, t.value


def opevo_tuner_history(tuner) -> Tuple[np.ndarray, np.ndarray]:
    n = opevo_tuner_num_trials(tuner)
    cfgs = np.empty((max(n, 1), tuner._width), dtype=np.int32)
    fit = np.empty(max(n, 1), dtype=np.float64)
    got = C.c_int()
    _check(lib.opevo_tuner_history(tuner, _ip(cfgs), _dp(fit), max(n, 1), C.byref(got)))
    return cfgs[:n].copy(), fit[:n].copy()


# -------------------------------------------------------------------------- operators
def opevo_op_create(kind: int, dims: Sequence[int], in_dtype: int):
    arr = (C.c_int64 * len(dims))(*[int(d) for d in dims])
    h = _vp()
    _check(lib.opevo_op_create(kind, arr, len(dims), in_dtype, C.byref(h)))
    return h


def opevo_op_destroy(op) -> None:
    _check(lib.opevo_op_destroy(op))


def opevo_op_flops(op) -> float:
    v = C.c_double()
    _check(lib.opevo_op_flops(op, C.byref(v)))
    return v.value


def opevo_op_bytes(op) -> float:
    v = C.c_double()
    _check(lib.opevo_op_bytes(op, C.byref(v)))
    return v.value


def opevo_op_sizes(op) -> Tuple[int, int, int]:
    a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
    _check(lib.opevo_op_sizes(op, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def opevo_op_space(op, variant: int):
    h = _vp()
    _check(lib.opevo_op_space(op, variant, C.byref(h)))
    return h


def opevo_compile_pool_start(n_workers: int) -> int:
    n = C.c_int()
    _check(lib.opevo_compile_pool_start(n_workers, C.byref(n)))
    return n.value


def opevo_compile_pool_stop() -> None:
    _check(lib.opevo_compile_pool_stop())


def opevo_compile_pool_deadline(seconds: float) -> None:
    _check(lib.opevo_compile_pool_deadline(seconds))


def opevo_compile_pool_kind() -> int:
    k = C.c_int()
    _check(lib.opevo_compile_pool_kind(C.byref(k)))
    return k.value


def opevo_code_cache_configure(directory=None, max_memory_bytes: int = -1) -> None:
    _check(lib.opevo_code_cache_configure(directory.encode() if directory else None, max_memory_bytes))


def opevo_code_cache_clear() -> None:
    _check(lib.opevo_code_cache_clear())


def opevo_code_cache_stats() -> dict:
    v = [C.c_int64() for _ in range(5)]
    _check(lib.opevo_code_cache_stats(*[C.byref(x) for x in v]))
    return dict(zip(("hits", "disk_hits", "misses", "entries", "bytes"), (x.value for x in v)))


def opevo_kernel_plan(op, variant: int, cfg) -> opevo_plan:
    cfg = _cfg(cfg)
    plan = opevo_plan()
    _check(lib.opevo_kernel_plan(op, variant, _ip(cfg), C.byref(plan)))
    return plan


def opevo_kernel_defines(op, variant: int, cfg) -> str:
    cfg = _cfg(cfg)
    buf = C.create_string_buffer(4096)
    _check(lib.opevo_kernel_defines(op, variant, _ip(cfg), buf, 4096))
    return buf.value.decode()


def opevo_kernel_build(op, variant: int, cfg):
    """Returns (kernel handle, compile_ms); raises OpevoError (status E_INVALID for an invalid
    configuration, E_HIPRTC for a compile failure)."""
    cfg = _cfg(cfg)
    h, ms = _vp(), C.c_double()
    _check(lib.opevo_kernel_build(op, variant, _ip(cfg), C.byref(h), C.byref(ms)))
    return h, ms.value


def opevo_kernel_destroy(kernel) -> None:
    _check(lib.opevo_kernel_destroy(kernel))


def opevo_kernel_code_size(kernel) -> int:
    v = C.c_size_t()
    _check(lib.opevo_kernel_code_size(kernel, C.byref(v)))
    return v.value


def opevo_kernel_resources(kernel) -> dict:
    v, s, sp, l = C.c_int(), C.c_int(), C.c_int(), C.c_int()
    _check(lib.opevo_kernel_resources(kernel, C.byref(v), C.byref(s), C.byref(sp), C.byref(l)))
    return {"vgprs": v.value, "sgprs": s.value, "spill_bytes": sp.value, "static_lds": l.value}


def opevo_kernel_launch(kernel, a: int, b: int, c: int, stream: int = 0) -> None:
    _check(lib.opevo_kernel_launch(kernel, a, b, c, stream))


def opevo_kernel_time(kernel, a: int, b: int, c: int, stream: int = 0, warmup: int = 3,
                      launches_per_sample: int = 0, samples: int = 5, timeout_ms: float = 0.0,
                      warmup_ms: float = 25.0) -> Tuple[float, np.ndarray]:
    med = C.c_double()
    per = np.empty(samples, dtype=np.float64)
    _check(lib.opevo_kernel_time(kernel, a, b, c, stream, warmup, warmup_ms, launches_per_sample, samples, timeout_ms,
                                 C.byref(med), _dp(per)))
    return med.value, per


def opevo_mfma_ceiling(in_dtype: int = OPEVO_BF16, stream: int = 0, random_data: bool = True) -> float:
    v = C.c_double()
    _check(lib.opevo_mfma_ceiling(in_dtype, 1 if random_data else 0, stream, C.byref(v)))
    return v.value


def opevo_mfma_ceiling_atom(in_dtype: int = OPEVO_BF16, stream: int = 0, random_data: bool = True, atom: int = 32) -> float:
    v = C.c_double()
    _check(lib.opevo_mfma_ceiling_atom(in_dtype, 1 if random_data else 0, atom, stream, C.byref(v)))
    return v.value


def opevo_compare_f32(c: int, ref: int, n: int, stream: int = 0) -> Tuple[float, float]:
    mx, fro = C.c_double(), C.c_double()
    _check(lib.opevo_compare_f32(c, ref, n, stream, C.byref(mx), C.byref(fro)))
    return mx.value, fro.value


def opevo_compare_f32_static(c: int, ref: int, n: int, stream: int, result: int) -> None:
    """`result` is a DEVICE pointer to two doubles; nothing is copied back and nothing synchronises."""
    _check(lib.opevo_compare_f32_static(c, ref, n, stream, result))


def opevo_compare_rows_f32(c: int, ref_rows: int, row_index: int, n_rows: int, row_len: int,
                           stream: int = 0) -> Tuple[float, float]:
    mx, fro = C.c_double(), C.c_double()
    _check(lib.opevo_compare_rows_f32(c, ref_rows, row_index, n_rows, row_len, stream, C.byref(mx), C.byref(fro)))
    return mx.value, fro.value


def opevo_tune(op, variant: int, a: int, b: int, c: int, ref: Optional[int] = None, stream: int = 0,
               ref_row_index: Optional[int] = None, n_ref_rows: int = 0, ref_row_len: int = 0,
               trials: int = 500, lambda_: int = 8, rho: int = 8, q: float = 0.5, seed: int = 0,
               compile_threads: int = 8, warmup: int = 3, launches_per_sample: int = 0, samples: int = 5,
               warmup_ms: float = 25.0, trial_timeout_ms: float = 0.0, tol_max_scaled: float = 2e-2, tol_rel_fro: float = 5e-3,
               progress_every: int = 0, mutation: int = 0, speculate_threads: int = 0) -> dict:
    """Runs Alg. 1 on the GPU; returns the result struct fields, the best configuration and the
    per-trial logs as numpy arrays."""
    space = opevo_op_space(op, variant)
    try:
        w = opevo_space_width(space)
    finally:
        opevo_space_destroy(space)
    logs = {"cfg": np.zeros((trials, w), dtype=np.int32), "fitness": np.zeros(trials),
            "status": np.zeros(trials, dtype=np.int32), "compile_ms": np.zeros(trials),
            "run_ms": np.zeros(trials), "wall_s": np.zeros(trials)}
    args = opevo_tune_args(a=a, b=b, c=c, ref=ref, ref_row_index=ref_row_index, n_ref_rows=n_ref_rows,
                           ref_row_len=ref_row_len, stream=stream, trials=trials, lambda_=lambda_, rho=rho,
                           q=q, seed=seed, compile_threads=compile_threads, warmup=warmup,
                           launches_per_sample=launches_per_sample, samples=samples,
                           warmup_ms=warmup_ms, trial_timeout_ms=trial_timeout_ms, tol_max_scaled=tol_max_scaled, tol_rel_fro=tol_rel_fro,
                           cfg_log=_ip(logs["cfg"]), fitness_log=_dp(logs["fitness"]),
                           status_log=_ip(logs["status"]), compile_ms_log=_dp(logs["compile_ms"]),
                           run_ms_log=_dp(logs["run_ms"]), wall_s_log=_dp(logs["wall_s"]), progress_every=progress_every, mutation=mutation,
                           speculate_threads=speculate_threads)
    best = np.zeros(w, dtype=np.int32)
    res = opevo_tune_result()
    _check(lib.opevo_tune(op, variant, C.byref(args), _ip(best), C.byref(res)))
    out = {f: getattr(res, f) for f, _ in opevo_tune_result._fields_}
    n = res.n_trials
    out["best_cfg"] = best
    out["logs"] = {k: v[:n] for k, v in logs.items()}
    return out
