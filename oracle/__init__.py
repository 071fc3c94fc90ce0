"""CPU oracle for the SESGD step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``se_oracle.c`` (plain C, fp32, fixed evaluation order) plus
``brute`` (exact rational arithmetic, definition level, tiny inputs only).

Only ``tests/``, the smoke check and the benchmark's CPU-baseline leg may import this
package.  It imports nothing from the GPU package and the GPU package imports nothing
from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "se_oracle.c")
_SO = os.path.join(_HERE, "libse_oracle.so")
_lib_handle = None
_lock = threading.Lock()

ORACLE_OK = 0
ORACLE_ERR_ARG = -1
ORACLE_ERR_DIVISIBILITY = -2


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc.  No contraction, no fast-math, no -march flags."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra",
               "-shared", "-fPIC", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def bind(path: str):
    """Load a build of se_oracle.c and declare its signatures."""
    lib = ctypes.CDLL(path)
    i64, u64, i32 = ctypes.c_int64, ctypes.c_uint64, ctypes.c_int
    vp, f32 = ctypes.c_void_p, ctypes.c_float
    lib.oracle_key.restype = ctypes.c_uint32
    lib.oracle_key.argtypes = [u64, i64, i32, i32]
    lib.oracle_plan.restype = i32
    lib.oracle_plan.argtypes = [u64, i32, i32, i64, vp, vp, vp, vp]
    lib.oracle_step.restype = i32
    lib.oracle_step.argtypes = [vp, vp, i32, vp, i64, i64, i64, i32, i32, u64, i64, f32, f32]
    lib.oracle_ring_step.restype = i32
    lib.oracle_ring_step.argtypes = [vp, vp, i32, vp, i64, i64, i64, i32, f32, f32]
    lib.oracle_step_ex.restype = i32
    lib.oracle_step_ex.argtypes = [vp, vp, i32, vp, i64, i64, i64, i32, i32, u64, i64, f32, f32, f32,
                                   ctypes.c_uint]
    lib.oracle_global_average.restype = i32
    lib.oracle_global_average.argtypes = [vp, i64, i64, i64, i32]
    lib.oracle_consensus.restype = i32
    lib.oracle_consensus.argtypes = [vp, i64, i64, i64, i32, vp]
    lib.oracle_ring_time.restype = ctypes.c_double
    lib.oracle_ring_time.argtypes = [ctypes.c_double, i32, ctypes.c_double, ctypes.c_double]
    lib.oracle_handshakes.restype = ctypes.c_long
    lib.oracle_handshakes.argtypes = [i32, i32]
    return lib


def _lib():
    global _lib_handle
    with _lock:
        if _lib_handle is None:
            build(force=False)
            _lib_handle = bind(_SO)
    return _lib_handle


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__(f"oracle error {code}")
        self.code = code


def key(seed: int, it: int, n: int, i: int) -> int:
    return int(_lib().oracle_key(seed, it, n, i))


def plan(n: int, m: int, it: int, seed: int = 0) -> dict:
    """Regrouping of n workers into n/m groups of m for iteration ``it``."""
    nn = max(n, 1)
    keys = np.zeros(nn, np.uint32)
    rank = np.zeros(nn, np.int32)
    group_of = np.zeros(nn, np.int32)
    members = np.zeros(nn, np.int32)
    rc = _lib().oracle_plan(seed, n, m, it, keys.ctypes.data, rank.ctypes.data,
                            group_of.ctypes.data, members.ctypes.data)
    if rc != ORACLE_OK:
        raise OracleError(rc)
    return {"keys": keys, "rank": rank, "group_of": group_of,
            "members": members.reshape(n // m, m)}


def _check_rows(a, n, name, dtypes):
    if not isinstance(a, np.ndarray) or a.ndim != 2 or a.shape[0] != n:
        raise ValueError(f"{name}: need a 2-D array with {n} rows")
    if a.dtype not in dtypes or not a.flags.c_contiguous:
        raise ValueError(f"{name}: need C-contiguous {dtypes}")


def _grad_args(grads, n):
    _check_rows(grads, n, "grads", (np.float32, np.uint16))
    return grads.ctypes.data, int(grads.dtype == np.uint16)


def step(params, grads, momentum, m: int, it: int, lr: float, mu: float,
         seed: int = 0, cols=None) -> None:
    """One SESGD iteration, in place.  params/momentum: float32 [n, pitch]; grads float32
    or uint16 (bf16 bit patterns) [n, pitch]; momentum may be None."""
    n, pitch = params.shape
    _check_rows(params, n, "params", (np.float32,))
    gptr, gbf = _grad_args(grads, n)
    if grads.shape != params.shape:
        raise ValueError("grads shape")
    mptr = None
    if momentum is not None:
        _check_rows(momentum, n, "momentum", (np.float32,))
        if momentum.shape != params.shape:
            raise ValueError("momentum shape")
        mptr = momentum.ctypes.data
    c0, c1 = (0, pitch) if cols is None else cols
    rc = _lib().oracle_step(params.ctypes.data, gptr, gbf, mptr, pitch, c0, c1,
                            n, m, seed, it, lr, mu)
    if rc != ORACLE_OK:
        raise OracleError(rc)


def ring_step(params, grads, momentum, lr: float, mu: float, cols=None) -> None:
    """One Ring-SGD (full mean-gradient) iteration, in place."""
    n, pitch = params.shape
    _check_rows(params, n, "params", (np.float32,))
    gptr, gbf = _grad_args(grads, n)
    mptr = None
    if momentum is not None:
        _check_rows(momentum, n, "momentum", (np.float32,))
        mptr = momentum.ctypes.data
    c0, c1 = (0, pitch) if cols is None else cols
    rc = _lib().oracle_ring_step(params.ctypes.data, gptr, gbf, mptr, pitch, c0, c1, n, lr, mu)
    if rc != ORACLE_OK:
        raise OracleError(rc)


FLAG_GRAD_AVG = 1


def step_ex(params, grads, momentum, m: int, it: int, lr: float, mu: float, wd: float = 0.0,
            flags: int = 0, seed: int = 0, cols=None) -> None:
    """General step: optional weight decay; flags=FLAG_GRAD_AVG selects the uncorrected
    variant that averages gradients instead of parameters."""
    n, pitch = params.shape
    _check_rows(params, n, "params", (np.float32,))
    gptr, gbf = _grad_args(grads, n)
    mptr = None
    if momentum is not None:
        _check_rows(momentum, n, "momentum", (np.float32,))
        mptr = momentum.ctypes.data
    c0, c1 = (0, pitch) if cols is None else cols
    rc = _lib().oracle_step_ex(params.ctypes.data, gptr, gbf, mptr, pitch, c0, c1, n, m, seed, it,
                               lr, mu, wd, flags)
    if rc != ORACLE_OK:
        raise OracleError(rc)


def global_average(params, cols=None) -> None:
    n, pitch = params.shape
    _check_rows(params, n, "params", (np.float32,))
    c0, c1 = (0, pitch) if cols is None else cols
    rc = _lib().oracle_global_average(params.ctypes.data, pitch, c0, c1, n)
    if rc != ORACLE_OK:
        raise OracleError(rc)


def consensus(params, cols=None):
    """(sum over workers and columns of (x - xbar)^2, sum of all parameters), float64."""
    n, pitch = params.shape
    _check_rows(params, n, "params", (np.float32,))
    c0, c1 = (0, pitch) if cols is None else cols
    out = np.zeros(2, np.float64)
    rc = _lib().oracle_consensus(params.ctypes.data, pitch, c0, c1, n, out.ctypes.data)
    if rc != ORACLE_OK:
        raise OracleError(rc)
    return float(out[0]), float(out[1])


def ring_time(layer_bytes: float, workers: int, nu: float, t_tau: float) -> float:
    return float(_lib().oracle_ring_time(layer_bytes, workers, nu, t_tau))


def handshakes(layers: int, workers: int) -> int:
    return int(_lib().oracle_handshakes(layers, workers))


def step_threaded(params, grads, momentum, m, it, lr, mu, seed=0, threads=1, ring=False):
    """The same oracle function called on disjoint column blocks from ``threads`` host
    threads (columns are independent; ctypes drops the GIL during the call)."""
    n, pitch = params.shape
    threads = max(1, min(int(threads), max(pitch, 1)))
    bounds = [pitch * q // threads for q in range(threads + 1)]
    errs = []

    def work(q):
        try:
            if ring:
                ring_step(params, grads, momentum, lr, mu, cols=(bounds[q], bounds[q + 1]))
            else:
                step(params, grads, momentum, m, it, lr, mu, seed, cols=(bounds[q], bounds[q + 1]))
        except Exception as exc:  # pragma: no cover
            errs.append(exc)

    ts = [threading.Thread(target=work, args=(q,)) for q in range(threads)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    if errs:
        raise errs[0]
