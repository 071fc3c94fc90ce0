"""ctypes binding of libsesgd.so: the same names as include/sesgd.h, argument marshalling
only.  Buffers are torch tensors (device memory) or raw integer addresses; nothing here
computes.  Importing this module without a built library raises: there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np
import torch  # noqa: F401  -- must come first: torch ships its own HIP runtime, and two
#                              HIP runtimes in one process cannot both open the GPU.  Loaded
#                              after torch, libsesgd.so binds to torch's runtime by soname.

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsesgd.so")

SE_OK = 0
SE_ERR_ARG = -1
SE_ERR_DIVISIBILITY = -2
SE_ERR_NULL = -3
SE_ERR_LAYOUT = -4
SE_ERR_UNSUPPORTED = -5
SE_ERR_HIP = -6
SE_MAX_WORKERS = 64

EXPORTS = ("se_plan", "se_plan_noalloc", "se_plan_device", "se_step", "se_step_bf16g", "se_ring_step",
           "se_ring_step_bf16g", "se_set_seed", "se_get_seed", "se_pitch", "se_step_bytes",
           "se_set_tuning", "se_get_tuning", "se_strerror", "se_last_error", "se_calib_copy", "se_calib_oneway",
           "se_step_ex", "se_global_average", "se_consensus", "se_comm_model", "se_layer_buckets")


SE_FLAG_GRAD_AVG = 1
TUNING_KNOBS = ("max_blocks_per_cu", "nontemporal", "cooperative", "coop_tiles",
                "cache_resident_mib", "split", "split_scratch_mib", "split_sub_tiles",
                "split_cap_reduce", "split_cap_finish", "split_finish_rows", "batch_rows",
                "unaligned_wide")


class SesgdError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"sesgd error {code}: {text}")
        self.code = code


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_2007_00433_amd.build` "
                          "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    runtimes = set()
    with open("/proc/self/maps") as maps:
        for line in maps:
            if "libamdhip64" in line:
                runtimes.add(line.split()[-1])
    if len(runtimes) > 1:
        raise ImportError(f"two HIP runtimes are loaded in this process: {sorted(runtimes)}")
    i32, i64, u64 = ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
    vp, f32, cp = ctypes.c_void_p, ctypes.c_float, ctypes.c_char_p
    lib.se_plan.restype = i32
    lib.se_plan.argtypes = [i32, i32, i64, vp, vp]
    lib.se_plan_noalloc.restype = i32
    lib.se_plan_noalloc.argtypes = [i32, i32, i64, vp, vp]
    lib.se_plan_device.restype = i32
    lib.se_plan_device.argtypes = [i32, i32, i64, vp, vp, vp]
    for name in ("se_step", "se_step_bf16g"):
        fn = getattr(lib, name)
        fn.restype = i32
        fn.argtypes = [vp, vp, vp, vp, i32, i32, i32, i64, f32, f32, vp]
    for name in ("se_ring_step", "se_ring_step_bf16g"):
        fn = getattr(lib, name)
        fn.restype = i32
        fn.argtypes = [vp, vp, vp, vp, i32, i32, f32, f32, vp]
    lib.se_set_seed.restype = i32
    lib.se_set_seed.argtypes = [u64]
    lib.se_get_seed.restype = u64
    lib.se_get_seed.argtypes = []
    lib.se_pitch.restype = i64
    lib.se_pitch.argtypes = [i64]
    lib.se_step_bytes.restype = i64
    lib.se_step_bytes.argtypes = [i64, i32, i32, i32]
    lib.se_set_tuning.restype = i32
    lib.se_set_tuning.argtypes = [cp, i32]
    lib.se_get_tuning.restype = i32
    lib.se_get_tuning.argtypes = [cp]
    lib.se_step_ex.restype = i32
    lib.se_step_ex.argtypes = [vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i64, f32, f32, f32,
                               ctypes.c_uint, vp]
    lib.se_global_average.restype = i32
    lib.se_global_average.argtypes = [vp, vp, i32, i32, vp]
    lib.se_consensus.restype = i32
    lib.se_consensus.argtypes = [vp, vp, i32, i32, vp, vp]
    lib.se_comm_model.restype = i32
    lib.se_comm_model.argtypes = [vp, i32, i32, i32, i32, ctypes.c_double, ctypes.c_double,
                                  vp, vp, vp, vp]
    lib.se_layer_buckets.restype = i32
    lib.se_layer_buckets.argtypes = [vp, i32, i64, vp, i32, vp]
    lib.se_calib_copy.restype = i32
    lib.se_calib_copy.argtypes = [vp, vp, i64, vp]
    lib.se_calib_oneway.restype = i32
    lib.se_calib_oneway.argtypes = [vp, vp, i64, i32, vp]
    lib.se_strerror.restype = cp
    lib.se_strerror.argtypes = [i32]
    lib.se_last_error.restype = cp
    lib.se_last_error.argtypes = []
    return lib


lib = _load()


def _ptr(buf) -> Optional[int]:
    """Address of a torch tensor / numpy array, an int passed through, or None."""
    if buf is None:
        return None
    if isinstance(buf, int):
        return buf
    if hasattr(buf, "data_ptr"):
        return int(buf.data_ptr())
    if isinstance(buf, np.ndarray):
        return int(buf.ctypes.data)
    raise TypeError(f"cannot take the address of {type(buf)}")


def _rows(buf, n: int, pitch: int, elem_bytes: int, what: str) -> Optional[int]:
    """Address of a device buffer of n rows of pitch elements.  The C ABI sees addresses only
    and cannot know how much memory stands behind them, so a torch tensor is checked here for
    device, contiguity, element size and length before its address is taken (a kernel that
    runs past an allocation faults the GPU).  Integers and None pass through."""
    if buf is not None and not isinstance(buf, int) and hasattr(buf, "data_ptr"):
        if not buf.is_cuda:
            raise ValueError(f"{what} must be a device tensor")
        if not buf.is_contiguous():
            raise ValueError(f"{what} must be contiguous")
        if buf.element_size() != elem_bytes:
            raise ValueError(f"{what} must have {elem_bytes}-byte elements, not {buf.dtype}")
        if n > 0 and pitch > 0 and buf.numel() < n * pitch:
            raise ValueError(f"{what} holds {buf.numel()} elements, fewer than n * pitch = {n * pitch}")
    return _ptr(buf)


def _offsets(layer_offsets: Sequence[int]) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(layer_offsets, dtype=np.int64))


def _stream(stream) -> Optional[int]:
    """hipStream_t of a torch stream or an integer handle; None means torch's current stream
    (not HIP's null stream, with which torch's side streams do not synchronise)."""
    if stream is None:
        if not torch.cuda.is_available():
            return None
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None      # torch.cuda.Stream


def check(code: int) -> None:
    if code != SE_OK:
        text = lib.se_strerror(code).decode()
        if code == SE_ERR_HIP:
            text += ": " + lib.se_last_error().decode()
        raise SesgdError(code, text)


def se_strerror(code: int) -> str:
    return lib.se_strerror(code).decode()


def se_last_error() -> str:
    return lib.se_last_error().decode()


def se_set_seed(seed: int) -> None:
    check(lib.se_set_seed(seed & 0xFFFFFFFFFFFFFFFF))


def se_get_seed() -> int:
    return int(lib.se_get_seed())


def se_pitch(P: int) -> int:
    return int(lib.se_pitch(P))


def se_step_bytes(columns: int, n: int, grad_elem_bytes: int = 4, has_momentum: bool = True) -> int:
    return int(lib.se_step_bytes(columns, n, grad_elem_bytes, int(has_momentum)))


def se_set_tuning(name: str, value: int) -> None:
    check(lib.se_set_tuning(name.encode(), value))


def se_get_tuning(name: str) -> int:
    return int(lib.se_get_tuning(name.encode()))


def se_calib_copy(dst, src, nbytes: int, stream=None) -> None:
    for buf, what in ((dst, "dst"), (src, "src")):
        if hasattr(buf, "data_ptr") and buf.numel() * buf.element_size() < nbytes:
            raise ValueError(f"{what} is shorter than {nbytes} bytes")
    check(lib.se_calib_copy(_rows(dst, 0, 0, dst.element_size() if hasattr(dst, "element_size") else 1, "dst"),
                            _rows(src, 0, 0, src.element_size() if hasattr(src, "element_size") else 1, "src"),
                            nbytes, _stream(stream)))


def se_calib_oneway(dst, src, nbytes: int, direction: int, stream=None) -> None:
    """direction 1: read nbytes of src; direction 2: overwrite nbytes of dst with a pattern."""
    for buf, what in ((dst, "dst"), (src, "src")):
        if hasattr(buf, "data_ptr") and buf.numel() * buf.element_size() < nbytes:
            raise ValueError(f"{what} is shorter than {nbytes} bytes")
    check(lib.se_calib_oneway(_rows(dst, 0, 0, dst.element_size() if hasattr(dst, "element_size") else 1, "dst"),
                              _rows(src, 0, 0, src.element_size() if hasattr(src, "element_size") else 1, "src"),
                              nbytes, direction, _stream(stream)))


def se_plan_raw(n, group_size, it, group_of_ptr, members_ptr) -> int:
    return int(lib.se_plan(n, group_size, it, group_of_ptr, members_ptr))


def se_plan(n: int, group_size: int, it: int, want_members: bool = True):
    """Returns (group_of[n], members[n/group_size, group_size]) as int32 numpy arrays."""
    group_of = np.full(max(n, 1), -1, np.int32)
    members = np.full(max(n, 1), -1, np.int32) if want_members else None
    check(lib.se_plan(n, group_size, it, group_of.ctypes.data,
                      members.ctypes.data if want_members else None))
    if want_members:
        return group_of[:n], members[:n].reshape(n // group_size, group_size)
    return group_of[:n], None


def se_plan_noalloc(n: int, group_size: int, it: int, want_members: bool = True):
    """se_plan through the entry point that allocates no device memory."""
    group_of = np.full(max(n, 1), -1, np.int32)
    members = np.full(max(n, 1), -1, np.int32) if want_members else None
    check(lib.se_plan_noalloc(n, group_size, it, group_of.ctypes.data,
                              members.ctypes.data if want_members else None))
    if want_members:
        return group_of[:n], members[:n].reshape(n // group_size, group_size)
    return group_of[:n], None


def se_plan_noalloc_raw(n, group_size, it, group_of_ptr, members_ptr) -> int:
    return int(lib.se_plan_noalloc(n, group_size, it, group_of_ptr, members_ptr))


def se_plan_device(n: int, group_size: int, it: int, group_of_dev, members_dev=None, stream=None):
    check(lib.se_plan_device(n, group_size, it, _rows(group_of_dev, 1, n, 4, "group_of_dev"),
                             _rows(members_dev, 1, n, 4, "members_dev"), _stream(stream)))


def se_step_raw(fn_name, params, grads, momentum, layer_offsets, num_layers, n, group_size, it,
                lr, mu, stream) -> int:
    """Unchecked call returning the status code (for error-path tests)."""
    offs = None if layer_offsets is None else _offsets(layer_offsets)
    return int(getattr(lib, fn_name)(_ptr(params), _ptr(grads), _ptr(momentum),
                                     None if offs is None else offs.ctypes.data, num_layers,
                                     n, group_size, it, lr, mu, _stream(stream)))


def se_ring_step_raw(fn_name, params, grads, momentum, layer_offsets, num_layers, n, lr, mu,
                     stream) -> int:
    offs = None if layer_offsets is None else _offsets(layer_offsets)
    return int(getattr(lib, fn_name)(_ptr(params), _ptr(grads), _ptr(momentum),
                                     None if offs is None else offs.ctypes.data, num_layers,
                                     n, lr, mu, _stream(stream)))


def se_step(params, grads, momentum, layer_offsets, n: int, group_size: int, it: int,
            lr: float, mu: float, stream=None) -> None:
    offs = _offsets(layer_offsets)
    pitch = int(offs[-1])
    check(lib.se_step(_rows(params, n, pitch, 4, "params"), _rows(grads, n, pitch, 4, "grads"),
                      _rows(momentum, n, pitch, 4, "momentum"), offs.ctypes.data,
                      len(offs) - 1, n, group_size, it, lr, mu, _stream(stream)))


def se_step_bf16g(params, grads_bf16, momentum, layer_offsets, n: int, group_size: int, it: int,
                  lr: float, mu: float, stream=None) -> None:
    offs = _offsets(layer_offsets)
    pitch = int(offs[-1])
    check(lib.se_step_bf16g(_rows(params, n, pitch, 4, "params"),
                            _rows(grads_bf16, n, pitch, 2, "grads_bf16"),
                            _rows(momentum, n, pitch, 4, "momentum"), offs.ctypes.data,
                            len(offs) - 1, n, group_size, it, lr, mu, _stream(stream)))


def se_ring_step(params, grads, momentum, layer_offsets, n: int, lr: float, mu: float,
                 stream=None) -> None:
    offs = _offsets(layer_offsets)
    pitch = int(offs[-1])
    check(lib.se_ring_step(_rows(params, n, pitch, 4, "params"), _rows(grads, n, pitch, 4, "grads"),
                           _rows(momentum, n, pitch, 4, "momentum"), offs.ctypes.data,
                           len(offs) - 1, n, lr, mu, _stream(stream)))


def se_ring_step_bf16g(params, grads_bf16, momentum, layer_offsets, n: int, lr: float, mu: float,
                       stream=None) -> None:
    offs = _offsets(layer_offsets)
    pitch = int(offs[-1])
    check(lib.se_ring_step_bf16g(_rows(params, n, pitch, 4, "params"),
                                 _rows(grads_bf16, n, pitch, 2, "grads_bf16"),
                                 _rows(momentum, n, pitch, 4, "momentum"),
                                 offs.ctypes.data, len(offs) - 1, n, lr, mu, _stream(stream)))


def se_step_ex_raw(params, grads, grads_are_bf16, momentum, layer_offsets, num_layers, first_layer,
                   last_layer, n, group_size, it, lr, mu, weight_decay, flags, stream) -> int:
    offs = None if layer_offsets is None else _offsets(layer_offsets)
    return int(lib.se_step_ex(_ptr(params), _ptr(grads), int(grads_are_bf16), _ptr(momentum),
                              None if offs is None else offs.ctypes.data, num_layers, first_layer,
                              last_layer, n, group_size, it, lr, mu, weight_decay, flags,
                              _stream(stream)))


def se_step_ex(params, grads, momentum, layer_offsets, n: int, group_size: int, it: int,
               lr: float, mu: float, weight_decay: float = 0.0, flags: int = 0,
               first_layer: int = 0, last_layer: Optional[int] = None,
               grads_are_bf16: bool = False, stream=None) -> None:
    offs = _offsets(layer_offsets)
    pitch = int(offs[-1])
    last = len(offs) - 1 if last_layer is None else last_layer
    check(lib.se_step_ex(_rows(params, n, pitch, 4, "params"),
                         _rows(grads, n, pitch, 2 if grads_are_bf16 else 4, "grads"),
                         int(grads_are_bf16), _rows(momentum, n, pitch, 4, "momentum"),
                         offs.ctypes.data, len(offs) - 1, first_layer, last, n, group_size, it,
                         lr, mu, weight_decay, flags, _stream(stream)))


def se_global_average(params, layer_offsets, n: int, stream=None) -> None:
    offs = _offsets(layer_offsets)
    check(lib.se_global_average(_rows(params, n, int(offs[-1]), 4, "params"), offs.ctypes.data,
                                len(offs) - 1, n, _stream(stream)))


def se_consensus(params, layer_offsets, n: int, out_dev, stream=None) -> None:
    """out_dev: device tensor of two float64 (distance to the mean, sum of parameters)."""
    offs = _offsets(layer_offsets)
    check(lib.se_consensus(_rows(params, n, int(offs[-1]), 4, "params"), offs.ctypes.data,
                           len(offs) - 1, n, _rows(out_dev, 1, 2, 8, "out_dev"), _stream(stream)))


def se_layer_buckets_raw(layer_offsets, num_layers, min_elements, first_layer_ptr, capacity, num_ranges_ptr) -> int:
    offs = None if layer_offsets is None else _offsets(layer_offsets)
    return int(lib.se_layer_buckets(None if offs is None else offs.ctypes.data, num_layers, min_elements,
                                    first_layer_ptr, capacity, num_ranges_ptr))


def se_layer_buckets(layer_offsets, min_elements: int) -> list:
    """[(first_layer, last_layer), ...] in stepping order (back to front), for se_step_ex."""
    offs = _offsets(layer_offsets)
    L = len(offs) - 1
    first = np.zeros(max(L, 1), np.int32)
    count = ctypes.c_int(0)
    check(lib.se_layer_buckets(offs.ctypes.data, L, int(min_elements), first.ctypes.data, L,
                               ctypes.addressof(count)))
    ends = [L] + [int(f) for f in first[:count.value]]
    return [(int(first[i]), ends[i]) for i in range(count.value)]


def se_comm_model(layer_offsets, elem_bytes: int, n: int, groups: int, bandwidth: float,
                  latency: float) -> dict:
    offs = _offsets(layer_offsets)
    ring, sesgd = ctypes.c_double(), ctypes.c_double()
    rh, sh = ctypes.c_int64(), ctypes.c_int64()
    check(lib.se_comm_model(offs.ctypes.data, len(offs) - 1, elem_bytes, n, groups, bandwidth,
                            latency, ctypes.addressof(ring), ctypes.addressof(sesgd),
                            ctypes.addressof(rh), ctypes.addressof(sh)))
    return {"ring_seconds": ring.value, "sesgd_seconds": sesgd.value,
            "ring_handshakes": rh.value, "sesgd_handshakes": sh.value}
