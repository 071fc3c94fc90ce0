"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2007_00433_amd import binding as se

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-NULL, 16-byte aligned address that is never dereferenced:
                        # every call below fails validation before any HIP call


def header_symbols(names=("sesgd.h", "sesgd_tuning.h")):
    found = set()
    for name in names:
        text = open(os.path.join(ROOT, "include", name)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        found |= set(re.findall(r"\b(se_[a-z0-9_]+)\s*\(", text))
    return sorted(found)


def test_library_exports_every_declared_symbol():
    names = header_symbols()
    assert "se_plan" in names and "se_step" in names and "se_ring_step" in names
    lib = ctypes.CDLL(se.LIB_PATH)
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(se.EXPORTS) == names
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["sesgd.h", "sesgd_tuning.h"]
    # the method's header carries no measurement scaffolding
    scaffolding = ["se_calib_copy", "se_calib_oneway", "se_get_tuning", "se_set_tuning"]
    assert header_symbols(("sesgd_tuning.h",)) == scaffolding
    assert not set(header_symbols(("sesgd.h",))) & set(scaffolding)
    for name in names:                      # the Python binding carries the same names
        assert hasattr(se, name), name


def test_error_strings():
    for code in range(0, -7, -1):
        assert se.se_strerror(code) and "unknown" not in se.se_strerror(code)
    assert "unknown" in se.se_strerror(-99)


def test_pitch_and_bytes():
    assert se.se_pitch(0) == 0 and se.se_pitch(1) == 1024 and se.se_pitch(1024) == 1024
    assert se.se_pitch(5106) == 5120 and se.se_pitch(25557032) == 25558016
    assert se.se_pitch(-1) == -1
    assert se.se_step_bytes(25557032, 16, 4, True) == 8178250240      # headline config
    assert se.se_step_bytes(109482240, 64, 2, True) == 126123540480   # bf16 gradients
    assert se.se_step_bytes(5106, 4, 4, False) == 245088
    assert se.se_step_bytes(10, 4, 3, True) == -1


def test_seed_and_tuning_state():
    se.se_set_seed(12345678901234567890)
    assert se.se_get_seed() == 12345678901234567890
    se.se_set_seed(0)
    assert len(se.TUNING_KNOBS) == 13
    for name, good, bad in (("nontemporal", 0, 3),
                            ("max_blocks_per_cu", 2, 33), ("cooperative", 1, -1),
                            ("cache_resident_mib", 0, -1), ("coop_tiles", 3, -1),
                            ("split", 0, 2), ("split_scratch_mib", 16, 0), ("split_sub_tiles", 64, -1),
                            ("split_cap_reduce", 3, 33), ("split_cap_finish", 0, -2),
                            ("split_finish_rows", 16, 65), ("batch_rows", 2, 9),
                            ("unaligned_wide", 0, 2)):
        assert name in se.TUNING_KNOBS
        old = se.se_get_tuning(name)
        se.se_set_tuning(name, good)
        assert se.se_get_tuning(name) == good
        with pytest.raises(se.SesgdError):
            se.se_set_tuning(name, bad)
        se.se_set_tuning(name, old)
    with pytest.raises(se.SesgdError):
        se.se_set_tuning("no_such_knob", 1)


OFFS = [0, 100, 228]


def step_rc(fn="se_step", params=FAKE, grads=FAKE + (1 << 20), momentum=FAKE + (2 << 20),
            offs=OFFS, num_layers=None, n=4, m=2, it=0, lr=0.1, mu=0.9):
    nl = (len(offs) - 1) if num_layers is None and offs is not None else (num_layers or 0)
    return se.se_step_raw(fn, params, grads, momentum, offs, nl, n, m, it, lr, mu, None)


@pytest.mark.parametrize("fn", ["se_step", "se_step_bf16g"])
def test_step_rejects_bad_arguments_without_a_device(fn):
    assert step_rc(fn, n=0) == se.SE_ERR_ARG
    assert step_rc(fn, m=0) == se.SE_ERR_ARG
    assert step_rc(fn, m=8) == se.SE_ERR_ARG
    assert step_rc(fn, it=-1) == se.SE_ERR_ARG
    assert step_rc(fn, num_layers=-1) == se.SE_ERR_ARG
    assert step_rc(fn, n=6, m=4) == se.SE_ERR_DIVISIBILITY
    assert step_rc(fn, params=None) == se.SE_ERR_NULL
    assert step_rc(fn, grads=None) == se.SE_ERR_NULL
    assert step_rc(fn, offs=None) == se.SE_ERR_NULL
    assert step_rc(fn, momentum=None, mu=0.9) == se.SE_ERR_NULL
    assert step_rc(fn, offs=[1, 100, 228]) == se.SE_ERR_LAYOUT
    assert step_rc(fn, offs=[0, 300, 228]) == se.SE_ERR_LAYOUT
    assert step_rc(fn, n=128, m=2) == se.SE_ERR_UNSUPPORTED
    assert step_rc(fn, offs=[0, 1 << 30]) == se.SE_ERR_UNSUPPORTED
    # overlapping buffers: 4 rows * 228 elements * 4 bytes = 3648 bytes each
    assert step_rc(fn, grads=FAKE + 3000) == se.SE_ERR_LAYOUT
    assert step_rc(fn, momentum=FAKE + 3644) == se.SE_ERR_LAYOUT
    assert step_rc(fn, momentum=FAKE) == se.SE_ERR_LAYOUT
    # misaligned element pointers
    assert step_rc(fn, params=FAKE + 2) == se.SE_ERR_LAYOUT
    assert step_rc(fn, grads=FAKE + (1 << 20) + 1) == se.SE_ERR_LAYOUT
    # an empty model is a no-op, not an error (nothing is launched)
    assert step_rc(fn, offs=[0]) == se.SE_OK
    assert step_rc(fn, offs=[0, 0, 0]) == se.SE_OK


@pytest.mark.parametrize("fn", ["se_ring_step", "se_ring_step_bf16g"])
def test_ring_rejects_bad_arguments_without_a_device(fn):
    def rc(params=FAKE, grads=FAKE + (1 << 20), momentum=FAKE + (2 << 20), offs=OFFS, n=4, mu=0.9,
           num_layers=None):
        nl = (len(offs) - 1) if num_layers is None and offs is not None else (num_layers or 0)
        return se.se_ring_step_raw(fn, params, grads, momentum, offs, nl, n, 0.1, mu, None)
    assert rc(n=0) == se.SE_ERR_ARG
    assert rc(num_layers=-2) == se.SE_ERR_ARG
    assert rc(params=None) == se.SE_ERR_NULL
    assert rc(momentum=None) == se.SE_ERR_NULL
    assert rc(offs=[0, 5, 4]) == se.SE_ERR_LAYOUT
    assert rc(grads=FAKE + 16) == se.SE_ERR_LAYOUT
    assert rc(n=65) == se.SE_ERR_UNSUPPORTED
    assert rc(offs=[0]) == se.SE_OK


def test_plan_rejects_bad_arguments_without_a_device():
    out = np.zeros(64, np.int32)
    p = out.ctypes.data
    assert se.se_plan_raw(0, 1, 0, p, p) == se.SE_ERR_ARG
    assert se.se_plan_raw(4, 0, 0, p, p) == se.SE_ERR_ARG
    assert se.se_plan_raw(4, 5, 0, p, p) == se.SE_ERR_ARG
    assert se.se_plan_raw(4, 2, -3, p, p) == se.SE_ERR_ARG
    assert se.se_plan_raw(6, 4, 0, p, p) == se.SE_ERR_DIVISIBILITY
    assert se.se_plan_raw(4, 2, 0, None, p) == se.SE_ERR_NULL
    assert se.se_plan_raw(128, 2, 0, p, p) == se.SE_ERR_UNSUPPORTED
    assert not out.any()                     # nothing written on error


def test_extended_calls_reject_bad_arguments_without_a_device():
    G, V = FAKE + (1 << 20), FAKE + (2 << 20)

    def ex(first=0, last=2, flags=0, n=4, m=2, offs=OFFS, grads=G, bf16=0):
        return se.se_step_ex_raw(FAKE, grads, bf16, V, offs, len(offs) - 1, first, last, n, m, 0,
                                 0.1, 0.9, 0.0, flags, None)
    assert ex(first=-1) == se.SE_ERR_ARG
    assert ex(first=2, last=1) == se.SE_ERR_ARG
    assert ex(last=3) == se.SE_ERR_ARG
    assert ex(flags=2) == se.SE_ERR_ARG
    assert ex(n=6, m=4) == se.SE_ERR_DIVISIBILITY
    assert ex(grads=None) == se.SE_ERR_NULL
    assert ex(grads=G + 2, bf16=0) == se.SE_ERR_LAYOUT
    assert ex(first=1, last=1) == se.SE_OK            # empty layer range: nothing to launch
    offs = np.asarray(OFFS, np.int64)
    assert se.lib.se_global_average(None, offs.ctypes.data, 2, 4, None) == se.SE_ERR_NULL
    assert se.lib.se_global_average(FAKE, offs.ctypes.data, 2, 0, None) == se.SE_ERR_ARG
    assert se.lib.se_global_average(FAKE, offs.ctypes.data, 2, 65, None) == se.SE_ERR_UNSUPPORTED
    assert se.lib.se_consensus(FAKE, offs.ctypes.data, 2, 4, None, None) == se.SE_ERR_NULL
    assert se.lib.se_consensus(FAKE, offs.ctypes.data, 2, 4, FAKE + 100, None) == se.SE_ERR_LAYOUT
    assert se.lib.se_consensus(FAKE, offs.ctypes.data, 2, 4, V + 4, None) == se.SE_ERR_LAYOUT
    assert se.lib.se_consensus(None, offs.ctypes.data, 2, 4, V, None) == se.SE_ERR_NULL


def test_comm_model_matches_the_oracle_and_the_paper():
    """Host-only calculator (no device): Sec. 2.2 ring cost per layer, Sec. 2.3's 1500
    handshakes for 50 layers on 16 workers, against the oracle's independent function."""
    import oracle
    from paper_2007_00433_amd import workloads as wl
    fifty = list(range(0, 51 * 1000, 1000))
    r = se.se_comm_model(fifty, 4, 16, 4, 125e6, 1e-4)
    assert r["ring_handshakes"] == 1500 == oracle.handshakes(50, 16)
    assert r["sesgd_handshakes"] == 300 == oracle.handshakes(50, 4)
    w = wl.WORKLOADS["resnet50"]
    offs = w.layer_offsets()
    for lat in (1e-4, 5e-3):
        r = se.se_comm_model(offs, 4, 16, 4, 125e6, lat)
        ring = sum(oracle.ring_time(4.0 * s, 16, 125e6, lat) for s in w.sizes)
        ses = sum(oracle.ring_time(4.0 * s, 4, 125e6, lat) for s in w.sizes)
        assert abs(r["ring_seconds"] - ring) <= 1e-12 * ring
        assert abs(r["sesgd_seconds"] - ses) <= 1e-12 * ses
        assert r["sesgd_seconds"] < r["ring_seconds"]
    offs_arr = np.asarray(offs, np.int64)
    assert se.lib.se_comm_model(offs_arr.ctypes.data, len(offs) - 1, 4, 16, 3, 1e9, 0.0,
                                None, None, None, None) == se.SE_ERR_DIVISIBILITY
    assert se.lib.se_comm_model(offs_arr.ctypes.data, len(offs) - 1, 4, 16, 4, 0.0, 0.0,
                                None, None, None, None) == se.SE_ERR_ARG
    assert se.lib.se_comm_model(None, 1, 4, 16, 4, 1e9, 0.0, None, None, None, None) == se.SE_ERR_NULL
    assert se.lib.se_comm_model(offs_arr.ctypes.data, len(offs) - 1, 4, 16, 4, 1e9, 0.0,
                                None, None, None, None) == se.SE_OK


def test_layer_buckets_cover_the_model_back_to_front():
    """Host-only helper for layer-range stepping (Sec. 2.1): ranges are consecutive, run from the
    last layer to the first, cover every layer once, hold at least min_elements each except the
    front-most one, and are as small as that allows (dropping the first layer of a range would
    take it below min_elements)."""
    import ctypes
    from paper_2007_00433_amd import workloads as wl
    rng = np.random.default_rng(3)
    models = [list(w.sizes) for w in wl.WORKLOADS.values()]
    models += [list(rng.integers(0, 5000, size=int(L))) for L in rng.integers(1, 60, size=30)]
    models += [[0, 0, 0], [7], [0], [5, 0, 0, 5], []]
    for sizes in models:
        offs = np.concatenate([[0], np.cumsum(np.asarray(sizes, np.int64))]).astype(np.int64)
        L = len(sizes)
        for min_elems in (1, 100, 4096, 1 << 20, 1 << 40):
            ranges = se.se_layer_buckets(offs, min_elems)
            if L == 0:
                assert ranges == []
                continue
            assert ranges[0][1] == L and ranges[-1][0] == 0
            for (f0, l0), (f1, l1) in zip(ranges, ranges[1:]):
                assert l1 == f0                                   # consecutive, back to front
            for q, (f, l) in enumerate(ranges):
                assert 0 <= f < l <= L
                size = int(offs[l] - offs[f])
                if q < len(ranges) - 1:
                    assert size >= min_elems
                    assert int(offs[l] - offs[f + 1]) < min_elems  # closed as early as possible
            if min_elems == 1 << 40:
                assert ranges == [(0, L)]
    # the ResNet-50 shape in ranges of 2^20 elements: 19 calls instead of 161
    w = wl.WORKLOADS["resnet50"]
    assert len(se.se_layer_buckets(w.layer_offsets(), 1 << 20)) == 19
    assert len(se.se_layer_buckets(w.layer_offsets(), 1)) == 161
    # a hand-checked case: sizes 10, 3, 4, 20, 1 with at least 5 per range
    assert se.se_layer_buckets([0, 10, 13, 17, 37, 38], 5) == [(3, 5), (1, 3), (0, 1)]
    # errors: nothing is written when the ranges do not fit
    offs = np.asarray([0, 10, 13, 17, 37, 38], np.int64)
    first = np.full(8, -7, np.int32)
    count = ctypes.c_int(-1)
    cnt = ctypes.addressof(count)
    assert se.se_layer_buckets_raw(offs, 5, 5, first.ctypes.data, 2, cnt) == se.SE_ERR_ARG
    assert count.value == 3 and (first == -7).all()
    assert se.se_layer_buckets_raw(offs, 5, 0, first.ctypes.data, 8, cnt) == se.SE_ERR_ARG
    assert se.se_layer_buckets_raw(offs, -1, 5, first.ctypes.data, 8, cnt) == se.SE_ERR_ARG
    assert se.se_layer_buckets_raw(None, 5, 5, first.ctypes.data, 8, cnt) == se.SE_ERR_NULL
    assert se.se_layer_buckets_raw(offs, 5, 5, None, 8, cnt) == se.SE_ERR_NULL
    assert se.se_layer_buckets_raw(offs, 5, 5, first.ctypes.data, 8, None) == se.SE_ERR_NULL
    assert se.se_layer_buckets_raw(np.asarray([0, 5, 3], np.int64), 2, 5, first.ctypes.data, 8, cnt) == se.SE_ERR_LAYOUT
    assert (first == -7).all()
    assert se.se_layer_buckets_raw(offs, 5, 5, first.ctypes.data, 3, cnt) == se.SE_OK
    assert list(first[:3]) == [3, 1, 0] and (first[3:] == -7).all()


def test_binding_checks_tensors_before_taking_their_address():
    """The checked wrappers refuse tensors the kernels would run past or misread (no GPU needed:
    a host tensor is refused first of all)."""
    import torch
    offs = [0, 8]
    host = torch.zeros(4, 8)
    with pytest.raises(ValueError, match="device tensor"):
        se.se_step(host, host, None, offs, 4, 2, 0, 0.1, 0.0)
    with pytest.raises(ValueError, match="device tensor"):
        se.se_global_average(host, offs, 4)

    class Fake:            # stands in for a device tensor on a box without one
        is_cuda = True
        dtype = "fake"
        def __init__(self, numel, elem=4, contiguous=True):
            self._n, self._e, self._c = numel, elem, contiguous
        def data_ptr(self): return 0x1000
        def is_contiguous(self): return self._c
        def element_size(self): return self._e
        def numel(self): return self._n

    with pytest.raises(ValueError, match="fewer than n \\* pitch"):
        se.se_step(Fake(31), Fake(32), None, offs, 4, 2, 0, 0.1, 0.0)
    with pytest.raises(ValueError, match="contiguous"):
        se.se_ring_step(Fake(32), Fake(32, contiguous=False), None, offs, 4, 0.1, 0.0)
    with pytest.raises(ValueError, match="2-byte elements"):
        se.se_step_bf16g(Fake(32), Fake(32, elem=4), None, offs, 4, 2, 0, 0.1, 0.0)
    with pytest.raises(ValueError, match="4-byte elements"):
        se.se_step_ex(Fake(32), Fake(32, elem=2), None, offs, 4, 2, 0, 0.1, 0.0)
    with pytest.raises(ValueError, match="8-byte elements"):
        se.se_consensus(Fake(32), offs, 4, Fake(2, elem=4))
