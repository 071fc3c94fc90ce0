"""The synthetic workloads have the shapes of the public architectures they are named after:
tensor counts and parameter totals (the figures those architectures are usually quoted with),
and the seeded generators are reproducible and independent across workers and iterations."""
import numpy as np

from paper_2007_00433_amd import workloads as wl


def test_parameter_totals_of_the_architectures():
    want = {"tiny": (3, 5106), "resnet20": (59, 269722), "resnet18": (62, 11689512),
            "resnet50": (161, 25557032), "densenet121": (364, 7978856), "vgg16": (32, 138357544),
            "bert_base": (199, 109482240), "bert_base_full": (199, 109482240)}
    assert set(wl.WORKLOADS) == set(want)
    for name, (tensors, total) in want.items():
        w = wl.WORKLOADS[name]
        assert (len(w.sizes), w.P) == (tensors, total), name
        assert all(s > 0 for s in w.sizes)
        assert w.n % w.group_size == 0
    # configurations as stated: workers, group size, iterations, gradient storage
    got = {k: (w.n, w.group_size, w.iters, w.grad_dtype) for k, w in wl.WORKLOADS.items()}
    assert got["tiny"] == (4, 2, 5, "f32") and got["resnet20"] == (16, 4, 100, "f32")
    assert got["resnet50"] == (16, 4, 50, "f32") and got["vgg16"] == (32, 4, 20, "f32")
    assert got["bert_base"] == (64, 8, 10, "bf16") and got["bert_base_full"] == (64, 64, 10, "bf16")
    # ResNet-50: 53 convolutions + 2 x 53 batch-norm vectors + the classifier's two tensors
    r50 = wl.WORKLOADS["resnet50"].sizes
    assert sum(1 for s in r50 if s < 1024) == 85 and max(r50) == 2359296 and min(r50) == 64


def test_layer_offsets_and_padding():
    w = wl.WORKLOADS["resnet20"]
    offs = w.layer_offsets()
    assert offs[0] == 0 and offs[-1] == w.P and len(offs) == len(w.sizes) + 1
    assert np.all(np.diff(offs) == np.asarray(w.sizes))
    padded = w.layer_offsets(270336)
    assert padded[-1] == 270336 and padded[-2] == w.P and len(padded) == len(offs) + 1


def test_generators_are_seeded_and_independent():
    a = wl.host_grads(4, 1000, 1e-2, 0, 3)
    assert np.array_equal(a, wl.host_grads(4, 1000, 1e-2, 0, 3))
    assert not np.array_equal(a, wl.host_grads(4, 1000, 1e-2, 0, 4))          # fresh per iteration
    assert not np.array_equal(a, wl.host_grads(4, 1000, 1e-2, 1, 3))          # and per seed
    assert not np.array_equal(a[0], a[1])                                     # and per worker
    assert abs(float(a.std()) - 1e-2) < 1e-3
    x = wl.host_params(5, 300, 0.05, 0, pitch=320)
    assert np.array_equal(x[0], x[4]) and not x[:, 300:].any()                # identical starts, zero padding
    cols = wl.stratified_columns(1 << 20, 16, 100, seed=1)
    assert cols[0] == 0 and cols[-1] == (1 << 20) - 1 and np.all(np.diff(cols) > 0)
    assert np.array_equal(cols[:256], np.arange(256)) and np.array_equal(cols[-256:], np.arange((1 << 20) - 256, 1 << 20))
    assert np.array_equal(wl.stratified_columns(1000, 16, 10), np.arange(1000))
