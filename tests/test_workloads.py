"""The synthetic gradient sets have the shapes the paper's workloads have (CPU only)."""
import numpy as np
import pytest

from workloads import gradients
from workloads.shapes import ALL, EXTRA, workload


def test_tensor_counts_and_sizes():
    expect = {"mlp": (6, 269322), "resnet50": (161, 25557032), "vgg16": (32, 138357544),
              "inception_v3": (284, 23834568), "transformer": (391, 335141888)}
    for name in ALL:
        wl = workload(name)
        assert (len(wl.tensors), wl.total_elems) == expect[name]


def test_vgg16_matches_the_papers_model_table():
    # section 6, "DNN models": VGG-16 has 32 parameters totalling 527.8 MiB
    wl = workload("vgg16")
    assert len(wl.tensors) == 32
    assert round(wl.total_elems * 4 / 2 ** 20, 1) == 527.8
    assert wl.algorithmic_bytes() == 8854882816


def test_extra_models_match_the_papers_model_table():
    # section 6, "DNN models": AlexNet-v2 16 parameters / 191.9 MiB, ResNet-v2-152 363 / 229.5 MiB
    for name, count, mib in (("alexnet_v2", 16, 191.9), ("resnet_v2_152", 363, 229.5)):
        wl = workload(name)
        assert len(wl.tensors) == count
        assert round(wl.total_elems * 4 / 2 ** 20, 1) == mib


@pytest.mark.parametrize("name", ALL + EXTRA)
def test_half_of_the_parameters_are_under_20_kb(name):
    # section 3.3.2 (C): at least 50 % of parameters are smaller than 20 KB in every model
    wl = workload(name)
    small = sum(1 for n in wl.elems() if n * wl.elem_size < 20 * 1024)
    assert 2 * small >= len(wl.elems())


def test_values_are_reproducible_and_distributed_as_stated():
    a = gradients.tensor_values(1, 2, 3, 200000)
    b = gradients.tensor_values(1, 2, 3, 200000)
    c = gradients.tensor_values(1, 3, 3, 200000)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    s = float(gradients.sigma(1, 3))
    assert 1e-4 <= s <= 1e-1
    assert abs(a.std() / s - 1) < 0.02 and abs(c.std() / s - 1) < 0.02 and abs(a.mean()) < 0.01 * s
    h = gradients.tensor_values(1, 2, 3, 1000, bf16=True)
    assert h.dtype == np.uint16 and np.array_equal(h, a[:1000].view(np.uint32) >> 16)
    sig = [float(gradients.sigma(0, t)) for t in range(400)]
    assert min(sig) < 3e-4 and max(sig) > 3e-2
