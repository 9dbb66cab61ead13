"""GPU parity of DGC_k (hierarchical sampling, Sec. 3.3 / Sec. 4.3) against the CPU oracle:
record, pairs (ascending index), accumulator and residual bit for bit, for sample strides from
the whole vector down to 0.1 %, both outcomes (second selection run / not run), ties, special
values, tilings, and an error-feedback chain on the ResNet-20-sized workload."""
import numpy as np
import pytest

from gpu_harness import FlatGpu, check_flat
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu


def test_sizes_strides_and_ranks():
    seen = set()
    for d in (1, 2, 5, 64, 257, 4096, 4097, 12_289, 100_003, 1_000_003):
        g = synth.student_t3(d, 201, d, 1e-3)
        eps = synth.normal(d, 202, d, 3e-4)
        gpu = FlatGpu(d, cap=d)
        for k in sorted({1, max(1, d // 1000), max(1, d // 10), d}):
            for stride in (1, 7, 100, 1000):
                for seed in (0, 12345678901234567):
                    gpu.set_residual(eps)
                    check_flat("dgck", gpu, g, eps, k, what=f"dgck d={d} k={k} S={stride} seed={seed}",
                               sample_stride=stride, sample_seed=seed)
                    seen.add(int(S.decode_results(gpu.b.result)[0]["rounds"]))
    assert seen == {1, 2}


@pytest.mark.parametrize("d", [777, 20_011, 300_007])
def test_ties_and_special_values(d):
    rng = np.random.default_rng(d)
    zero = np.zeros(d, np.float32)
    vecs = {"small_ints": rng.integers(-3, 4, d).astype(np.float32),
            "zeros": zero.copy(), "constant": np.full(d, -0.375, np.float32)}
    w = (rng.integers(-4, 5, d) * np.float32(1e-45)).astype(np.float32)
    w[::7] = np.float32(-0.0)
    vecs["denormals"] = w
    u = rng.standard_normal(d).astype(np.float32)
    u[rng.integers(0, d, 5)] = np.float32(np.inf)
    u[rng.integers(0, d, 3)] = np.float32(np.nan)
    vecs["inf_nan"] = u
    gpu = FlatGpu(d, cap=d)
    for name, acc in vecs.items():
        for k in sorted({1, d // 100 + 1, d // 3, d - 1, d}):
            for stride in (3, 100):
                gpu.set_residual(zero)
                check_flat("dgck", gpu, acc, zero, k, what=f"dgck {name} d={d} k={k} S={stride}",
                           sample_stride=stride, sample_seed=d)


@pytest.mark.parametrize("tile_chunks", [1, 3, 16])
def test_results_do_not_depend_on_the_tiling(tile_chunks):
    for d in (70_001, 1_000_003):
        g = synth.normal(d, 203, d, 1e-3)
        eps = synth.normal(d, 204, d, 3e-4)
        gpu = FlatGpu(d, cap=d)
        for k in (max(1, d // 1000), d // 20):
            gpu.set_residual(eps)
            check_flat("dgck", gpu, g, eps, k, what=f"dgck d={d} k={k} tc={tile_chunks}",
                       tile_chunks=tile_chunks, sample_seed=5)


def test_cfg1_error_feedback_chain_default_sample():
    """ResNet-20-sized vector, the default 1 % sample, residual carried over 10 iterations."""
    wl = synth.workload("cfg1_resnet20")
    gpu = FlatGpu(wl.d, cap=max(4 * wl.k, 1024))
    eps = np.zeros(wl.d, np.float32)
    for step in range(wl.steps + 1):
        eps = check_flat("dgck", gpu, wl.grad(step), eps, wl.k, what=f"cfg1 dgck step {step}",
                         sample_seed=step)


def test_cfg3_headline_size_two_steps():
    wl = synth.workload("cfg3_resnet50")
    gpu = FlatGpu(wl.d, cap=4 * wl.k)
    eps = np.zeros(wl.d, np.float32)
    g = np.empty(wl.d, np.float32)
    for step in range(2):
        wl.grad(step, out=g)
        eps = check_flat("dgck", gpu, g, eps, wl.k, what=f"cfg3 dgck step {step}", sample_seed=step)


def test_cfg2_chain_of_five_steps():
    """VGG-16-sized mixture workload: the residual grows heavy-tailed over the steps."""
    wl = synth.workload("cfg2_vgg16")
    gpu = FlatGpu(wl.d, cap=4 * wl.k)
    eps = np.zeros(wl.d, np.float32)
    g = np.empty(wl.d, np.float32)
    for step in range(5):
        wl.grad(step, out=g)
        eps = check_flat("dgck", gpu, g, eps, wl.k, what=f"cfg2 dgck step {step}", sample_seed=100 + step)


def test_lstm_sized_heavy_tails_three_steps():
    """The sampling comparator at the LSTM-sized length (66 M elements, Student-t(3) gradients):
    three error-feedback steps, bit-exact record, pairs, accumulator and residual."""
    wl = synth.workload("cfg5_lstm")
    gpu = FlatGpu(wl.d, cap=wl.k)
    eps = np.zeros(wl.d, np.float32)
    for step in range(3):
        eps = check_flat("dgck", gpu, wl.grad(step), eps, wl.k, what=f"cfg5 dgck step {step}")
