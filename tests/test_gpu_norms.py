"""The optional squared-norm reductions: ||acc||^2 and ||acc - Comp_k(acc)||^2 = ||residual'||^2
(the two sides of the contraction property, Eq. (3)-(5) and Theorem 1) against the oracle's fp64
sums, for both selectors, flat and layer-wise; and that asking for them changes nothing else."""
import math

import numpy as np
import pytest

from gpu_harness import FlatGpu, SegGpu, check_flat, check_segmented
from oracle import oracle as O
from paper_1911_08772_amd import sparsify as S
from paper_1911_08772_amd import synth

pytestmark = pytest.mark.gpu
RTOL = 1e-12   # fp64 sums of d terms in different orders


@pytest.mark.parametrize("selector", ["gaussiank", "topk"])
def test_flat_norms_match_oracle(selector):
    for d, rho_den in [(5, 2), (4097, 100), (269_722, 1000), (3_000_017, 1000), (3_000_017, 10)]:
        k = synth.k_of(d, rho_den)
        g = synth.normal(d, 501, d, 1.0)
        eps = synth.normal(d, 502, d, 0.3)
        for inplace in (False, True):
            gpu = FlatGpu(d, cap=d, inplace=inplace)
            gpu.set_residual(eps)
            eps_o = check_flat(selector, gpu, g, eps, k, what=f"norms {selector} d={d}", error_norms=True)
            res = S.decode_results(gpu.b.result)[0]
            acc_o = O.accumulate(g, eps)
            assert math.isclose(float(res["acc_sqnorm"]), O.sqnorm(acc_o), rel_tol=RTOL)
            assert math.isclose(float(res["residual_sqnorm"]), O.sqnorm(eps_o), rel_tol=RTOL, abs_tol=1e-300)
            if selector == "topk":
                ratio = float(res["residual_sqnorm"]) / float(res["acc_sqnorm"])
                assert ratio <= (1 - k / d) ** 2 + 1e-12 <= (1 - k / d) + 1e-12  # Theorem 1 on Gaussian data
            # off by default: the fields stay zero
            gpu.set_residual(eps)
            gpu.step(selector, g, k)
            res = S.decode_results(gpu.b.result)[0]
            assert float(res["acc_sqnorm"]) == 0.0 and float(res["residual_sqnorm"]) == 0.0


@pytest.mark.parametrize("mode", [0, 1])
def test_segmented_norms_match_oracle(mode):
    sizes = np.array([64, 1, 1000, 37, 40_000, 5000, 3, 300_001], np.int64)
    seg_off = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    seg_k = np.maximum(1, (sizes + 99) // 100).astype(np.int64)
    caps = np.maximum(4 * seg_k, 16)
    caps[3] = 0   # nothing can be selected there: residual' = acc
    d = int(seg_off[-1])
    g = synth.student_t3(d, 503, 0, 1e-2)
    eps = np.zeros(d, np.float32)
    gpu = SegGpu(seg_off, seg_k, caps)
    eps_o = check_segmented(mode, gpu, g, eps, what=f"seg norms mode {mode}", error_norms=True)
    res = S.decode_results(gpu.b.result)
    for l in range(sizes.size):
        a, b = int(seg_off[l]), int(seg_off[l + 1])
        assert math.isclose(float(res[l]["acc_sqnorm"]), O.sqnorm(g[a:b].copy()), rel_tol=RTOL)
        assert math.isclose(float(res[l]["residual_sqnorm"]), O.sqnorm(eps_o[a:b].copy()), rel_tol=RTOL,
                            abs_tol=1e-300)
