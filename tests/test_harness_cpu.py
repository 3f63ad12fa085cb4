"""The parity criterion of the GPU tests, exercised on the CPU: a second valid evaluation of a
step (the oracle with its products in float32, the contraction cut in two) stands in for the
device.  The criterion must accept it and must reject a planted error."""
import numpy as np
import pytest

import oracle as O
import vf_inputs as I
import vfharness as H


def _lin_two_halves(x, W, b=None):
    h = x.shape[1] // 2
    x32, W32 = np.asarray(x, dtype=np.float32), np.asarray(W, dtype=np.float32)
    y = (x32[:, :h] @ W32[:h] + x32[:, h:] @ W32[h:]).astype(np.float64)
    return y if b is None else y + b


@pytest.fixture(scope="module")
def case():
    from dataclasses import replace
    wl = replace(I.workload("mlp_mid_bn_bf16"), name="deep", dims=(256, 768, 768, 768, 768, 100))
    theta = I.make_params(wl, jitter=0.1)
    x, y = I.make_batch(wl)
    ref = H.oracle_steps(wl, theta, x, y)
    with H.oracle_layers_patched(linear_fwd=_lin_two_halves):
        other = O.oracle_step(wl, theta.astype(np.float32), x, y)
    return wl, theta, x, y, ref, other


def test_second_valid_evaluation_is_accepted_and_its_misses_are_explained(case):
    wl, theta, x, y, ref, other = case
    errs = H.tensor_errors(wl, other["G"], ref["G"])
    assert max(m for _, _, m in errs) > 0.02, "the case should need the explained exception"
    used = H.assert_explained(wl, other["G"], ref, 0.02, "second evaluation")
    assert used > 0
    assert ref["band"]["tau"][0] < 1e-4 < ref["band"]["tau"][-1]      # the distance grows with depth


def test_planted_errors_are_rejected(case):
    wl, theta, x, y, ref, other = case
    views = O.unflatten(wl, np.arange(ref["G"].size))
    big = 0.5 * np.abs(ref["G"]).max()
    # an entry of the first layer: no ambiguous unit of its column can account for that much
    g = other["G"].copy()
    g[int(views["l0.W"][3, 5])] += big
    with pytest.raises(AssertionError, match="no ambiguous ReLU unit explains"):
        H.assert_explained(wl, g, ref, 0.02, "planted")
    # an entry of a column of the deepest hidden layer that has no ambiguous unit at all
    allow = O.unflatten(wl, ref["band"]["allow"])["l3.W"]
    free = np.nonzero(allow.sum(axis=0) == 0)[0]
    assert free.size > 0
    g = other["G"].copy()
    g[int(views["l3.W"][7, free[0]])] += big
    with pytest.raises(AssertionError, match="no ambiguous ReLU unit explains"):
        H.assert_explained(wl, g, ref, 0.02, "planted")
    # a whole tensor scaled by 5 percent fails the L2 bound
    g = other["G"].copy()
    lo = int(views["l1.W"][0, 0])
    g[lo:lo + views["l1.W"].size] *= 1.05
    with pytest.raises(AssertionError, match="rel-L2"):
        H.assert_explained(wl, g, ref, 0.02, "scaled")


def test_weights_only_gradient_is_the_oracle_without_operand_rounding(case):
    wl, theta, x, y, ref, other = case
    gw = H.weights_only_gradient(wl, theta, x, y)
    d = np.linalg.norm(ref["G"] - gw) / np.linalg.norm(gw)
    assert 1e-4 < d < 0.2            # operand rounding matters, and stays a perturbation
    H.check_independent_bound(wl, other["G"], ref["G"], gw, "second evaluation")
    # the same oracle on a float32 workload does not round operands at all: bit-identical twice
    assert np.array_equal(gw, H.weights_only_gradient(wl, theta, x, y))
