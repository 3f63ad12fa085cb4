"""Pins for the CPU oracle: paper's worked example, invariants, finite differences,
closed forms, brute force.  None of these re-types an oracle formula."""
import os
from dataclasses import replace
from fractions import Fraction

import numpy as np
import pytest

import oracle as O
import vf_inputs as I

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _f64(wl):
    return replace(wl, dtype="f64")


def _tiny_mlp(bn, sizes, dims=(5, 4, 6, 3)):
    return I.Workload(name="tiny", kind="mlp", dims=tuple(dims), batchnorm=bn,
                      node_sizes=tuple(sizes), dtype="f64", lr=0.1)


def _tiny_enc(sizes):
    return I.Workload(name="tinyenc", kind="encoder", n_layers=2, d_model=8, n_heads=2, d_ffn=12,
                      seq_len=4, vocab=11, n_masked=2, node_sizes=tuple(sizes), dtype="f64",
                      optimizer="adam", lr=1e-3)


def _setup(wl, jitter=0.3):
    theta = I.make_params(wl, jitter=jitter).astype(np.float64)
    rng = np.random.Generator(np.random.PCG64(7))
    theta = theta + 0.01 * rng.standard_normal(theta.size)      # genuinely fp64 values
    x, y = I.make_batch(wl)
    return theta, x, y


# ---- Section 5.2 worked example -----------------------------------------------------

def _read_golden():
    rows = {}
    with open(os.path.join(GOLDEN, "weighted_average_6_2.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, a, b = line.split()
            rows[name] = (Fraction(a), Fraction(b))
    return rows


def test_worked_example_6_plus_2():
    gold = _read_golden()
    wl = _tiny_mlp(False, [6, 2])
    theta, x, y = _setup(wl)
    # per-example gradients g_1..g_8: eight nodes of one sample each, read back
    # from the node losses' gradients by giving every node weight 1 (V = 1, B = 1).
    g = []
    for j in range(8):
        r = O.oracle_step(replace(wl, node_sizes=(1,)), theta, x[j:j + 1], y[j:j + 1])
        g.append(r["G"])
    g = np.array(g)
    r = O.oracle_step(wl, theta, x, y)
    # weights the method uses
    assert [Fraction(float(v)).limit_denominator(64) for v in r["w"]] == list(gold["weights"])
    cw, cw2 = (float(v) for v in gold["weighted"])
    expect = cw * g[:6].sum(0) + cw2 * g[6:].sum(0)
    np.testing.assert_allclose(r["G"], expect, rtol=1e-12, atol=1e-14)
    # negative control: the plain average of local averages is a different vector
    cu, cu2 = (float(v) for v in gold["unweighted"])
    wrong = cu * g[:6].sum(0) + cu2 * g[6:].sum(0)
    assert np.linalg.norm(r["G"] - wrong) > 1e-3 * np.linalg.norm(expect)


# ---- invariants ---------------------------------------------------------------------

@pytest.mark.parametrize("sizes", [[64], [16] * 4, [1] * 64, [48, 16], [1, 2, 3, 58], [13, 17, 34]])
def test_partition_invariance_without_batchnorm(sizes):
    """Without BatchNorm G equals the full-batch mean gradient for any partition."""
    wl = _f64(I.workload("C1"))
    theta, x, y = _setup(wl, jitter=0.1)
    full = O.oracle_step(replace(wl, node_sizes=(64,)), theta, x, y)
    r = O.oracle_step(replace(wl, node_sizes=tuple(sizes)), theta, x, y)
    assert np.linalg.norm(r["G"] - full["G"]) <= 1e-12 * np.linalg.norm(full["G"])
    assert abs(r["loss"] - full["loss"]) <= 1e-12 * abs(full["loss"])
    np.testing.assert_allclose(r["theta"], full["theta"], rtol=0, atol=1e-13)


def test_partition_invariance_encoder():
    wl = _tiny_enc([6])
    theta, x, y = _setup(wl)
    full = O.oracle_step(wl, theta, x, y)
    for sizes in ([3, 3], [1, 5], [2, 1, 3]):
        r = O.oracle_step(replace(wl, node_sizes=tuple(sizes)), theta, x, y)
        assert np.linalg.norm(r["G"] - full["G"]) <= 1e-12 * np.linalg.norm(full["G"])


def test_uneven_sizes_on_bn_free_copy_of_c3_shape():
    """C3's size vector on a narrow BatchNorm-free MLP."""
    sizes = I.workload("C3").node_sizes
    wl = I.Workload(name="c3free", kind="mlp", dims=(64, 96, 96, 50), batchnorm=False,
                    node_sizes=sizes, dtype="f64")
    theta, x, y = _setup(wl)
    full = O.oracle_step(replace(wl, node_sizes=(256,)), theta, x, y)
    r = O.oracle_step(wl, theta, x, y)
    assert np.linalg.norm(r["G"] - full["G"]) <= 1e-12 * np.linalg.norm(full["G"])


def test_batchnorm_statistics_are_per_node():
    """With BatchNorm and V > 1 the result differs from one full-batch pass
    (negative control); V copies of the same rows as V nodes give exactly the
    single node's gradient (positive control)."""
    wl = _tiny_mlp(True, [4, 4, 4], dims=(5, 8, 6, 3))
    theta, x, y = _setup(wl)
    per_node = O.oracle_step(wl, theta, x, y)
    full = O.oracle_step(replace(wl, node_sizes=(12,)), theta, x, y)
    assert np.linalg.norm(per_node["G"] - full["G"]) > 1e-3 * np.linalg.norm(full["G"])
    xs, ys = np.tile(x[:4], (3, 1)), np.tile(y[:4], 3)
    rep = O.oracle_step(wl, theta, xs, ys)
    one = O.oracle_step(replace(wl, node_sizes=(4,)), theta, x[:4], y[:4])
    np.testing.assert_allclose(rep["G"], one["G"], rtol=1e-12, atol=1e-15)
    # swapping rows between nodes changes G with BatchNorm (scope is the node)
    perm = np.arange(12); perm[[0, 4]] = perm[[4, 0]]
    sw = O.oracle_step(wl, theta, x[perm], y[perm])
    assert np.linalg.norm(sw["G"] - per_node["G"]) > 1e-4 * np.linalg.norm(per_node["G"])


def test_node_order_does_not_matter():
    wl = _tiny_mlp(True, [3, 5, 4], dims=(5, 8, 6, 3))
    theta, x, y = _setup(wl)
    a = O.oracle_step(wl, theta, x, y)
    order = np.r_[8:12, 0:3, 3:8]
    b = O.oracle_step(replace(wl, node_sizes=(4, 3, 5)), theta, x[order], y[order])
    np.testing.assert_allclose(a["G"], b["G"], rtol=1e-12, atol=1e-15)


def test_v1_is_the_ordinary_step_and_one_update_per_step():
    wl = _f64(I.workload("mlp_small_f32"))
    theta, x, y = _setup(wl)
    one = O.oracle_step(replace(wl, node_sizes=(wl.batch,)), theta, x, y)
    many = O.oracle_step(wl, theta, x, y)
    assert one["state"]["t"] == many["state"]["t"] == 1
    np.testing.assert_allclose(one["state"]["v"], many["state"]["v"], rtol=1e-11, atol=1e-14)


# ---- finite differences of the combined loss ------------------------------------------

def _fd_check(wl, n_probe=None, h=1e-5, tol=1e-6):
    theta, x, y = _setup(wl)
    r = O.oracle_step(wl, theta, x, y)
    G = r["G"]
    rng = np.random.Generator(np.random.PCG64(3))
    idx = np.arange(theta.size) if n_probe is None else rng.choice(theta.size, n_probe, replace=False)
    fd = np.empty(len(idx))
    for k, j in enumerate(idx):
        tp, tm = theta.copy(), theta.copy()
        tp[j] += h
        tm[j] -= h
        fd[k] = (O.oracle_step(wl, tp, x, y)["loss"] - O.oracle_step(wl, tm, x, y)["loss"]) / (2 * h)
    err = np.linalg.norm(fd - G[idx]) / np.linalg.norm(G[idx])
    assert err < tol, err
    assert np.max(np.abs(fd - G[idx])) < tol * np.max(np.abs(G)) * 10
    # every tensor got probed and has a non-zero gradient somewhere
    pos = 0
    for name, shape in O.layout(wl):
        n = int(np.prod(shape))
        sel = (idx >= pos) & (idx < pos + n)
        assert sel.any(), name
        assert np.abs(G[pos:pos + n]).max() > 0, name
        pos += n


def test_finite_differences_mlp_plain():
    _fd_check(_tiny_mlp(False, [3, 2, 1]))


def test_finite_differences_mlp_batchnorm():
    _fd_check(_tiny_mlp(True, [3, 3]))
    _fd_check(_tiny_mlp(True, [2, 4, 5]))


def test_finite_differences_encoder():
    _fd_check(_tiny_enc([2, 1, 3]), tol=2e-6)


# ---- closed forms -----------------------------------------------------------------------

@pytest.mark.parametrize("n_cls", [10, 1000])
def test_uniform_logits_give_ln_n(n_cls):
    wl = _tiny_mlp(False, [3, 2], dims=(5, 4, n_cls))
    theta, x, y = _setup(wl)
    p = O.unflatten(wl, theta)
    p["l1.W"][:] = 0.0
    p["l1.b"][:] = 0.7                       # equal logits
    r = O.oracle_step(wl, theta, x, y)
    assert abs(r["loss"] - np.log(n_cls)) < 1e-12
    # gradient of the last bias: softmax - onehot, averaged: sums to zero over classes
    pos = theta.size - n_cls
    assert abs(r["G"][pos:].sum()) < 1e-13
    counts = np.bincount(y, minlength=n_cls) / len(y)
    np.testing.assert_allclose(r["G"][pos:], 1.0 / n_cls - counts, atol=1e-14)


def test_encoder_uniform_logits_give_ln_vocab():
    wl = _tiny_enc([2, 2])
    theta, x, y = _setup(wl)
    p = O.unflatten(wl, theta)
    p["Wout"][:] = 0.0
    p["bout"][:] = -0.2
    assert abs(O.oracle_step(wl, theta, x, y)["loss"] - np.log(wl.vocab)) < 1e-12


def test_batchnorm_backward_sums_vanish():
    """Per node the gradient w.r.t. the pre-normalisation values sums to zero over
    rows; seen from outside: a bias added before BatchNorm has zero gradient, so
    shifting the first-layer pre-activations leaves the loss unchanged."""
    wl = _tiny_mlp(True, [4, 3])
    theta, x, y = _setup(wl)
    base = O.oracle_step(wl, theta, x, y)["loss"]
    # adding c * W-row direction == shifting inputs by a constant vector per node
    x2 = x.copy().astype(np.float64)
    x2[:4] += 0.37                            # same shift for all rows of node 0
    shifted = O.oracle_step(wl, theta, x2, y)["loss"]
    assert abs(base - shifted) < 1e-12        # BN removes a per-node constant shift of z


def test_sgdm_closed_form_two_steps():
    rng = np.random.Generator(np.random.PCG64(1))
    th0, g1, g2 = rng.standard_normal((3, 50))
    lr, mu = 0.1, 0.9
    th1, v1 = O.sgdm_update(th0, g1, np.zeros(50), lr, mu)
    np.testing.assert_allclose(th1, th0 - lr * g1, rtol=1e-15)
    th2, v2 = O.sgdm_update(th1, g2, v1, lr, mu)
    np.testing.assert_allclose(th2, th1 - lr * (mu * g1 + g2), rtol=1e-14)


def test_adam_closed_form_first_step():
    rng = np.random.Generator(np.random.PCG64(2))
    th0, g = rng.standard_normal((2, 50))
    lr, eps = 1e-3, 1e-8
    th1, m, u = O.adam_update(th0, g, np.zeros(50), np.zeros(50), 1, lr, 0.9, 0.999, eps)
    np.testing.assert_allclose(th1 - th0, -lr * g / (np.abs(g) + eps), rtol=1e-12)
    # constant gradient: bias-corrected moments stay g and g^2 at every step
    th = th0
    mm, uu = np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        th, mm, uu = O.adam_update(th, g, mm, uu, t, lr, 0.9, 0.999, eps)
    np.testing.assert_allclose(th - th0, -5 * lr * g / (np.abs(g) + eps), rtol=1e-10)


# ---- partition: brute force and bit patterns ---------------------------------------------

@pytest.mark.parametrize("sizes", [[16] * 4, [48, 48, 32, 32, 16, 16, 48, 16], [1], [1, 1, 1], [128] * 64,
                                   [5, 1, 250]])
def test_partition_brute_force(sizes):
    B = sum(sizes)
    off, w = O.partition(sizes, B)
    assert off.dtype == np.int32 and w.dtype == np.float32
    owner = O.node_of_sample(sizes, B)
    for j in range(B):
        i = int(np.searchsorted(off, j, side="right") - 1)
        assert owner[j] == i
    assert off[0] == 0 and off[-1] == B and list(np.diff(off)) == sizes
    for i, b in enumerate(sizes):
        assert w[i].tobytes() == (np.float32(b) / np.float32(B)).tobytes()
        assert Fraction(float(w[i])) == Fraction(b, B) or (B & (B - 1)) != 0


def test_c3_offsets_and_weights_exact():
    off, w = O.partition(I.workload("C3").node_sizes, 256)
    assert list(off) == [0, 48, 96, 128, 160, 176, 192, 240, 256]
    assert [Fraction(float(v)) for v in w] == [Fraction(3, 16), Fraction(3, 16), Fraction(1, 8), Fraction(1, 8),
                                               Fraction(1, 16), Fraction(1, 16), Fraction(3, 16), Fraction(1, 16)]


@pytest.mark.parametrize("sizes,B", [([], 0), ([0, 4], 4), ([3, 3], 7), ([-1, 5], 4)])
def test_partition_rejects(sizes, B):
    with pytest.raises(ValueError):
        O.partition(sizes, B)


def test_round_to_bf16_matches_library_cast():
    import torch
    rng = np.random.Generator(np.random.PCG64(5))
    x = np.concatenate([rng.standard_normal(10000).astype(np.float32) * 10.0 ** rng.integers(-6, 6, 10000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.0078125, 1.01171875, 3.3895314e38],
                                 dtype=np.float32)]).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_bf16(x), want)


def test_layouts_agree():
    for name, wl in I.WORKLOADS.items():
        a = [(n, tuple(s)) for n, s, _ in I.param_layout(wl)]
        assert a == O.layout(wl), name
    assert I.num_params(I.workload("C1")) == 203530
    assert I.num_params(I.workload("C2")) == 41870312
    assert I.num_params(I.workload("C4")) == 75363642
    assert I.num_params(I.workload("C5")) == 360612840


def test_bf16_operand_rounding_is_a_small_perturbation_and_exact_when_representable():
    """bf16 workloads round contraction operands.  (i) On a workload the result stays within
    a few percent of the unrounded one; (ii) when every operand is exactly representable
    (weights and inputs are small integers / powers of two, one Linear layer so that no
    intermediate needs rounding) both modes agree to float64 rounding."""
    wl = I.workload("mlp_mid_bn_bf16")
    theta = I.make_params(wl, jitter=0.1)
    x, y = I.make_batch(wl)
    a = O.oracle_step(wl, theta, x, y)
    theta_r = O.round_to_bf16(theta).astype(np.float32)
    b = O.oracle_step(replace(wl, dtype="f32"), theta_r, x, y)
    err = np.linalg.norm(a["G"] - b["G"]) / np.linalg.norm(b["G"])
    assert 1e-5 < err < 0.08, err
    wl1 = I.Workload(name="one", kind="mlp", dims=(8, 4), batchnorm=False, node_sizes=(2, 2), dtype="bf16")
    rng = np.random.Generator(np.random.PCG64(4))
    th1 = np.concatenate([rng.integers(-4, 5, 32) / 8.0, np.zeros(4)]).astype(np.float32)
    x1 = rng.integers(-3, 4, (4, 8)).astype(np.float32)
    y1 = np.array([0, 1, 2, 3], dtype=np.int32)
    r16 = O.oracle_step(wl1, th1, x1, y1)
    r32 = O.oracle_step(replace(wl1, dtype="f32"), th1, x1, y1)
    assert abs(r16["loss"] - r32["loss"]) < 1e-14
    # the bias gradient never passes through a rounded operand
    np.testing.assert_allclose(r16["G"][32:], r32["G"][32:], rtol=1e-13, atol=1e-16)
    # the weight gradient uses the rounded output gradient: within bf16 rounding of it
    assert np.max(np.abs(r16["G"][:32] - r32["G"][:32])) <= 2.0 ** -8 * np.max(np.abs(r32["G"][:32]))


# ---- moving BatchNorm statistics (Section 4.1: per-device state, updated by every pass) -------

def _bn_workload(node_sizes, lr=0.0):
    from dataclasses import replace
    return replace(I.workload("mlp_small_bn_f32"), node_sizes=tuple(node_sizes), lr=lr, momentum=0.0,
                   dtype="f64")


def test_moving_stats_of_identical_nodes_follow_the_geometric_closed_form():
    """k passes over the same samples from (mean 0, variance 1) with share s leave
    mean = (1-(1-s)^k) mu and var = (1-s)^k + (1-(1-s)^k) sigma^2, with mu and sigma^2 the
    library mean / biased variance of the first Linear's output over ONE node."""
    wl = _bn_workload([6, 6, 6])
    theta = I.make_params(wl, jitter=0.1).astype(np.float64)
    x, y = I.make_batch(wl)
    x = np.tile(x[:6], (3, 1)).astype(np.float64)
    y = np.tile(y[:6], 3)
    r = O.oracle_step(wl, theta, x, y)
    W0 = O.unflatten(wl, theta)["l0.W"]
    z = x[:6] @ W0
    keep = (1 - wl.bn_momentum) ** 3
    np.testing.assert_allclose(r["state"]["bn_mean"][0], (1 - keep) * z.mean(axis=0), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["state"]["bn_var"][0], keep + (1 - keep) * z.var(axis=0), rtol=1e-12)
    # a second step with a zero learning rate continues the same series (k = 6)
    r2 = O.oracle_step(wl, r["theta"], x, y, state=r["state"])
    keep = (1 - wl.bn_momentum) ** 6
    np.testing.assert_allclose(r2["state"]["bn_mean"][0], (1 - keep) * z.mean(axis=0), rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r2["state"]["bn_var"][0], keep + (1 - keep) * z.var(axis=0), rtol=1e-12)


def test_moving_stats_use_each_nodes_own_samples_in_node_order():
    wl = _bn_workload([5, 9])
    theta = I.make_params(wl, jitter=0.1).astype(np.float64)
    x, y = I.make_batch(wl)
    x = x.astype(np.float64)
    r = O.oracle_step(wl, theta, x, y)
    W0 = O.unflatten(wl, theta)["l0.W"]
    z1, z2 = x[:5] @ W0, x[5:] @ W0
    s = wl.bn_momentum
    want_mean = (1 - s) * (s * z1.mean(axis=0)) + s * z2.mean(axis=0)
    want_var = (1 - s) * ((1 - s) * 1.0 + s * z1.var(axis=0)) + s * z2.var(axis=0)
    np.testing.assert_allclose(r["state"]["bn_mean"][0], want_mean, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(r["state"]["bn_var"][0], want_var, rtol=1e-12)
    # not the statistics of the whole batch, and not order-free
    zb = x @ W0
    assert not np.allclose(r["state"]["bn_mean"][0], s * zb.mean(axis=0))
    swapped = O.oracle_step(wl.with_nodes([9, 5]), theta, np.concatenate([x[5:], x[:5]]),
                            np.concatenate([y[5:], y[:5]]))
    assert not np.allclose(swapped["state"]["bn_mean"][0], r["state"]["bn_mean"][0])


def test_models_without_batchnorm_carry_no_moving_stats():
    wl = I.workload("mlp_small_f32")
    x, y = I.make_batch(wl)
    r = O.oracle_step(wl, I.make_params(wl), x, y)
    assert "bn_mean" not in r["state"]
