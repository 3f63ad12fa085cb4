"""Pins of the oracle's convolutional family (CPU): the 3x3 convolution against its definition
written as plain loops and against the library convolution with library autograd; finite
differences of the combined loss; BatchNorm statistics scoped to the node's positions; the
bf16 operand rounding as a small perturbation.  (The whole model against library autograd per
node slice: test_oracle_autograd.py.)"""
from dataclasses import replace

import numpy as np
import torch
import torch.nn.functional as F

import oracle as O
from oracle import layers as L
import vf_inputs as I


def test_conv3x3_against_its_definition_as_loops():
    rng = np.random.Generator(np.random.PCG64(5))
    x = rng.standard_normal((2, 4, 3, 2))
    W = rng.standard_normal((3, 3, 3, 2))
    y = L.conv3x3_fwd(x, W)
    ref = np.zeros((2, 4, 3, 3))
    for n in range(2):
        for h in range(4):
            for w in range(3):
                for o in range(3):
                    acc = 0.0
                    for kh in range(3):
                        for kw in range(3):
                            hh, ww = h + kh - 1, w + kw - 1
                            if 0 <= hh < 4 and 0 <= ww < 3:
                                for c in range(2):
                                    acc += x[n, hh, ww, c] * W[o, kh, kw, c]
                    ref[n, h, w, o] = acc
    np.testing.assert_allclose(y, ref, rtol=1e-13, atol=1e-13)


def test_conv3x3_forward_and_backward_against_the_library():
    rng = np.random.Generator(np.random.PCG64(6))
    x = rng.standard_normal((3, 5, 7, 4))
    W = rng.standard_normal((6, 3, 3, 4))
    dy = rng.standard_normal((3, 5, 7, 6))
    xt = torch.tensor(x, requires_grad=True)
    Wt = torch.tensor(W, requires_grad=True)
    yt = F.conv2d(xt.permute(0, 3, 1, 2), Wt.permute(0, 3, 1, 2), padding=1).permute(0, 2, 3, 1)
    yt.backward(torch.tensor(dy))
    np.testing.assert_allclose(L.conv3x3_fwd(x, W), yt.detach().numpy(), rtol=1e-12, atol=1e-12)
    dx, dW = L.conv3x3_bwd(x, W, dy)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(dW, Wt.grad.numpy(), rtol=1e-12, atol=1e-12)
    assert L.conv3x3_bwd(x, W, dy, need_dx=False)[0] is None


def _setup(name, jitter=0.2):
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=jitter).astype(np.float64 if wl.dtype == "f64" else np.float32)
    x, y = I.make_batch(wl)
    return wl, theta, x, y


def test_finite_differences_of_the_combined_loss():
    wl, theta, x, y = _setup("conv_tiny_f64")
    r = O.oracle_step(wl, theta, x, y)
    G = r["G"]
    rng = np.random.Generator(np.random.PCG64(3))
    idx = rng.choice(theta.size, 160, replace=False)
    # every tensor gets probed
    pos = 0
    extra = []
    for name, shape in O.layout(wl):
        n = int(np.prod(shape))
        if not ((idx >= pos) & (idx < pos + n)).any():
            extra.append(pos + n // 2)
        assert np.abs(G[pos:pos + n]).max() > 0, name
        pos += n
    idx = np.concatenate([idx, np.array(extra, dtype=idx.dtype)])
    h = 1e-5
    fd = np.empty(len(idx))
    for k, j in enumerate(idx):
        tp, tm = theta.copy(), theta.copy()
        tp[j] += h
        tm[j] -= h
        fd[k] = (O.oracle_step(wl, tp, x, y)["loss"] - O.oracle_step(wl, tm, x, y)["loss"]) / (2 * h)
    assert np.linalg.norm(fd - G[idx]) <= 2e-6 * np.linalg.norm(G[idx])


def test_batchnorm_statistics_are_taken_over_the_nodes_positions_only():
    """V copies of one node give that node's gradient; one node of all samples does not."""
    wl, theta, x, y = _setup("conv_tiny_f64")
    b = wl.node_sizes[0]
    x1, y1 = x[:b], y[:b]
    one = O.oracle_step(replace(wl, node_sizes=(b,)), theta, x1, y1)
    three = O.oracle_step(replace(wl, node_sizes=(b, b, b)), theta, np.concatenate([x1] * 3), np.concatenate([y1] * 3))
    np.testing.assert_allclose(three["G"], one["G"], rtol=1e-12, atol=1e-15)
    split = O.oracle_step(wl, theta, x, y)
    whole = O.oracle_step(replace(wl, node_sizes=(wl.batch,)), theta, x, y)
    assert np.linalg.norm(split["G"] - whole["G"]) > 1e-3 * np.linalg.norm(whole["G"])
    # moving statistics: one blend per node and BatchNorm layer, in node order
    st = split["state"]
    assert len(st["bn_mean"]) == 1 + 2 * wl.n_blocks and st["bn_mean"][0].shape == (wl.width,)


def test_bf16_rounding_is_a_small_perturbation():
    wl, theta, x, y = _setup("conv_small_bf16")
    lo = O.oracle_step(wl, theta, x, y)
    hi = O.oracle_step(replace(wl, dtype="f32"), theta, x, y)
    rel = np.linalg.norm(lo["G"] - hi["G"]) / np.linalg.norm(hi["G"])
    assert 1e-5 < rel < 5e-2, rel
    assert abs(lo["loss"] - hi["loss"]) < 2e-2 * abs(hi["loss"])


def test_layouts_agree():
    for name in ("C6", "conv_tiny_bf16", "conv_small_bf16"):
        wl = I.workload(name)
        assert [(n, tuple(s)) for n, s, _ in I.param_layout(wl)] == [(n, tuple(s)) for n, s in O.layout(wl)]
