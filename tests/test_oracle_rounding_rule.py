"""The oracle's bf16 rule, checked on the oracle itself (CPU): exactly the operands of contractions
are bf16 -- every array that enters a Linear, convolution or attention product (forward or
backward) is bf16-representable, and the tensors that are not operands of a product (the
pre-activations read by GELU / BatchNorm, the logits, the LayerNorm inputs) are not rounded.

The float64 pins of the oracle run without any rounding, so a rounding that is missing, or one that
sits on a tensor which is no operand, would fail none of them; here it fails."""
import numpy as np
import pytest

import oracle as O
import oracle.layers as OL
import vf_inputs as I
from vfharness import oracle_layers_patched


def _is_bf16(x):
    x = np.asarray(x, dtype=np.float64)
    return np.array_equal(O.round_to_bf16(x.astype(np.float32)), x)


def _needs_more_bits(x):
    """true for an array that has NOT been rounded to bf16 (a float64 result has entries that bf16
    cannot hold; an array of a few entries could be representable by chance, these are large)"""
    x = np.asarray(x, dtype=np.float64)
    return x.size >= 16 and np.mean(O.round_to_bf16(x.astype(np.float32)) != x) > 0.5


@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_mid_bf16", "enc_small_bf16", "conv_tiny_bf16"])
def test_exactly_the_operands_of_contractions_are_bf16(name):
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=0.1)
    x, y = I.make_batch(wl)
    seen = {"products": 0, "unrounded": 0}
    real = {k: getattr(OL, k) for k in ("linear_fwd", "linear_bwd", "attention_fwd", "attention_bwd", "conv3x3_fwd",
                                        "conv3x3_bwd", "gelu_fwd", "batchnorm_fwd", "layernorm_fwd",
                                        "softmax_xent_fwd_bwd")}

    def operands(*arrays):
        for a in arrays:
            assert _is_bf16(a), "an operand of a contraction is not bf16"
        seen["products"] += 1

    def linear_fwd(x_, W, b=None):
        operands(x_, W)
        return real["linear_fwd"](x_, W, b)

    def linear_bwd(x_, W, dy, has_bias):
        operands(x_, W, dy)
        return real["linear_bwd"](x_, W, dy, has_bias)

    def conv3x3_fwd(x_, W):
        operands(x_, W)
        return real["conv3x3_fwd"](x_, W)

    def conv3x3_bwd(x_, W, dy, need_dx=True):
        operands(x_, W, dy)
        return real["conv3x3_bwd"](x_, W, dy, need_dx)

    def attention_fwd(q, k, v, operand=OL._identity):
        operands(q, k, v)
        o, p = real["attention_fwd"](q, k, v, operand)
        assert _is_bf16(p)                       # the probabilities enter the product with v rounded
        assert not _is_bf16(o)                   # ... and its result is not rounded inside
        return o, p

    def attention_bwd(do, q, k, v, p, operand=OL._identity):
        operands(do, q, k, v, p)
        marks = []

        def spy(a):
            r = operand(a)
            marks.append(_is_bf16(r))
            return r
        out = real["attention_bwd"](do, q, k, v, p, spy)
        assert marks == [True]                   # the score gradient, once, before its two products
        return out

    def not_rounded(fn):
        def f(a, *rest):
            assert _needs_more_bits(a), f"the input of {fn} was rounded although it is no operand of a product"
            seen["unrounded"] += 1
            return real[fn](a, *rest)
        return f

    patches = dict(linear_fwd=linear_fwd, linear_bwd=linear_bwd, conv3x3_fwd=conv3x3_fwd, conv3x3_bwd=conv3x3_bwd,
                   attention_fwd=attention_fwd, attention_bwd=attention_bwd,
                   gelu_fwd=not_rounded("gelu_fwd"), batchnorm_fwd=not_rounded("batchnorm_fwd"),
                   layernorm_fwd=not_rounded("layernorm_fwd"), softmax_xent_fwd_bwd=not_rounded("softmax_xent_fwd_bwd"))
    with oracle_layers_patched(**patches):
        cp = O.step.compute_copy(wl, theta)
        b0 = wl.node_sizes[0]
        O.node_loss_and_grads(wl, cp, x[:b0], y[:b0])
    assert seen["products"] >= 4 and seen["unrounded"] >= 1


def test_fp32_workloads_round_nothing():
    wl = I.workload("mlp_small_bn_f32")
    theta = I.make_params(wl, jitter=0.1)
    x, y = I.make_batch(wl)
    real = OL.linear_fwd
    seen = []

    def linear_fwd(x_, W, b=None):
        seen.append(_needs_more_bits(W))
        return real(x_, W, b)
    with oracle_layers_patched(linear_fwd=linear_fwd):
        b0 = wl.node_sizes[0]
        O.node_loss_and_grads(wl, O.step.compute_copy(wl, theta), x[:b0], y[:b0])
    assert seen and all(seen)
