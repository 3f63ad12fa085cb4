"""Seeded synthetic inputs for the virtual-node training step.

This module is shared by the CPU oracle's tests and by the HIP path's tests and
benchmark.  It holds no arithmetic of the method: it only names the workloads
(model shapes, batch sizes, node sizes, hyper-parameters) and draws random
parameters, inputs and labels from `numpy.random.Generator(PCG64(seed))`.

The workloads are synthetic stand-ins that keep the shapes of the paper's
experiments (global batch 8192 in nodes of 128 as in Section 6.2 / Table 1,
BERT-BASE-like encoder blocks at sequence length 128 as in Table 2, unequal
node sizes as in Table 4); no dataset item is reproduced.

Flat parameter layout (fp32, tensors in forward order):
  MLP:     per hidden layer  W[K_in, N_out] row-major, then bias[N_out] (only
           when the model has no BatchNorm), then gamma[N_out], beta[N_out]
           (only with BatchNorm); last layer W, bias.
  encoder: tok_emb[vocab, d], pos_emb[T, d]; per layer ln1.gamma, ln1.beta,
           Wqkv[d, 3d], bqkv[3d], Wo[d, d], bo[d], ln2.gamma, ln2.beta,
           W1[d, ffn], b1[ffn], W2[ffn, d], b2[d]; then lnf.gamma, lnf.beta,
           Wout[d, vocab], bout[vocab].
  conv:    (residual network of 3x3 convolutions, stride 1, zero padding 1, inputs NHWC)
           stem.W[width, 3, 3, in_ch], stem.gamma[width], stem.beta[width]; per block b
           b.W1[width, 3, 3, width], b.gamma1, b.beta1, b.W2[width, 3, 3, width], b.gamma2,
           b.beta2; then fc.W[width, classes], fc.b[classes].
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Tuple

import numpy as np

SEED_PARAMS = 9523
SEED_INPUTS = 9524
SEED_LABELS = 9525
SEED_MASK = 9526


@dataclass(frozen=True)
class Workload:
    """One configuration of the step: model, batch split, numerics, optimizer."""
    name: str
    kind: str                       # "mlp" | "encoder" | "conv"
    # MLP
    dims: Tuple[int, ...] = ()      # [in, h1, ..., out]
    batchnorm: bool = False
    # encoder
    n_layers: int = 0
    d_model: int = 0
    n_heads: int = 0
    d_ffn: int = 0
    seq_len: int = 0
    vocab: int = 0
    n_masked: int = 0               # masked positions per sequence
    # conv (residual network on img x img inputs with in_ch channels)
    img: int = 0
    in_ch: int = 0
    width: int = 0                  # channels of every convolution
    n_blocks: int = 0               # residual blocks of two 3x3 convolutions each
    classes: int = 0
    # step
    node_sizes: Tuple[int, ...] = ()
    dtype: str = "f32"              # "f32" | "bf16"
    optimizer: str = "sgdm"         # "sgdm" | "adam"
    lr: float = 0.01
    momentum: float = 0.9
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    bn_eps: float = 1e-5
    bn_momentum: float = 0.1        # share of a node's statistics blended into the moving ones
    ln_eps: float = 1e-5

    @property
    def batch(self) -> int:
        return int(sum(self.node_sizes))

    @property
    def n_nodes(self) -> int:
        return len(self.node_sizes)

    def with_nodes(self, node_sizes) -> "Workload":
        return replace(self, node_sizes=tuple(int(b) for b in node_sizes))


def _mlp(name, dims, bn, node_sizes, dtype, **kw) -> Workload:
    return Workload(name=name, kind="mlp", dims=tuple(dims), batchnorm=bn,
                    node_sizes=tuple(node_sizes), dtype=dtype, **kw)


def _enc(name, n_layers, d, h, ffn, T, vocab, node_sizes, dtype, **kw) -> Workload:
    return Workload(name=name, kind="encoder", n_layers=n_layers, d_model=d, n_heads=h,
                    d_ffn=ffn, seq_len=T, vocab=vocab, n_masked=int(0.15 * T),
                    node_sizes=tuple(node_sizes), dtype=dtype, **kw)


def _conv(name, img, in_ch, width, n_blocks, classes, node_sizes, dtype, **kw) -> Workload:
    return Workload(name=name, kind="conv", img=img, in_ch=in_ch, width=width, n_blocks=n_blocks,
                    classes=classes, batchnorm=True, node_sizes=tuple(node_sizes), dtype=dtype, **kw)


# The five named configurations (C1..C5) and small relatives used by the tests.
WORKLOADS: Dict[str, Workload] = {
    "C1": _mlp("C1", [784, 256, 10], False, [16] * 4, "f32", lr=0.1, momentum=0.9),
    "C2": _mlp("C2", [1024, 4096, 4096, 4096, 1000], True, [128] * 8, "bf16"),
    "C3": _mlp("C3", [1024, 4096, 4096, 4096, 1000], True,
               [48, 48, 32, 32, 16, 16, 48, 16], "bf16"),
    "C4": _enc("C4", 4, 768, 12, 3072, 128, 30522, [16] * 16, "bf16",
               optimizer="adam", lr=1e-4),
    "C5": _mlp("C5", [2048] + [8192] * 6 + [1000], True, [128] * 64, "bf16"),
    # small relatives: several tiles, ragged tails, seconds on the CPU
    "mlp_small_f32": _mlp("mlp_small_f32", [200, 136, 72, 10], False, [16, 7, 1, 24], "f32",
                          lr=0.1),
    "mlp_small_bn_f32": _mlp("mlp_small_bn_f32", [200, 136, 72, 10], True, [16, 7, 2, 23], "f32",
                             lr=0.1),
    # more than 1024 classes, an odd number of them: the loss kernel that keeps a row in registers,
    # writing the reduced logits to a buffer of their own
    "mlp_classes_f32": _mlp("mlp_classes_f32", [40, 48, 2051], False, [5, 3, 1, 7], "f32", lr=0.1),
    "mlp_mid_bn_bf16": _mlp("mlp_mid_bn_bf16", [256, 520, 392, 1000], True,
                            [48, 16, 128, 40, 8], "bf16"),
    "mlp_mid_bf16": _mlp("mlp_mid_bf16", [256, 520, 392, 1000], False,
                         [48, 16, 128, 40, 8], "bf16"),
    # layers wide enough for the 256 x 256 product tiles in one round per unit of sixteen 128-row nodes
    # (the input-gradient products whose epilogue takes the BatchNorm / ReLU backward pass)
    "mlp_wide_bn_bf16": _mlp("mlp_wide_bn_bf16", [64, 8192, 8192, 16], True, [128] * 16, "bf16"),
    "mlp_wide_bf16": _mlp("mlp_wide_bf16", [64, 8192, 8192, 16], False, [128] * 16, "bf16"),
    "mlp_big_node_bf16": _mlp("mlp_big_node_bf16", [256, 520, 392, 100], True,
                              [300, 212], "bf16"),
    "enc_tiny_f32": _enc("enc_tiny_f32", 2, 64, 2, 136, 16, 211, [3, 1, 2], "f32",
                         optimizer="adam", lr=1e-3),
    "enc_small_bf16": _enc("enc_small_bf16", 2, 128, 2, 264, 32, 1003, [4, 2, 3], "bf16",
                           optimizer="adam", lr=1e-4),
    "enc_mid_bf16": _enc("enc_mid_bf16", 2, 192, 3, 264, 64, 1003, [2, 1, 2], "bf16",
                         optimizer="adam", lr=1e-4),
    "enc_small_f32": _enc("enc_small_f32", 2, 128, 2, 264, 32, 1003, [4, 2, 3], "f32",
                          optimizer="adam", lr=1e-4),
    # nodes of 1024 and 1088 token rows, feed-forward width 1024: products on the 128 x 128 tiles, the
    # second node ending inside a tile
    "enc_wide_bf16": _enc("enc_wide_bf16", 1, 512, 8, 1024, 64, 1003, [16, 17], "bf16",
                          optimizer="adam", lr=1e-4),
    # widths that are not multiples of 4: the kernels' scalar paths
    "enc_odd_f32": _enc("enc_odd_f32", 1, 66, 2, 70, 8, 37, [2, 1, 1], "f32",
                        optimizer="adam", lr=1e-3),
    # vocabularies beyond 1024 entries, odd, so the logits' rows end inside a pair of columns
    "enc_vocab_f32": _enc("enc_vocab_f32", 1, 64, 2, 136, 16, 4099, [2, 1, 3], "f32",
                          optimizer="adam", lr=1e-3),
    "enc_vocab_bf16": _enc("enc_vocab_bf16", 1, 64, 2, 136, 16, 9001, [2, 1, 3], "bf16",
                           optimizer="adam", lr=1e-4),
    # second workload family: a residual network of 3x3 convolutions (the paper's headline
    # workloads are ResNets); C6 = 32 x 32 x 3 inputs, width 64, two blocks, nodes as in C2
    "C6": _conv("C6", 32, 3, 64, 2, 10, [128] * 8, "bf16"),
    "conv_tiny_f64": _conv("conv_tiny_f64", 5, 2, 8, 1, 4, [3, 2], "f64"),
    "conv_tiny_bf16": _conv("conv_tiny_bf16", 6, 3, 16, 1, 10, [5, 3, 8], "bf16"),
    "conv_small_bf16": _conv("conv_small_bf16", 12, 3, 24, 2, 10, [9, 16, 7], "bf16"),
    "conv_w64_bf16": _conv("conv_w64_bf16", 6, 3, 64, 1, 10, [3, 2, 4], "bf16"),
    # image sides that are powers of two: a stage of 64 positions is a whole image (8) or a quarter of one (16)
    "conv_w64_img8_bf16": _conv("conv_w64_img8_bf16", 8, 3, 64, 1, 10, [3, 2, 4], "bf16"),
    "conv_w64_img16_bf16": _conv("conv_w64_img16_bf16", 16, 3, 64, 1, 10, [2, 1], "bf16"),
    "conv_w64_img64_bf16": _conv("conv_w64_img64_bf16", 64, 3, 64, 1, 10, [1, 2], "bf16"),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


# ----------------------------------------------------------------------------
# parameter layout (names, shapes, init kind) -- structure only, no arithmetic
# ----------------------------------------------------------------------------

def param_layout(wl: Workload) -> List[Tuple[str, Tuple[int, ...], str]]:
    """List of (name, shape, init) in flat order.  init is one of
    'he' (normal, variance 2/fan_in with fan_in = shape[0]), 'he_conv' (the same with
    fan_in = the entries of one output channel's filter), 'emb' (normal, std 0.02), 'zeros',
    'ones'."""
    out: List[Tuple[str, Tuple[int, ...], str]] = []
    if wl.kind == "mlp":
        nl = len(wl.dims) - 1
        for l in range(nl):
            k, n = wl.dims[l], wl.dims[l + 1]
            out.append((f"l{l}.W", (k, n), "he"))
            last = l == nl - 1
            if last or not wl.batchnorm:
                out.append((f"l{l}.b", (n,), "zeros"))
            if wl.batchnorm and not last:
                out.append((f"l{l}.gamma", (n,), "ones"))
                out.append((f"l{l}.beta", (n,), "zeros"))
    elif wl.kind == "encoder":
        d, f = wl.d_model, wl.d_ffn
        out.append(("tok_emb", (wl.vocab, d), "emb"))
        out.append(("pos_emb", (wl.seq_len, d), "emb"))
        for l in range(wl.n_layers):
            out += [(f"l{l}.ln1.gamma", (d,), "ones"), (f"l{l}.ln1.beta", (d,), "zeros"),
                    (f"l{l}.Wqkv", (d, 3 * d), "he"), (f"l{l}.bqkv", (3 * d,), "zeros"),
                    (f"l{l}.Wo", (d, d), "he"), (f"l{l}.bo", (d,), "zeros"),
                    (f"l{l}.ln2.gamma", (d,), "ones"), (f"l{l}.ln2.beta", (d,), "zeros"),
                    (f"l{l}.W1", (d, f), "he"), (f"l{l}.b1", (f,), "zeros"),
                    (f"l{l}.W2", (f, d), "he"), (f"l{l}.b2", (d,), "zeros")]
        out += [("lnf.gamma", (d,), "ones"), ("lnf.beta", (d,), "zeros"),
                ("Wout", (d, wl.vocab), "he"), ("bout", (wl.vocab,), "zeros")]
    elif wl.kind == "conv":
        c = wl.width
        out += [("stem.W", (c, 3, 3, wl.in_ch), "he_conv"), ("stem.gamma", (c,), "ones"), ("stem.beta", (c,), "zeros")]
        for b in range(wl.n_blocks):
            out += [(f"b{b}.W1", (c, 3, 3, c), "he_conv"), (f"b{b}.gamma1", (c,), "ones"), (f"b{b}.beta1", (c,), "zeros"),
                    (f"b{b}.W2", (c, 3, 3, c), "he_conv"), (f"b{b}.gamma2", (c,), "ones"), (f"b{b}.beta2", (c,), "zeros")]
        out += [("fc.W", (c, wl.classes), "he"), ("fc.b", (wl.classes,), "zeros")]
    else:
        raise ValueError(wl.kind)
    return out


def num_params(wl: Workload) -> int:
    return int(sum(int(np.prod(s)) for _, s, _ in param_layout(wl)))


def make_params(wl: Workload, seed: int = SEED_PARAMS, jitter: float = 0.0) -> np.ndarray:
    """Flat fp32 parameter vector.  Normal draws are made in fp64 and cast to
    fp32.  `jitter` > 0 adds N(0, jitter^2) to the 'zeros'/'ones' tensors so that
    tests exercise bias / gamma / beta paths with non-trivial values."""
    rng = np.random.Generator(np.random.PCG64(seed))
    parts = []
    for _, shape, init in param_layout(wl):
        n = int(np.prod(shape))
        if init == "he":
            v = rng.standard_normal(n) * np.sqrt(2.0 / shape[0])
        elif init == "he_conv":
            v = rng.standard_normal(n) * np.sqrt(2.0 / int(np.prod(shape[1:])))
        elif init == "emb":
            v = rng.standard_normal(n) * 0.02
        elif init == "zeros":
            v = np.zeros(n) if jitter == 0.0 else rng.standard_normal(n) * jitter
        elif init == "ones":
            v = np.ones(n) if jitter == 0.0 else 1.0 + rng.standard_normal(n) * jitter
        else:
            raise ValueError(init)
        parts.append(v.astype(np.float32))
    return np.concatenate(parts)


def _to_bf16_representable(x32: np.ndarray) -> np.ndarray:
    """fp32 array whose values are exactly representable in bf16 (library cast)."""
    import torch
    return torch.from_numpy(x32).to(torch.bfloat16).to(torch.float32).numpy()


def make_batch(wl: Workload, seed_x: int = SEED_INPUTS, seed_y: int = SEED_LABELS,
               seed_mask: int = SEED_MASK) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (x, y).

    MLP:     x fp32 [B, D_in] ~ N(0,1) (bf16-representable when wl.dtype is
             bf16); y int32 [B] uniform in [0, n_classes).
    conv:    x fp32 [B, img, img, in_ch] ~ N(0,1) (bf16-representable when wl.dtype is bf16);
             y int32 [B] uniform in [0, classes).
    encoder: x int32 ids [B, T] uniform in [0, vocab) with the masked positions
             already replaced by id 0; y int32 [B, 2, n_masked] with
             y[:, 0, :] the masked positions (first n_masked entries of a seeded
             permutation of 0..T-1, sorted ascending) and y[:, 1, :] the
             original ids at those positions (the targets).
    """
    B = wl.batch
    if wl.kind == "mlp":
        rx = np.random.Generator(np.random.PCG64(seed_x))
        ry = np.random.Generator(np.random.PCG64(seed_y))
        x = rx.standard_normal((B, wl.dims[0])).astype(np.float32)
        if wl.dtype == "bf16":
            x = _to_bf16_representable(x)
        y = ry.integers(0, wl.dims[-1], size=B, dtype=np.int64).astype(np.int32)
        return x, y
    if wl.kind == "conv":
        rx = np.random.Generator(np.random.PCG64(seed_x))
        ry = np.random.Generator(np.random.PCG64(seed_y))
        x = rx.standard_normal((B, wl.img, wl.img, wl.in_ch)).astype(np.float32)
        if wl.dtype == "bf16":
            x = _to_bf16_representable(x)
        y = ry.integers(0, wl.classes, size=B, dtype=np.int64).astype(np.int32)
        return x, y
    rx = np.random.Generator(np.random.PCG64(seed_x))
    rm = np.random.Generator(np.random.PCG64(seed_mask))
    ids = rx.integers(0, wl.vocab, size=(B, wl.seq_len), dtype=np.int64).astype(np.int32)
    y = np.empty((B, 2, wl.n_masked), dtype=np.int32)
    for s in range(B):
        pos = np.sort(rm.permutation(wl.seq_len)[: wl.n_masked]).astype(np.int32)
        y[s, 0] = pos
        y[s, 1] = ids[s, pos]
        ids[s, pos] = 0
    return ids, y


def make_flat_gradients(n: int, count: int, seed: int = SEED_INPUTS) -> np.ndarray:
    """`count` random fp32 vectors of length n (stand-ins for node gradients)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    return rng.standard_normal((count, n)).astype(np.float32)
