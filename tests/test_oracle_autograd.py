"""Pin: library autograd (torch CPU, float64) run on every node's slice on its own,
combined with b_i/B -- the equal-size case is textbook gradient accumulation, which the
paper says virtual-node execution generalises (Section 8).  An independent third
implementation: no formula of the oracle is re-typed here, only library layers."""
from dataclasses import replace

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import vf_inputs as I


def _views(wl, flat_t):
    out, pos = {}, 0
    for name, shape, _ in I.param_layout(wl):
        n = int(np.prod(shape))
        out[name] = flat_t[pos:pos + n].view(*shape)
        pos += n
    return out


def _mlp_loss(wl, p, x, y):
    h = x
    nl = len(wl.dims) - 1
    for l in range(nl - 1):
        h = F.linear(h, p[f"l{l}.W"].t(), None if wl.batchnorm else p[f"l{l}.b"])
        if wl.batchnorm:
            h = F.batch_norm(h, None, None, p[f"l{l}.gamma"], p[f"l{l}.beta"], training=True,
                             eps=wl.bn_eps)
        h = F.relu(h)
    z = F.linear(h, p[f"l{nl-1}.W"].t(), p[f"l{nl-1}.b"])
    return F.cross_entropy(z, y, reduction="mean")


def _enc_loss(wl, p, ids, y):
    n, T = ids.shape
    d, nh = wl.d_model, wl.n_heads
    h = F.embedding(ids, p["tok_emb"]) + p["pos_emb"][:T]
    for l in range(wl.n_layers):
        a = F.layer_norm(h, (d,), p[f"l{l}.ln1.gamma"], p[f"l{l}.ln1.beta"], wl.ln_eps)
        qkv = F.linear(a, p[f"l{l}.Wqkv"].t(), p[f"l{l}.bqkv"])
        q, k, v = (t.view(n, T, nh, d // nh).transpose(1, 2) for t in qkv.split(d, dim=-1))
        o = F.scaled_dot_product_attention(q, k, v)
        o = o.transpose(1, 2).reshape(n, T, d)
        h = h + F.linear(o, p[f"l{l}.Wo"].t(), p[f"l{l}.bo"])
        f = F.layer_norm(h, (d,), p[f"l{l}.ln2.gamma"], p[f"l{l}.ln2.beta"], wl.ln_eps)
        u = F.gelu(F.linear(f, p[f"l{l}.W1"].t(), p[f"l{l}.b1"]))
        h = h + F.linear(u, p[f"l{l}.W2"].t(), p[f"l{l}.b2"])
    h = F.layer_norm(h, (d,), p["lnf.gamma"], p["lnf.beta"], wl.ln_eps)
    pos = y[:, 0, :]
    rows = torch.gather(h, 1, pos.unsqueeze(-1).expand(-1, -1, d)).reshape(-1, d)
    z = F.linear(rows, p["Wout"].t(), p["bout"])
    return F.cross_entropy(z, y[:, 1, :].reshape(-1), reduction="mean")


def _conv_loss(wl, p, x, y):
    """Library convolution (NCHW, filters [out, in, kh, kw]), batch statistics per call."""
    def conv_bn(h, W, gamma, beta):
        z = F.conv2d(h, W.permute(0, 3, 1, 2), padding=1)
        return F.batch_norm(z, None, None, gamma, beta, training=True, eps=wl.bn_eps)
    h = F.relu(conv_bn(x.permute(0, 3, 1, 2), p["stem.W"], p["stem.gamma"], p["stem.beta"]))
    for b in range(wl.n_blocks):
        t = F.relu(conv_bn(h, p[f"b{b}.W1"], p[f"b{b}.gamma1"], p[f"b{b}.beta1"]))
        h = F.relu(conv_bn(t, p[f"b{b}.W2"], p[f"b{b}.gamma2"], p[f"b{b}.beta2"]) + h)
    z = F.linear(h.mean(dim=(2, 3)), p["fc.W"].t(), p["fc.b"])
    return F.cross_entropy(z, y, reduction="mean")


def _autograd_step(wl, theta, x, y):
    sizes = wl.node_sizes
    B = sum(sizes)
    G = np.zeros(theta.size)
    loss = 0.0
    node_losses = []
    lo = 0
    for b in sizes:
        t = torch.tensor(theta, dtype=torch.float64, requires_grad=True)
        p = _views(wl, t)
        if wl.kind == "mlp":
            li = _mlp_loss(wl, p, torch.tensor(x[lo:lo + b], dtype=torch.float64),
                           torch.tensor(y[lo:lo + b], dtype=torch.int64))
        elif wl.kind == "conv":
            li = _conv_loss(wl, p, torch.tensor(x[lo:lo + b], dtype=torch.float64),
                            torch.tensor(y[lo:lo + b], dtype=torch.int64))
        else:
            li = _enc_loss(wl, p, torch.tensor(x[lo:lo + b], dtype=torch.int64),
                           torch.tensor(y[lo:lo + b], dtype=torch.int64))
        li.backward()
        G += (b / B) * t.grad.numpy()
        loss += (b / B) * float(li.detach())
        node_losses.append(float(li.detach()))
        lo += b
    return loss, G, np.array(node_losses)


@pytest.mark.parametrize("name", ["mlp_small_f32", "mlp_small_bn_f32", "mlp_mid_bn_bf16", "enc_tiny_f32",
                                  "enc_small_bf16", "C1", "conv_tiny_bf16", "conv_small_bf16"])
def test_oracle_matches_autograd_per_node(name):
    wl = replace(I.workload(name), dtype="f64")
    theta = I.make_params(wl, jitter=0.2).astype(np.float64)
    x, y = I.make_batch(wl)
    r = O.oracle_step(wl, theta, x, y)
    loss, G, node_losses = _autograd_step(wl, theta, x, y)
    assert abs(r["loss"] - loss) <= 1e-12 * abs(loss)
    np.testing.assert_allclose(r["node_losses"], node_losses, rtol=1e-12)
    assert np.linalg.norm(r["G"] - G) <= 1e-11 * np.linalg.norm(G)
    assert np.max(np.abs(r["G"] - G)) <= 1e-11 * np.max(np.abs(G))


def test_optimizers_match_library():
    rng = np.random.Generator(np.random.PCG64(11))
    th0 = rng.standard_normal(200)
    grads = rng.standard_normal((4, 200))
    # SGD with momentum, no dampening, no Nesterov
    t = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.SGD([t], lr=0.05, momentum=0.9)
    th, v = th0, np.zeros(200)
    for g in grads:
        t.grad = torch.tensor(g)
        opt.step()
        th, v = O.sgdm_update(th, g, v, 0.05, 0.9)
        np.testing.assert_allclose(th, t.detach().numpy(), rtol=1e-12, atol=1e-14)
    # Adam
    t = torch.tensor(th0, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([t], lr=1e-3, betas=(0.9, 0.999), eps=1e-8)
    th, m, u = th0, np.zeros(200), np.zeros(200)
    for k, g in enumerate(grads):
        t.grad = torch.tensor(g)
        opt.step()
        th, m, u = O.adam_update(th, g, m, u, k + 1, 1e-3, 0.9, 0.999, 1e-8)
        np.testing.assert_allclose(th, t.detach().numpy(), rtol=1e-10, atol=1e-13)
