"""One virtual-node training step, by definition (Section 3.2 steps 1-5, Section 5.2)."""
import numpy as np

from . import layers as L
from .numerics import round_to_bf16
from .optim import adam_update, sgdm_update
from .partition import partition


# ---- flat parameter layout (the oracle's own statement of it) -------------------------

def layout(wl):
    """[(name, shape)] in flat order: tensors in forward order; a Linear's weight
    [K_in, N_out] row-major, then its bias, then the normalisation scale and shift."""
    out = []
    if wl.kind == "mlp":
        n_lin = len(wl.dims) - 1
        for l in range(n_lin):
            k, n = wl.dims[l], wl.dims[l + 1]
            hidden = l < n_lin - 1
            out.append((f"l{l}.W", (k, n)))
            if not (hidden and wl.batchnorm):
                out.append((f"l{l}.b", (n,)))     # a bias feeding BatchNorm would have zero gradient
            if hidden and wl.batchnorm:
                out.append((f"l{l}.gamma", (n,)))
                out.append((f"l{l}.beta", (n,)))
        return out
    if wl.kind == "conv":
        # filters [out channel, kh, kw, in channel]; every convolution feeds a BatchNorm (no bias)
        c = wl.width
        out += [("stem.W", (c, 3, 3, wl.in_ch)), ("stem.gamma", (c,)), ("stem.beta", (c,))]
        for b in range(wl.n_blocks):
            out += [(f"b{b}.W1", (c, 3, 3, c)), (f"b{b}.gamma1", (c,)), (f"b{b}.beta1", (c,)),
                    (f"b{b}.W2", (c, 3, 3, c)), (f"b{b}.gamma2", (c,)), (f"b{b}.beta2", (c,))]
        out += [("fc.W", (c, wl.classes)), ("fc.b", (wl.classes,))]
        return out
    d, f = wl.d_model, wl.d_ffn
    out.append(("tok_emb", (wl.vocab, d)))
    out.append(("pos_emb", (wl.seq_len, d)))
    for l in range(wl.n_layers):
        out += [(f"l{l}.ln1.gamma", (d,)), (f"l{l}.ln1.beta", (d,)),
                (f"l{l}.Wqkv", (d, 3 * d)), (f"l{l}.bqkv", (3 * d,)),
                (f"l{l}.Wo", (d, d)), (f"l{l}.bo", (d,)),
                (f"l{l}.ln2.gamma", (d,)), (f"l{l}.ln2.beta", (d,)),
                (f"l{l}.W1", (d, f)), (f"l{l}.b1", (f,)),
                (f"l{l}.W2", (f, d)), (f"l{l}.b2", (d,))]
    out += [("lnf.gamma", (d,)), ("lnf.beta", (d,)),
            ("Wout", (d, wl.vocab)), ("bout", (wl.vocab,))]
    return out


def unflatten(wl, flat):
    """dict name -> view of `flat` with the tensor's shape."""
    views, pos = {}, 0
    for name, shape in layout(wl):
        n = int(np.prod(shape))
        views[name] = flat[pos:pos + n].reshape(shape)
        pos += n
    if pos != flat.size:
        raise ValueError(f"parameter vector has {flat.size} entries, layout needs {pos}")
    return views


def _flatten(wl, grads):
    return np.concatenate([np.asarray(grads[name], dtype=np.float64).reshape(-1)
                           for name, _ in layout(wl)])


# ---- one node: loss L_i (mean over the node) and g_i = dL_i/dtheta ----------------------

def _operand(wl):
    """How a tensor enters a contraction.  bf16 workloads are defined with bf16 weights
    AND activations, fp32 accumulation, their contractions (Linear, convolution and
    attention products; forward, input gradient and weight gradient) being bf16 products:
    every operand of a contraction -- the activation fed to a Linear or convolution, q, k, v
    and the probabilities of an attention product, and the gradient fed to a backward
    contraction -- is a bf16 tensor, rounded to nearest even once, where it is produced.
    Nothing else is rounded: what a contraction puts out, normalisation statistics, softmax,
    losses, the residual stream and sums over rows are float64.  This also puts the one
    discontinuous decision of the MLP, the ReLU mask of the next layer, at the same
    precision on both sides of a parity check."""
    if wl.dtype == "bf16":
        return lambda a: round_to_bf16(np.asarray(a, dtype=np.float32))
    return lambda a: a


def _mlp_node(wl, p, x, y):
    q = _operand(wl)
    n_lin = len(wl.dims) - 1
    h = np.asarray(x, dtype=np.float64)
    saved = []
    margin = np.inf
    for l in range(n_lin - 1):
        z = L.linear_fwd(h, p[f"l{l}.W"], None if wl.batchnorm else p[f"l{l}.b"])
        if wl.batchnorm:
            pre, bn_cache = L.batchnorm_fwd(z, p[f"l{l}.gamma"], p[f"l{l}.beta"], wl.bn_eps)
        else:
            pre, bn_cache = z, None
        saved.append((h, pre, bn_cache))
        # diagnostic: how close any ReLU input of this node is to the kink, relative to the
        # layer's typical magnitude (a fp32 implementation may legitimately flip such a unit)
        margin = min(margin, float(np.min(np.abs(pre)) / np.sqrt(np.mean(pre * pre))))
        h = q(L.relu_fwd(pre))
    last = n_lin - 1
    logits = L.linear_fwd(h, p[f"l{last}.W"], p[f"l{last}.b"])
    loss, dlogits = L.softmax_xent_fwd_bwd(logits, np.asarray(y, dtype=np.int64))

    g = {}
    dh, g[f"l{last}.W"], _ = L.linear_bwd(h, p[f"l{last}.W"], q(dlogits), False)
    g[f"l{last}.b"] = dlogits.sum(axis=0)
    for l in range(n_lin - 2, -1, -1):
        h_in, pre, bn_cache = saved[l]
        dpre = L.relu_bwd(dh, pre)
        if wl.batchnorm:
            dz, g[f"l{l}.gamma"], g[f"l{l}.beta"] = L.batchnorm_bwd(dpre, p[f"l{l}.gamma"], bn_cache)
        else:
            dz = dpre
            g[f"l{l}.b"] = dz.sum(axis=0)
        dh, g[f"l{l}.W"], _ = L.linear_bwd(h_in, p[f"l{l}.W"], q(dz), False)
    stats = [(c[2], c[3]) for _, _, c in saved] if wl.batchnorm else []
    return loss, g, margin, stats


def _bn_rows(z, gamma, beta, eps):
    """BatchNorm of an NHWC tensor: statistics per channel over all rows (n, h, w) of the node."""
    pre, cache = L.batchnorm_fwd(z.reshape(-1, z.shape[-1]), gamma, beta, eps)
    return pre.reshape(z.shape), cache


def _bn_rows_bwd(dpre, gamma, cache):
    dz, dg, db = L.batchnorm_bwd(dpre.reshape(-1, dpre.shape[-1]), gamma, cache)
    return dz.reshape(dpre.shape), dg, db


def _conv_node(wl, p, x, y):
    """Residual network of 3x3 convolutions on one node's images x [n, H, W, in_ch]:
    stem (convolution, BatchNorm, ReLU); blocks of convolution-BatchNorm-ReLU-convolution-
    BatchNorm, the block's input added, ReLU; mean over the positions; Linear; mean
    cross-entropy over the node.  Every BatchNorm takes its statistics over the node's
    n*H*W positions (Section 4.1).  bf16 workloads: the stored activations (operands of the
    next convolution, and the addend of the skip connection), the pooled features and every
    gradient handed to a backward contraction are rounded to bf16; convolution outputs,
    statistics, sums and the gradients between contractions stay float64."""
    q = _operand(wl)
    n, H, Wd, _ = x.shape
    rms = lambda t: float(np.min(np.abs(t)) / np.sqrt(np.mean(t * t)))
    stats = []
    h0 = np.asarray(x, dtype=np.float64)
    z = L.conv3x3_fwd(h0, p["stem.W"])
    pre, c0 = _bn_rows(z, p["stem.gamma"], p["stem.beta"], wl.bn_eps)
    stats.append((c0[2], c0[3]))
    margin = rms(pre)
    a = q(L.relu_fwd(pre))
    saved = []
    for b in range(wl.n_blocks):
        z1 = L.conv3x3_fwd(a, p[f"b{b}.W1"])
        pre1, c1 = _bn_rows(z1, p[f"b{b}.gamma1"], p[f"b{b}.beta1"], wl.bn_eps)
        a1 = q(L.relu_fwd(pre1))
        z2 = L.conv3x3_fwd(a1, p[f"b{b}.W2"])
        pre2, c2 = _bn_rows(z2, p[f"b{b}.gamma2"], p[f"b{b}.beta2"], wl.bn_eps)
        s = pre2 + a                                   # skip connection: the block's (stored) input
        stats += [(c1[2], c1[3]), (c2[2], c2[3])]
        margin = min(margin, rms(pre1), rms(s))
        saved.append((a, pre1, c1, a1, c2, s))
        a = q(L.relu_fwd(s))
    pooled = q(a.sum(axis=(1, 2)) / (H * Wd))          # [n, width]
    logits = L.linear_fwd(pooled, p["fc.W"], p["fc.b"])
    loss, dlogits = L.softmax_xent_fwd_bwd(logits, np.asarray(y, dtype=np.int64))

    g = {}
    dpooled, g["fc.W"], g["fc.b"] = L.linear_bwd(pooled, p["fc.W"], q(dlogits), True)
    g["fc.b"] = dlogits.sum(axis=0)                    # bias gradient from the unrounded dlogits, as in the MLP
    da = np.broadcast_to(dpooled[:, None, None, :] / (H * Wd), (n, H, Wd, dpooled.shape[1]))
    for b in range(wl.n_blocks - 1, -1, -1):
        a_in, pre1, c1, a1, c2, s = saved[b]
        ds = L.relu_bwd(da, s)
        dz2, g[f"b{b}.gamma2"], g[f"b{b}.beta2"] = _bn_rows_bwd(ds, p[f"b{b}.gamma2"], c2)
        da1, g[f"b{b}.W2"] = L.conv3x3_bwd(a1, p[f"b{b}.W2"], q(dz2))
        dpre1 = L.relu_bwd(da1, pre1)
        dz1, g[f"b{b}.gamma1"], g[f"b{b}.beta1"] = _bn_rows_bwd(dpre1, p[f"b{b}.gamma1"], c1)
        dconv, g[f"b{b}.W1"] = L.conv3x3_bwd(a_in, p[f"b{b}.W1"], q(dz1))
        da = dconv + ds                                # through the convolutions + through the skip
    dpre = L.relu_bwd(da, pre)
    dz, g["stem.gamma"], g["stem.beta"] = _bn_rows_bwd(dpre, p["stem.gamma"], c0)
    _, g["stem.W"] = L.conv3x3_bwd(h0, p["stem.W"], q(dz), need_dx=False)
    return loss, g, margin, stats


def _split_heads(t, n_heads):
    n, T, d = t.shape
    return t.reshape(n, T, n_heads, d // n_heads).transpose(0, 2, 1, 3)


def _merge_heads(t):
    n, nh, T, dh = t.shape
    return t.transpose(0, 2, 1, 3).reshape(n, T, nh * dh)


def _encoder_node(wl, p, ids, y):
    """ids [n, T] token ids (masked positions already hold id 0); y [n, 2, m]:
    y[:,0] positions, y[:,1] target ids.  Pre-LayerNorm encoder, GELU FFN, final
    LayerNorm, untied output projection on the masked rows, mean cross-entropy
    over the node's n*m masked rows.

    bf16 workloads: the operands of every contraction are rounded to bf16 by `q_`
    -- forward: the LayerNorm outputs, q/k/v, the attention probabilities, the merged
    attention output, the GELU output and the gathered final rows; backward: the
    gradient at every Linear layer's output, the gradient of the attention output
    and the score gradient.  The FFN pre-activation (a Linear layer's output, read
    only by the GELU), the logits, the residual stream and the statistics stay
    float64."""
    q_ = _operand(wl)
    ids = np.asarray(ids, dtype=np.int64)
    y = np.asarray(y, dtype=np.int64)
    n, T = ids.shape
    d, nh, ffn = wl.d_model, wl.n_heads, wl.d_ffn
    h = p["tok_emb"][ids] + p["pos_emb"][None, :T, :]
    saved = []
    for l in range(wl.n_layers):
        a, c1 = L.layernorm_fwd(h, p[f"l{l}.ln1.gamma"], p[f"l{l}.ln1.beta"], wl.ln_eps)
        a = q_(a)
        qkv = q_(L.linear_fwd(a, p[f"l{l}.Wqkv"], p[f"l{l}.bqkv"]))
        q, k, v = (_split_heads(qkv[..., i * d:(i + 1) * d], nh) for i in range(3))
        o, prob = L.attention_fwd(q, k, v, q_)
        om = q_(_merge_heads(o))
        h_mid = h + L.linear_fwd(om, p[f"l{l}.Wo"], p[f"l{l}.bo"])
        f, c2 = L.layernorm_fwd(h_mid, p[f"l{l}.ln2.gamma"], p[f"l{l}.ln2.beta"], wl.ln_eps)
        f = q_(f)
        u = L.linear_fwd(f, p[f"l{l}.W1"], p[f"l{l}.b1"])
        gl = q_(L.gelu_fwd(u))
        h_out = h_mid + L.linear_fwd(gl, p[f"l{l}.W2"], p[f"l{l}.b2"])
        saved.append((a, c1, q, k, v, prob, om, f, c2, u, gl))
        h = h_out
    hf, cf = L.layernorm_fwd(h, p["lnf.gamma"], p["lnf.beta"], wl.ln_eps)
    seq = np.repeat(np.arange(n), y.shape[2])
    pos = y[:, 0, :].reshape(-1)
    tgt = y[:, 1, :].reshape(-1)
    rows = q_(hf[seq, pos, :])                              # [n*m, d]
    logits = L.linear_fwd(rows, p["Wout"], p["bout"])
    loss, dlogits = L.softmax_xent_fwd_bwd(logits, tgt)

    g = {}
    drows, g["Wout"], g["bout"] = L.linear_bwd(rows, p["Wout"], q_(dlogits), True)
    dhf = np.zeros_like(hf)
    np.add.at(dhf, (seq, pos), drows)
    dh, g["lnf.gamma"], g["lnf.beta"] = L.layernorm_bwd(dhf, p["lnf.gamma"], cf)
    for l in range(wl.n_layers - 1, -1, -1):
        a, c1, q, k, v, prob, om, f, c2, u, gl = saved[l]
        dgl, g[f"l{l}.W2"], _ = L.linear_bwd(gl.reshape(-1, ffn), p[f"l{l}.W2"], q_(dh.reshape(-1, d)), False)
        g[f"l{l}.b2"] = dh.reshape(-1, d).sum(axis=0)
        du = q_(L.gelu_bwd(dgl, u.reshape(-1, ffn)))
        df, g[f"l{l}.W1"], g[f"l{l}.b1"] = L.linear_bwd(f.reshape(-1, d), p[f"l{l}.W1"], du, True)
        dmid, g[f"l{l}.ln2.gamma"], g[f"l{l}.ln2.beta"] = L.layernorm_bwd(
            df.reshape(n, T, d), p[f"l{l}.ln2.gamma"], c2)
        dmid = dmid + dh                                     # residual around the FFN
        dom, g[f"l{l}.Wo"], _ = L.linear_bwd(om.reshape(-1, d), p[f"l{l}.Wo"], q_(dmid.reshape(-1, d)), False)
        g[f"l{l}.bo"] = dmid.reshape(-1, d).sum(axis=0)
        dq, dk, dv = L.attention_bwd(_split_heads(q_(dom.reshape(n, T, d)), nh), q, k, v, prob, q_)
        dqkv = q_(np.concatenate([_merge_heads(dq), _merge_heads(dk), _merge_heads(dv)], axis=-1))
        da, g[f"l{l}.Wqkv"], g[f"l{l}.bqkv"] = L.linear_bwd(a.reshape(-1, d), p[f"l{l}.Wqkv"],
                                                            dqkv.reshape(-1, 3 * d), True)
        din, g[f"l{l}.ln1.gamma"], g[f"l{l}.ln1.beta"] = L.layernorm_bwd(
            da.reshape(n, T, d), p[f"l{l}.ln1.gamma"], c1)
        dh = din + dmid                                      # residual around attention
    g["pos_emb"] = np.zeros_like(p["pos_emb"])
    g["pos_emb"][:T] = dh.sum(axis=0)
    g["tok_emb"] = np.zeros_like(p["tok_emb"])
    np.add.at(g["tok_emb"], ids.reshape(-1), dh.reshape(-1, d))
    return loss, g, np.inf


def node_loss_and_grads(wl, compute_params, x_node, y_node, diag=None):
    """(L_i, flat g_i) for one node given float64 compute parameters (flat).  `diag`, if a
    dict, receives 'relu_margin': the smallest |ReLU input| of the node relative to its
    layer's rms (inf for models without ReLU)."""
    p = unflatten(wl, compute_params)
    if wl.kind == "mlp":
        loss, g, margin, stats = _mlp_node(wl, p, x_node, y_node)
    elif wl.kind == "conv":
        loss, g, margin, stats = _conv_node(wl, p, np.asarray(x_node), y_node)
    else:
        loss, g, margin = _encoder_node(wl, p, x_node, y_node)
        stats = []
    if diag is not None:
        diag["relu_margin"] = margin
        diag["bn_stats"] = stats          # per BatchNorm layer: (mean, biased variance) of this node
    return loss, _flatten(wl, g)


def compute_copy(wl, theta):
    """Parameters the forward/backward passes see: fp32 master values, rounded to
    bf16 for bf16 workloads; returned as float64."""
    if wl.dtype == "f64":                                    # tests only: no rounding at all
        return np.asarray(theta, dtype=np.float64).copy()
    theta32 = np.asarray(theta, dtype=np.float32)
    if wl.dtype == "bf16":
        return round_to_bf16(theta32)
    return theta32.astype(np.float64)


def new_state(wl, n):
    st = {"t": 0, "v": np.zeros(n)} if wl.optimizer == "sgdm" else {"t": 0, "m": np.zeros(n), "u": np.zeros(n)}
    if wl.kind in ("mlp", "conv") and wl.batchnorm:      # moving statistics start at mean 0, variance 1
        widths = wl.dims[1:-1] if wl.kind == "mlp" else [wl.width] * (1 + 2 * wl.n_blocks)
        st["bn_mean"] = [np.zeros(n_) for n_ in widths]
        st["bn_var"] = [np.ones(n_) for n_ in widths]
    return st


def blend_moving_stats(moving_mean, moving_var, node_stats, share):
    """Section 4.1: moving mean / variance belong to the device and are updated by every pass
    it runs, i.e. once per virtual node, in node order, from that node's own statistics
    (biased variance): moving <- (1 - share) * moving + share * node."""
    mean = [(1.0 - share) * m + share * s[0] for m, s in zip(moving_mean, node_stats)]
    var = [(1.0 - share) * v + share * s[1] for v, s in zip(moving_var, node_stats)]
    return mean, var


def oracle_step(wl, theta, x, y, node_sizes=None, state=None, nodes=None):
    """One step.  theta: flat fp32 master parameters.  Returns a dict with
    off, w (bit-exact data), loss, node_losses, G (float64 [P]), theta (float64
    [P] after the update), state (after the update).  `nodes` limits the nodes
    that are evaluated (timing a sample of the work); G and the update are then
    partial and must not be compared.  'relu_margin' is a diagnostic for parity checks:
    the smallest |ReLU input| relative to its layer's rms over the whole step."""
    sizes = list(wl.node_sizes if node_sizes is None else node_sizes)
    off, w = partition(sizes, len(x))
    cp = compute_copy(wl, theta)
    n = cp.size
    G = np.zeros(n)
    loss = 0.0
    node_losses = []
    relu_margin = np.inf
    which = range(len(sizes)) if nodes is None else nodes
    state = new_state(wl, n) if state is None else state
    bn_mean, bn_var = state.get("bn_mean"), state.get("bn_var")
    for i in which:                                          # node after node (Section 3.2)
        lo, hi = int(off[i]), int(off[i + 1])
        diag = {}
        L_i, g_i = node_loss_and_grads(wl, cp, x[lo:hi], y[lo:hi], diag)
        weight = sizes[i] / float(len(x))                    # b_i / B (Section 5.2)
        G += weight * g_i
        loss += weight * L_i
        node_losses.append(L_i)
        relu_margin = min(relu_margin, diag["relu_margin"])
        if bn_mean is not None:
            bn_mean, bn_var = blend_moving_stats(bn_mean, bn_var, diag["bn_stats"], wl.bn_momentum)
    t = state["t"] + 1
    theta64 = (np.asarray(theta, dtype=np.float64) if wl.dtype == "f64"
               else np.asarray(theta, dtype=np.float32).astype(np.float64))
    if wl.optimizer == "sgdm":
        theta_new, v = sgdm_update(theta64, G, state["v"], wl.lr, wl.momentum)
        new = {"t": t, "v": v}
    else:
        theta_new, m, u = adam_update(theta64, G, state["m"], state["u"], t, wl.lr,
                                      wl.beta1, wl.beta2, wl.adam_eps)
        new = {"t": t, "m": m, "u": u}
    if bn_mean is not None:
        new["bn_mean"], new["bn_var"] = bn_mean, bn_var
    return {"off": off, "w": w, "loss": loss, "node_losses": np.array(node_losses),
            "G": G, "theta": theta_new, "state": new, "relu_margin": relu_margin}
