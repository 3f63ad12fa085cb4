"""GPU parity: the HIP path through the C ABI against the CPU oracle, MLP workloads."""
import numpy as np
import pytest

import oracle as O
import vf_inputs as I
from vfharness import (TOL, check_against_oracle, check_independent_bound, check_update_from_own_gradient,
                       float32_products, oracle_steps, run_gpu, weights_only_gradient)

pytestmark = pytest.mark.gpu

FUSED = 1
NO_GRAPH = 2


def _case(name, jitter=0.1):
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=jitter)
    x, y = I.make_batch(wl)
    return wl, theta, x, y


@pytest.mark.parametrize("flags", [NO_GRAPH, 0, FUSED | NO_GRAPH, FUSED])
@pytest.mark.parametrize("name", ["C1", "mlp_small_f32", "mlp_small_bn_f32", "mlp_mid_bf16", "mlp_mid_bn_bf16",
                                  "mlp_big_node_bf16", "mlp_classes_f32"])
def test_mlp_step_matches_oracle(name, flags):
    print(f"case {name} flags={flags}", flush=True)
    wl, theta, x, y = _case(name)
    gpu = run_gpu(wl, theta, x, y, flags=flags)
    ref = oracle_steps(wl, theta, x, y)
    check_against_oracle(wl, gpu, ref)
    check_update_from_own_gradient(wl, gpu, theta)


def test_c1_exact_configuration():
    """MLP 784-256-10, fp32, B=64 in 4 nodes of 16, He init, one SGD step lr 0.1 mu 0.9."""
    wl, theta, x, y = _case("C1", jitter=0.0)
    gpu = run_gpu(wl, theta, x, y)
    ref = oracle_steps(wl, theta, x, y)
    check_against_oracle(wl, gpu, ref, tol=1e-4)


@pytest.mark.parametrize("name", ["mlp_small_bn_f32", "mlp_mid_bn_bf16"])
def test_two_steps_carry_momentum(name):
    wl, theta, x, y = _case(name)
    gpu = run_gpu(wl, theta, x, y, steps=2)
    ref = oracle_steps(wl, theta, x, y, steps=2)
    check_against_oracle(wl, gpu, ref, tol=2 * TOL[wl.dtype])


def test_fused_and_staged_accumulation_agree_bitwise():
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    a = run_gpu(wl, theta, x, y, flags=0)
    b = run_gpu(wl, theta, x, y, flags=FUSED)
    assert a["G"].tobytes() == b["G"].tobytes()
    assert a["theta"].tobytes() == b["theta"].tobytes()


def test_graph_replay_is_repeatable():
    """Several replays of the captured node sequence, with eager work between them."""
    import torch
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    eager = run_gpu(wl, theta, x, y, flags=NO_GRAPH, steps=3)
    torch.cuda.synchronize()
    graph = run_gpu(wl, theta, x, y, flags=0, steps=3)
    assert eager["G"].tobytes() == graph["G"].tobytes()
    assert eager["theta"].tobytes() == graph["theta"].tobytes()


@pytest.mark.parametrize("flags,window", [(0, 0), (FUSED, 0), (FUSED, 4), (FUSED | NO_GRAPH | 4, 4)])
@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_mid_bf16"])
def test_ragged_node_sizes(name, flags, window):
    """Node sizes that are no multiple of anything (13, 7, 1, 33, 50 rows) and one longer than the
    register-resident BatchNorm path and the single-trip weight-gradient kernels take (136):
    every 16-byte access of the transposed copies ends in padding, never in a neighbour's rows."""
    wl, theta, x, y = _case(name)
    sizes = [13, 7, 1, 33, 50, 136]
    assert sum(sizes) == wl.batch
    gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=flags, fold_window=window, steps=2)
    ref = oracle_steps(wl, theta, x, y, node_sizes=sizes, steps=2)
    check_against_oracle(wl, gpu, ref, tol=2 * TOL[wl.dtype])


def test_partition_invariance_on_device_without_batchnorm():
    wl, theta, x, y = _case("mlp_small_f32")
    a = run_gpu(wl, theta, x, y, node_sizes=[wl.batch])
    b = run_gpu(wl, theta, x, y, node_sizes=[1] * wl.batch)
    c = run_gpu(wl, theta, x, y)
    for other in (b, c):
        assert np.linalg.norm(other["G"] - a["G"]) <= 1e-5 * np.linalg.norm(a["G"])


def test_workspace_independent_of_node_count():
    """The gradient buffer and the per-node workspace do not grow with V (Section 3.3)."""
    wl, theta, x, y = _case("mlp_small_bn_f32")
    sizes = {}
    for V in (1, 2, 4, 16, 64):
        r = run_gpu(wl, theta, x[:16], y[:16], node_sizes=[16], max_node_size=16, max_nodes=V,
                    max_batch=16 * 64)
        sizes[V] = r["workspace_bytes"]
    assert len(set(sizes.values())) == 1, sizes


def test_rejected_step_leaves_state_untouched():
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import VF_EINVAL, config_from_workload
    wl, theta, x, y = _case("mlp_small_f32")
    stream = torch.cuda.Stream()
    eng = vf.VirtualNodeStep(config_from_workload(wl, stream=stream))
    params = torch.from_numpy(theta).cuda()
    before = params.clone()
    xt, yt = torch.from_numpy(x).cuda(), torch.from_numpy(y).cuda()
    B = wl.batch
    for sizes, V in (([B - 1], 1), ([B, 0], 2), ([B + 1, -1], 2), (list(wl.node_sizes) + [1], 5),
                     ([B], 1)):   # last: b_i > max_node_size
        rc = eng.step_raw(params.data_ptr(), xt.data_ptr(), yt.data_ptr(), B, V, sizes)
        assert rc == VF_EINVAL, (sizes, rc)
    assert eng.step_raw(0, xt.data_ptr(), yt.data_ptr(), B, 1, [B]) == VF_EINVAL
    torch.cuda.synchronize()
    assert torch.equal(params, before) and eng.step_count == 0
    with pytest.raises(vf.VfError):
        eng.loss()
    eng.close()


BENCH = FUSED | NO_GRAPH | 4        # what bench.py times: fused fold, two streams, eager launches, window 8


BENCH_GROUP = 32                    # ... and up to 32 nodes through their passes together


@pytest.mark.parametrize("name,flags,window,group", [("C2", BENCH, 8, BENCH_GROUP), ("C3", BENCH, 8, BENCH_GROUP),
                                                     ("C2", BENCH, 8, 1), ("C2", 0, 0, 0), ("C3", FUSED, 0, 0)])
def test_full_size_configurations(name, flags, window, group):
    """The 8 x 128 configuration (C2) and the heterogeneous split (C3) at full size, in the
    launch configuration bench.py times (and node after node, and in the plain staged / fused
    modes), every gradient entry against the oracle."""
    print(f"full size {name} flags={flags} window={window} group={group}", flush=True)
    wl, theta, x, y = _case(name, jitter=0.0)
    gpu = run_gpu(wl, theta, x, y, flags=flags, fold_window=window, node_group=group)
    ref = oracle_steps(wl, theta, x, y)
    check_against_oracle(wl, gpu, ref)
    check_update_from_own_gradient(wl, gpu, theta)
    off, w = O.partition(wl.node_sizes, wl.batch)
    import paper_2009_09523_amd as vf
    off2, w2 = vf.vf_partition(wl.node_sizes, wl.batch)
    assert off.tobytes() == off2.tobytes() and w.tobytes() == w2.tobytes()
    if flags == BENCH and group == BENCH_GROUP:
        check_independent_bound(wl, gpu["G"], ref["G"], weights_only_gradient(wl, theta, x, y), name)


def test_c5_full_size_launch_configuration():
    """Large-batch emulation: MLP 2048-8192x6-1000 + BatchNorm, 64 nodes of 128 (B = 8192), in the
    launch configuration bench.py times (fused fold, two streams, launches one by one, units
    of 32 nodes per pass, one window over the two units).  The oracle can afford single nodes of this
    model: it evaluates the eight distinct nodes 0..7, and the device runs V = 64 nodes of which node i
    holds the rows of node i mod 8 (a unit of the device's passes is these eight nodes twice, its
    BatchNorm launches take eight nodes each) -- the combined gradient is then
    (g_0 + .. + g_7)/8 (Section 5.2 with 64 weights of 1/64), every fold of step 3 and the update of
    step 5 run over all 64 nodes.

    Tolerance.  Six BatchNorm+ReLU layers with bf16 operands are sensitive to rounding: a
    difference delta of a pre-activation moves about delta/ulp of the bf16 roundings of the
    layer's output, i.e. it leaves the layer with size sqrt(delta*ulp), so ANY two correct
    evaluations (a different summation order is enough) drift apart layer by layer until they
    differ at the bf16 ulp level.  Per tensor the test therefore first measures, on the CPU, how
    far a second valid evaluation (the oracle with its forward products in float32) lies from
    the oracle: tensors for which that distance is below half of 2e-2 are held to 2e-2; the
    others -- stated as NOT meeting 2e-2, here and in the design notes -- to twice that distance.
    The loss is held to 1e-3."""
    print("full size C5", flush=True)
    from oracle.step import compute_copy
    from vfharness import tensor_errors
    wl = I.workload("C5")
    theta = I.make_params(wl)
    x, y = I.make_batch(wl)
    cp = compute_copy(wl, theta)
    K = 8
    Ls, want, alt = [], 0.0, 0.0
    for k in range(K):
        lo, hi = 128 * k, 128 * (k + 1)
        L_k, g_k = O.node_loss_and_grads(wl, cp, x[lo:hi], y[lo:hi])
        with float32_products():
            _, a_k = O.node_loss_and_grads(wl, cp, x[lo:hi], y[lo:hi])
        Ls.append(L_k)
        want = want + g_k / K                     # (b_i / B with eight equal nodes)
        alt = alt + a_k / K
        del g_k, a_k
        print(f"oracle node {k} done", flush=True)
    del cp
    Lw = sum(Ls) / K
    tol = TOL["bf16"]
    second = {n: r for n, r, _ in tensor_errors(wl, alt, want)}
    bounds = {n: (tol if r <= tol / 2 else 2.0 * r) for n, r in second.items()}
    print("second CPU evaluation, rel-L2 per tensor:", {k: round(v, 4) for k, v in second.items()}, flush=True)
    print("tensors held to 2e-2:", sorted(n for n, b in bounds.items() if b == tol), flush=True)
    print("tensors NOT held to 2e-2 (bound = twice the second evaluation's distance):",
          {n: round(b, 4) for n, b in bounds.items() if b != tol}, flush=True)
    assert bounds["l6.W"] == tol and bounds["l6.b"] == tol

    xa = np.tile(x[:128 * K], (64 // K, 1))
    ya = np.tile(y[:128 * K], 64 // K)
    gpu = run_gpu(wl, theta, xa, ya, flags=BENCH, fold_window=8, node_group=BENCH_GROUP)
    assert gpu["streams"] == 2
    assert abs(gpu["loss"] - Lw) <= 1e-3 * abs(Lw)
    np.testing.assert_allclose(gpu["node_losses"], np.tile(np.array(Ls), 64 // K), rtol=1e-3)
    errs = tensor_errors(wl, gpu["G"], want)
    print("device, rel-L2 per tensor:", {n: round(r, 4) for n, r, _ in errs}, flush=True)
    bad = [(n, r, bounds[n]) for n, r, _ in errs if r > bounds[n]]
    assert not bad, bad
    check_update_from_own_gradient(wl, gpu, theta)
    G64 = gpu["G"].copy()
    del gpu, xa, ya
    # the same nodes as ONE unit: four such units in one window against that (fp32 rounding only;
    # a unit of another shape would not do: at this depth another shape of the products, which means
    # another order of fp32 sums, already moves the early layers by percents)
    U = BENCH_GROUP // K
    once = run_gpu(wl.with_nodes([128] * BENCH_GROUP), theta, np.tile(x[:128 * K], (U, 1)), np.tile(y[:128 * K], U),
                   flags=BENCH, fold_window=8, node_group=BENCH_GROUP)
    assert np.linalg.norm(G64 - once["G"]) <= 1e-6 * np.linalg.norm(once["G"])
    del once
    # the bound that does not depend on where operands are rounded (nodes 0 .. 7, weights only)
    gw = weights_only_gradient(wl.with_nodes([128] * K), theta, x[:128 * K], y[:128 * K])
    check_independent_bound(wl, G64, want, gw, "C5")


OVERLAP = 4


def test_overlap_and_single_stream_agree_bitwise():
    """Weight gradients on the side stream change scheduling only, never a bit of the result."""
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    base = run_gpu(wl, theta, x, y, flags=NO_GRAPH, steps=2)
    for flags in (0, FUSED, FUSED | NO_GRAPH, OVERLAP, OVERLAP | NO_GRAPH, FUSED | OVERLAP,
                  FUSED | OVERLAP | NO_GRAPH):
        other = run_gpu(wl, theta, x, y, flags=flags, steps=2)
        assert base["G"].tobytes() == other["G"].tobytes(), flags
        assert base["theta"].tobytes() == other["theta"].tobytes(), flags
        assert base["loss"] == other["loss"], flags


@pytest.mark.parametrize("window", [1, 2, 3, 8])
@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_mid_bf16", "mlp_big_node_bf16"])
def test_two_streams_with_fold_windows_agree_bitwise(name, window):
    """Forward passes on one stream, backward passes and weight gradients on the other, with and
    without graph replay, three steps (buffer sets and operand copies are reused across steps):
    the same bits as one stream with the same window."""
    wl, theta, x, y = _case(name)
    base = run_gpu(wl, theta, x, y, flags=FUSED | NO_GRAPH, steps=3, fold_window=window)
    for flags in (FUSED | OVERLAP, FUSED | OVERLAP | NO_GRAPH):
        other = run_gpu(wl, theta, x, y, flags=flags, steps=3, fold_window=window)
        assert base["G"].tobytes() == other["G"].tobytes(), flags
        assert base["theta"].tobytes() == other["theta"].tobytes(), flags
        assert base["loss"] == other["loss"], flags
        assert base["node_losses"].tobytes() == other["node_losses"].tobytes(), flags


# ---- fold window: the weight gradients of several nodes folded in one pass over the buffer -------

@pytest.mark.parametrize("window", [2, 3, 4, 8])
@pytest.mark.parametrize("name,flags", [("mlp_mid_bn_bf16", FUSED), ("mlp_mid_bf16", FUSED),
                                        ("mlp_mid_bn_bf16", FUSED | NO_GRAPH)])
def test_fold_window_gives_the_node_by_node_result_bitwise(name, flags, window):
    """The ordered fold: the same chain of fused multiply-adds, so the same bits: five unequal nodes
    (the last window is ragged), two steps so that the buffer is overwritten, not accumulated, by
    the second.  Also with node sizes that are no multiples of 8, where it is the only windowed path."""
    wl, theta, x, y = _case(name)
    one = run_gpu(wl, theta, x, y, flags=flags, steps=2)
    win = run_gpu(wl, theta, x, y, flags=flags | 8, steps=2, fold_window=window)
    odd = [44, 20, 125, 43, 8]
    assert sum(odd) == wl.batch
    one_odd = run_gpu(wl, theta, x, y, node_sizes=odd, flags=flags, steps=2)
    win_odd = run_gpu(wl, theta, x, y, node_sizes=odd, flags=flags, steps=2, fold_window=window)
    assert one_odd["G"].tobytes() == win_odd["G"].tobytes()
    assert one["G"].tobytes() == win["G"].tobytes()
    assert one["theta"].tobytes() == win["theta"].tobytes()
    assert one["loss"] == win["loss"]


ORDERED = 8


@pytest.mark.parametrize("window", [2, 4, 8])
@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_mid_bf16"])
def test_window_of_equal_nodes_as_one_product(name, window):
    """Nodes of one size share one weight b_i/B, and a window of them takes its weight gradients
    as one product over all its rows (Section 5.2: the same weighted sum).  Against the oracle;
    against the node-by-node chain to fp32 rounding; the ordered-fold flag restores that chain
    bit for bit; two streams change nothing.  Six nodes: windows of 4 and 8 are ragged."""
    wl, theta, x, y = _case(name)
    b = 8 * max(1, wl.batch // 6 // 8)
    sizes = [b] * 6
    xs, ys = x[:6 * b], y[:6 * b]
    one = run_gpu(wl, theta, xs, ys, node_sizes=sizes, flags=FUSED, steps=2)
    joined = run_gpu(wl, theta, xs, ys, node_sizes=sizes, flags=FUSED, steps=2, fold_window=window)
    ordered = run_gpu(wl, theta, xs, ys, node_sizes=sizes, flags=FUSED | ORDERED, steps=2, fold_window=window)
    assert one["G"].tobytes() == ordered["G"].tobytes()
    assert one["theta"].tobytes() == ordered["theta"].tobytes()
    scale = np.abs(one["G"]).max()
    assert np.abs(joined["G"] - one["G"]).max() <= 1e-5 * scale
    assert joined["loss"] == one["loss"]
    ref = oracle_steps(wl, theta, xs, ys, node_sizes=sizes, steps=2)
    check_against_oracle(wl, joined, ref, tol=2 * TOL[wl.dtype])      # second step: the trajectories have drifted
    # a single step of the joined window, whose inputs are bit-identical on both sides, at the tolerance itself
    check_against_oracle(wl, run_gpu(wl, theta, xs, ys, node_sizes=sizes, flags=FUSED, fold_window=window),
                         oracle_steps(wl, theta, xs, ys, node_sizes=sizes))
    for flags in (FUSED | OVERLAP, FUSED | OVERLAP | NO_GRAPH, FUSED | NO_GRAPH):
        other = run_gpu(wl, theta, xs, ys, node_sizes=sizes, flags=flags, steps=2, fold_window=window)
        assert joined["G"].tobytes() == other["G"].tobytes(), flags
        assert joined["theta"].tobytes() == other["theta"].tobytes(), flags


@pytest.mark.parametrize("window", [2, 3, 8])
@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_mid_bf16"])
def test_window_of_unequal_nodes_as_one_product(name, window):
    """Unequal nodes whose sizes are multiples of 8: the window's weighted gradient sum as one
    product over all its rows, node i's rows of the transposed output gradients holding
    (b_i/B) dz -- the per-sample gradient of the step's loss (Section 5.2) -- rounded to bf16
    once.  Against the oracle, against the ordered chain (one bf16 rounding apart), and the same
    bits on two streams, replayed or launched one by one."""
    wl, theta, x, y = _case(name)
    assert all(b % 8 == 0 for b in wl.node_sizes) and len(set(wl.node_sizes)) > 1
    first = run_gpu(wl, theta, x, y, flags=FUSED, fold_window=window)
    ordered = run_gpu(wl, theta, x, y, flags=FUSED | ORDERED, fold_window=window)
    scale = np.abs(ordered["G"]).max()
    print("joined - ordered, largest entry relative to the largest gradient:",
          np.abs(first["G"] - ordered["G"]).max() / scale, flush=True)
    assert np.abs(first["G"] - ordered["G"]).max() <= 1e-2 * scale     # two bf16 roundings of 2^-9 each, over the rows
    assert first["G"].tobytes() != ordered["G"].tobytes()
    assert first["loss"] == ordered["loss"]
    check_against_oracle(wl, first, oracle_steps(wl, theta, x, y))     # one step: the tolerance itself
    joined = run_gpu(wl, theta, x, y, flags=FUSED, steps=2, fold_window=window)
    ref = oracle_steps(wl, theta, x, y, steps=2)
    check_against_oracle(wl, joined, ref, tol=2 * TOL[wl.dtype])      # second step: the trajectories have drifted
    for flags in (FUSED | OVERLAP, FUSED | OVERLAP | NO_GRAPH, FUSED | NO_GRAPH):
        other = run_gpu(wl, theta, x, y, flags=flags, steps=2, fold_window=window)
        assert joined["G"].tobytes() == other["G"].tobytes(), flags
        assert joined["theta"].tobytes() == other["theta"].tobytes(), flags


def test_fold_window_with_long_nodes_and_other_modes_falls_back_to_node_by_node():
    """Nodes longer than the single-trip kernel takes (300, 212 rows), the staged fold and the fp32
    path ignore the window: results equal those without it."""
    wl, theta, x, y = _case("mlp_big_node_bf16")
    assert run_gpu(wl, theta, x, y, flags=FUSED)["G"].tobytes() == \
        run_gpu(wl, theta, x, y, flags=FUSED, fold_window=4)["G"].tobytes()
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    assert run_gpu(wl, theta, x, y, flags=0)["G"].tobytes() == \
        run_gpu(wl, theta, x, y, flags=0, fold_window=4)["G"].tobytes()
    wl, theta, x, y = _case("mlp_small_bn_f32")
    assert run_gpu(wl, theta, x, y, flags=FUSED)["G"].tobytes() == \
        run_gpu(wl, theta, x, y, flags=FUSED, fold_window=4)["G"].tobytes()


def test_fold_window_against_the_oracle_at_benchmark_size():
    wl, theta, x, y = _case("C2", jitter=0.0)
    gpu = run_gpu(wl, theta, x, y, flags=FUSED, fold_window=8)
    ref = oracle_steps(wl, theta, x, y)
    check_against_oracle(wl, gpu, ref)


def test_fold_window_workspace_does_not_depend_on_the_number_of_nodes():
    wl, theta, x, y = _case("mlp_mid_bf16")
    few = run_gpu(wl, theta, x, y, node_sizes=[120, 120], flags=FUSED, fold_window=4, max_node_size=128,
                  max_batch=240, max_nodes=16)
    many = run_gpu(wl, theta, x, y, node_sizes=[16] * 15, flags=FUSED, fold_window=4, max_node_size=128,
                   max_batch=240, max_nodes=16)
    assert few["workspace_bytes"] == many["workspace_bytes"]
    assert np.linalg.norm(few["G"] - many["G"]) > 0          # different splits really ran


def test_changing_the_split_between_steps_replays_the_right_graph():
    """Three different splits of the same batch in rotation (more than the two captured sets the
    context keeps), against the same calls launched kernel by kernel."""
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import config_from_workload
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    B = wl.batch
    splits = [list(wl.node_sizes), [B // 2, B - B // 2], [64] * (B // 64) + ([B % 64] if B % 64 else [])]
    order = [0, 1, 0, 2, 1, 0, 0, 2]

    def run(flags):
        stream = torch.cuda.Stream()
        eng = vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, fold_window=2,
                                                      max_node_size=max(max(s) for s in splits),
                                                      max_nodes=max(len(s) for s in splits)))
        from vfharness import to_device_batch
        p = torch.from_numpy(theta).cuda()
        xt, yt = to_device_batch(wl, x, y)
        torch.cuda.synchronize()
        for k in order:
            eng.step(p, xt, yt, splits[k])
        stream.synchronize()
        out = p.cpu().numpy()
        eng.close()
        return out

    assert run(FUSED).tobytes() == run(FUSED | NO_GRAPH).tobytes()


# ---- node groups: consecutive nodes through their passes together ---------------------

@pytest.mark.parametrize("group", [2, 4, 8])
@pytest.mark.parametrize("name,sizes", [("mlp_mid_bn_bf16", [40] * 6), ("mlp_mid_bf16", [40] * 6),
                                        ("mlp_mid_bn_bf16", [40, 40, 40, 16, 16, 8, 8, 8, 8, 56]),
                                        ("mlp_mid_bn_bf16", [112, 112, 16]), ("mlp_mid_bn_bf16", [24] * 10)])
def test_node_groups_match_the_oracle(name, sizes, group):
    """Up to 2, 4 or 8 consecutive nodes, of one size or of several, taken through their passes as one
    unit (ten nodes go as 8 + 2; sizes that are no multiple of 8 would go alone), in every fold mode, on one and two streams, replayed and
    launched one by one: BatchNorm statistics, node losses and the weights b_i/B stay per node, so
    the oracle's node-by-node result must come out; the modes agree bitwise with one another."""
    wl, theta, x, y = _case(name)
    B = sum(sizes)
    x, y = x[:B], y[:B]
    ref = oracle_steps(wl, theta, x, y, node_sizes=sizes)
    plain = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED)
    base = None
    for flags, window in ((FUSED, 0), (FUSED | NO_GRAPH, 0), (FUSED | NO_GRAPH | OVERLAP, 0), (FUSED | OVERLAP, 0), (0, 0),
                          (FUSED | ORDERED, 4)):
        gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=flags, fold_window=window, node_group=group)
        check_against_oracle(wl, gpu, ref)
        np.testing.assert_allclose(gpu["node_losses"], plain["node_losses"], rtol=1e-5)
        if base is None:
            base = gpu
        assert gpu["G"].tobytes() == base["G"].tobytes(), (flags, window)
        assert gpu["theta"].tobytes() == base["theta"].tobytes(), (flags, window)
    # a windowed product over groups against the oracle as well
    gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED | NO_GRAPH | OVERLAP, fold_window=4, node_group=group)
    check_against_oracle(wl, gpu, ref)
    assert np.linalg.norm(gpu["G"] - plain["G"]) <= 2e-2 * np.linalg.norm(plain["G"])


@pytest.mark.parametrize("group", [16, 32])
@pytest.mark.parametrize("name,sizes", [("mlp_mid_bn_bf16", [8] * 30), ("mlp_mid_bf16", [8] * 30),
                                        ("mlp_mid_bn_bf16", [16, 8, 8] * 7 + [16]), ("mlp_mid_bn_bf16", [24] * 9)])
def test_units_of_more_than_eight_nodes_match_the_oracle(name, sizes, group):
    """Units of up to 16 or 32 nodes (the BatchNorm kernels then take a unit in launches of eight nodes,
    the last one ragged; 30 nodes go as 16 + 14 or as one unit, 9 nodes as 8 + 1): the oracle's
    node-by-node result, the same bits in every launch mode, per-node losses unchanged."""
    wl, theta, x, y = _case(name)
    B = sum(sizes)
    x, y = x[:B], y[:B]
    ref = oracle_steps(wl, theta, x, y, node_sizes=sizes)
    plain = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED)
    base = None
    for flags, window in ((FUSED, 0), (FUSED | NO_GRAPH | OVERLAP, 0), (FUSED | OVERLAP, 0), (0, 0)):
        gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=flags, fold_window=window, node_group=group)
        check_against_oracle(wl, gpu, ref)
        np.testing.assert_allclose(gpu["node_losses"], plain["node_losses"], rtol=1e-5)
        if base is None:
            base = gpu
        if flags & FUSED:
            assert gpu["G"].tobytes() == base["G"].tobytes(), (flags, window)
            assert gpu["theta"].tobytes() == base["theta"].tobytes(), (flags, window)
        else:
            # staged fold: the BatchNorm scale / shift gradients of a unit's launches of eight nodes are
            # added in the staging vector before the weight is applied, not weighted one by one
            assert np.abs(gpu["G"] - base["G"]).max() <= 1e-6 * np.abs(base["G"]).max()
    gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED | NO_GRAPH | OVERLAP, fold_window=4, node_group=group)
    check_against_oracle(wl, gpu, ref)
    assert np.linalg.norm(gpu["G"] - plain["G"]) <= 2e-2 * np.linalg.norm(plain["G"])


@pytest.mark.parametrize("name", ["mlp_wide_bn_bf16", "mlp_wide_bf16"])
def test_wide_units_of_whole_nodes_match_the_oracle(name):
    """Sixteen nodes of 128 rows on layers of 8192 columns, as one unit: the input-gradient products run
    on the 256 x 256 tiles with the BatchNorm / ReLU backward pass in their epilogue (two whole nodes
    per tile; with and without BatchNorm), the forward pass on the two-column BatchNorm kernel.  The
    oracle's node-by-node result, per-node losses, and the same bits from every launch mode; with the
    last node cut in two (units of unequal nodes: the separate backward kernel) the oracle again."""
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=0.1)
    x, y = I.make_batch(wl)
    print(f"wide units {name}", flush=True)
    ref = oracle_steps(wl, theta, x, y)
    base = None
    for flags in (FUSED | NO_GRAPH | OVERLAP, FUSED, 0):
        gpu = run_gpu(wl, theta, x, y, flags=flags, node_group=16)
        check_against_oracle(wl, gpu, ref)
        np.testing.assert_allclose(gpu["node_losses"], ref["node_losses"], rtol=1e-3)
        if base is None:
            base = gpu
        assert gpu["G"].tobytes() == base["G"].tobytes(), flags
        assert gpu["theta"].tobytes() == base["theta"].tobytes(), flags
    sizes = [128] * 15 + [64, 64]
    ref = oracle_steps(wl, theta, x, y, node_sizes=sizes)
    gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED | NO_GRAPH | OVERLAP, node_group=32)
    check_against_oracle(wl, gpu, ref)
    if name == "mlp_wide_bn_bf16":
        # a unit of sixteen whole nodes and a unit of sixteen nodes of 64 rows in one fold window: the
        # window's joint weight-gradient product takes the nodes' weights b_i/B inside its operand, i.e.
        # the fused epilogue writes its transposed copy scaled
        sizes = [128] * 16 + [64] * 16
        wl2 = wl.with_nodes(sizes)
        x2, y2 = I.make_batch(wl2)
        ref = oracle_steps(wl2, theta, x2, y2)
        gpu = run_gpu(wl2, theta, x2, y2, flags=BENCH, fold_window=8, node_group=16)
        check_against_oracle(wl2, gpu, ref)


def test_node_groups_keep_the_workspace_independent_of_the_node_count():
    wl, theta, x, y = _case("mlp_mid_bn_bf16")
    few = run_gpu(wl, theta, x[:80], y[:80], node_sizes=[40, 40], flags=FUSED, node_group=4, max_node_size=40,
                  max_batch=240, max_nodes=6)
    many = run_gpu(wl, theta, x, y, node_sizes=[40] * 6, flags=FUSED, node_group=4, max_node_size=40,
                   max_batch=240, max_nodes=6)
    assert few["workspace_bytes"] == many["workspace_bytes"]
