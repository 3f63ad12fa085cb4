"""GPU parity: the HIP path through the C ABI against the CPU oracle, MLP workloads."""
import numpy as np
import pytest

import oracle as O
import vf_inputs as I
from vfharness import (TOL, check_against_oracle, check_update_from_own_gradient, oracle_steps, run_gpu)

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
                                  "mlp_big_node_bf16"])
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


@pytest.mark.parametrize("name,flags", [("C2", 0), ("C3", 0), ("C3", FUSED)])
def test_full_size_configurations(name, flags):
    """The benchmark configuration (C2) and the heterogeneous split (C3) at full size, in the
    launch configuration bench.py times, every gradient entry against the oracle."""
    print(f"full size {name} flags={flags}", flush=True)
    wl, theta, x, y = _case(name, jitter=0.0)
    gpu = run_gpu(wl, theta, x, y, flags=flags)
    ref = oracle_steps(wl, theta, x, y)
    check_against_oracle(wl, gpu, ref)
    check_update_from_own_gradient(wl, gpu, theta)
    off, w = O.partition(wl.node_sizes, wl.batch)
    import paper_2009_09523_amd as vf
    off2, w2 = vf.vf_partition(wl.node_sizes, wl.batch)
    assert off.tobytes() == off2.tobytes() and w.tobytes() == w2.tobytes()


def test_c5_full_size_launch_configuration():
    """Large-batch emulation: MLP 2048-8192x6-1000 + BatchNorm, 64 nodes of 128 (B = 8192).
    The oracle can afford single nodes of this model, so: (a) the step is run in the launch
    configuration bench.py times (V = 64) on a batch whose 64 nodes all hold the rows of
    node 0 -- the combined gradient must then equal the oracle's g_0, and the update the
    oracle's update with it; (b) two different nodes (V = 2) against (g_0 + g_1)/2."""
    print("full size C5", flush=True)
    wl = I.workload("C5")
    theta = I.make_params(wl)
    x, y = I.make_batch(wl)
    from oracle.step import compute_copy
    cp = compute_copy(wl, theta)
    L0, g0 = O.node_loss_and_grads(wl, cp, x[:128], y[:128])
    print("oracle node 0 done", flush=True)
    L1, g1 = O.node_loss_and_grads(wl, cp, x[128:256], y[128:256])
    print("oracle node 1 done", flush=True)
    del cp
    from vfharness import assert_close_per_tensor
    tol = TOL["bf16"]
    # (a)
    xa, ya = np.tile(x[:128], (64, 1)), np.tile(y[:128], 64)
    gpu = run_gpu(wl, theta, xa, ya)
    assert abs(gpu["loss"] - L0) <= tol * abs(L0)
    np.testing.assert_allclose(gpu["node_losses"], np.full(64, L0), rtol=tol)
    assert_close_per_tensor(wl, gpu["G"], g0, tol, "G (64 equal nodes)", ambiguous=True)
    check_update_from_own_gradient(wl, gpu, theta)
    th_new, v_new = O.sgdm_update(theta.astype(np.float64), g0, np.zeros(g0.size), wl.lr, wl.momentum)
    assert_close_per_tensor(wl, gpu["theta"], th_new, tol, "theta", ambiguous=True)
    del gpu, xa, ya
    # (b)
    w2 = wl.with_nodes([128, 128])
    gpu = run_gpu(w2, theta, x[:256], y[:256])
    assert abs(gpu["loss"] - 0.5 * (L0 + L1)) <= tol * abs(L0)
    assert_close_per_tensor(wl, gpu["G"], 0.5 * (g0 + g1), tol, "G (two nodes)", ambiguous=True)
