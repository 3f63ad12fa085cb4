"""Per-device training state (Section 4.1): BatchNorm moving statistics updated by every virtual
node, and the export / import of everything a device needs to continue a job."""
from dataclasses import replace

import numpy as np
import pytest

import vf_inputs as I
from vfharness import TOL, oracle_steps, to_device_batch

pytestmark = pytest.mark.gpu

NO_GRAPH, FUSED = 2, 1


def _engine(wl, flags=0, node_group=0):
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import config_from_workload
    stream = torch.cuda.Stream()
    return vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, node_group=node_group)), stream


def _setup(wl, jitter=0.1):
    import torch
    theta = I.make_params(wl, jitter=jitter)
    x, y = I.make_batch(wl)
    xt, yt = to_device_batch(wl, x, y)
    return theta, x, y, torch.from_numpy(theta).cuda(), xt, yt


@pytest.mark.parametrize("name", ["mlp_small_bn_f32", "mlp_mid_bn_bf16", "mlp_big_node_bf16"])
@pytest.mark.parametrize("flags", [0, NO_GRAPH, FUSED, FUSED | 4])
def test_moving_statistics_match_the_oracle_after_two_steps(name, flags):
    import paper_2009_09523_amd as vf
    wl = I.workload(name)
    theta, x, y, params, xt, yt = _setup(wl)
    eng, stream = _engine(wl, flags)
    for _ in range(2):
        eng.step(params, xt, yt, list(wl.node_sizes))
    st = vf.parse_state(eng.state_export(params))
    eng.close()
    ref = oracle_steps(wl, theta, x, y, steps=2)
    assert st["steps"] == 2
    tol = TOL[wl.dtype]
    want_mean = np.concatenate(ref["state"]["bn_mean"])
    want_var = np.concatenate(ref["state"]["bn_var"])
    assert st["bn_mean"].size == want_mean.size == sum(wl.dims[1:-1])
    assert np.max(np.abs(st["bn_mean"] - want_mean)) <= tol * np.max(np.abs(want_mean))
    assert np.max(np.abs(st["bn_var"] - want_var)) <= tol * np.max(np.abs(want_var))


@pytest.mark.parametrize("group,nodes", [(2, [48] * 5), (4, [48] * 5), (8, [24] * 10)])
def test_moving_statistics_of_grouped_nodes_are_blended_node_after_node(group, nodes):
    """Equal nodes taken 2, 4 or 8 at a time: every node still blends its own statistics into the
    moving ones, in node order (Section 4.1), so the oracle's values come out."""
    import paper_2009_09523_amd as vf
    wl = I.workload("mlp_mid_bn_bf16").with_nodes(nodes)
    theta, x, y, params, xt, yt = _setup(wl)
    eng, stream = _engine(wl, FUSED, node_group=group)
    for _ in range(2):
        eng.step(params, xt, yt, list(wl.node_sizes))
    st = vf.parse_state(eng.state_export(params))
    eng.close()
    ref = oracle_steps(wl, theta, x, y, steps=2)
    want_mean, want_var = np.concatenate(ref["state"]["bn_mean"]), np.concatenate(ref["state"]["bn_var"])
    tol = TOL[wl.dtype]
    assert np.max(np.abs(st["bn_mean"] - want_mean)) <= tol * np.max(np.abs(want_mean))
    assert np.max(np.abs(st["bn_var"] - want_var)) <= tol * np.max(np.abs(want_var))


def test_moving_statistics_of_wide_units_are_blended_node_after_node():
    """Sixteen whole nodes of 128 rows on 8192-wide layers, one unit: the forward products take BatchNorm in
    their epilogue and leave per-node statistics, which a small launch blends into the moving ones in node
    order -- the oracle's values after one step."""
    import paper_2009_09523_amd as vf
    wl = I.workload("mlp_wide_bn_bf16")
    theta, x, y, params, xt, yt = _setup(wl)
    eng, stream = _engine(wl, FUSED, node_group=16)
    eng.step(params, xt, yt, list(wl.node_sizes))
    st = vf.parse_state(eng.state_export(params))
    eng.close()
    ref = oracle_steps(wl, theta, x, y, steps=1)
    want_mean, want_var = np.concatenate(ref["state"]["bn_mean"]), np.concatenate(ref["state"]["bn_var"])
    tol = TOL[wl.dtype]
    assert np.max(np.abs(st["bn_mean"] - want_mean)) <= tol * np.max(np.abs(want_mean))
    assert np.max(np.abs(st["bn_var"] - want_var)) <= tol * np.max(np.abs(want_var))


def test_zero_share_freezes_the_moving_statistics():
    import paper_2009_09523_amd as vf
    wl = replace(I.workload("mlp_small_bn_f32"), bn_momentum=0.0)
    theta, x, y, params, xt, yt = _setup(wl)
    eng, _ = _engine(wl)
    eng.step(params, xt, yt, list(wl.node_sizes))
    st = vf.parse_state(eng.state_export(params))
    eng.close()
    assert np.all(st["bn_mean"] == 0.0) and np.all(st["bn_var"] == 1.0)


@pytest.mark.parametrize("name", ["mlp_mid_bn_bf16", "mlp_small_f32", "enc_tiny_f32", "conv_small_bf16"])
def test_export_import_round_trip_continues_bitwise(name):
    """Two steps, export, two more steps -- against a fresh context that imports the payload
    (through a device buffer) and runs the same two steps: identical bits everywhere."""
    import torch
    import paper_2009_09523_amd as vf
    wl = I.workload(name)
    theta, x, y, params, xt, yt = _setup(wl)
    sizes = list(wl.node_sizes)
    eng, _ = _engine(wl)
    for _ in range(2):
        eng.step(params, xt, yt, sizes)
    payload = eng.state_export(params)
    dev = torch.empty(eng.state_bytes, dtype=torch.uint8, device="cuda")
    eng.state_export(params, dev)
    assert np.array_equal(dev.cpu().numpy(), payload)
    for _ in range(2):
        eng.step(params, xt, yt, sizes)
    final_a = eng.state_export(params)
    eng.close()

    eng2, _ = _engine(wl)
    params2 = torch.zeros_like(params)
    eng2.state_import(params2, dev)
    assert eng2.step_count == 2
    assert np.array_equal(eng2.state_export(params2), payload)
    for _ in range(2):
        eng2.step(params2, xt, yt, sizes)
    final_b = eng2.state_export(params2)
    eng2.close()
    a, b = vf.parse_state(final_a), vf.parse_state(final_b)
    assert a["steps"] == b["steps"] == 4
    assert np.array_equal(final_a, final_b)
    assert not np.array_equal(a["theta"], vf.parse_state(payload)["theta"])


def test_import_rejects_a_payload_of_another_model_and_changes_nothing():
    import torch
    import paper_2009_09523_amd as vf
    wl_a, wl_b = I.workload("mlp_small_bn_f32"), I.workload("mlp_small_f32")
    theta, x, y, params, xt, yt = _setup(wl_a)
    eng_a, _ = _engine(wl_a)
    eng_a.step(params, xt, yt, list(wl_a.node_sizes))
    payload = eng_a.state_export(params)
    before = eng_a.state_export(params).copy()
    eng_b, _ = _engine(wl_b)
    pb = torch.zeros(eng_b.num_params, device="cuda")
    big = np.zeros(max(payload.size, eng_b.state_bytes), dtype=np.uint8)
    big[:payload.size] = payload
    with pytest.raises(vf.VfError):
        eng_b.state_import(pb, big)
    assert eng_b.step_count == 0 and float(pb.abs().max()) == 0.0
    with pytest.raises(vf.VfError):                       # too short
        eng_a.state_import(params, payload[:-4])
    garbage = payload.copy()
    garbage[:8] = 0                                       # wrong magic
    with pytest.raises(vf.VfError):
        eng_a.state_import(params, garbage)
    assert np.array_equal(eng_a.state_export(params), before)
    eng_a.close(); eng_b.close()
