"""Input prefetch (Section 3.2 step 1): the next batch is copied from pinned host memory into one of
two device staging buffers on a copy stream while the current step runs; results are those of
vf_step on device-resident batches."""
import numpy as np
import pytest

import oracle as O
import vf_inputs as I
from vfharness import TOL, to_device_batch

pytestmark = pytest.mark.gpu


def _batches(wl, n):
    return [I.make_batch(wl, seed_x=I.SEED_INPUTS + 10 * t, seed_y=I.SEED_LABELS + 10 * t,
                         seed_mask=I.SEED_MASK + 10 * t) for t in range(n)]


def _pinned(wl, x, y):
    import torch
    xt, yt = to_device_batch(wl, x, y, device="cpu")
    return xt.pin_memory(), yt.pin_memory()


@pytest.mark.parametrize("name,flags", [("mlp_mid_bn_bf16", 1), ("mlp_small_f32", 0), ("enc_tiny_f32", 0),
                                        ("mlp_mid_bn_bf16", 1 | 2)])
def test_prefetched_steps_equal_steps_on_resident_batches(name, flags):
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import config_from_workload
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=0.1)
    batches = _batches(wl, 4)
    sizes = list(wl.node_sizes)

    def engine():
        stream = torch.cuda.Stream()
        return vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, fold_window=2)), stream

    # reference: every batch resident before its step
    eng, stream = engine()
    p_ref = torch.from_numpy(theta).cuda()
    for x, y in batches:
        xt, yt = to_device_batch(wl, x, y)
        torch.cuda.synchronize()
        eng.step(p_ref, xt, yt, sizes)
        stream.synchronize()
    ref = p_ref.cpu().numpy()
    eng.close()

    # prefetch: batch t+1 is handed over while step t is in flight
    eng, stream = engine()
    p = torch.from_numpy(theta).cuda()
    host = [_pinned(wl, x, y) for x, y in batches]
    torch.cuda.synchronize()
    eng.prefetch(*host[0])
    for t in range(len(host)):
        eng.step_prefetched(p, sizes)
        if t + 1 < len(host):
            eng.prefetch(*host[t + 1])
    stream.synchronize()
    torch.cuda.synchronize()
    got = p.cpu().numpy()
    assert eng.step_count == len(host)
    G_last = torch.empty_like(p)
    eng.grads(G_last)
    loss_last = eng.loss()
    eng.close()
    assert got.tobytes() == ref.tobytes()
    assert not np.array_equal(ref, theta)

    # and against the oracle stepping through the same batches (Section 3.2: one update per batch,
    # each batch split into the same virtual nodes): the last step's combined gradient and loss,
    # and the total parameter movement
    th, state, r = theta.astype(np.float32), None, None
    for x, y in batches:
        r = O.oracle_step(wl, th, x, y, state=state)
        state, th = r["state"], r["theta"].astype(np.float32)
    tol = 5 * TOL[wl.dtype]        # four steps: the trajectories drift apart at the tolerance of one
    g = G_last.cpu().numpy().astype(np.float64)
    assert abs(loss_last - r["loss"]) <= tol * abs(r["loss"])
    assert np.linalg.norm(g - r["G"]) <= tol * np.linalg.norm(r["G"])
    if wl.optimizer == "sgdm":     # (Adam's first steps move noise-level entries by +-lr either way)
        moved, want = got.astype(np.float64) - theta, r["theta"] - theta
        assert np.linalg.norm(moved - want) <= tol * np.linalg.norm(want)


def test_prefetch_order_errors_and_rejected_step_keeps_the_batch():
    import torch
    import paper_2009_09523_amd as vf
    from paper_2009_09523_amd.binding import config_from_workload
    wl = I.workload("mlp_small_bn_f32")
    theta = I.make_params(wl, jitter=0.1)
    (x, y), = _batches(wl, 1)
    hx, hy = _pinned(wl, x, y)
    stream = torch.cuda.Stream()
    eng = vf.VirtualNodeStep(config_from_workload(wl, stream=stream))
    p = torch.from_numpy(theta).cuda()
    sizes = list(wl.node_sizes)
    with pytest.raises(vf.VfError):
        eng.step_prefetched(p, sizes)                    # nothing staged
    eng.prefetch(hx, hy)
    with pytest.raises(vf.VfError):
        eng.prefetch(hx, hy)                             # one batch ahead at most
    with pytest.raises(vf.VfError):
        eng.step_prefetched(p, sizes[:-1])               # sizes do not add up: rejected ...
    before = p.cpu().numpy().copy()
    assert np.array_equal(before, theta) and eng.step_count == 0
    eng.step_prefetched(p, sizes)                        # ... and the batch is still there
    stream.synchronize()
    assert eng.step_count == 1 and not np.array_equal(p.cpu().numpy(), theta)
    # same result as the resident path
    eng2 = vf.VirtualNodeStep(config_from_workload(wl, stream=stream))
    p2 = torch.from_numpy(theta).cuda()
    xt, yt = to_device_batch(wl, x, y)
    eng2.step(p2, xt, yt, sizes)
    stream.synchronize()
    assert p2.cpu().numpy().tobytes() == p.cpu().numpy().tobytes()
    eng.close(); eng2.close()
