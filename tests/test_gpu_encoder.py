"""GPU parity: the encoder workloads through the C ABI against the CPU oracle."""
import numpy as np
import pytest

import oracle as O
import vf_inputs as I
from vfharness import (TOL, check_against_oracle, check_independent_bound, check_update_from_own_gradient,
                       oracle_steps, run_gpu, weights_only_gradient)

pytestmark = pytest.mark.gpu

FUSED = 1
NO_GRAPH = 2


def _case(name, jitter=0.1):
    wl = I.workload(name)
    theta = I.make_params(wl, jitter=jitter)
    x, y = I.make_batch(wl)
    return wl, theta, x, y


@pytest.mark.parametrize("flags", [NO_GRAPH, 0, FUSED])
@pytest.mark.parametrize("name", ["enc_tiny_f32", "enc_small_f32", "enc_small_bf16", "enc_mid_bf16", "enc_vocab_f32",
                                  "enc_vocab_bf16", "enc_odd_f32", "enc_wide_bf16"])
def test_encoder_step_matches_oracle(name, flags):
    print(f"case {name} flags={flags}", flush=True)
    wl, theta, x, y = _case(name)
    gpu = run_gpu(wl, theta, x, y, flags=flags)
    ref = oracle_steps(wl, theta, x, y)
    # Adam: new parameters are compared through the device's own gradient (an entry whose
    # gradient is within rounding of zero moves by +lr on one side and -lr on the other)
    check_against_oracle(wl, gpu, ref)
    check_update_from_own_gradient(wl, gpu, theta, tol=1e-4)


def test_encoder_fused_and_staged_agree_bitwise():
    wl, theta, x, y = _case("enc_small_bf16")
    a = run_gpu(wl, theta, x, y, flags=0)
    b = run_gpu(wl, theta, x, y, flags=FUSED)
    assert a["G"].tobytes() == b["G"].tobytes()


OVERLAP = 4


@pytest.mark.parametrize("name,sizes", [("enc_small_bf16", None), ("enc_small_bf16", [2, 2, 1, 3, 1]),
                                        ("enc_mid_bf16", [1, 1, 1, 1, 1]), ("enc_wide_bf16", None)])
def test_encoder_two_streams_agree_bitwise(name, sizes):
    """Forward passes on one stream, backward passes on the other (two sets of what passes from a
    node's forward to its backward part), staged and fused, replayed and launched one by one,
    three steps: the same bits as one stream."""
    print(f"case {name} sizes={sizes}", flush=True)
    wl, theta, x, y = _case(name)
    if sizes is not None:
        assert sum(sizes) == wl.batch
    base = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=FUSED | NO_GRAPH, steps=3)
    assert base["streams"] == 1
    for flags in (OVERLAP, OVERLAP | NO_GRAPH, FUSED | OVERLAP, FUSED | OVERLAP | NO_GRAPH):
        other = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=flags, steps=3)
        assert other["streams"] == 2, flags
        assert base["G"].tobytes() == other["G"].tobytes(), flags
        assert base["theta"].tobytes() == other["theta"].tobytes(), flags
        assert base["loss"] == other["loss"], flags
        assert base["node_losses"].tobytes() == other["node_losses"].tobytes(), flags


def test_encoder_fp32_keeps_one_stream():
    """The fp32 attention path shares its score scratch between the two passes: no second stream."""
    wl, theta, x, y = _case("enc_small_f32")
    assert run_gpu(wl, theta, x, y, flags=FUSED | OVERLAP | NO_GRAPH)["streams"] == 1


def test_encoder_two_steps():
    wl, theta, x, y = _case("enc_small_f32")
    gpu = run_gpu(wl, theta, x, y, steps=2)
    ref = oracle_steps(wl, theta, x, y, steps=2)
    check_against_oracle(wl, gpu, ref, tol=5e-4)


def test_encoder_partition_invariance_on_device():
    wl, theta, x, y = _case("enc_small_f32")
    a = run_gpu(wl, theta, x, y, node_sizes=[wl.batch])
    b = run_gpu(wl, theta, x, y, node_sizes=[1] * wl.batch)
    assert np.linalg.norm(b["G"] - a["G"]) <= 2e-5 * np.linalg.norm(a["G"])


def test_c4_full_size():
    """4-layer encoder 768/12/3072, T=128, vocab 30522, B=256 in 16 nodes of 16, Adam."""
    print("full size C4", flush=True)
    wl, theta, x, y = _case("C4", jitter=0.0)
    ref = oracle_steps(wl, theta, x, y)
    for flags, group in ((0, 0), (FUSED | OVERLAP | NO_GRAPH, 8)):      # the second is what bench.py times (the encoder takes 4 of the 8)
        print(f"flags {flags} group {group}", flush=True)
        gpu = run_gpu(wl, theta, x, y, flags=flags, node_group=group)
        check_against_oracle(wl, gpu, ref)
        check_update_from_own_gradient(wl, gpu, theta, tol=1e-4)
    # the bound that does not depend on where operands are rounded
    check_independent_bound(wl, gpu["G"], ref["G"], weights_only_gradient(wl, theta, x, y), "C4")


@pytest.mark.parametrize("group", [2, 4])
@pytest.mark.parametrize("name,sizes", [("enc_small_bf16", [2, 2, 2, 1, 1, 1]), ("enc_small_f32", [1] * 9),
                                        ("enc_mid_bf16", [1, 1, 1, 1, 1])])
def test_encoder_node_groups_match_the_oracle(name, sizes, group):
    """Groups of equal-sized nodes as one unit of the passes (the sequences of an encoder node are
    independent: only the loss bookkeeping tells the nodes apart): per-node losses and the combined
    gradient against the oracle, one and two streams bitwise equal."""
    wl, theta, x, y = _case(name)
    assert sum(sizes) == wl.batch
    ref = oracle_steps(wl, theta, x, y, node_sizes=sizes)
    base = None
    for flags in (FUSED, FUSED | NO_GRAPH, FUSED | OVERLAP | NO_GRAPH, 0):
        gpu = run_gpu(wl, theta, x, y, node_sizes=sizes, flags=flags, node_group=group)
        check_against_oracle(wl, gpu, ref)
        if base is None:
            base = gpu
        assert gpu["G"].tobytes() == base["G"].tobytes(), flags
        assert gpu["node_losses"].tobytes() == base["node_losses"].tobytes(), flags
