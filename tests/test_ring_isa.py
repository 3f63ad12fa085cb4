"""The register-staged load rings of the product kernels, checked in the compiler's output.

`gemm_bf16_pipe_kernel` issues its global loads from inline assembly and waits with explicit
`s_waitcnt vmcnt(n)`.  A build of it once read a load's destination register before the wait
that covered it (a `v_and` of the edge masking, scheduled ahead of a wait that named no
registers): products with a contraction length that is no multiple of 8 came out wrong whenever
the operand was not yet in a near cache.  These tests compile the kernels for gfx950 and prove
on the assembly that no instruction touches a register a load in flight still has to write, on
any path, and that the kernels spill nothing (a spilled ring register would be the same bug).
"""
import os
import re
import subprocess

import pytest

import isa_ring_check as R

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


# ---- the checker itself, on hand-written snippets ---------------------------------------------

def _kernel(body: str) -> str:
    return "_Z4testv:\n" + body + "\n\ts_endpgm\n.Lfunc_end0:\n"


def _asm(line: str) -> str:
    return f"\t;;#ASMSTART\n\t{line}\n\t;;#ASMEND\n"


def _check(body: str):
    ks = R.kernels_with_asm_loads(_kernel(body))
    assert list(ks) == ["_Z4testv"]
    return R.check_kernel(ks["_Z4testv"])


def test_checker_flags_a_read_before_the_wait():
    body = (_asm("global_load_dwordx4 v[4:7], v[0:1], off") +
            "\tv_and_b32_e32 v8, v4, v9\n" +
            _asm("s_waitcnt vmcnt(0)") +
            "\tds_write_b128 v10, v[4:7]\n")
    bad = _check(body)
    assert len(bad) == 1 and bad[0][1].startswith("v_and_b32") and bad[0][2] == (4,)


def test_checker_accepts_use_after_the_wait_and_counts_in_order():
    body = (_asm("global_load_dwordx4 v[4:7], v[0:1], off") +
            _asm("global_load_dwordx4 v[8:11], v[0:1], off") +
            _asm("s_waitcnt vmcnt(1)") +
            "\tv_and_b32_e32 v12, v4, v13\n" +          # the older load has landed
            _asm("s_waitcnt vmcnt(0)") +
            "\tv_and_b32_e32 v12, v8, v13\n")
    assert _check(body) == []
    body_bad = body.replace("v_and_b32_e32 v12, v4, v13", "v_and_b32_e32 v12, v8, v13")
    assert len(_check(body_bad)) == 1                   # the younger one has not


def test_checker_follows_a_ring_around_its_loop():
    ring = (_asm("global_load_dwordx4 v[4:7], v[0:1], off") +
            _asm("global_load_dwordx4 v[8:11], v[0:1], off") +
            ".LBB0_1:\n" +
            _asm("s_waitcnt vmcnt(1)") +
            "\tds_write_b128 v20, v[4:7]\n" +
            _asm("global_load_dwordx4 v[4:7], v[0:1], off") +
            _asm("s_waitcnt vmcnt(1)") +
            "\tds_write_b128 v20, v[8:11]\n" +
            _asm("global_load_dwordx4 v[8:11], v[0:1], off") +
            "\ts_cbranch_scc1 .LBB0_1\n" +
            _asm("s_waitcnt vmcnt(0)"))
    assert _check(ring) == []
    # a compiler-made copy of a register in flight is a violation as well
    moved = ring.replace("\tds_write_b128 v20, v[8:11]\n", "\tv_mov_b32_e32 v30, v5\n\tds_write_b128 v20, v[8:11]\n")
    assert [b[1] for b in _check(moved)] == ["v_mov_b32_e32 v30, v5"]


# ---- the kernels as compiled -------------------------------------------------------------------

@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    from paper_2009_09523_amd import build as vfbuild
    if not os.path.exists(vfbuild.HIPCC):
        pytest.skip("hipcc not available")
    out = tmp_path_factory.mktemp("isa") / "k_gemm_bf16.s"
    src = os.path.join(vfbuild.CSRC, "k_gemm_bf16.hip")
    cmd = [vfbuild.HIPCC, *vfbuild.FLAGS, "-x", "hip", "--cuda-device-only", "-S", src, "-o", str(out)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return out.read_text()


def test_no_instruction_touches_a_register_with_a_load_in_flight(gemm_asm):
    ks = R.kernels_with_asm_loads(gemm_asm)
    assert len(ks) >= 12, sorted(ks)                    # every instantiation of the pipelined kernel
    for name, body in ks.items():
        assert R.check_kernel(body) == [], name


def test_product_kernels_use_no_scratch_memory(gemm_asm):
    sizes = [int(v) for v in re.findall(r"; ScratchSize: (\d+)", gemm_asm)]
    assert sizes and all(v == 0 for v in sizes), sizes
