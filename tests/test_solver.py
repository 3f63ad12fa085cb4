"""Heterogeneous split solver: the library's host-side search against the brute-force oracle, and
both against the configurations the paper lists (Table 4) under its stated 4:1 speed ratio."""
import os

import numpy as np
import pytest

import paper_2009_09523_amd as vf
from oracle.solver import power_of_two_like, solve_split

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table4_heterogeneous_splits.txt")
NODES = [16, 24, 32, 48, 64, 96, 128, 192, 256]          # node batches that fit in memory


def _linear(speed):
    return {b: b / speed for b in NODES}


def _lib(types, B, comm=0.0):
    return vf.vf_solve_split([(n, sorted(p), [p[b] for b in sorted(p)]) for n, p in types], B, comm)


def _rows():
    rows = []
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            name, nv, bv, npp, bp = line.split()
            rows.append((name, int(nv), int(bv), int(npp), int(bp)))
    return rows


@pytest.mark.parametrize("name,nv,bv,npp,bp", _rows())
def test_table4_splits_are_optimal_under_the_papers_speed_ratio(name, nv, bv, npp, bp):
    types = [(nv, _linear(4.0)), (npp, _linear(1.0))]
    best, winners = solve_split(types, 8192)
    assert nv * bv + npp * bp == 8192
    assert any(w[0][0] == bv and w[1][0] == bp for w in winners), (name, winners)
    b, v, t = _lib(types, 8192)
    assert t == best
    assert [(bi, vi) for bi, vi in zip(b, v)] in winners
    if len({(w[0][0], w[1][0]) for w in winners}) == 1:
        assert b == [bv, bp]


def test_uneven_split_beats_even_split_by_the_papers_margin():
    """2 V100 + 2 P100: the uneven split's step is at least 44 % shorter than the even one."""
    types = [(2, _linear(4.0)), (2, _linear(1.0))]
    even = max(2048 / 4.0, 2048 / 1.0)
    best, _ = solve_split(types, 8192)
    assert best <= (1 - 0.44) * even
    assert _lib(types, 8192)[2] == best


def test_falls_back_to_homogeneous_when_the_slow_type_cannot_help():
    types = [(2, _linear(100.0)), (1, _linear(1.0))]
    b, v, t = _lib(types, 4096)
    assert b == [2048, 0] and v[1] == 0
    best, winners = solve_split(types, 4096)
    assert t == best and [(b[0], v[0]), (0, 0)] in winners


def test_random_instances_match_brute_force():
    rng = np.random.Generator(np.random.PCG64(12))
    for _ in range(40):
        n_types = int(rng.integers(1, 4))
        types = []
        for _ in range(n_types):
            nodes = sorted(rng.choice(NODES, size=int(rng.integers(2, 6)), replace=False).tolist())
            base = float(rng.uniform(0.5, 4.0))
            prof = {b: base * (20.0 + b) * float(rng.uniform(0.9, 1.1)) for b in nodes}   # sub-linear curve
            types.append((int(rng.integers(1, 5)), prof))
        B = int(rng.choice([256, 384, 512, 1024, 1536, 2048]))
        comm = float(rng.choice([0.0, 5.0]))
        try:
            best, winners = solve_split(types, B, comm)
        except ValueError:
            with pytest.raises(vf.VfError):
                _lib(types, B, comm)
            continue
        b, v, t = _lib(types, B, comm)
        assert abs(t - best) <= 1e-12 * best
        assert sum(n * bi for (n, _), bi in zip(types, b)) == B
        assert [(bi, vi) for bi, vi in zip(b, v)] in winners


def test_candidate_sizes():
    assert power_of_two_like(64) == [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]


def test_rejects_malformed_input():
    with pytest.raises(vf.VfError):
        vf.vf_solve_split([(0, [16], [1.0])], 64)
    with pytest.raises(vf.VfError):
        vf.vf_solve_split([(1, [32, 16], [1.0, 2.0])], 64)
    with pytest.raises(vf.VfError):
        vf.vf_solve_split([(1, [16], [-1.0])], 64)
    with pytest.raises(vf.VfError):
        vf.vf_solve_split([(1, [16], [1.0])], 24)          # 24 is not a multiple of a profiled size
