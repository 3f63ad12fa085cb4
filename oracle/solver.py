"""Heterogeneous split by exhaustive search (Section 5.1.2), test infrastructure only.

min over per-device batches b_i and nodes per device v_i of
    max_i ( t_i(b_i / v_i) * v_i ) + comm     subject to   sum_i n_i b_i = B,
with t_i from an offline profile (Section 5.1.1).  Reading: the paper prints t_i(b_i) * v_i;
t_i is taken at the node batch b_i / v_i (nodes of a device run one after another).  b_i is 0
(type unused) or a power of two or the mid-point between two powers of two, b_i / v_i must be
a profiled size, comm counts when more than one device takes part.
"""
import itertools


def power_of_two_like(limit):
    out, p = [], 1
    while p <= limit:
        out.append(p)
        if p >= 2 and p * 3 // 2 <= limit:
            out.append(p * 3 // 2)
        p *= 2
    return out


def solve_split(types, B, comm=0.0):
    """types: [(n_devices, {node_batch: time})].  Returns (best time, list of every optimal
    assignment [(b_i, v_i), ...])."""
    sizes = [0] + power_of_two_like(B)
    per_type = []
    for n, prof in types:
        options = [(0, 0, 0.0)]
        for b in sizes[1:]:
            best = None
            for node, t in prof.items():
                if b % node == 0:
                    v = b // node
                    if best is None or t * v < best[2] or (t * v == best[2] and v < best[1]):
                        best = (b, v, t * v)
            if best:
                options.append(best)
        per_type.append(options)
    best_time, winners = None, []
    for combo in itertools.product(*per_type):
        if sum(n * c[0] for (n, _), c in zip(types, combo)) != B:
            continue
        devices = sum(n for (n, _), c in zip(types, combo) if c[0])
        if devices == 0:
            continue
        total = max(c[2] for c in combo if c[0]) + (comm if devices > 1 else 0.0)
        if best_time is None or total < best_time:
            best_time, winners = total, [combo]
        elif total == best_time:
            winners.append(combo)
    if best_time is None:
        raise ValueError("no combination of profiled sizes adds up to the batch")
    return best_time, [[(c[0], c[1]) for c in w] for w in winners]
