"""Pins for the oracle's two CPU policies: hand-worked examples (tests/golden/policy_examples.txt),
brute force over all subsets / all placements on small instances, and the bound the paper's
appendix states for the placement."""
import itertools
import math
import os
import random

from oracle import policy_oracle as po


def parse_examples():
    path = os.path.join(os.path.dirname(__file__), "golden", "policy_examples.txt")
    ex, cur = [], None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        w = line.split()
        if w[0] in ("arbitrate", "place"):
            cur = {"kind": w[0], "head": [float(x) for x in w[1:]], "rows": []}
            ex.append(cur)
        elif w[0] in ("accept", "gpus"):
            cur["expect"] = [int(x) for x in w[1:]]
        else:
            cur["rows"].append([float(x) for x in w])
    return ex


def test_hand_worked_examples():
    ex = parse_examples()
    assert len(ex) == 2
    for e in ex:
        cols = list(zip(*e["rows"]))
        if e["kind"] == "arbitrate":
            assert po.arbitrate(cols[0], cols[1], cols[2], cols[3], e["head"][0]) == e["expect"]
        else:
            n, cap, tau = int(e["head"][0]), e["head"][1], e["head"][2]
            got = po.place(n, cap, tau, cols[0], cols[1], cols[2], cols[3], [int(x) for x in cols[4]])
            assert got == e["expect"]


def feasible(subset, arrival, slo, e, now):
    t = now
    for i in sorted(subset, key=lambda i: (arrival[i] + slo[i], i)):     # earliest deadline first is optimal for feasibility
        t += e[i]
        if t > arrival[i] + slo[i]:
            return False
    return True


def test_arbitration_accepts_as_many_as_any_subset_can():
    rng = random.Random(5)
    for trial in range(150):
        n = rng.randint(1, 9)
        arrival = [rng.uniform(0, 3) for _ in range(n)]
        slo = [rng.uniform(0.5, 6) for _ in range(n)]
        p = [rng.randint(1, 40) * 10.0 for _ in range(n)]
        c = [rng.choice([50.0, 100.0, 200.0]) for _ in range(n)]
        now = rng.uniform(0, 3)
        e = [p[i] / c[i] for i in range(n)]
        S = po.arbitrate(arrival, slo, p, c, now)
        assert len(set(S)) == len(S)
        t = now
        for i in S:                                   # dispatched in this order, every one of them is on time
            t += e[i]
            assert t <= arrival[i] + slo[i] + 1e-12
        best = max(len(sub) for k in range(n + 1) for sub in itertools.combinations(range(n), k)
                   if feasible(sub, arrival, slo, e, now))
        assert len(S) == best, (trial, S, best)


def test_placement_bound_against_exhaustive_search():
    """Appendix, KVPR bound: with every model unplaced (tau irrelevant), the greedy maximum is at most
    KVPR_OPT * (1 + C / (S - w_k)), S and w_k taken at the last assignment to the worst GPU."""
    rng = random.Random(11)
    for trial in range(120):
        n_gpus = rng.randint(2, 3)
        M = rng.randint(2, 7)
        C = 100.0
        rate = [rng.uniform(1, 100) for _ in range(M)]
        size = [1.0] * M
        slo = [rng.choice([0.05, 0.1, 0.2]) for _ in range(M)]
        weight = [rng.uniform(1, 20) for _ in range(M)]
        got = po.place(n_gpus, C, 0.0, rate, size, slo, weight)
        assert sorted(set(got)) == sorted(set(got)) and all(0 <= g < n_gpus for g in got)
        greedy = po.max_kvpr(n_gpus, C, got, rate, size, slo, weight)
        opt = min(po.max_kvpr(n_gpus, C, pl, rate, size, slo, weight) for pl in itertools.product(range(n_gpus), repeat=M))
        assert greedy >= opt - 1e-12
        # the last model assigned to the worst GPU
        d = [rate[j] * size[j] / slo[j] for j in range(M)]
        order = sorted(range(M), key=lambda j: (-d[j], j))
        worst = max(range(n_gpus), key=lambda i: sum(d[j] for j in range(M) if got[j] == i) /
                    (C - sum(weight[j] for j in range(M) if got[j] == i)))
        k = [j for j in order if got[j] == worst][-1]
        s_before = C - sum(weight[j] for j in order[:order.index(k)] if got[j] == worst)
        assert greedy <= opt * (1 + C / (s_before - weight[k])) + 1e-9, (trial, greedy, opt)


def test_placement_rules():
    # hysteresis: with a huge threshold nobody moves
    got = po.place(3, 100.0, 1e9, [50, 40, 30, 20], [1] * 4, [0.1] * 4, [10] * 4, current_gpu=[2, 2, 2, 1])
    assert got == [2, 2, 2, 1]
    # tensor-parallel parts never share a GPU, even when one GPU is by far the least loaded
    got = po.place(3, 100.0, 0.0, [90, 30, 30, 30], [1] * 4, [0.1] * 4, [5] * 4, tp_group=[-1, 7, 7, 7])
    assert sorted(got[1:]) == [0, 1, 2]
    # a GPU whose memory is used up is never chosen while another has room
    got = po.place(2, 100.0, 0.0, [10, 9, 8], [1] * 3, [0.1] * 3, [100, 10, 10])
    assert got[0] != got[1] and got[1] == got[2]
    assert math.isinf(po.max_kvpr(2, 100.0, [0, 0, 1], [10, 9, 8], [1] * 3, [0.1] * 3, [100, 10, 10]))
