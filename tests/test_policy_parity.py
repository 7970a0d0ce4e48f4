"""The library's two CPU policies (host code in libprismkv.so, no GPU needed) against the oracle's
step-by-step definitions: identical decisions on random instances, the golden examples, error codes."""
import random

import numpy as np
import pytest

from oracle import policy_oracle as po
from paper_2505_04021_amd import binding
from test_oracle_policy import parse_examples


def test_golden_examples_through_the_library():
    for e in parse_examples():
        cols = list(zip(*e["rows"]))
        if e["kind"] == "arbitrate":
            assert binding.arbitrate_requests(cols[0], cols[1], cols[2], cols[3], e["head"][0]) == e["expect"]
        else:
            got = binding.place_models(int(e["head"][0]), e["head"][1], e["head"][2], cols[0], cols[1], cols[2], cols[3],
                                       [int(x) for x in cols[4]])
            assert got == e["expect"]


def test_arbitration_matches_oracle():
    rng = random.Random(21)
    for trial in range(300):
        n = rng.randint(0, 60)
        arrival = [rng.uniform(0, 5) for _ in range(n)]
        slo = [rng.choice([0.5, 1.0, 2.0, 4.0]) for _ in range(n)]          # many equal deadlines and lengths
        p = [rng.randint(1, 20) * 32.0 for _ in range(n)]
        c = [rng.choice([256.0, 512.0, 1024.0]) for _ in range(n)]
        if trial % 3 == 0:
            arrival = [round(a) * 1.0 for a in arrival]
        now = rng.uniform(0, 5)
        assert binding.arbitrate_requests(arrival, slo, p, c, now) == po.arbitrate(arrival, slo, p, c, now), trial


def test_placement_matches_oracle():
    rng = random.Random(22)
    for trial in range(300):
        n_gpus = rng.randint(1, 8)
        M = rng.randint(0, 40)
        rate = [rng.choice([10.0, 20.0, 50.0, rng.uniform(1, 100)]) for _ in range(M)]
        size = [rng.choice([1.0, 2.0]) for _ in range(M)]
        slo = [rng.choice([0.05, 0.1]) for _ in range(M)]
        weight = [rng.uniform(0, 30) for _ in range(M)]
        cur = [rng.randint(-1, n_gpus - 1) for _ in range(M)] if trial % 2 else None
        tp = None
        if trial % 5 == 0 and M >= 4 and n_gpus >= 2:
            tp = [-1] * M
            for part in rng.sample(range(M), min(n_gpus, 3)):
                tp[part] = 4
        tau = rng.choice([0.0, 0.05, 0.5])
        want = po.place(n_gpus, 100.0, tau, rate, size, slo, weight, cur, tp)
        assert binding.place_models(n_gpus, 100.0, tau, rate, size, slo, weight, cur, tp) == want, trial


def test_policy_argument_errors():
    with pytest.raises(ValueError):
        binding.arbitrate_requests([0.0], [1.0], [10.0], [0.0], 0.0)           # zero speed
    with pytest.raises(ValueError):
        binding.place_models(2, 100.0, 0.0, [1.0, 1.0, 1.0], [1.0] * 3, [0.1] * 3, [1.0] * 3, None, [3, 3, 3])   # 3 parts, 2 GPUs
    with pytest.raises(ValueError):
        binding.place_models(0, 100.0, 0.0, [], [], [], [])
