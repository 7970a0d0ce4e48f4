"""Pins for the oracle's page-pool / balloon bookkeeping (CPU only)."""
import os
import random

import numpy as np
import pytest

from pool_model import PoolModel
from state_image import check_invariants, parse

BF16 = 0
GOLD = os.path.join(os.path.dirname(__file__), "golden", "pool_trace.txt")


def test_hand_worked_trace(oracle):
    o = oracle
    pool = o.pool_create(6 * 2048, 16, 2048)
    A = o.model_register(pool, 2, 1, 16, BF16, 4, 8)
    B = o.model_register(pool, 2, 1, 32, BF16, 4, 8)
    ids = {"A": A, "B": B}
    assert (o.slots(A), o.slots(B)) == (2, 1)
    final = {"frames": {}, "bits": {}, "row": {}, "address": []}
    for line in open(GOLD):
        tok = line.split("#")[0].split()
        if not tok:
            continue
        op, a = tok[0], tok[1:]
        if op == "resize":
            assert o.balloon_resize(ids[a[0]], int(a[1])) == int(a[2]), line
        elif op == "reserve":
            assert o.seq_reserve(ids[a[0]], int(a[1]), int(a[2])) == int(a[3]), line
        elif op == "release":
            assert o.seq_release(ids[a[0]], int(a[1])) == int(a[2]), line
        elif op == "free":
            final["free"] = [int(x) for x in a]
        elif op == "owner":
            final["owner"] = [int(x) if int(x) < 0 else [A, B][int(x)] for x in a]
        elif op in ("frames", "bits"):
            final[op][ids[a[0]]] = [int(x) for x in a[1:]]
        elif op == "row":
            final["row"][(ids[a[0]], int(a[1]))] = [int(x) for x in a[2:]]
        elif op == "address":
            final["address"].append((ids[a[0]], int(a[1]), int(a[2])))
    st = parse(o.pool_export_state(pool))
    check_invariants(st)
    assert st["free"] == final["free"] and st["owner"] == final["owner"]
    for m in (A, B):
        assert st["models"][m]["frames"] == final["frames"][m]
        assert st["models"][m]["bits"] == final["bits"][m]
    rows = {(m, s): r for m in (A, B) for s, r in st["models"][m]["rows"].items()}
    assert rows == final["row"]
    for m, blk, addr in final["address"]:
        assert o.block_address(m, blk) == addr
    for m in (A, B):
        for s in range(4):
            o.seq_release(m, s)
        assert o.balloon_resize(m, 0) == 0
        assert o.model_unregister(m) == 0
    assert o.pool_destroy(pool) == 0


def _fresh(o, n_frames=16, frame=4096, order=None):
    pool = o.pool_create(n_frames * frame, 16, frame)
    if order is not None:
        assert o.pool_seed_free_order(pool, np.array(order, dtype=np.uint32)) == 0
    return pool


def _drop(o, pool, models, max_seqs):
    for m in models:
        for s in range(max_seqs):
            o.seq_release(m, s)
        assert o.balloon_resize(m, 0) == 0
        assert o.model_unregister(m) == 0
    assert o.pool_destroy(pool) == 0


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_ops_match_independent_model(oracle, seed):
    """1000 random calls on a 16-frame pool shared by three models of different
    block sizes: return codes and the full exported state must equal the
    list-and-set model after every call, and the invariants must hold."""
    o, rnd = oracle, random.Random(seed)
    n_frames, frame, T, max_seqs, max_blocks = 16, 4096, 16, 5, 12
    order = list(range(n_frames))
    rnd.shuffle(order)
    pool = _fresh(o, n_frames, frame, order)
    ref = PoolModel(n_frames, order)
    shapes = [(2, 1, 16), (4, 2, 16), (4, 1, 64)]      # block bytes 1024, 2048, 4096
    mids = []
    for hq, hkv, d in shapes:
        m = o.model_register(pool, hq, hkv, d, BF16, max_seqs, max_blocks)
        mids.append(m)
        ref.register(m, frame // (2 * T * hkv * d * 2), T, max_blocks)
        assert o.slots(m) == ref.models[m]["slots"]
    for step in range(1000):
        m = rnd.choice(mids)
        r = rnd.random()
        if r < 0.30:
            tgt = rnd.randint(0, 9)
            got, want = o.balloon_resize(m, tgt), ref.resize(m, tgt)
        elif r < 0.75:
            s, c = rnd.randrange(max_seqs), rnd.randint(0, 200)
            got, want = o.seq_reserve(m, s, c), ref.reserve(m, s, c)
        else:
            s = rnd.randrange(max_seqs)
            got, want = o.seq_release(m, s), ref.release(m, s)
        assert got == want, (step, got, want)
        st = parse(o.pool_export_state(pool))
        check_invariants(st)
        assert st["free"] == ref.free[:], step
        for mm in mids:
            assert st["models"][mm]["frames"] == ref.models[mm]["frames"], step
            assert st["models"][mm]["bits"] == ref.bits(mm), step
            want_rows = {s: r for s, r in ref.models[mm]["rows"].items() if r}
            assert st["models"][mm]["rows"] == want_rows, step
    _drop(o, pool, mids, max_seqs)


def test_round_trip_restores_free_stack(oracle):
    """Inflate, use, release everything, deflate to zero: a single model on a fresh
    pool gets the original stack back in the original order."""
    o = oracle
    order = [3, 0, 7, 5, 1, 6, 2, 4]
    pool = _fresh(o, 8, 4096, order)
    before = parse(o.pool_export_state(pool))["free"]
    assert before == order[::-1]
    m = o.model_register(pool, 2, 1, 16, BF16, 4, 32)
    assert o.balloon_resize(m, 6) == 6
    assert parse(o.pool_export_state(pool))["models"][m]["frames"] == order[:6]
    assert o.seq_reserve(m, 0, 300) == 19
    assert o.balloon_resize(m, 0) == 5          # 19 blocks at 4 per frame pin 5 frames
    assert o.seq_release(m, 0) == 19
    assert o.balloon_resize(m, 0) == 0
    assert parse(o.pool_export_state(pool))["free"] == before
    _drop(o, pool, [m], 4)


def test_batch_reserve_equals_sequential_reserves(oracle):
    o = oracle
    out = []
    for batch in (False, True):
        pool = _fresh(o, 8, 4096)
        m = o.model_register(pool, 2, 1, 16, BF16, 4, 16)
        assert o.balloon_resize(m, 5) == 5
        assert o.seq_reserve(m, 1, 20) == 2
        seqs, ctx = [2, 0, 1, 2], [33, 16, 70, 64]
        if batch:
            assert o.seq_reserve_batch(m, seqs, ctx) == 3 + 1 + 3 + 1
        else:
            assert [o.seq_reserve(m, s, c) for s, c in zip(seqs, ctx)] == [3, 1, 3, 1]
        out.append(parse(o.pool_export_state(pool)))
        # a batch that does not fit changes nothing
        img = o.pool_export_state(pool)
        assert o.seq_reserve_batch(m, [3, 0], [16 * 9, 16 * 12]) == -4
        assert np.array_equal(img, o.pool_export_state(pool))
        _drop(o, pool, [m], 4)
    assert out[0] == out[1]


def test_error_paths_leave_state_untouched(oracle):
    o = oracle
    pool = _fresh(o, 4, 4096)
    assert o.model_register(pool, 3, 2, 16, BF16, 2, 4) == -5       # Hq % Hkv
    assert o.model_register(pool, 8, 8, 128, BF16, 2, 4) == -5      # block larger than a frame
    m = o.model_register(pool, 2, 1, 16, BF16, 2, 4)
    assert o.balloon_resize(m, 2) == 2
    img = o.pool_export_state(pool)
    assert o.balloon_resize(m, 5) == -3
    assert o.balloon_resize(m, -1) == -1
    assert o.balloon_resize(99, 1) == -2
    assert o.seq_reserve(m, 0, 16 * 5) == -6                        # row too long
    assert o.seq_reserve(m, 2, 16) == -1                            # no such row
    assert o.seq_reserve(m, 0, 16 * 4) == 4
    assert o.seq_reserve(m, 1, 16 * 4) == 4
    assert o.seq_release(m, 0) == 4 and o.seq_release(m, 0) == 0    # second release is a no-op
    assert o.seq_release(m, 1) == 4
    assert np.array_equal(img, o.pool_export_state(pool))
    assert o.model_unregister(m) == -7 and o.pool_destroy(pool) == -7
    _drop(o, pool, [m], 2)
    assert o.pool_destroy(pool) == -2


def test_scenarios_keep_invariants(oracle):
    """The dynamic workloads (small sizes) on the oracle alone: invariants hold at
    every step and the clamp path of deflate is exercised."""
    from workloads.scenarios import Runner, make_config
    for cfg_id in (3, 5):
        cfg = make_config(cfg_id, "small")
        r = Runner(oracle, cfg, write_kv=False).setup()
        seen_active = set()
        for t in range(cfg.steps):
            r.step(t)
            st = parse(oracle.pool_export_state(r.pool))
            check_invariants(st)
            seen_active.add(tuple(r.active_models()))
        assert len(seen_active) > (3 if cfg_id == 3 else 0)
        r.teardown()


def test_one_call_admission_equals_the_growth_rounds(oracle):
    """A batched reserve is defined as its single reserves in order, so the growth rounds of an
    admission in one list, and the departures in one release list, leave the very state the
    round-by-round calls leave: the bursty scenario in all three runner modes, step by step."""
    from workloads.scenarios import Runner, make_config
    images = {}
    for mode in ("calls", "batched", "enqueue"):
        cfg = make_config(3, "small")
        r = Runner(oracle, cfg, write_kv=False, mode=mode).setup()
        images[mode] = []
        for t in range(cfg.steps):
            r.step(t).flush()
            images[mode].append(oracle.pool_export_state(r.pool).copy())
        r.teardown()
    for t, ref in enumerate(images["calls"]):
        assert np.array_equal(ref, images["batched"][t]) and np.array_equal(ref, images["enqueue"][t]), t
