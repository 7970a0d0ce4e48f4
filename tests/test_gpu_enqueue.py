"""The enqueue-only bookkeeping calls and the one-call admission against the CPU oracle.

The batched calls are defined as their single calls in order, so a scenario driven in any of
the runner's three modes must leave the same pool state and return the same values; here the
GPU runs "batched" / "enqueue" and the oracle the same mode (its batched calls are the
sequential definition written out).  Refusals must change nothing and raise the sticky flag.
"""
import numpy as np
import pytest

from parity import TOL, assert_same_state, row_rel_err, run_pair
from state_image import check_invariants, parse
from workloads import gen
from workloads.scenarios import Runner, make_config

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1
E_ARG, E_NOMEM, E_BALLOON, E_RANGE = -1, -3, -4, -6


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


@pytest.mark.parametrize("cfg_id,mode", [(3, "batched"), (3, "enqueue"), (5, "batched"), (5, "enqueue")])
def test_scenarios_in_one_call_modes(gpu, oracle, cfg_id, mode):
    """The bursty and the cycling workload with every admission as one reserve call and every
    departure as one release call; state and return values after every step, attention on some."""
    cfg = make_config(cfg_id, "small")
    rg, ro = Runner(gpu, cfg, mode=mode).setup(), Runner(oracle, cfg, mode=mode).setup()
    attn = set(range(6)) | {10, 11, 20, cfg.steps - 1}
    try:
        for t in range(cfg.steps):
            rg.step(t)
            ro.step(t)
            rg.flush()
            ro.flush()
            assert rg.log == ro.log, f"step {t}: return values differ"
            img = assert_same_state(gpu, oracle, rg.pool, ro.pool, f"step {t}")
            check_invariants(parse(img))
            if t in attn:
                for mi in rg.active_models():
                    q = rg.queries(t, mi)
                    rc_g, out_g = gpu.decode_attention(rg.models[mi], q, rg.ctx[mi])
                    rc_o, out_o = oracle.decode_attention(ro.models[mi], q, ro.ctx[mi])
                    assert rc_g == 0 and rc_o == 0
                    assert row_rel_err(out_g, out_o) <= TOL[cfg.models[mi].dtype]
        assert gpu.device_errors() == 0
    finally:
        rg.teardown()
        ro.teardown()


def test_long_reserve_lists_with_repeated_sequences(gpu, oracle):
    """Lists that span several chunks of the reserve kernel (1024 entries each), sequences repeated
    in and across chunks, wants that do not rise monotonically, rows that already hold blocks."""
    rng = np.random.default_rng(77)
    frame, n_frames, n_seq, max_blocks = 256 << 10, 512, 48, 400
    perm = gen.free_order(n_frames, gen.generator(77))
    pools, ms = [], []
    for be in (gpu, oracle):
        pool = be.pool_create(n_frames * frame, 16, frame)
        assert pool >= 0 and be.pool_seed_free_order(pool, perm) == 0
        ms.append(be.model_register(pool, 8, 2, 64, BF16, n_seq, max_blocks))
        assert ms[-1] >= 0 and be.balloon_resize(ms[-1], 400) == 400
        pools.append(pool)
    try:
        for case, n in enumerate((1, 63, 1024, 1025, 3000, 4096)):
            seqs = rng.integers(0, n_seq, size=n).astype(np.int32)
            # mostly growing, sometimes falling back: the entry then needs nothing
            ctx = (np.sort(rng.integers(0, 16 * max_blocks // 4, size=n)) + rng.integers(-200, 200, size=n)).clip(0, 16 * max_blocks // 4)
            ctx = (ctx + case * 300).astype(np.int32)
            r = [be.seq_reserve_batch(m, seqs, ctx) for be, m in zip((gpu, oracle), ms)]
            assert r[0] == r[1], (n, r)
            assert_same_state(gpu, oracle, pools[0], pools[1], f"list of {n}")
            if case % 2 == 1:                     # release some rows, two of them twice in one list
                out = rng.integers(0, n_seq, size=9).astype(np.int32)
                out[7], out[8] = out[0], out[3]
                r = [be.seq_release_batch(m, out) for be, m in zip((gpu, oracle), ms)]
                assert r[0] == r[1] and r[0] > 0
                assert_same_state(gpu, oracle, pools[0], pools[1], f"release after {n}")
        # limits and refusals: nothing changes
        before = gpu.pool_export_state(pools[0])
        assert gpu.seq_reserve_batch(ms[0], np.zeros(4097, np.int32), np.zeros(4097, np.int32)) == E_ARG
        assert gpu.seq_reserve_batch(ms[0], [0, n_seq], [16, 16]) == E_ARG
        assert gpu.seq_reserve_batch(ms[0], [0, 1], [16, 16 * max_blocks + 1]) == E_RANGE
        assert oracle.seq_reserve_batch(ms[1], [0, 1], [16, 16 * max_blocks + 1]) == E_RANGE
        assert gpu.seq_release_batch(ms[0], [0, -1]) == E_ARG and oracle.seq_release_batch(ms[1], [0, -1]) == E_ARG
        assert np.array_equal(before, gpu.pool_export_state(pools[0]))
        assert gpu.device_errors() == 0          # the synchronous forms return their code and raise no flag
    finally:
        for be, m, pool in zip((gpu, oracle), ms, pools):
            be.seq_release_batch(m, np.arange(n_seq, dtype=np.int32))
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0


def test_refused_enqueued_calls(gpu, oracle):
    """An inflate beyond the pool, a reserve beyond the balloon and a list with a bad entry, all
    enqueue-only: the tickets carry the oracle's codes, the state stays the oracle's, bit 2 of the
    device flags is up, and the calls that follow run against the unchanged state."""
    frame, n_frames = 64 << 10, 32
    pools, ms = [], []
    for be in (gpu, oracle):
        pool = be.pool_create(n_frames * frame, 16, frame)
        ms.append(be.model_register(pool, 8, 2, 64, BF16, 8, 64))       # 8 KiB blocks: 8 slots per frame
        pools.append(pool)
    calls = [
        ("balloon_resize_enqueue", (4,)),                      # fine
        ("balloon_resize_enqueue", (40,)),                     # beyond the pool: refused at once, NOMEM
        ("balloon_resize_enqueue", (33,)),                     # (also beyond)
        ("seq_reserve_batch_enqueue", ([0, 1], [16 * 20, 16 * 20])),   # 40 blocks > 32 slots: BALLOON
        ("seq_reserve_batch_enqueue", ([0, 1], [16 * 10, 16 * 10])),   # fits
        ("seq_reserve_batch_enqueue", ([0, 9], [16, 16])),     # bad sequence: ARG
        ("balloon_resize_enqueue", (1,)),                      # clamps at the frames in use
        ("seq_release_batch_enqueue", ([1, 1, 0],)),
        ("balloon_resize_enqueue", (0,)),
    ]
    try:
        tickets = [[getattr(be, name)(m, *args) for name, args in calls] for be, m in zip((gpu, oracle), ms)]
        assert min(tickets[0]) >= 0
        res = [[be.ticket_result(t) for t in ts] for be, ts in zip((gpu, oracle), tickets)]
        assert res[0] == res[1], res
        assert res[1][1] == E_NOMEM and res[1][3] == E_BALLOON and res[1][5] == E_ARG and res[1][6] == 3
        assert_same_state(gpu, oracle, pools[0], pools[1])
        assert gpu.device_errors() == 4 and gpu.device_errors() == 0
        assert gpu.ticket_result(10 ** 6) == E_RANGE
        # the synchronous calls after a refused enqueued one see the true state
        assert gpu.balloon_resize(ms[0], 2) == 2 and oracle.balloon_resize(ms[1], 2) == 2
        assert gpu.seq_reserve(ms[0], 3, 100) == oracle.seq_reserve(ms[1], 3, 100) == 7
        kv = gen.seq_kv((5, 5), 100, 2, 64, BF16, 16)
        assert gpu.kv_write(ms[0], 3, 0, kv["k"], kv["v"]) == 100
        assert gpu.kv_write(ms[0], 2, 0, kv["k"], kv["v"]) == E_RANGE      # a row that holds nothing
        assert_same_state(gpu, oracle, pools[0], pools[1])
    finally:
        for be, m, pool in zip((gpu, oracle), ms, pools):
            be.seq_release_batch(m, np.arange(8, dtype=np.int32))
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0


def test_ticket_ring_wraps(gpu, oracle):
    """More enqueued calls than the library remembers tickets for: the calls still run in order."""
    frame, n_frames = 64 << 10, 64
    pools, ms = [], []
    for be in (gpu, oracle):
        pool = be.pool_create(n_frames * frame, 16, frame)
        ms.append(be.model_register(pool, 8, 2, 64, BF16, 4, 64))
        pools.append(pool)
    try:
        last = None
        for i in range(300):
            target = (i * 7) % 50
            last = [be.balloon_resize_enqueue(m, target) for be, m in zip((gpu, oracle), ms)]
        assert gpu.ticket_result(last[0]) == oracle.ticket_result(last[1]) == 299 * 7 % 50
        assert_same_state(gpu, oracle, pools[0], pools[1])
        assert gpu.device_errors() == 0
    finally:
        for be, m, pool in zip((gpu, oracle), ms, pools):
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0
