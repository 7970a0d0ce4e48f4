"""GPU tests of elastic pools: a pool whose frames are backed by device memory only while a model
owns them (HIP virtual memory management behind balloon_resize).  The bookkeeping state and the
attention results must be what they are with an ordinary pool — the oracle knows no difference —
and, once the pre-allocation thread has caught up, the memory mapped must be exactly the frames that
are owned plus the buffer on top of the free stack."""
import numpy as np
import pytest

from parity import TOL, assert_same_state, row_rel_err, run_pair
from state_image import parse
from workloads import gen
from workloads.scenarios import Runner, make_config

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1


class Elastic:
    """The GPU backend with every pool created elastic."""

    def __init__(self, gpu):
        self._gpu = gpu
        self.name = "gpu-elastic"

    def __getattr__(self, k):
        return getattr(self._gpu, k)

    def pool_create(self, nbytes, page_tokens, frame_bytes=None, storage=None):
        assert storage is None
        return self._gpu.pool_create_elastic(nbytes, page_tokens, frame_bytes or (2 << 20))


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


def mapped_matches_owned(gpu, pool, frame_bytes, buffer=0):
    """After the pre-allocation thread has caught up: memory backs the owned frames and the `buffer`
    frames on top of the free stack (as many as there are), nothing else."""
    held = gpu.pool_prealloc_wait(pool)
    st = gpu.pool_stats(pool)
    assert held == st["idle_frames"] == min(buffer, st["n_free"]), (held, buffer, st["idle_frames"], st["n_free"])
    assert st["mapped_bytes"] == (st["n_frames"] - st["n_free"] + st["idle_frames"]) * frame_bytes, st
    return st


def test_frames_are_mapped_while_owned(gpu, oracle):
    """Inflate, fill, attend, release, deflate with a clamp, reuse by a second model."""
    fb = 2 << 20
    pools = [gpu.pool_create_elastic(64 * fb, 16, fb), oracle.pool_create(64 * fb, 16, fb)]
    assert min(pools) >= 0
    perm = gen.free_order(64, gen.generator(9))
    bes = (gpu, oracle)
    for be, pool in zip(bes, pools):
        assert be.pool_seed_free_order(pool, perm) == 0
    assert gpu.pool_stats(pools[0])["mapped_bytes"] == 0
    ms = [be.model_register(pool, 32, 8, 128, BF16, 4, 64) for be, pool in zip(bes, pools)]
    m2 = [be.model_register(pool, 12, 4, 64, E4M3, 4, 64) for be, pool in zip(bes, pools)]
    ctx = np.array([300, 17, 1000, 64], dtype=np.int32)
    for be, m in zip(bes, ms):
        assert be.balloon_resize(m, 5) == 5
        assert be.seq_reserve_batch(m, [0, 1, 2, 3], ctx) >= 0
    mapped_matches_owned(gpu, pools[0], fb)
    for s, c in enumerate(ctx):
        kv = gen.seq_kv((9, s), int(c), 8, 128, BF16, 16)
        for be, m in zip(bes, ms):
            assert be.kv_write(m, s, 0, kv["k"], kv["v"]) == c
    q = gen.queries((9, 9), 4, 32, 128)
    out_g, out_o = gpu.decode_attention(ms[0], q, ctx), oracle.decode_attention(ms[1], q, ctx)
    assert out_g[0] == 0 and out_o[0] == 0 and row_rel_err(out_g[1], out_o[1]) <= TOL[BF16]
    # the second model grows while the first still holds its frames
    for be, m in zip(bes, m2):
        assert be.balloon_resize(m, 20) == 20
    assert mapped_matches_owned(gpu, pools[0], fb)["mapped_bytes"] == 25 * fb
    # the first gives back what it can: sequences 0 and 2 leave, the deflate clamps at the frames still in use
    for be, m in zip(bes, ms):
        assert be.seq_release(m, 0) > 0 and be.seq_release(m, 2) > 0
    r = [be.balloon_resize(m, 0) for be, m in zip(bes, ms)]
    assert r[0] == r[1] and 0 < r[0] < 5
    assert_same_state(gpu, oracle, pools[0], pools[1])
    mapped_matches_owned(gpu, pools[0], fb)
    sel = [1, 3]
    q2 = gen.queries((9, 10), 4, 32, 128)
    ctx2 = ctx.copy()
    ctx2[[0, 2]] = 0
    out_g, out_o = gpu.decode_attention(ms[0], q2, ctx2), oracle.decode_attention(ms[1], q2, ctx2)
    assert out_g[0] == 0 and out_o[0] == 0 and row_rel_err(out_g[1], out_o[1]) <= TOL[BF16]
    assert gpu.device_errors() == 0
    for be, m, mm in zip(bes, ms, m2):
        for s in range(4):
            be.seq_release(m, s)
        assert be.balloon_resize(m, 0) == 0 and be.balloon_resize(mm, 0) == 0
        assert be.model_unregister(m) == 0 and be.model_unregister(mm) == 0
    assert mapped_matches_owned(gpu, pools[0], fb)["mapped_bytes"] == 0
    for be, pool in zip(bes, pools):
        assert be.pool_destroy(pool) == 0


def test_prealloc_buffer(gpu):
    """The buffer is the top n frames of the free stack kept mapped: inflates within it map nothing,
    deflates unmap nothing, and the library's thread restores the rule behind the calls."""
    fb = 2 << 20
    pool = gpu.pool_create_elastic(32 * fb, 16, fb)
    assert pool >= 0
    assert gpu.pool_stats(pool)["mapped_bytes"] == 0
    assert gpu.pool_set_prealloc(pool, 6) == 6
    assert gpu.pool_stats(pool)["mapped_bytes"] == 6 * fb              # nobody owns a frame yet; six are ready
    m = gpu.model_register(pool, 32, 8, 128, BF16, 2, 64)
    assert gpu.balloon_resize(m, 4) == 4                     # all four were ready
    st = mapped_matches_owned(gpu, pool, fb, 6)              # ... and the thread has made six ready again
    assert st["mapped_bytes"] == 10 * fb
    assert gpu.balloon_resize(m, 14) == 14                   # 6 from the buffer, 4 mapped by the call itself
    assert mapped_matches_owned(gpu, pool, fb, 6)["mapped_bytes"] == 20 * fb
    assert gpu.balloon_resize(m, 1) == 1                     # 13 come back with their memory ...
    st = gpu.pool_stats(pool)
    assert st["mapped_bytes"] >= 7 * fb                      # (the thread may already be taking it from the deeper ones)
    assert mapped_matches_owned(gpu, pool, fb, 6)["mapped_bytes"] == 7 * fb       # ... of which the top six keep it
    assert gpu.balloon_resize(m, 5) == 5                     # the free stack hands the latest frames out first:
    assert mapped_matches_owned(gpu, pool, fb, 6)["mapped_bytes"] == 11 * fb      # those that were left mapped
    assert gpu.pool_set_prealloc(pool, 0) == 0               # no buffer: only what is owned stays mapped
    assert mapped_matches_owned(gpu, pool, fb, 0)["mapped_bytes"] == 5 * fb
    assert gpu.pool_set_prealloc(pool, 32) == 27             # the whole free stack
    assert mapped_matches_owned(gpu, pool, fb, 32)["mapped_bytes"] == 32 * fb
    assert gpu.pool_set_prealloc(pool, 2) == 2
    assert gpu.balloon_resize(m, 0) == 0 and gpu.model_unregister(m) == 0
    assert mapped_matches_owned(gpu, pool, fb, 2)["mapped_bytes"] == 2 * fb
    assert gpu.pool_destroy(pool) == 0
    assert gpu.pool_create_elastic(32 * fb, 16, fb + 512) < 0          # not a multiple of the granularity


def test_a_cold_inflate_and_any_deflate_stay_off_the_driver(gpu):
    """With a buffer of 176 frames (one admission of the bursty workload) a model that has never held a
    frame inflates by 176, and deflates by 176, without a single mapping call on its path: both return in
    a time that no 176 driver calls would fit into."""
    import time
    fb = 2 << 20
    pool = gpu.pool_create_elastic(2048 * fb, 16, fb)
    assert pool >= 0 and gpu.pool_set_prealloc(pool, 176) == 176
    a = gpu.model_register(pool, 32, 8, 128, BF16, 2, 64)
    b = gpu.model_register(pool, 32, 8, 64, BF16, 2, 64)
    t_inf, t_def = [], []
    for m in (a, b, a, b):
        t0 = time.perf_counter()
        assert gpu.balloon_resize(m, 176) == 176
        t1 = time.perf_counter()
        gpu.pool_prealloc_wait(pool)                  # the thread refills the buffer for the next one
        t2 = time.perf_counter()
        assert gpu.balloon_resize(m, 0) == 0
        t3 = time.perf_counter()
        gpu.pool_prealloc_wait(pool)
        t_inf.append((t1 - t0) * 1e6)
        t_def.append((t3 - t2) * 1e6)
        assert mapped_matches_owned(gpu, pool, fb, 176)["mapped_bytes"] == 176 * fb
    print(f"inflate by 176 frames {t_inf} us, deflate {t_def} us")
    assert max(t_inf) < 1000 and max(t_def) < 1000    # 176 mappings take ~7 ms, 176 unmappings ~44 ms
    assert gpu.model_unregister(a) == 0 and gpu.model_unregister(b) == 0 and gpu.pool_destroy(pool) == 0


@pytest.mark.parametrize("cfg_id", [3, 5])
def test_dynamic_scenarios_on_an_elastic_pool(gpu, oracle, cfg_id):
    """cfg 3 (models switching on and off) and cfg 5 (release, deflate, re-inflate every tenth step)
    at the small sizes, the GPU side on an elastic pool: state bit-exact after every step, attention
    within tolerance, mapped memory equal to the frames owned."""
    cfg = make_config(cfg_id, "small")
    eg = Elastic(gpu)
    rg, ro = Runner(eg, cfg).setup(), Runner(oracle, cfg).setup()
    assert gpu.pool_set_prealloc(rg.pool, 16) == 16
    try:
        for t in range(cfg.steps):
            rg.step(t)
            ro.step(t)
            assert rg.log == ro.log
            assert_same_state(gpu, oracle, rg.pool, ro.pool, f"step {t}")
            if t % 3 == 0:          # (other steps go on while the thread is still at work)
                mapped_matches_owned(gpu, rg.pool, cfg.frame_bytes, 16)
            if t % 7 == 0:
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


def test_inflate_without_memory_is_undone(gpu, oracle):
    """A frame mapping that fails in the middle of an inflate (forced from the host) leaves pool,
    balloon and mappings as they were: the oracle, which never saw the call, still agrees bit for bit."""
    fb = 2 << 20
    pools = [gpu.pool_create_elastic(32 * fb, 16, fb), oracle.pool_create(32 * fb, 16, fb)]
    assert min(pools) >= 0
    bes = (gpu, oracle)
    perm = gen.free_order(32, gen.generator(12))
    ms = []
    for be, pool in zip(bes, pools):
        assert be.pool_seed_free_order(pool, perm) == 0
        m = be.model_register(pool, 32, 8, 128, BF16, 2, 64)
        assert be.balloon_resize(m, 4) == 4
        assert be.seq_reserve(m, 0, 700) >= 0
        ms.append(m)
    try:
        for fail_at in (0, 3):
            assert gpu.debug_fail_frame_map(fail_at) == 0
            assert gpu.balloon_resize(ms[0], 10) == -3             # PKV_E_NOMEM
            assert "refused" in gpu.last_error()
            assert_same_state(gpu, oracle, pools[0], pools[1], f"after the refused inflate ({fail_at})")
            st = mapped_matches_owned(gpu, pools[0], fb)
            assert st["mapped_bytes"] == 4 * fb and st["owned"][ms[0]] == 4
        for be, m in zip(bes, ms):                                  # the hook fired once; now there is memory
            assert be.balloon_resize(m, 10) == 10
            assert be.seq_reserve(m, 1, 900) >= 0
        assert_same_state(gpu, oracle, pools[0], pools[1], "after the inflate that went through")
        assert mapped_matches_owned(gpu, pools[0], fb)["mapped_bytes"] == 10 * fb
        kv = gen.seq_kv((12, 1), 900, 8, 128, BF16, 16)
        assert gpu.kv_write(ms[0], 1, 0, kv["k"], kv["v"], None, None) == 900
        rc, k, v, _, _ = gpu.kv_read(ms[0], 1, 0, 900)
        assert rc == 900 and np.array_equal(k, kv["k"]) and np.array_equal(v, kv["v"])
        assert gpu.device_errors() == 0
    finally:
        gpu.debug_fail_frame_map(-1)
        for be, m, pool in zip(bes, ms, pools):
            be.seq_release(m, 0), be.seq_release(m, 1)
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0
