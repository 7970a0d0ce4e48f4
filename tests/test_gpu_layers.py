"""GPU parity for models of several layers that share one block table (paper Sec. 4.2, D3:
the K and V of all layers of a token block lie side by side, one allocation for all).

Two co-located models of different depth and cache type go through the same calls on the
HIP library and on the oracle.  Bookkeeping must agree bit for bit; on every layer the
cache must read back exactly, decode and chunked-prefill attention must agree within
2e-3 (bf16 cache) / 2e-2 (e4m3 cache), and an appended token must produce the same codes
and scales bit for bit.
"""
import copy

import numpy as np
import pytest

from parity import TOL, assert_same_state, row_rel_err
from workloads import gen
from workloads.scenarios import Runner, make_config
from test_gpu_full_size import compare_sampled, sample_longest_median_shortest

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1
SHAPES = [(32, 8, 128, BF16, 3), (12, 4, 64, E4M3, 5)]      # q heads, kv heads, head dim, cache type, layers
CTX = [[300, 0, 17, 1024, 64], [33, 700, 16, 1, 257]]


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


class TwoModels:
    def __init__(self, gpu, oracle, elastic=False):
        self.be = (gpu, oracle)
        self.pools, self.models = [], []
        pool_bytes, frame = 256 << 20, 2 << 20
        perm = gen.free_order(pool_bytes // frame, gen.generator(17))
        for be in self.be:
            pool = be.pool_create_elastic(pool_bytes, 16, frame) if (elastic and be is gpu) else \
                be.pool_create(pool_bytes, 16, frame)
            assert pool >= 0
            assert be.pool_seed_free_order(pool, perm) == 0
            ms = [be.model_register(pool, hq, hkv, d, dt, 5, 80, n_layers=L) for hq, hkv, d, dt, L in SHAPES]
            assert min(ms) >= 0
            want = [0, 0]
            for mi, (hq, hkv, d, dt, L) in enumerate(SHAPES):
                bb = L * (2 * 16 * hkv * d * (2 if dt == BF16 else 1) + (128 if dt == E4M3 else 0))
                slots = frame // bb
                blocks = sum((c + 15) // 16 for c in CTX[mi]) + 5
                want[mi] = (blocks + slots - 1) // slots
            have = [0, 0]
            while have != want:                     # alternate so the balloons interleave
                for mi in range(2):
                    if have[mi] < want[mi]:
                        have[mi] += 1
                        assert be.balloon_resize(ms[mi], have[mi]) == have[mi]
            for upto in range(80, 1024 + 80, 80):
                for mi in range(2):
                    assert be.seq_reserve_batch(ms[mi], list(range(5)), [min(c, upto) for c in CTX[mi]]) >= 0
            self.pools.append(pool)
            self.models.append(ms)
        self.kv = {}
        for mi, (hq, hkv, d, dt, L) in enumerate(SHAPES):
            for layer in (L - 1,) + tuple(range(L - 1)):          # not in address order
                for s, c in enumerate(CTX[mi]):
                    kv = gen.seq_kv((41, mi, layer, s), c, hkv, d, dt, 16)
                    self.kv[mi, layer, s] = kv
                    for be, ms in zip(self.be, self.models):
                        assert be.set_layer(ms[mi], layer) == 0
                        if c:
                            assert be.kv_write(ms[mi], s, 0, kv["k"], kv["v"], kv["k_scale"], kv["v_scale"]) == c

    def same_state(self, what):
        assert_same_state(self.be[0], self.be[1], self.pools[0], self.pools[1], what)

    def close(self):
        for be, ms, pool in zip(self.be, self.models, self.pools):
            for m in ms:
                for s in range(5):
                    be.seq_release(m, s)
                assert be.balloon_resize(m, 0) == 0
                assert be.model_unregister(m) == 0
            assert be.pool_destroy(pool) == 0


@pytest.mark.parametrize("elastic", [False, True])
def test_layers_decode_readback_append_prefill(gpu, oracle, elastic):
    tm = TwoModels(gpu, oracle, elastic)
    try:
        tm.same_state("after the set-up")
        for mi, (hq, hkv, d, dt, L) in enumerate(SHAPES):
            ctx = np.array(CTX[mi], dtype=np.int32)
            q = gen.queries((41, 7, mi), 5, hq, d)
            outs = []
            for layer in range(L):
                res = []
                for be, ms in zip(tm.be, tm.models):
                    assert be.set_layer(ms[mi], layer) == 0
                    for s, c in enumerate(CTX[mi]):                # the layer holds exactly what was written to it
                        if c:
                            rc, k, v, ks, vs = be.kv_read(ms[mi], s, 0, c)
                            assert rc == c
                            kv = tm.kv[mi, layer, s]
                            assert np.array_equal(k, kv["k"]) and np.array_equal(v, kv["v"]), (mi, layer, s)
                            if dt == E4M3:
                                blk = np.arange(c) // 16
                                assert np.array_equal(ks, kv["k_scale"][blk]) and np.array_equal(vs, kv["v_scale"][blk])
                    rc, out = be.decode_attention(ms[mi], q, ctx)
                    assert rc == 0
                    res.append(out)
                err = row_rel_err(res[0], res[1])
                assert err <= TOL[dt], (mi, layer, err)
                outs.append(res[0])
            assert not np.allclose(outs[0], outs[-1])              # the layers really differ

        # one grouped launch, the two models on different layers
        layers = (2, 4)
        qs = [gen.queries((41, 8, mi), 5, SHAPES[mi][0], SHAPES[mi][2]) for mi in range(2)]
        ctxs = [np.array(CTX[mi], dtype=np.int32) for mi in range(2)]
        for be, ms in zip(tm.be, tm.models):
            for mi in range(2):
                assert be.set_layer(ms[mi], layers[mi]) == 0
        import torch
        dq = [torch.from_numpy(q.view(np.int16)).cuda() for q in qs]
        dc = [torch.from_numpy(c).cuda() for c in ctxs]
        do = [torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda") for q in qs]
        assert gpu.decode_attention_multi_dev(tm.models[0], dq, dc, do) == 0
        torch.cuda.synchronize()
        got = [o.cpu().numpy() for o in do]
        for mi in range(2):
            rc, ref = oracle.decode_attention(tm.models[1][mi], qs[mi], ctxs[mi])
            assert rc == 0 and row_rel_err(got[mi], ref) <= TOL[SHAPES[mi][3]]

        # a decode step's append on layer 1 of both models: same codes and scales, other layers untouched
        for mi, (hq, hkv, d, dt, L) in enumerate(SHAPES):
            ctx1 = np.array(CTX[mi], dtype=np.int32) + 1
            new_k = gen.randn_bf16((5, hkv, d), gen.generator(43, mi))
            new_v = gen.randn_bf16((5, hkv, d), gen.generator(44, mi))
            for be, ms in zip(tm.be, tm.models):
                assert be.seq_reserve_batch(ms[mi], list(range(5)), ctx1) >= 0
                assert be.set_layer(ms[mi], 1) == 0
                assert be.kv_append(ms[mi], new_k, new_v, ctx1) >= 0
            for layer in (0, 1, L - 1):
                for s in range(5):
                    n = int(ctx1[s]) if layer == 1 else CTX[mi][s]
                    if n == 0:
                        continue
                    back = []
                    for be, ms in zip(tm.be, tm.models):
                        be.set_layer(ms[mi], layer)
                        back.append(be.kv_read(ms[mi], s, 0, n))
                    assert back[0][0] == back[1][0] == n
                    for a, b in zip(back[0][1:], back[1][1:]):
                        assert (a is None and b is None) or np.array_equal(a, b), (mi, layer, s)
            # chunked prefill on layer 1: the last tokens (the appended one included) as queries
            q_lens = np.minimum(np.array([40, 1, 9, 130, 0], dtype=np.int32), ctx1)
            qc = gen.queries((41, 9, mi), int(q_lens.sum()), hq, d)
            res = []
            for be, ms in zip(tm.be, tm.models):
                be.set_layer(ms[mi], 1)
                rc, out = be.prefill_attention(ms[mi], qc, q_lens, ctx1)
                assert rc == 0
                res.append(out)
            assert row_rel_err(res[0], res[1]) <= TOL[dt]
        tm.same_state("after the appends")
        assert gpu.set_layer(tm.models[0][0], 3) == -1 and gpu.set_layer(tm.models[0][0], -1) == -1
        assert gpu.set_layer(63, 0) == -2
        assert gpu.device_errors() == 0
    finally:
        tm.close()


def test_refusals_match_oracle(gpu, oracle):
    res = []
    for be in (gpu, oracle):
        pool = be.pool_create(4 << 20, 16, 64 << 10)
        r = [be.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=0),
             be.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=9)]      # 9 x 8 KiB > one frame
        m = be.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=8)
        r.append(m >= 0)
        r.append(be.set_layer(m, 8))
        r.append(be.model_unregister(m))
        r.append(be.pool_destroy(pool))
        res.append(r)
    assert res[0] == res[1] == [-1, -5, True, -1, 0, 0]


def test_full_size_two_models_four_layers(gpu, oracle):
    """The two-model workload at its full size with four layers per model: bookkeeping bit
    for bit, attention on the sampled sequences on the first and the last layer."""
    cfg = copy.deepcopy(make_config(2, "full"))
    for spec in cfg.models:
        spec.layers = 4
    fill = sample_longest_median_shortest(cfg, 3)
    rg, ro = Runner(gpu, cfg, fill=fill).setup(), Runner(oracle, cfg, fill=fill).setup()
    try:
        assert rg.log == ro.log
        assert np.array_equal(gpu.pool_export_state(rg.pool), oracle.pool_export_state(ro.pool))
        for layer in (0, 3):
            for r in (rg, ro):
                for mi in range(len(cfg.models)):
                    r.set_layer(mi, layer)
            print(f"layer {layer}: sampled rel err {compare_sampled(gpu, oracle, rg, ro, layer):.2e}")
        assert gpu.device_errors() == 0
    finally:
        rg.teardown()
        ro.teardown()
