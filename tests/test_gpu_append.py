"""GPU parity of the write path: kv_write / kv_read round trip, and the decode step's
kv_append against the oracle — stored values and e4m3 codes and scales bit for bit,
then decode attention over what was appended."""
import numpy as np
import pytest
import torch

from parity import TOL, assert_same_state, row_rel_err
from workloads import gen

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


class Twin:
    """One model on both backends, rows reserved up to `cap` tokens, `start` of them written in bulk."""

    def __init__(self, gpu, oracle, hq, hkv, d, dtype, start, cap, seed=5):
        self.be = (gpu, oracle)
        self.hq, self.hkv, self.d, self.dtype = hq, hkv, d, dtype
        self.pools, self.models = [], []
        pool_bytes, frame_bytes = 64 << 20, 2 << 20
        perm = gen.free_order(pool_bytes // frame_bytes, gen.generator(seed, 1))
        for be in self.be:
            pool = be.pool_create(pool_bytes, 16, frame_bytes)
            assert pool >= 0 and be.pool_seed_free_order(pool, perm) == 0
            m = be.model_register(pool, hq, hkv, d, dtype, len(start), 64)
            assert m >= 0
            assert be.balloon_resize(m, 16) == 16
            assert be.seq_reserve_batch(m, list(range(len(start))), cap) >= 0
            self.pools.append(pool)
            self.models.append(m)
        self.ctx = np.array(start, dtype=np.int32)
        for s, c in enumerate(start):
            if c:
                kv = gen.seq_kv((seed, s), c, hkv, d, dtype, 16)
                for be, m in zip(self.be, self.models):
                    assert be.kv_write(m, s, 0, kv["k"], kv["v"], kv.get("k_scale"), kv.get("v_scale")) == c

    def compare_cache(self):
        for s, c in enumerate(self.ctx):
            if c == 0:
                continue
            a = self.be[0].kv_read(self.models[0], s, 0, int(c))
            b = self.be[1].kv_read(self.models[1], s, 0, int(c))
            assert a[0] == c and b[0] == c
            assert np.array_equal(a[1], b[1]), f"seq {s}: K differs"
            assert np.array_equal(a[2], b[2]), f"seq {s}: V differs"
            if self.dtype == E4M3:
                assert np.array_equal(a[3], b[3]) and np.array_equal(a[4], b[4]), f"seq {s}: scales differ"

    def close(self):
        for be, m, pool in zip(self.be, self.models, self.pools):
            for s in range(len(self.ctx)):
                be.seq_release(m, s)
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0


@pytest.mark.parametrize("hq,hkv,d,dtype", [(32, 8, 128, BF16), (8, 2, 64, BF16), (32, 8, 128, E4M3), (12, 4, 64, E4M3)])
def test_write_read_round_trip(gpu, oracle, hq, hkv, d, dtype):
    t = Twin(gpu, oracle, hq, hkv, d, dtype, [37, 16, 1, 100], [37, 16, 1, 100])
    t.compare_cache()
    kv = gen.seq_kv((5, 3), 100, hkv, d, dtype, 16)
    rc, k, v, ks, vs = gpu.kv_read(t.models[0], 3, 0, 100)
    assert rc == 100 and np.array_equal(k, kv["k"]) and np.array_equal(v, kv["v"])
    if dtype == E4M3:
        assert np.array_equal(ks, np.repeat(kv["k_scale"], 16, axis=0)[:100])
    rc, k2, _, _, _ = gpu.kv_read(t.models[0], 3, 21, 30)        # a range that starts inside a block
    assert rc == 30 and np.array_equal(k2, kv["k"][21:51])
    t.close()


@pytest.mark.parametrize("hq,hkv,d,dtype", [(32, 8, 128, BF16), (8, 2, 64, BF16), (32, 8, 128, E4M3), (12, 4, 64, E4M3)])
def test_append_matches_oracle(gpu, oracle, hq, hkv, d, dtype):
    """40 decode steps on sequences that start empty, inside a block and on a block boundary;
    token magnitudes wander so that e4m3 scales grow inside blocks and codes get re-encoded."""
    start = [0, 5, 16, 31, 47]
    steps = 40
    t = Twin(gpu, oracle, hq, hkv, d, dtype, start, [c + steps for c in start])
    g = gen.generator(91, d, dtype)
    B = len(start)
    for step in range(steps):
        mag = torch.exp(torch.randn((B, 1, 1), generator=g))             # per-token magnitude, log-normal
        kx = gen.to_bf16_bits(torch.randn((B, hkv, d), generator=g) * mag)
        vx = gen.to_bf16_bits(torch.randn((B, hkv, d), generator=g) * mag)
        if step == 7:
            kx[1] = 0                                                      # an all-zero token
        t.ctx += 1
        for be, m in zip(t.be, t.models):
            assert be.kv_append(m, kx, vx, t.ctx) == B
        if step in (0, 1, 10, 15, 16, 17, 39):
            t.compare_cache()
    assert gpu.device_errors() == 0
    assert_same_state(gpu, oracle, t.pools[0], t.pools[1])                 # appending moves no block
    q = gen.queries((91, 2), B, hq, d)
    rc_g, out_g = gpu.decode_attention(t.models[0], q, t.ctx)
    rc_o, out_o = oracle.decode_attention(t.models[1], q, t.ctx)
    assert rc_g == 0 and rc_o == 0 and row_rel_err(out_g, out_o) <= TOL[dtype]
    t.close()


def test_append_encoder_ties_and_range(gpu, oracle):
    """Every e4m3 midpoint and its neighbours, the saturation edge and the subnormal range go
    through the append path with scale 1 (a 448 in the row pins amax)."""
    hq, hkv, d = 8, 1, 128
    vals = sorted({oracle.e4m3_decode(c) for c in range(0x7F)})
    mids = [(a + b) / 2 for a, b in zip(vals[:-1], vals[1:])]             # 126 midpoints, all exact in bf16
    rows = []
    row = np.array([448.0] + mids + [0.0], dtype=np.float32)
    rows.append(row)
    rows.append(-row)
    up = np.nextafter(row.astype(np.float32), np.float32(1e9)).astype(np.float32)
    rows.append(np.concatenate([[448.0], up[1:]]))                          # bf16 rounding of these is part of the input
    rows.append(np.concatenate([[448.0], np.linspace(0, 2.0 ** -5, 127, dtype=np.float32)]))
    t = Twin(gpu, oracle, hq, hkv, d, E4M3, [0] * len(rows), [16] * len(rows))
    x = gen.to_bf16_bits(torch.from_numpy(np.stack(rows)).view(len(rows), 1, d))
    t.ctx += 1
    for be, m in zip(t.be, t.models):
        assert be.kv_append(m, x, x, t.ctx) == len(rows)
    t.compare_cache()
    rc, k, _, ks, _ = gpu.kv_read(t.models[0], 0, 0, 1)
    assert ks[0, 0] == np.float32(1.0) and k[0, 0, 0] == 0x7E
    t.close()


def test_append_bad_context_is_reported_not_written(gpu, oracle):
    t = Twin(gpu, oracle, 8, 2, 64, BF16, [4, 4], [20, 20])
    kx = gen.randn_bf16((2, 2, 64), gen.generator(3))
    before = gpu.kv_read(t.models[0], 0, 0, 4)
    assert gpu.kv_append(t.models[0], kx, kx, np.array([0, 33], dtype=np.int32)) == 2
    assert gpu.device_errors() == 2 and gpu.device_errors() == 0
    after = gpu.kv_read(t.models[0], 0, 0, 4)
    assert np.array_equal(before[1], after[1]) and np.array_equal(before[2], after[2])
    assert oracle.kv_append(t.models[1], kx, kx, np.array([0, 33], dtype=np.int32)) < 0
    t.close()


@pytest.mark.parametrize("hq,hkv,d,dtype", [(32, 8, 128, BF16), (32, 8, 128, E4M3), (12, 4, 64, E4M3)])
def test_chunk_append_then_prefill(gpu, oracle, hq, hkv, d, dtype):
    """Prefill chunks are written with kv_append_chunk (stored values, e4m3 codes and scales equal the
    oracle's bit for bit), attended with prefill_attention, then a decode step follows."""
    start = [0, 7, 16, 40]
    chunks = [[33, 0, 16, 5], [1, 20, 31, 0]]
    t = Twin(gpu, oracle, hq, hkv, d, dtype, start, [c + 70 for c in start])
    g = gen.generator(57, d, dtype)
    for ql in chunks:
        ql = np.array(ql, dtype=np.int32)
        n = int(ql.sum())
        mag = torch.exp(torch.randn((n, 1, 1), generator=g))
        kx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        vx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        t.ctx += ql
        for be, m in zip(t.be, t.models):
            assert be.kv_append_chunk(m, kx, vx, ql, t.ctx) == n
        t.compare_cache()
        q = gen.queries((57, n), n, hq, d)
        rc_g, out_g = gpu.prefill_attention(t.models[0], q, ql, t.ctx)
        rc_o, out_o = oracle.prefill_attention(t.models[1], q, ql, t.ctx)
        assert rc_g == 0 and rc_o == 0 and row_rel_err(out_g, out_o) <= TOL[dtype]
    q = gen.queries((57, 1), len(start), hq, d)
    rc_g, out_g = gpu.decode_attention(t.models[0], q, t.ctx)
    rc_o, out_o = oracle.decode_attention(t.models[1], q, t.ctx)
    assert rc_g == 0 and rc_o == 0 and row_rel_err(out_g, out_o) <= TOL[dtype]
    assert gpu.device_errors() == 0
    # a chunk longer than the cache is reported and skipped
    assert gpu.kv_append_chunk(t.models[0], kx[:3], vx[:3], [3, 0, 0, 0], np.array([2, 9, 9, 9], dtype=np.int32)) == 3
    assert gpu.device_errors() == 2
    t.close()


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_long_chunk_over_many_pages(gpu, oracle, dtype):
    """A chunk that starts inside a block and runs over more than a dozen pages (each page of the
    chunk is written by a wave of its own): the cache equals the oracle's token-by-token result
    bit for bit, codes and scales included, and a second chunk continues the last block's scale."""
    hq, hkv, d = 16, 4, 128
    start = [13, 0, 32]
    t = Twin(gpu, oracle, hq, hkv, d, dtype, start, [c + 400 for c in start])
    g = gen.generator(61, dtype)
    for ql in ([200, 129, 1], [150, 17, 250]):
        ql = np.array(ql, dtype=np.int32)
        n = int(ql.sum())
        mag = torch.exp(torch.randn((n, 1, 1), generator=g))
        kx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        vx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        t.ctx += ql
        for be, m in zip(t.be, t.models):
            assert be.kv_append_chunk(m, kx, vx, ql, t.ctx) == n
        t.compare_cache()
    assert gpu.device_errors() == 0
    t.close()
