"""GPU parity of chunked-prefill attention (causal, against the paged cache) with the oracle."""
import numpy as np
import pytest
import torch

from parity import TOL, row_rel_err
from workloads import gen

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1
UNEVEN = [1.25, 0.75, 1.1, 0.9, 1.2, 0.8, 1.0, 1.0]


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


class Twin:
    def __init__(self, gpu, oracle, hq, hkv, d, dtype, ctx, seed=13, poison=True, pool_bytes=64 << 20, max_blocks=64):
        self.be = (gpu, oracle)
        self.ctx = np.array(ctx, dtype=np.int32)
        self.pools, self.models = [], []
        frame_bytes = 2 << 20
        perm = gen.free_order(pool_bytes // frame_bytes, gen.generator(seed, 1))
        for be in self.be:
            storage = None
            if be is gpu and poison:          # every byte decodes to NaN until written
                storage = torch.full((pool_bytes,), 0xFF, dtype=torch.uint8, device="cuda")
            pool = be.pool_create(pool_bytes, 16, frame_bytes, storage) if be is gpu else be.pool_create(pool_bytes, 16, frame_bytes)
            assert pool >= 0 and be.pool_seed_free_order(pool, perm) == 0
            m = be.model_register(pool, hq, hkv, d, dtype, len(ctx), max_blocks)
            assert m >= 0
            assert be.balloon_resize(m, pool_bytes // frame_bytes) > 0
            for upto in range(48, max(max(ctx), 1) + 48, 48):       # interleave the rows' blocks
                assert be.seq_reserve_batch(m, list(range(len(ctx))), [min(c, upto) for c in ctx]) >= 0
            self.pools.append(pool)
            self.models.append(m)
        for s, c in enumerate(ctx):
            if c:
                kv = gen.seq_kv((seed, s), c, hkv, d, dtype, 16)
                for be, m in zip(self.be, self.models):
                    assert be.kv_write(m, s, 0, kv["k"], kv["v"], kv.get("k_scale"), kv.get("v_scale")) == c

    def close(self):
        for be, m, pool in zip(self.be, self.models, self.pools):
            for s in range(len(self.ctx)):
                be.seq_release(m, s)
            assert be.balloon_resize(m, 0) == 0 and be.model_unregister(m) == 0 and be.pool_destroy(pool) == 0


CASES = [(13, 5), (6, 6), (9, 1), (300, 37), (64, 64), (33, 17), (16, 16), (100, 0), (257, 256), (48, 32)]


@pytest.mark.parametrize("hq,hkv,d,dtype", [
    (32, 8, 128, BF16), (8, 2, 64, BF16), (64, 8, 128, BF16), (16, 1, 128, BF16), (3, 3, 64, BF16),
    (12, 4, 64, E4M3), (32, 8, 128, E4M3)])
def test_prefill_matches_oracle(gpu, oracle, hq, hkv, d, dtype):
    """Chunks that start at 0, inside and on page boundaries, of 0, 1 and many tokens; tiles of 1 to 16
    query tokens per MFMA pass (g = 16 ... 1); the pool starts as NaN."""
    ctx = [c for c, _ in CASES]
    qlen = [q for _, q in CASES]
    t = Twin(gpu, oracle, hq, hkv, d, dtype, ctx)
    q = gen.queries((17, d, hq), sum(qlen), hq, d)
    rc_o, out_o = oracle.prefill_attention(t.models[1], q, qlen, ctx)
    assert rc_o == 0
    for items, share, seg, w in ((0, 0, -1, None), (100000, 1, 0, None), (37, 3, 2, None), (64, 16, 5, UNEVEN)):
        assert gpu.set_split(items, share) == 0 and gpu.set_segment_cost(seg) == 0 and gpu.set_xcd_weights(w) == 0
        rc_g, out_g = gpu.prefill_attention(t.models[0], q, qlen, ctx)
        assert rc_g == 0
        err = row_rel_err(out_g, out_o)
        assert err <= TOL[dtype], (items, share, err)
    gpu.set_split(0, 0)
    gpu.set_segment_cost(-1)
    gpu.set_xcd_weights(None)
    assert gpu.device_errors() == 0
    # the last query of every chunk is a decode step
    sel = [i for i, ql in enumerate(qlen) if ql > 0]
    last = (np.cumsum(qlen) - 1)[sel]
    rc_d, out_d = gpu.decode_attention(t.models[0], q[last], np.array(ctx, dtype=np.int32)[sel]) if len(sel) == len(ctx) else (0, None)
    if out_d is not None:
        assert rc_d == 0 and row_rel_err(out_d, out_o[last]) <= TOL[dtype]
    t.close()


def test_prefill_then_decode_steps(gpu, oracle):
    """A sequence is prefilled in two chunks, then decoded: append, attend, repeat."""
    hq, hkv, d = 32, 8, 128
    total, c1, c2, steps = 90, 50, 40, 6
    t = Twin(gpu, oracle, hq, hkv, d, BF16, [total + steps, total + steps], poison=False)
    ctx_full = np.array([total + steps] * 2, dtype=np.int32)
    for (lo, n) in ((0, c1), (c1, c2)):
        q = gen.queries((23, lo), 2 * n, hq, d)
        ctx = np.array([lo + n] * 2, dtype=np.int32)
        rc_g, g_ = gpu.prefill_attention(t.models[0], q, [n, n], ctx)
        rc_o, o_ = oracle.prefill_attention(t.models[1], q, [n, n], ctx)
        assert rc_g == 0 and rc_o == 0 and row_rel_err(g_, o_) <= TOL[BF16]
    g = gen.generator(29)
    ctx = np.array([total] * 2, dtype=np.int32)
    for step in range(steps):
        kx = gen.to_bf16_bits(torch.randn((2, hkv, d), generator=g))
        vx = gen.to_bf16_bits(torch.randn((2, hkv, d), generator=g))
        ctx += 1
        for be, m in zip(t.be, t.models):
            assert be.kv_append(m, kx, vx, ctx) == 2
        q = gen.queries((23, 100 + step), 2, hq, d)
        rc_g, g_ = gpu.decode_attention(t.models[0], q, ctx)
        rc_o, o_ = oracle.decode_attention(t.models[1], q, ctx)
        assert rc_g == 0 and rc_o == 0 and row_rel_err(g_, o_) <= TOL[BF16]
    assert np.array_equal(ctx, ctx_full)
    t.close()


def test_prefill_arguments(gpu, oracle):
    t = Twin(gpu, oracle, 8, 2, 64, BF16, [40, 40], poison=False)
    q = gen.queries((1, 2), 8, 8, 64)
    qd = torch.from_numpy(q.view(np.int16)).cuda()
    ctx = torch.tensor([40, 40], dtype=torch.int32, device="cuda")
    out = torch.empty((8, 8, 64), dtype=torch.float32, device="cuda")
    assert gpu.prefill_attention_dev(t.models[0], qd, np.array([4, -1], dtype=np.int32), ctx, out) < 0
    assert gpu.prefill_attention_dev(9999, qd, np.array([4, 4], dtype=np.int32), ctx, out) < 0
    assert gpu.prefill_attention_dev(t.models[0], qd, np.array([0, 0], dtype=np.int32), ctx, out) == 0
    t.close()


LONG = [(1500, 3), (1024, 40), (2047, 1), (777, 16), (640, 0), (999, 33)]


@pytest.mark.parametrize("hq,hkv,d,dtype", [(32, 8, 128, BF16), (16, 2, 64, BF16), (12, 4, 64, E4M3), (32, 8, 128, E4M3)])
def test_few_queries_in_front_of_long_contexts(gpu, oracle, hq, hkv, d, dtype):
    """Few query groups and long contexts: every group is walked by several work-groups, each with a
    part of the context, and their partial results are joined.  The second call asks with shorter
    contexts than the rows hold, so that the last parts of some groups see no token at all."""
    ctx = [c for c, _ in LONG]
    qlen = [q for _, q in LONG]
    t = Twin(gpu, oracle, hq, hkv, d, dtype, ctx, max_blocks=128, pool_bytes=128 << 20)
    q = gen.queries((19, d, hq), sum(qlen), hq, d)
    for shrink in (0, 600):
        c2 = [max(ql, c - shrink) for c, ql in LONG]
        rc_o, out_o = oracle.prefill_attention(t.models[1], q, qlen, c2)
        rc_g, out_g = gpu.prefill_attention(t.models[0], q, qlen, c2)
        assert rc_o == 0 and rc_g == 0
        err = row_rel_err(out_g, out_o)
        assert err <= TOL[dtype], (shrink, err)
    assert gpu.device_errors() == 0
    t.close()


@pytest.mark.parametrize("d,dtype", [(128, BF16), (64, BF16), (128, E4M3)])
def test_scores_that_rise_and_fall_along_the_context(gpu, oracle, d, dtype):
    """Keys along a fixed direction with a length that grows (or shrinks) with the token's position: the
    logits of a query head ramp up or down along the context, depending on the sign of its component in
    that direction, by a little per page pair in one sequence (the running maximum creeps: the reference
    point of the exponentials lags behind it by design and is moved only now and then), by more than the
    allowed lag per pair in another (it moves in every step), and not at all in a third.  Decode and
    chunked prefill against the oracle."""
    import torch
    hq, hkv = 16, 4
    ctx = [1500, 700, 900, 333]
    slope = [0.1, 0.6, 0.0, -0.3]                       # growth of a key's length per token
    t = Twin(gpu, oracle, hq, hkv, d, dtype, ctx, max_blocks=96)
    g = gen.generator(91, d, dtype)
    e = torch.randn((hkv, d), generator=g)
    e = e / e.norm(dim=-1, keepdim=True)
    for s, (c, sl) in enumerate(zip(ctx, slope)):
        pos = torch.arange(c, dtype=torch.float32)
        length = (sl * pos if sl >= 0 else -sl * (c - pos))[:, None, None]
        k = length * e[None] * (d ** 0.5) / 4 + 0.05 * torch.randn((c, hkv, d), generator=g)
        v = torch.randn((c, hkv, d), generator=g)
        if dtype == BF16:
            kb, vb, ks, vs = gen.to_bf16_bits(k), gen.to_bf16_bits(v), None, None
        else:
            (kb, ks), (vb, vs) = gen.quantise_e4m3(k, 16), gen.quantise_e4m3(v, 16)
        for be, m in zip(t.be, t.models):
            assert be.kv_write(m, s, 0, kb, vb, ks, vs) == c
    # decode: one query per sequence; prefill: the last 40 tokens of every sequence as a chunk
    q = gen.queries((92, d), len(ctx), hq, d)
    cl = np.array(ctx, dtype=np.int32)
    for form in (0, 1):
        assert gpu.set_kernel_form(form) == 0
        rc_g, out_g = gpu.decode_attention(t.models[0], q, cl)
        rc_o, out_o = oracle.decode_attention(t.models[1], q, cl)
        assert rc_g == 0 and rc_o == 0
        err = row_rel_err(out_g, out_o)
        assert err <= TOL[dtype], (form, err)
    gpu.set_kernel_form(-1)
    qlen = [40] * len(ctx)
    qp = gen.queries((93, d), sum(qlen), hq, d)
    rc_g, out_g = gpu.prefill_attention(t.models[0], qp, qlen, ctx)
    rc_o, out_o = oracle.prefill_attention(t.models[1], qp, qlen, ctx)
    assert rc_g == 0 and rc_o == 0
    err = row_rel_err(out_g, out_o)
    assert err <= TOL[dtype], err
    assert gpu.device_errors() == 0
    t.close()


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_prefill_at_the_size_the_bench_times(gpu, oracle, dtype):
    """The chunk of bench.py's prefill leg — 512 new tokens behind 2048 cached ones, 32 q heads, 8 kv heads,
    128-wide heads, every group of 32 query tokens on the mask-free path for most of its context — for
    three sequences (the bench has eight of the same kind), every output row against the oracle."""
    from parity import elementwise_rel_err
    hq, hkv, d, prefix, chunk = 32, 8, 128, 2048, 512
    ctx = [prefix + chunk] * 3
    qlen = [chunk] * 3
    t = Twin(gpu, oracle, hq, hkv, d, dtype, ctx, max_blocks=(prefix + chunk) // 16, pool_bytes=256 << 20)
    q = gen.queries((23, dtype), sum(qlen), hq, d)
    rc_o, out_o = oracle.prefill_attention(t.models[1], q, qlen, ctx)
    rc_g, out_g = gpu.prefill_attention(t.models[0], q, qlen, ctx)
    assert rc_o == 0 and rc_g == 0
    err = row_rel_err(out_g, out_o)
    print(f"dtype {dtype}: worst row error {err:.3e}, floored per-element error {elementwise_rel_err(out_g, out_o):.3e}")
    assert err <= TOL[dtype], err
    assert gpu.device_errors() == 0
    t.close()
