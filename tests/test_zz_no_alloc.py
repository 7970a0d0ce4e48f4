"""decode_attention_static, the entry point that allocates nothing, through the C-ABI.

Its output must equal decode_attention_ex's (the same kernel code with its partials and
counters elsewhere) to the bar of the attention tests: 2e-3 (bf16 cache) / 2e-2 (e4m3 cache)
per output row, and both must agree with the CPU oracle.  Two calls in a row share the one
scratch array, the second with a smaller input; then a caller's block table, a forced split
that makes nearly every segment a merged one, and the size limit.
"""
import ctypes as C

import numpy as np
import pytest

from parity import TOL, row_rel_err
from workloads import gen

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


def _setup(gpu, oracle, hq, hkv, d, dtype, ctx, seed):
    """One model with the same bookkeeping and KV on both backends."""
    pool_bytes, frame_bytes = 256 << 20, 2 << 20
    perm = gen.free_order(pool_bytes // frame_bytes, gen.generator(seed))
    bb = 2 * 16 * hkv * d * (2 if dtype == BF16 else 1) + (128 if dtype == E4M3 else 0)
    slots = frame_bytes // bb
    blocks = int(sum((c + 15) // 16 for c in ctx))
    res = []
    for be in (gpu, oracle):
        pool = be.pool_create(pool_bytes, 16, frame_bytes)
        assert pool >= 0 and be.pool_seed_free_order(pool, perm) == 0
        m = be.model_register(pool, hq, hkv, d, dtype, len(ctx), 256)
        assert m >= 0
        assert be.balloon_resize(m, (blocks + slots - 1) // slots + 1) > 0
        for upto in range(64, max(ctx) + 64, 64):      # grow in rounds: blocks of different sequences interleave
            assert be.seq_reserve_batch(m, list(range(len(ctx))), [min(c, upto) for c in ctx]) >= 0
        for s, c in enumerate(ctx):
            kv = gen.seq_kv((seed, s), c, hkv, d, dtype, 16)
            assert be.kv_write(m, s, 0, kv["k"], kv["v"], kv["k_scale"], kv["v_scale"]) == c
        res.append((pool, m))
    return res


def _teardown(be, pool, m, n):
    for s in range(n):
        be.seq_release(m, s)
    assert be.balloon_resize(m, 0) == 0
    assert be.model_unregister(m) == 0
    assert be.pool_destroy(pool) == 0


def _static_call(gpu, m, q, ctx, hq, d, block_table=None):
    """Raw C-ABI call: device buffers from torch, nothing else."""
    t = gpu.torch
    qd = t.from_numpy(np.ascontiguousarray(q).view(np.int16)).cuda()
    cd = t.from_numpy(np.ascontiguousarray(ctx, dtype=np.int32)).cuda()
    out = t.full((len(ctx), hq, d), float("nan"), dtype=t.float32, device="cuda")
    bt, stride = None, 0
    if block_table is not None:
        btd = t.from_numpy(np.ascontiguousarray(block_table, dtype=np.int32)).cuda()
        bt, stride = C.c_void_p(btd.data_ptr()), btd.shape[1]
    rc = gpu.lib.decode_attention_static(m, len(ctx), C.c_void_p(qd.data_ptr()), bt, stride,
                                         C.c_void_p(cd.data_ptr()), C.c_void_p(out.data_ptr()))
    t.cuda.synchronize()
    return rc, out.cpu().numpy()


@pytest.mark.parametrize("hq,hkv,d,dtype", [(32, 8, 128, BF16), (32, 8, 64, BF16), (32, 8, 128, E4M3), (16, 1, 128, BF16)])
def test_static_entry_point_matches_the_allocating_one(gpu, oracle, hq, hkv, d, dtype):
    rng = np.random.default_rng(hq * 1000 + d + dtype)
    ctx_big = [int(x) for x in rng.integers(1, 3000, size=24)] + [0, 1, 16, 17]
    ctx_small = ctx_big[:5]
    (gp, gm), (op, om) = _setup(gpu, oracle, hq, hkv, d, dtype, ctx_big, seed=91)
    tol = TOL[dtype]
    try:
        for call, ctx in enumerate((ctx_big, ctx_small)):        # two calls in a row, the second smaller
            print(f"static call {call}: {hq}/{hkv}/{d} dtype {dtype}, batch {len(ctx)}", flush=True)
            q = gen.queries((91, call), len(ctx), hq, d)
            rc_s, out_s = _static_call(gpu, gm, q, ctx, hq, d)
            rc_e, out_e = gpu.decode_attention(gm, q, np.array(ctx, dtype=np.int32))
            rc_o, out_o = oracle.decode_attention(om, q, np.array(ctx, dtype=np.int32))
            assert rc_s == 0 and rc_e == 0 and rc_o == 0, (rc_s, rc_e, rc_o, gpu.last_error())
            assert row_rel_err(out_s, out_e) <= tol
            assert row_rel_err(out_s, out_o) <= tol
            assert row_rel_err(out_e, out_o) <= tol
        # a split that cuts nearly every segment: most rows come out of the merge through the scratch array
        assert gpu.set_split(100000, 1) == 0
        q = gen.queries((91, 7), len(ctx_big), hq, d)
        rc_s, out_s = _static_call(gpu, gm, q, ctx_big, hq, d)
        rc_o, out_o = oracle.decode_attention(om, q, np.array(ctx_big, dtype=np.int32))
        assert rc_s == 0 and row_rel_err(out_s, out_o) <= tol
        gpu.set_split(37, 3)
        rc_s, out_s = _static_call(gpu, gm, q, ctx_big, hq, d)
        assert rc_s == 0 and row_rel_err(out_s, out_o) <= tol
        gpu.set_split(0, 0)
        # a caller's block table
        rows = oracle.block_table_rows(om, len(ctx_big))
        perm = rng.permutation(len(ctx_big))
        bt = np.ascontiguousarray(rows[perm][:, :192])
        rc_s, out_s = _static_call(gpu, gm, q[perm], [ctx_big[i] for i in perm], hq, d, block_table=bt)
        assert rc_s == 0 and row_rel_err(out_s, out_o[perm]) <= tol
        assert gpu.device_errors() == 0
    finally:
        gpu.set_split(0, 0)
        _teardown(gpu, gp, gm, len(ctx_big))
        _teardown(oracle, op, om, len(ctx_big))


def test_static_entry_point_rejects_what_does_not_fit(gpu):
    pool = gpu.pool_create(64 << 20, 16, 2 << 20)
    m = gpu.model_register(pool, 32, 8, 128, BF16, 16, 16)
    t = gpu.torch
    n = 32768 // 8 + 1                      # one sequence more than the arrival counters cover
    q = t.zeros((n, 32, 128), dtype=t.int16, device="cuda")
    ctx = t.zeros(n, dtype=t.int32, device="cuda")
    bt = t.zeros((n, 4), dtype=t.int32, device="cuda")
    out = t.zeros((n, 32, 128), dtype=t.float32, device="cuda")
    p = lambda x: C.c_void_p(x.data_ptr())
    rc = gpu.lib.decode_attention_static(m, n, p(q), p(bt), 4, p(ctx), p(out))
    assert rc == -6 and "arrival counters" in gpu.last_error()          # PKV_E_RANGE
    assert gpu.lib.decode_attention_static(m, n - 1, p(q), p(bt), 4, p(ctx), p(out)) == 0     # the largest that fits
    t.cuda.synchronize()
    assert float(out[: n - 1].abs().max()) == 0.0                        # empty contexts: zero rows
    assert gpu.lib.decode_attention_static(m, 17, p(q), None, 0, p(ctx), p(out)) == -6           # more rows than the model has
    assert gpu.lib.decode_attention_static(99, 1, p(q), None, 0, p(ctx), p(out)) == -2
    assert gpu.device_errors() == 0
    assert gpu.model_unregister(m) == 0 and gpu.pool_destroy(pool) == 0
