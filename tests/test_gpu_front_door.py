"""The four calls the library is named for, through raw ctypes exactly as they are spelled:
pool_create(bytes, page_tokens), model_register(q_heads, kv_heads, head_dim, dtype),
balloon_resize(model, pages), decode_attention(model, q, block_table, ctx_lens, out)
(with model_set_batch for the batch shape) — against the oracle, with two pools alive."""
import ctypes as C

import numpy as np
import pytest

from parity import TOL, row_rel_err
from workloads import gen

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


def test_named_calls_with_two_pools(gpu, oracle):
    lib, t = gpu.lib, gpu.torch
    first = lib.pool_create(C.c_size_t(64 << 20), 16)
    second = lib.pool_create(C.c_size_t(96 << 20), 16)
    assert first >= 0 and second >= 0 and first != second
    o_first, o_second = oracle.pool_create(64 << 20, 16), oracle.pool_create(96 << 20, 16)
    # model_register names no pool: the model lands in the pool created last
    m = lib.model_register(32, 8, 128, 0)
    om = oracle.model_register(o_second, 32, 8, 128, 0)
    assert m >= 0 and om >= 0
    gpu._shape[m] = (32, 8, 128, 0)          # the binding's note of the shape, for its kv_write convenience
    st = gpu.pool_stats(second)
    assert st["n_frames"] == 48 and gpu.pool_stats(first)["n_frames"] == 32
    assert lib.model_register(7, 2, 64, 0) == -5                     # q heads not a multiple of kv heads: PKV_E_SHAPE
    assert lib.balloon_resize(m, 49) == -3                           # more than the pool has: PKV_E_NOMEM
    assert lib.balloon_resize(m, 20) == 20 and oracle.balloon_resize(om, 20) == 20
    assert gpu.pool_stats(second)["n_free"] == 28 and gpu.pool_stats(first)["n_free"] == 32
    ctx = np.array([700, 1, 16, 333, 0, 2047], dtype=np.int32)
    assert gpu.seq_reserve_batch(m, np.arange(6), ctx) == oracle.seq_reserve_batch(om, np.arange(6), ctx) > 0
    for s, c in enumerate(ctx):
        if c:
            kv = gen.seq_kv((61, s), int(c), 8, 128, 0, 16)
            assert gpu.kv_write(m, s, 0, kv["k"], kv["v"]) == c and oracle.kv_write(om, s, 0, kv["k"], kv["v"]) == c
    assert np.array_equal(gpu.pool_export_state(second), oracle.pool_export_state(o_second))
    assert np.array_equal(gpu.pool_export_state(first), oracle.pool_export_state(o_first))
    q = gen.queries((61, 99), 6, 32, 128)
    qd = t.from_numpy(q.view(np.int16)).cuda()
    cd = t.from_numpy(ctx).cuda()
    out = t.full((6, 32, 128), float("nan"), dtype=t.float32, device="cuda")
    p = lambda x: C.c_void_p(x.data_ptr())
    assert lib.decode_attention(m, p(qd), None, p(cd), p(out)) == -1       # no batch shape yet: PKV_E_ARG
    assert lib.model_set_batch(m, 6, 0) == 0
    assert lib.decode_attention(m, p(qd), None, p(cd), p(out)) == 0        # the library's own table
    t.cuda.synchronize()
    rc, ref = oracle.decode_attention(om, q, ctx)
    assert rc == 0 and row_rel_err(out.cpu().numpy(), ref) <= TOL[0]
    # the same through a caller's table: rows reversed, a stride of the caller's choosing
    rows = oracle.block_table_rows(om, 6)[::-1, :130].copy()
    bt = t.from_numpy(rows).cuda()
    qr, cr = t.from_numpy(q[::-1].copy().view(np.int16)).cuda(), t.from_numpy(ctx[::-1].copy()).cuda()
    out2 = t.full((6, 32, 128), float("nan"), dtype=t.float32, device="cuda")
    assert lib.model_set_batch(m, 6, 130) == 0
    assert lib.decode_attention(m, p(qr), p(bt), p(cr), p(out2)) == 0
    t.cuda.synchronize()
    assert row_rel_err(out2.cpu().numpy(), ref[::-1]) <= TOL[0]
    assert gpu.device_errors() == 0
    # a pool with a model in it cannot go; the other one can, and the next model_register still finds `second`
    assert lib.pool_destroy(second) == -7 and lib.pool_destroy(first) == 0
    m2 = lib.model_register(8, 2, 64, 0)
    assert m2 >= 0 and lib.balloon_resize(m2, 3) == 3 and gpu.pool_stats(second)["n_free"] == 25
    assert lib.balloon_resize(m2, 0) == 0 and lib.model_unregister(m2) == 0
    for s in range(6):
        gpu.seq_release(m, s)
        oracle.seq_release(om, s)
    assert lib.balloon_resize(m, 0) == 0 and lib.model_unregister(m) == 0 and lib.pool_destroy(second) == 0
    assert lib.model_register(8, 2, 64, 0) == -2                      # no pool left: PKV_E_HANDLE
    oracle.balloon_resize(om, 0), oracle.model_unregister(om), oracle.pool_destroy(o_second), oracle.pool_destroy(o_first)
