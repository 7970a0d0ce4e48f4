"""Pins for the oracle's multi-layer blocks (CPU only).

Paper Sec. 4.2, D3, first optimisation: the K and V of all L layers of a token block sit
side by side, so one block id, one slot and one block-table row serve every layer and a
reserve is one allocation instead of 2L.  What that fixes, and what is checked here
against something other than the oracle's own layer arithmetic:
  * geometry: a block is L times one layer's bytes (closed form typed out below), the
    layer parts of all blocks of a frame tile it without overlap (brute force over bytes);
  * bookkeeping does not know about layers: it equals that of a one-layer model whose
    blocks have the same size (L times the kv heads), word for word;
  * every layer is a cache of its own: what was written to a layer is read back
    unchanged after the other layers were written, and attention on a layer equals the
    library attention routine on that layer's logical tensors.
"""
import numpy as np
import pytest
import torch

from workloads import gen
from tests.state_image import parse
from tests.test_oracle_attention import dense_reference, decode_kv

BF16, E4M3 = 0, 1
MiB = 1 << 20


def layer_bytes_by_hand(T, hkv, d, dtype):
    return 2 * T * hkv * d * 2 if dtype == BF16 else 2 * T * hkv * d + 128


@pytest.mark.parametrize("hkv,d,dtype,L", [(2, 16, BF16, 3), (8, 128, BF16, 4), (4, 64, E4M3, 5), (1, 8, E4M3, 2)])
def test_block_geometry(oracle, hkv, d, dtype, L):
    o, T, frame = oracle, 16, 2 * MiB
    pool = o.pool_create(8 * MiB, T, frame)
    m = o.model_register(pool, hkv * 2, hkv, d, dtype, 4, 8, n_layers=L)
    assert m >= 0 and o.lib.orc_model_layers(m) == L
    lb = layer_bytes_by_hand(T, hkv, d, dtype)
    assert o.block_bytes(m) == L * lb
    slots = o.slots(m)
    assert slots == frame // (L * lb)
    # every (block, layer) part of the first two frames: inside its frame, no byte shared
    taken = np.zeros(2 * frame, dtype=np.uint8)
    n_blocks = min(2 * slots, 96)
    ids = list(range(min(slots, 48))) + list(range(slots, slots + n_blocks - min(slots, 48)))
    for layer in range(L):
        assert o.set_layer(m, layer) == 0
        for b in ids:
            a = o.block_address(m, b)
            f = b // slots
            assert f * frame <= a and a + lb <= (f + 1) * frame
            assert not taken[a:a + lb].any()
            taken[a:a + lb] = 1
    # consecutive layers of one block are lb apart
    o.set_layer(m, 0)
    a0 = o.block_address(m, 1)
    o.set_layer(m, L - 1)
    assert o.block_address(m, 1) - a0 == (L - 1) * lb
    assert o.set_layer(m, L) == -1 and o.set_layer(m, -1) == -1 and o.set_layer(99, 0) == -2
    assert o.model_unregister(m) == 0
    assert o.pool_destroy(pool) == 0


def test_refusals(oracle):
    o = oracle
    pool = o.pool_create(4 * MiB, 16, 64 << 10)
    assert o.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=0) == -1
    # 2 kv heads x 64 x bf16 -> 8 KiB per layer: 8 layers fill a 64 KiB frame, 9 do not fit
    m = o.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=8)
    assert m >= 0 and o.slots(m) == 1
    assert o.model_unregister(m) == 0
    assert o.model_register(pool, 8, 2, 64, BF16, 2, 4, n_layers=9) == -5
    assert o.pool_destroy(pool) == 0


def random_ops(o, m, rng, n_ops, max_seqs, max_tokens, log):
    ctx = [0] * max_seqs
    for _ in range(n_ops):
        kind = rng.integers(0, 4)
        if kind == 0:
            log.append(o.balloon_resize(m, int(rng.integers(0, 12))))
        elif kind in (1, 2):
            s = int(rng.integers(0, max_seqs))
            want = min(max_tokens, ctx[s] + int(rng.integers(1, 70)))
            rc = o.seq_reserve(m, s, want)
            log.append(rc)
            if rc >= 0:
                ctx[s] = want
        else:
            s = int(rng.integers(0, max_seqs))
            log.append(o.seq_release(m, s))
            ctx[s] = 0
    for s in range(max_seqs):
        o.seq_release(m, s)


@pytest.mark.parametrize("L", [2, 5])
def test_bookkeeping_equals_one_layer_model_of_same_block_size(oracle, L):
    """Reserve, release, inflate and deflate see block sizes only: an L-layer model and a
    one-layer model with L times the kv heads go through identical states."""
    o, T = oracle, 16
    images, logs = [], []
    for hq, hkv, layers in ((4, 2, L), (4 * L, 2 * L, 1)):
        pool = o.pool_create(2 * MiB, T, 64 << 10)           # 32 frames
        n = o.n_frames(pool)
        assert o.pool_seed_free_order(pool, gen.free_order(n, gen.generator(3))) == 0
        m = o.model_register(pool, hq, hkv, 32, BF16, 6, 24, n_layers=layers)
        assert m >= 0
        log, imgs = [], []
        rng = np.random.default_rng(11)
        for _ in range(6):
            random_ops_log = []
            random_ops(o, m, rng, 40, 6, 24 * T, random_ops_log)
            log.append(random_ops_log)
            st = parse(o.pool_export_state(pool))
            for mm in st["models"].values():                 # the shape words differ by construction
                mm.pop("q_heads"), mm.pop("kv_heads")
            imgs.append(st)
        images.append(imgs)
        logs.append(log)
        assert o.balloon_resize(m, 0) == 0 and o.model_unregister(m) == 0 and o.pool_destroy(pool) == 0
    assert logs[0] == logs[1]
    assert images[0] == images[1]
    assert any(r >= 0 for r in logs[0][0]) and any(r < 0 for lg in logs[0] for r in lg)


@pytest.mark.parametrize("hq,hkv,d,dtype", [(4, 2, 16, BF16), (8, 2, 64, E4M3)])
def test_every_layer_is_a_cache_of_its_own(oracle, hq, hkv, d, dtype):
    o, T, L = oracle, 16, 3
    ctx = [1, 16, 17, 45]
    pool = o.pool_create(16 * MiB, T, 256 << 10)
    assert o.pool_seed_free_order(pool, gen.free_order(o.n_frames(pool), gen.generator(5))) == 0
    m = o.model_register(pool, hq, hkv, d, dtype, len(ctx), 8, n_layers=L)
    assert o.balloon_resize(m, 8) == 8
    for upto in (16, 32, 48):                                 # blocks of the sequences interleave
        for s, c in enumerate(ctx):
            assert o.seq_reserve(m, s, min(c, upto)) >= 0
    kv = [[gen.seq_kv((21, layer, s), c, hkv, d, dtype, T, 0.0) for s, c in enumerate(ctx)] for layer in range(L)]
    for layer in (1, 0, 2):                                   # not in address order
        assert o.set_layer(m, layer) == 0
        for s, c in enumerate(ctx):
            x = kv[layer][s]
            assert o.kv_write(m, s, 0, x["k"], x["v"], x["k_scale"], x["v_scale"]) == c
    q = gen.queries((21, 99), len(ctx), hq, d)
    ctx_a = np.array(ctx, dtype=np.int32)
    outs = []
    for layer in range(L):
        assert o.set_layer(m, layer) == 0
        for s, c in enumerate(ctx):                           # nothing of another layer leaked in
            rc, k, v, ks, vs = o.kv_read(m, s, 0, c)
            assert rc == c
            assert np.array_equal(k, kv[layer][s]["k"]) and np.array_equal(v, kv[layer][s]["v"])
            if dtype == E4M3:
                blk = np.arange(c) // T
                assert np.array_equal(ks, kv[layer][s]["k_scale"][blk]) and np.array_equal(vs, kv[layer][s]["v_scale"][blk])
        rc, out = o.decode_attention(m, q, ctx_a)
        assert rc == 0
        for s, c in enumerate(ctx):
            kk, vv = decode_kv(kv[layer][s], dtype, T)
            ref = dense_reference(q[s], kk, vv, hq // hkv)
            assert np.allclose(out[s], ref, rtol=2e-7, atol=1e-7), (layer, s)
        outs.append(out)
    assert not np.allclose(outs[0], outs[1]) and not np.allclose(outs[1], outs[2])
    # a prefill chunk on layer 2: the last 5 tokens of the longest sequence as queries
    o.set_layer(m, 2)
    C, s = 5, 3
    qc = gen.queries((21, 77), C, hq, d)
    q_lens = np.array([0, 0, 0, C], dtype=np.int32)
    rc, po = o.prefill_attention(m, qc, q_lens, ctx_a)
    assert rc == 0
    kk, vv = decode_kv(kv[2][s], dtype, T)
    for i in range(C):
        upto = ctx[s] - C + i + 1
        ref = dense_reference(qc[i], kk[:upto], vv[:upto], hq // hkv)
        assert np.allclose(po[i], ref, rtol=2e-7, atol=1e-7), i
    # an appended token lands in the current layer only
    o.set_layer(m, 1)
    assert o.seq_reserve(m, 0, 2) >= 0
    new = gen.randn_bf16((len(ctx), hkv, d), gen.generator(8))
    before = [o.kv_read(m, 0, 0, 1)[1:3]]
    assert o.kv_append(m, new[:1], new[:1], np.array([2], dtype=np.int32)) >= 0
    for layer in (0, 2):
        o.set_layer(m, layer)
        rc, k, v, _, _ = o.kv_read(m, 0, 0, 1)
        assert np.array_equal(k, kv[layer][0]["k"]) and np.array_equal(v, kv[layer][0]["v"])
    o.set_layer(m, 1)
    rc, k, v, ks, vs = o.kv_read(m, 0, 1, 1)
    assert rc == 1
    if dtype == BF16:
        assert np.array_equal(k[0], new[0]) and np.array_equal(v[0], new[0])
    else:
        dec = torch.from_numpy(k).view(torch.float8_e4m3fn).to(torch.float64).numpy()[0] * ks[0][:, None]
        assert np.allclose(dec, gen.bf16_bits_to_f64(new[0]), rtol=0.07, atol=float(ks.max()) * 2 ** -9 * 448 / 8)
    del before
    for s in range(len(ctx)):
        o.seq_release(m, s)
    assert o.balloon_resize(m, 0) == 0 and o.model_unregister(m) == 0 and o.pool_destroy(pool) == 0
