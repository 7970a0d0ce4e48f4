"""Pins for the oracle's write path (kv_append, kv_read, e4m3 encode) and its chunked
prefill attention (CPU only).

Each is fixed to something other than itself: the encoder to a library conversion, the
format's midpoints and the harness quantiser; the append rule to a hand-worked example
(tests/golden/kv_append_e4m3.txt) and to the closed form "scale = running maximum of
amax / 448"; prefill attention to a dense causal routine on tensors the test keeps itself,
and to decode attention in the special cases where both must coincide.
"""
import math
import os

import numpy as np
import pytest
import torch

from workloads import gen

BF16, E4M3 = 0, 1


# ------------------------------------------------------------------ encoder

def test_encode_round_trip_and_midpoints(oracle):
    vals = [oracle.e4m3_decode(c) for c in range(0x7F)]
    for c, v in enumerate(vals):
        assert oracle.e4m3_encode(v) == c
        assert oracle.e4m3_encode(-v) == (c | 0x80)
    for c in range(0x7E):
        lo, hi = vals[c], vals[c + 1]
        mid = (lo + hi) / 2                       # exact in fp32: both ends have <= 4 significant bits
        even = c if c % 2 == 0 else c + 1
        assert oracle.e4m3_encode(mid) == even, (c, mid)
        assert oracle.e4m3_encode(np.nextafter(np.float32(mid), np.float32(0))) == c
        assert oracle.e4m3_encode(np.nextafter(np.float32(mid), np.float32(1e9))) == c + 1
    assert oracle.e4m3_encode(448.0) == 0x7E and oracle.e4m3_encode(463.9) == 0x7E
    assert oracle.e4m3_encode(1e30) == 0x7E and oracle.e4m3_encode(-500.0) == 0xFE
    assert oracle.e4m3_encode(float("inf")) == 0x7E and oracle.e4m3_encode(float("nan")) == 0x7F
    assert oracle.e4m3_encode(0.0) == 0x00 and oracle.e4m3_encode(-0.0) == 0x80


def test_encode_matches_library_conversion(oracle):
    g = gen.generator(31, 1)
    y = torch.cat([torch.randn(4000, generator=g) * 100, torch.randn(2000, generator=g) * 0.02,
                   torch.empty(2000).uniform_(-448, 448, generator=g)]).clamp(-448, 448)
    lib = y.to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    for yi, ci in zip(y.tolist(), lib.tolist()):
        assert oracle.e4m3_encode(yi) == ci, (yi, ci)


# ------------------------------------------------------------------ append

def make(o, hq, hkv, d, dtype, T, n_seq, max_blocks=16, pool_bytes=1 << 20, frame_bytes=None):
    block = 2 * T * hkv * d * (2 if dtype == BF16 else 1) + (128 if dtype == E4M3 else 0)
    pool = o.pool_create(pool_bytes, T, frame_bytes or 4 * block)
    m = o.model_register(pool, hq, hkv, d, dtype, n_seq, max_blocks)
    assert pool >= 0 and m >= 0
    assert o.balloon_resize(m, o.n_frames(pool)) == o.n_frames(pool)
    return pool, m


def drop(o, pool, m, n_seq):
    for s in range(n_seq):
        o.seq_release(m, s)
    assert o.balloon_resize(m, 0) == 0 and o.model_unregister(m) == 0 and o.pool_destroy(pool) == 0


def parse_golden():
    path = os.path.join(os.path.dirname(__file__), "golden", "kv_append_e4m3.txt")
    steps, cur = [], None
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        if line.startswith("append"):
            head, rest = line.split("k:")
            ks, vs = rest.split("v:")
            cur = {"ctx": int(head.split()[1]), "k": [float(x) for x in ks.split()], "v": [float(x) for x in vs.split()],
                   "rows": []}
            steps.append(cur)
        elif line.startswith("expect"):
            _, first, n = line.split()
            cur["first"], cur["n"] = int(first), int(n)
        else:
            kc, ksc, vc, vsc = [x.strip() for x in line.split("|")]
            frac = lambda t: np.float32(np.float32(float(t.split("/")[0])) / np.float32(float(t.split("/")[1])))
            cur["rows"].append(([int(x, 16) for x in kc.split()], frac(ksc), [int(x, 16) for x in vc.split()], frac(vsc)))
    return steps


def test_append_e4m3_worked_example(oracle):
    o = oracle
    pool, m = make(o, 1, 1, 8, E4M3, 4, 1)
    steps = parse_golden()
    assert len(steps) == 5
    for st in steps:
        assert o.seq_reserve(m, 0, st["ctx"]) >= 0
        k = gen.to_bf16_bits(torch.tensor(st["k"]).view(1, 1, 8))
        v = gen.to_bf16_bits(torch.tensor(st["v"]).view(1, 1, 8))
        assert o.kv_append(m, k, v, [st["ctx"]]) == 1
        rc, kk, vv, ks, vs = o.kv_read(m, 0, st["first"], st["n"])
        assert rc == st["n"] and len(st["rows"]) == st["n"]
        for t, (kc, ksc, vc, vsc) in enumerate(st["rows"]):
            assert kk[t, 0].tolist() == kc, (st["ctx"], t, [hex(x) for x in kk[t, 0]])
            assert vv[t, 0].tolist() == vc, (st["ctx"], t, [hex(x) for x in vv[t, 0]])
            assert ks[t, 0] == ksc and vs[t, 0] == vsc, (st["ctx"], t, ks[t, 0], vs[t, 0])
    drop(o, pool, m, 1)


def test_append_bf16_is_a_copy_and_agrees_with_bulk_write(oracle):
    o = oracle
    T, hq, hkv, d, L = 4, 4, 2, 8, 11
    pool, m = make(o, hq, hkv, d, BF16, T, 2)
    kv = gen.seq_kv((5, 0), L, hkv, d, BF16, T)
    for t in range(L):
        for s in range(2):
            assert o.seq_reserve(m, s, t + 1) >= 0
        assert o.kv_append(m, np.stack([kv["k"][t]] * 2), np.stack([kv["v"][t]] * 2), [t + 1, t + 1]) == 2
    rc, k, v, _, _ = o.kv_read(m, 1, 0, L)
    assert rc == L and np.array_equal(k, kv["k"]) and np.array_equal(v, kv["v"])
    q = gen.queries((5, 9), 2, hq, d)
    rc, a = o.decode_attention(m, q, [L, L])
    assert o.kv_write(m, 0, 0, kv["k"], kv["v"]) == L          # the same tokens through the bulk path
    rc2, b = o.decode_attention(m, q, [L, L])
    assert rc == 0 and rc2 == 0 and np.array_equal(a, b)
    assert o.kv_append(m, kv["k"][:2], kv["v"][:2], [0, 3]) < 0            # ctx_len 0 has no last token
    assert o.kv_append(m, kv["k"][:2], kv["v"][:2], [3, L + T + 1]) < 0   # beyond what the row holds
    drop(o, pool, m, 2)


def test_append_e4m3_scale_is_running_maximum_and_error_is_bounded(oracle):
    o = oracle
    T, hq, hkv, d, L = 8, 4, 2, 16, 29
    pool, m = make(o, hq, hkv, d, E4M3, T, 1)
    g = gen.generator(77)
    x = torch.randn((L, 2, hkv, d), generator=g) * torch.rand((L, 2, hkv, 1), generator=g) * 4
    x[5] = 0.0
    xb = x.to(torch.bfloat16)
    for t in range(L):
        assert o.seq_reserve(m, 0, t + 1) >= 0
        assert o.kv_append(m, gen.to_bf16_bits(xb[t, 0:1].float()), gen.to_bf16_bits(xb[t, 1:2].float()), [t + 1]) == 1
        rc, k, v, ks, vs = o.kv_read(m, 0, 0, t + 1)
        b0 = (t // T) * T
        for which, codes, sc in ((0, k, ks), (1, v, vs)):
            blk = xb[b0:t + 1, which].float()                                   # tokens of the current block
            amax = blk.abs().amax(dim=(0, 2)).numpy()                             # [Hkv]
            want = np.where(amax > 0, (amax.astype(np.float32) / np.float32(448)), np.float32(1)).astype(np.float32)
            assert np.array_equal(sc[t], want), (t, which, sc[t], want)
            deq = torch.from_numpy(codes[b0:t + 1].copy()).view(torch.float8_e4m3fn).float().numpy() * sc[t][None, :, None]
            step = np.maximum(np.abs(blk.numpy()), sc[t][None, :, None] * 2.0 ** -6) * 2.0 ** -3
            # half a step from the final encode plus at most one step per earlier re-encode is a loose
            # but sufficient bound: what matters is that nothing is off by a binade, a sign or a slot
            assert np.all(np.abs(deq - blk.numpy()) <= 2.5 * step + 1e-12), (t, which)
    drop(o, pool, m, 1)


# ------------------------------------------------------------------ prefill

def causal_reference(qf, kf, vf, g, pos0):
    """Dense causal attention in long double on arrays the test holds itself.
    qf [C][Hq][D], kf/vf [L][Hkv][D]; query i sees t <= pos0 + i."""
    C, hq, d = qf.shape
    out = np.zeros((C, hq, d), dtype=np.longdouble)
    for i in range(C):
        n = pos0 + i + 1
        for h in range(hq):
            z = np.array([np.dot(qf[i, h].astype(np.longdouble), kf[t, h // g].astype(np.longdouble)) for t in range(n)])
            z = z / np.sqrt(np.longdouble(d))
            p = np.exp(z - z.max())
            p /= p.sum()
            out[i, h] = sum(p[t] * vf[t, h // g].astype(np.longdouble) for t in range(n))
    return out.astype(np.float64)


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_prefill_matches_dense_causal_attention(oracle, dtype):
    o = oracle
    T, hq, hkv, d = 4, 4, 2, 8
    ctx, qlen = [13, 6, 9], [5, 6, 1]
    pool, m = make(o, hq, hkv, d, dtype, T, 3)
    kvs = []
    for s, L in enumerate(ctx):
        assert o.seq_reserve(m, s, L) >= 0
        kv = gen.seq_kv((11, s), L, hkv, d, dtype, T)
        kvs.append(kv)
        assert o.kv_write(m, s, 0, kv["k"], kv["v"], kv.get("k_scale"), kv.get("v_scale")) == L
    q = gen.queries((11, 50), sum(qlen), hq, d)
    rc, out = o.prefill_attention(m, q, qlen, ctx)
    assert rc == 0
    r = 0
    for s, (L, C) in enumerate(zip(ctx, qlen)):
        kv = kvs[s]
        if dtype == BF16:
            kf, vf = gen.bf16_bits_to_f64(kv["k"]), gen.bf16_bits_to_f64(kv["v"])
        else:
            dec = lambda c, sc: torch.from_numpy(c).view(torch.float8_e4m3fn).to(torch.float64).numpy() * \
                np.repeat(sc.astype(np.float64), T, axis=0)[:c.shape[0], :, None]
            kf, vf = dec(kv["k"], kv["k_scale"]), dec(kv["v"], kv["v_scale"])
        ref = causal_reference(gen.bf16_bits_to_f64(q[r:r + C]), kf, vf, hq // hkv, L - C)
        assert np.max(np.abs(out[r:r + C] - ref)) <= 1e-6 * max(1.0, np.max(np.abs(ref)))
        if C == L:                                   # prefill from an empty cache: the first query sees token 0 only
            assert np.allclose(out[r], np.repeat(vf[0], hq // hkv, axis=0), rtol=0, atol=1e-7)
        r += C
    # the last query of every chunk is a decode step
    last = np.cumsum(qlen) - 1
    rc, dec_out = o.decode_attention(m, q[last], ctx)
    assert rc == 0 and np.array_equal(dec_out, out[last])
    # a chunk longer than the cache is refused
    assert o.prefill_attention(m, q, [4, 7, 1], ctx)[0] < 0
    drop(o, pool, m, 3)


@pytest.mark.parametrize("dtype", [BF16, E4M3])
def test_chunk_append_equals_token_by_token(oracle, dtype):
    """Two models on one pool get the same tokens, one in chunks, one a token at a time through
    kv_append (pinned above); a second sequence in the chunk calls checks the packing."""
    o = oracle
    T, hq, hkv, d = 4, 4, 2, 8
    block = 2 * T * hkv * d * (2 if dtype == BF16 else 1) + (128 if dtype == E4M3 else 0)
    pool = o.pool_create(1 << 20, T, 4 * block)
    ma = o.model_register(pool, hq, hkv, d, dtype, 2, 16)
    mb = o.model_register(pool, hq, hkv, d, dtype, 1, 16)
    mc = o.model_register(pool, hq, hkv, d, dtype, 1, 16)
    for m in (ma, mb, mc):
        assert o.balloon_resize(m, 16) == 16
    g = gen.generator(41, dtype)
    ctx = np.zeros(2, dtype=np.int32)
    for ql in ([3, 0], [6, 5], [1, 9], [0, 2]):
        ql = np.array(ql, dtype=np.int32)
        n = int(ql.sum())
        mag = torch.exp(torch.randn((n, 1, 1), generator=g))
        kx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        vx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g) * mag)
        new_ctx = ctx + ql
        for s in range(2):
            assert o.seq_reserve(ma, s, int(new_ctx[s])) >= 0
        assert o.seq_reserve(mb, 0, int(new_ctx[0])) >= 0 and o.seq_reserve(mc, 0, int(new_ctx[1])) >= 0
        assert o.kv_append_chunk(ma, kx, vx, ql, new_ctx) == n
        row = 0
        for s, m1 in ((0, mb), (1, mc)):                 # sequence s of the chunked model = the one sequence of m1
            for i in range(int(ql[s])):
                assert o.kv_append(m1, kx[row:row + 1], vx[row:row + 1], [int(ctx[s]) + i + 1]) == 1
                row += 1
        ctx = new_ctx
        for s, m1 in ((0, mb), (1, mc)):
            if ctx[s]:
                a, b = o.kv_read(ma, s, 0, int(ctx[s])), o.kv_read(m1, 0, 0, int(ctx[s]))
                assert np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
                if dtype == E4M3:
                    assert np.array_equal(a[3], b[3]) and np.array_equal(a[4], b[4])
    assert o.kv_append_chunk(ma, kx[:1], vx[:1], [1, 0], [0, 5]) < 0          # a chunk longer than the cache
    for m, n_seq in ((ma, 2), (mb, 1), (mc, 1)):
        for s in range(n_seq):
            o.seq_release(m, s)
        assert o.balloon_resize(m, 0) == 0 and o.model_unregister(m) == 0
    assert o.pool_destroy(pool) == 0
