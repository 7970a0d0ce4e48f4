"""Pins for the oracle's decode attention (CPU only).

The oracle is the definition softmax(q K^T / sqrt(D)) V evaluated through a block
table (paper: Background, "KV cache and PagedAttention").  Each test below fixes
it to something other than itself: a library attention routine on gathered dense
tensors, closed forms, and invariants.  A dropped scale, a wrong kv-head map, a
K/V swap, a wrong in-block index or a missing tail mask fails at least one.
"""
import math

import numpy as np
import pytest
import torch

from workloads import gen

BF16, E4M3 = 0, 1


def dense_reference(q_bits, k, v, g):
    """Library routine on contiguous fp64 tensors: q [Hq][D], k/v [L][Hkv][D]."""
    q = torch.from_numpy(gen.bf16_bits_to_f64(q_bits))                  # [Hq][D]
    kk = torch.from_numpy(k).repeat_interleave(g, dim=1).permute(1, 0, 2)  # [Hq][L][D]
    vv = torch.from_numpy(v).repeat_interleave(g, dim=1).permute(1, 0, 2)
    o = torch.nn.functional.scaled_dot_product_attention(q[:, None, :], kk, vv)
    return o[:, 0, :].numpy()


def decode_kv(kv, dtype, T):
    """Logical fp64 K, V [L][Hkv][D] from what the generator produced."""
    if dtype == BF16:
        return gen.bf16_bits_to_f64(kv["k"]), gen.bf16_bits_to_f64(kv["v"])
    out = []
    for c, s in ((kv["k"], kv["k_scale"]), (kv["v"], kv["v_scale"])):
        x = torch.from_numpy(c).view(torch.float8_e4m3fn).to(torch.float64).numpy()
        n = x.shape[0]
        out.append(x * np.repeat(s.astype(np.float64), T, axis=0)[:n, :, None])
    return out


class Setup:
    def __init__(self, o, hq, hkv, d, dtype, ctx_lens, T=16, frame_bytes=None, seed=7, perm_seed=1,
                 max_blocks=64, pool_bytes=64 << 20, peak=0.0):
        self.o, self.T, self.hq, self.hkv, self.d, self.dtype = o, T, hq, hkv, d, dtype
        self.pool = o.pool_create(pool_bytes, T, frame_bytes or (2 << 20))
        assert self.pool >= 0
        n = o.n_frames(self.pool)
        assert o.pool_seed_free_order(self.pool, gen.free_order(n, gen.generator(perm_seed))) == 0
        self.m = o.model_register(self.pool, hq, hkv, d, dtype, len(ctx_lens), max_blocks)
        assert self.m >= 0
        blocks = sum((c + T - 1) // T for c in ctx_lens)
        slots = o.slots(self.m)
        assert o.balloon_resize(self.m, (blocks + slots - 1) // slots + 1) > 0
        self.ctx = np.array(ctx_lens, dtype=np.int32)
        self.kv = []
        # grow the sequences in turns so their blocks interleave inside frames
        for upto in range(T * 2, max(ctx_lens) + T * 2, T * 2):
            for s, c in enumerate(ctx_lens):
                assert o.seq_reserve(self.m, s, min(c, upto)) >= 0
        for s, c in enumerate(ctx_lens):
            kv = gen.seq_kv((seed, s), c, hkv, d, dtype, T, peak)
            self.kv.append(kv)
            if c:
                assert o.kv_write(self.m, s, 0, kv["k"], kv["v"], kv["k_scale"], kv["v_scale"]) == c
        self.q = gen.queries((seed, 99), len(ctx_lens), hq, d)

    def run(self):
        rc, out = self.o.decode_attention(self.m, self.q, self.ctx)
        assert rc == 0
        return out

    def close(self):
        for s in range(len(self.ctx)):
            self.o.seq_release(self.m, s)
        assert self.o.balloon_resize(self.m, 0) == 0
        assert self.o.model_unregister(self.m) == 0
        assert self.o.pool_destroy(self.pool) == 0


@pytest.mark.parametrize("hq,hkv,d,dtype", [(4, 2, 8, BF16), (8, 2, 64, BF16), (6, 3, 16, BF16),
                                            (8, 1, 128, BF16), (4, 2, 64, E4M3), (8, 4, 128, E4M3)])
def test_matches_dense_library_attention(oracle, hq, hkv, d, dtype):
    ctx = [1, 15, 16, 17, 33, 40]
    s = Setup(oracle, hq, hkv, d, dtype, ctx)
    out = s.run()
    for i, L in enumerate(ctx):
        k, v = decode_kv(s.kv[i], dtype, s.T)
        ref = dense_reference(s.q[i], k, v, hq // hkv)
        assert np.allclose(out[i], ref, rtol=2e-7, atol=1e-7), (i, L, np.abs(out[i] - ref).max())
    s.close()


def test_softmax_rows_sum_to_one(oracle):
    ctx = [5, 31, 64]
    s = Setup(oracle, 4, 2, 32, BF16, ctx)
    rows = oracle.block_table_rows(s.m, len(ctx))
    for i, L in enumerate(ctx):
        for h in range(4):
            rc, p = oracle.attention_probs(s.m, s.q[i, h], rows[i], L, h)
            assert rc == 0
            assert abs(p.sum() - 1.0) < 1e-14 and (p >= 0).all()
            # the probabilities reproduce the output row through the logical V
            _, v = decode_kv(s.kv[i], BF16, s.T)
            assert np.allclose(p @ v[:, h // 2, :], s.run()[i, h], rtol=1e-6, atol=1e-7)
    s.close()


def test_uniform_keys_give_mean_of_v(oracle):
    """All keys equal => every logit equal => out = mean_t v[t] (closed form)."""
    T, L, hkv, d = 16, 37, 2, 16
    s = Setup(oracle, 4, hkv, d, BF16, [L])
    k1 = gen.randn_bf16((1, hkv, d), gen.generator(5))
    k = np.repeat(k1, L, axis=0)
    assert oracle.kv_write(s.m, 0, 0, k, s.kv[0]["v"]) == L
    out = s.run()
    v = gen.bf16_bits_to_f64(s.kv[0]["v"])
    for h in range(4):
        assert np.allclose(out[0, h], v[:, h // 2, :].mean(axis=0), rtol=1e-6, atol=1e-7)
    s.close()


def test_single_token_returns_its_value_row(oracle):
    s = Setup(oracle, 4, 2, 16, BF16, [1])
    out = s.run()
    v = gen.bf16_bits_to_f64(s.kv[0]["v"])
    for h in range(4):
        assert np.array_equal(out[0, h], v[0, h // 2].astype(np.float32))
    s.close()


def test_dominant_key_selects_its_value(oracle):
    """One key aligned with q and far above the rest: out -> that token's V row,
    and nothing overflows (max subtraction)."""
    L, hkv, d, hit = 50, 1, 64, 23
    s = Setup(oracle, 2, hkv, d, BF16, [L])
    q = gen.bf16_bits_to_f64(s.q[0, 0])
    k = gen.bf16_bits_to_f64(s.kv[0]["k"])
    k[hit, 0] = q * 256.0                     # logit ~ 256 |q|^2 / 8 ~ 2000: exp() alone would overflow
    kb = gen.to_bf16_bits(torch.from_numpy(k).float())
    assert oracle.kv_write(s.m, 0, 0, kb, s.kv[0]["v"]) == L
    out = s.run()
    v = gen.bf16_bits_to_f64(s.kv[0]["v"])
    assert np.isfinite(out).all()
    assert np.abs(out[0, 0] - v[hit, 0]).max() < 1e-6
    s.close()


def test_physical_placement_does_not_change_the_result(oracle):
    ctx = [40, 7, 100]
    a = Setup(oracle, 8, 2, 32, BF16, ctx, perm_seed=1)
    out_a = a.run()
    rows_a = oracle.block_table_rows(a.m, 3)
    a.close()
    b = Setup(oracle, 8, 2, 32, BF16, ctx, perm_seed=2, frame_bytes=64 << 10)
    out_b = b.run()
    rows_b = oracle.block_table_rows(b.m, 3)
    b.close()
    assert not np.array_equal(rows_a[:, :3], rows_b[:, :3])   # really placed elsewhere
    assert np.array_equal(out_a, out_b)                        # bit-identical: sums run in logical order


def test_power_of_two_rescaling_is_exact(oracle):
    """K * c with q / c (c a power of two) leaves every product unchanged."""
    ctx = [29]
    s = Setup(oracle, 4, 2, 16, BF16, ctx)
    base = s.run()
    k4 = gen.to_bf16_bits(torch.from_numpy(gen.bf16_bits_to_f64(s.kv[0]["k"]) * 4.0).float())
    s.q = gen.to_bf16_bits(torch.from_numpy(gen.bf16_bits_to_f64(s.q) / 4.0).float())
    assert oracle.kv_write(s.m, 0, 0, k4, s.kv[0]["v"]) == ctx[0]
    assert np.array_equal(s.run(), base)
    s.close()


def test_scale_is_one_over_sqrt_d(oracle):
    """Two tokens, k0 = 0 and k1 = c*q: p1/p0 = exp(c |q|^2 / sqrt(D)), so out is a
    known blend of v0 and v1; a missing or wrong scale changes the blend."""
    d = 64
    s = Setup(oracle, 1, 1, d, BF16, [2])
    q = np.zeros(d); q[:4] = [1.0, -2.0, 0.5, 1.5]            # exact in bf16
    s.q = gen.to_bf16_bits(torch.tensor(q).float().view(1, 1, d))
    k = np.zeros((2, 1, d)); k[1, 0] = q * 2.0
    v = gen.bf16_bits_to_f64(s.kv[0]["v"])
    assert oracle.kv_write(s.m, 0, 0, gen.to_bf16_bits(torch.from_numpy(k).float()), s.kv[0]["v"]) == 2
    z1 = 2.0 * float(q @ q) / math.sqrt(d)
    p1 = 1.0 / (1.0 + math.exp(-z1))
    want = (1 - p1) * v[0, 0] + p1 * v[1, 0]
    assert np.allclose(s.run()[0, 0], want, rtol=1e-6, atol=1e-7)
    s.close()


def test_tail_slots_are_never_read(oracle):
    """Tokens past ctx_len in the last block must not influence the result:
    poison them (NaN keys and values) and compare with the clean run."""
    L, T = 21, 16
    s = Setup(oracle, 4, 2, 16, BF16, [L])
    clean = s.run()
    assert oracle.seq_reserve(s.m, 0, 2 * T) == 0          # same two blocks
    nan = np.full((2 * T - L, 2, 16), 0x7FC0, dtype=np.uint16)
    assert oracle.kv_write(s.m, 0, L, nan, nan) == 2 * T - L
    assert np.array_equal(s.run(), clean)
    s.close()


def test_zero_length_sequence_gives_zero_row(oracle):
    s = Setup(oracle, 4, 2, 16, BF16, [0, 9])
    out = s.run()
    assert np.array_equal(out[0], np.zeros((4, 16), dtype=np.float32))
    assert np.abs(out[1]).max() > 0
    s.close()


def test_kv_head_mapping_is_contiguous_groups(oracle):
    """Make kv head 1's values a constant the other heads lack: exactly the query
    heads g..2g-1 must see it."""
    hq, hkv, d, L = 6, 3, 8, 10
    s = Setup(oracle, hq, hkv, d, BF16, [L])
    v = gen.bf16_bits_to_f64(s.kv[0]["v"]) * 0.0
    v[:, 1, :] = 3.0
    assert oracle.kv_write(s.m, 0, 0, s.kv[0]["k"], gen.to_bf16_bits(torch.from_numpy(v).float())) == L
    out = s.run()[0]
    assert np.allclose(out[[2, 3]], 3.0) and np.allclose(out[[0, 1, 4, 5]], 0.0)
    s.close()


def test_external_block_table_equals_own_rows(oracle):
    ctx = [33, 5]
    s = Setup(oracle, 4, 2, 16, BF16, ctx)
    rows = oracle.block_table_rows(s.m, 2)
    rc, out = oracle.decode_attention(s.m, s.q, s.ctx, rows[:, :8])
    assert rc == 0 and np.array_equal(out, s.run())
    rows[0, 0] = 10**8
    rc, _ = oracle.decode_attention(s.m, s.q, s.ctx, rows[:, :8])
    assert rc == -6
    s.close()
