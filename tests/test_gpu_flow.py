"""One serving loop over two co-located models on one pool, step for step on the HIP library and
on the oracle: a balloon per model, prefill in chunks (chunk append + causal attention), then
decode steps (row growth, token append, attention of both models in one launch) on every layer,
a burst of one model ending in the middle (release + deflate, the other model inflates into the
freed frames) and starting again.  Bookkeeping must agree bit for bit after every call that
changes it, caches bit for bit, attention within 2e-3 (bf16 cache) / 2e-2 (e4m3 cache).
"""
import numpy as np
import pytest
import torch

from parity import TOL, assert_same_state, row_rel_err
from workloads import gen

pytestmark = pytest.mark.gpu

BF16, E4M3 = 0, 1
#            q heads, kv heads, head dim, cache, layers, sequences
MODELS = [(32, 8, 128, BF16, 2, 3), (16, 4, 64, E4M3, 3, 4)]
PROMPT = [[70, 33, 150], [16, 200, 5, 90]]
CHUNK = 64


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


class Side:
    """One backend's handles."""

    def __init__(self, be, perm):
        self.be = be
        self.pool = be.pool_create(128 << 20, 16, 2 << 20)
        assert self.pool >= 0 and be.pool_seed_free_order(self.pool, perm) == 0
        self.m = [be.model_register(self.pool, hq, hkv, d, dt, nseq, 40, n_layers=L) for hq, hkv, d, dt, L, nseq in MODELS]
        assert min(self.m) >= 0


def both(sides, fn):
    res = [fn(s) for s in sides]
    assert res[0] == res[1], res
    return res[0]


def frames_for(mi, tokens):
    hq, hkv, d, dt, L, nseq = MODELS[mi]
    bb = L * (2 * 16 * hkv * d * (2 if dt == BF16 else 1) + (128 if dt == E4M3 else 0))
    slots = (2 << 20) // bb
    blocks = sum((t + 15) // 16 for t in tokens)
    return (blocks + slots - 1) // slots


def attend_decode(gpu, oracle, sides, ctx, step):
    """Every layer of both models: one grouped launch on the GPU, single calls on the oracle."""
    worst = 0.0
    for layer in range(max(m[4] for m in MODELS)):
        live = [mi for mi in range(2) if layer < MODELS[mi][4] and ctx[mi] is not None]
        if not live:
            continue
        for s in sides:
            for mi in live:
                assert s.be.set_layer(s.m[mi], layer) == 0
        qs = [gen.queries((91, step, layer, mi), MODELS[mi][5], MODELS[mi][0], MODELS[mi][2]) for mi in live]
        dq = [torch.from_numpy(q.view(np.int16)).cuda() for q in qs]
        dc = [torch.from_numpy(ctx[mi]).cuda() for mi in live]
        do = [torch.full(q.shape, float("nan"), dtype=torch.float32, device="cuda") for q in qs]
        assert gpu.decode_attention_multi_dev([sides[0].m[mi] for mi in live], dq, dc, do) == 0
        torch.cuda.synchronize()
        for k, mi in enumerate(live):
            rc, ref = oracle.decode_attention(sides[1].m[mi], qs[k], ctx[mi])
            assert rc == 0
            err = row_rel_err(do[k].cpu().numpy(), ref)
            assert err <= TOL[MODELS[mi][3]], (step, layer, mi, err)
            worst = max(worst, err)
    return worst


def same_cache(sides, mi, ctx):
    for layer in range(MODELS[mi][4]):
        for s in sides:
            s.be.set_layer(s.m[mi], layer)
        for seq, c in enumerate(ctx):
            if c == 0:
                continue
            a = sides[0].be.kv_read(sides[0].m[mi], seq, 0, int(c))
            b = sides[1].be.kv_read(sides[1].m[mi], seq, 0, int(c))
            assert a[0] == b[0] == c
            for x, y in zip(a[1:], b[1:]):
                assert (x is None and y is None) or np.array_equal(x, y), (mi, layer, seq)


def prefill(gpu, oracle, sides, mi, prompt, tag):
    """The prompts of model mi in chunks of CHUNK tokens, every layer: append, then attend."""
    hq, hkv, d, dt, L, nseq = MODELS[mi]
    done = np.zeros(nseq, dtype=np.int32)
    prompt = np.array(prompt, dtype=np.int32)
    while (done < prompt).any():
        ql = np.minimum(CHUNK, prompt - done).astype(np.int32)
        ctx = done + ql
        both(sides, lambda s: s.be.seq_reserve_batch(s.m[mi], list(range(nseq)), ctx))
        n = int(ql.sum())
        for layer in range(L):
            g = gen.generator(92, tag, mi, layer, int(done.sum()))
            kx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g))
            vx = gen.to_bf16_bits(torch.randn((n, hkv, d), generator=g))
            q = gen.queries((93, tag, mi, layer, int(done.sum())), n, hq, d)
            outs = []
            for s in sides:
                assert s.be.set_layer(s.m[mi], layer) == 0
                assert s.be.kv_append_chunk(s.m[mi], kx, vx, ql, ctx) == n
                rc, out = s.be.prefill_attention(s.m[mi], q, ql, ctx)
                assert rc == 0
                outs.append(out)
            assert row_rel_err(outs[0], outs[1]) <= TOL[dt], (mi, layer)
        done = ctx
    assert_same_state(sides[0].be, sides[1].be, sides[0].pool, sides[1].pool, f"after the prefill of model {mi}")
    same_cache(sides, mi, done)
    return done


def decode_steps(gpu, oracle, sides, ctx, n_steps, tag):
    for step in range(n_steps):
        for mi in range(2):
            if ctx[mi] is None:
                continue
            hq, hkv, d, dt, L, nseq = MODELS[mi]
            ctx[mi] = ctx[mi] + 1
            both(sides, lambda s: s.be.seq_reserve_batch(s.m[mi], list(range(nseq)), ctx[mi]))
            for layer in range(L):
                g = gen.generator(94, tag, step, mi, layer)
                kx = gen.to_bf16_bits(torch.randn((nseq, hkv, d), generator=g))
                vx = gen.to_bf16_bits(torch.randn((nseq, hkv, d), generator=g))
                for s in sides:
                    assert s.be.set_layer(s.m[mi], layer) == 0
                    assert s.be.kv_append(s.m[mi], kx, vx, ctx[mi]) == nseq
        attend_decode(gpu, oracle, sides, ctx, 100 * tag + step)
    assert_same_state(sides[0].be, sides[1].be, sides[0].pool, sides[1].pool, f"after decode steps {tag}")


def test_two_models_prefill_decode_burst(gpu, oracle):
    perm = gen.free_order((128 << 20) // (2 << 20), gen.generator(90))
    sides = [Side(gpu, perm), Side(oracle, perm)]
    try:
        grow = 24                                          # decode steps to come: room for them from the start
        for mi in range(2):
            want = frames_for(mi, [p + grow for p in PROMPT[mi]])
            assert both(sides, lambda s: s.be.balloon_resize(s.m[mi], want)) == want
        ctx = [prefill(gpu, oracle, sides, mi, PROMPT[mi], 0) for mi in range(2)]
        decode_steps(gpu, oracle, sides, ctx, 10, 0)
        for mi in range(2):
            same_cache(sides, mi, ctx[mi])

        # model 1's burst ends: its sequences are released and its frames go back to the pool ...
        for seq in range(MODELS[1][5]):
            both(sides, lambda s: s.be.seq_release(s.m[1], seq))
        assert both(sides, lambda s: s.be.balloon_resize(s.m[1], 0)) == 0
        ctx[1] = None
        # ... and model 0 takes some of them for longer contexts
        more = frames_for(0, [p + 200 for p in PROMPT[0]])
        assert both(sides, lambda s: s.be.balloon_resize(s.m[0], more)) == more
        assert_same_state(sides[0].be, sides[1].be, sides[0].pool, sides[1].pool, "after the hand-over")
        decode_steps(gpu, oracle, sides, ctx, 6, 1)

        # model 1 wakes up with new prompts while model 0 keeps decoding
        new_prompt = [40, 17, 64, 130]
        want = frames_for(1, [p + grow for p in new_prompt])
        assert both(sides, lambda s: s.be.balloon_resize(s.m[1], want)) == want
        ctx[1] = prefill(gpu, oracle, sides, 1, new_prompt, 1)
        decode_steps(gpu, oracle, sides, ctx, 8, 2)
        for mi in range(2):
            same_cache(sides, mi, ctx[mi])
        assert gpu.device_errors() == 0
    finally:
        for s in sides:
            for mi in range(2):
                for seq in range(MODELS[mi][5]):
                    s.be.seq_release(s.m[mi], seq)
                s.be.balloon_resize(s.m[mi], 0)
                s.be.model_unregister(s.m[mi])
            s.be.pool_destroy(s.pool)
