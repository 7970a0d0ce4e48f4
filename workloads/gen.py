"""Seeded synthetic inputs shared by the oracle-side and GPU-side harness code.

Nothing here computes any part of the method (no attention, no page-pool
bookkeeping): it only draws random numbers with fixed seeds and packs them
into the element formats the two libraries accept.  bf16 values travel as uint16
bit patterns, e4m3 values as uint8 codes plus fp32 scales.

The inputs stand in for the paper's production traces and model zoo, which are
not available: shapes follow the KV shapes the paper quotes (8 KV heads, head
dim 128 or 64), context lengths follow a capped lognormal, and the on/off
activity of co-located models follows a two-state Markov chain whose stationary
active fraction (0.4) lies inside the band the paper's trace analysis reports
(23-50 % of models active at a time).
"""
import math

import numpy as np
import torch

BF16, E4M3 = 0, 1
E4M3_MAX = 448.0


def generator(*key):
    """CPU generator seeded from a tuple of small integers."""
    seed = 0x9E3779B97F4A7C15
    for k in key:
        seed = (seed * 6364136223846793005 + int(k) + 1442695040888963407) % (1 << 63)
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


def to_bf16_bits(x):
    """fp32 tensor -> uint16 numpy array of bf16 bit patterns (round to nearest even)."""
    return x.to(torch.bfloat16).contiguous().view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f64(bits):
    """uint16 bf16 bit patterns -> float64 numpy (exact)."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16
    return u.view(np.float32).astype(np.float64)


def randn_bf16(shape, gen):
    return to_bf16_bits(torch.randn(shape, generator=gen, dtype=torch.float32))


def free_order(n_frames, gen):
    """Seeded permutation of the frame ids: the order in which pops hand frames out."""
    return torch.randperm(n_frames, generator=gen).numpy().astype(np.uint32)


def ctx_uniform(n, lo, hi, gen):
    return torch.randint(lo, hi + 1, (n,), generator=gen).numpy().astype(np.int32)


def ctx_lognormal(n, median, sigma, cap, gen):
    z = torch.randn(n, generator=gen, dtype=torch.float64)
    c = torch.round(torch.exp(math.log(median) + sigma * z)).clamp(1, cap)
    return c.numpy().astype(np.int32)


def quantise_e4m3(x, page_tokens):
    """Harness-side quantiser for e4m3 KV with one fp32 scale per (block, kv head).

    x: fp32 tensor [n_tok][Hkv][D] holding one sequence from token 0.
    Returns (codes uint8 [n_tok][Hkv][D], scale fp32 [n_blocks][Hkv]).
    scale = amax / 448 over the block's tokens (1 when the block is all zero);
    codes = round-to-nearest-even of x / scale, saturated at +-448.
    """
    n_tok, hkv, d = x.shape
    n_blk = (n_tok + page_tokens - 1) // page_tokens
    pad = n_blk * page_tokens - n_tok
    xp = torch.cat([x, torch.zeros(pad, hkv, d)]) if pad else x
    xb = xp.view(n_blk, page_tokens, hkv, d)
    amax = xb.abs().amax(dim=(1, 3))                       # [n_blk][Hkv]
    scale = torch.where(amax > 0, amax / E4M3_MAX, torch.ones_like(amax)).to(torch.float32)
    y = (xb / scale[:, None, :, None]).clamp(-E4M3_MAX, E4M3_MAX)
    codes = y.to(torch.float8_e4m3fn).view(torch.uint8).view(n_blk * page_tokens, hkv, d)[:n_tok]
    return codes.contiguous().numpy(), scale.contiguous().numpy()


def seq_kv(key, n_tok, kv_heads, head_dim, dtype, page_tokens, peak_frac=0.0, peak_scale=8.0):
    """Logical K and V of one sequence, reproducible from `key` alone.

    Returns dict(k, v[, k_scale, v_scale]).  With peak_frac > 0 a Bernoulli
    fraction of (token, kv head) key rows is multiplied by peak_scale (a power
    of two, exact in bf16) to create sharp softmax peaks.
    """
    g = generator(*key)
    k = torch.randn((n_tok, kv_heads, head_dim), generator=g, dtype=torch.float32)
    v = torch.randn((n_tok, kv_heads, head_dim), generator=g, dtype=torch.float32)
    if peak_frac > 0.0:
        hit = torch.rand((n_tok, kv_heads), generator=g) < peak_frac
        k = torch.where(hit[:, :, None], k * peak_scale, k)
    if dtype == BF16:
        return {"k": to_bf16_bits(k), "v": to_bf16_bits(v), "k_scale": None, "v_scale": None}
    kc, ks = quantise_e4m3(k, page_tokens)
    vc, vs = quantise_e4m3(v, page_tokens)
    return {"k": kc, "v": vc, "k_scale": ks, "v_scale": vs}


def queries(key, batch, q_heads, head_dim):
    return randn_bf16((batch, q_heads, head_dim), generator(*key))


def markov_activity(n_models, n_steps, p_on, p_off, gen):
    """bool [n_steps][n_models]: two-state chain per model, initial state from the
    stationary distribution p_on / (p_on + p_off)."""
    u = torch.rand((n_steps, n_models), generator=gen).numpy()
    act = np.zeros((n_steps, n_models), dtype=bool)
    act[0] = u[0] < p_on / (p_on + p_off)
    for t in range(1, n_steps):
        act[t] = np.where(act[t - 1], u[t] >= p_off, u[t] < p_on)
    return act
