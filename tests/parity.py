"""Helpers for the GPU-vs-oracle parity tests."""
import numpy as np

from state_image import check_invariants, parse
from workloads.scenarios import Runner

TOL = {0: 2e-3, 1: 2e-2}     # max relative error per KV dtype (bf16, e4m3)


def row_rel_err(gpu, orc):
    """Per output row r = (sequence, q head): ||gpu_r - orc_r||_inf / max(||orc_r||_inf, 1e-6);
    returns the maximum over rows.  NaN or Inf anywhere fails."""
    assert gpu.shape == orc.shape
    assert np.isfinite(gpu).all(), "non-finite value in GPU output"
    assert np.isfinite(orc).all(), "non-finite value in oracle output"
    num = np.abs(gpu.astype(np.float64) - orc.astype(np.float64)).max(axis=-1)
    den = np.maximum(np.abs(orc.astype(np.float64)).max(axis=-1), 1e-6)
    return float((num / den).max()) if num.size else 0.0


def elementwise_rel_err(gpu, orc):
    """Secondary measure: |gpu - orc| / max(|orc|, 1e-3 * ||orc_row||_inf) per element, maximum over all
    elements (the floor keeps elements that cancel to almost nothing from dominating).  Reported, not gated."""
    o = orc.astype(np.float64)
    floor = 1e-3 * np.maximum(np.abs(o).max(axis=-1, keepdims=True), 1e-6)
    e = np.abs(gpu.astype(np.float64) - o) / np.maximum(np.abs(o), floor)
    return float(e.max()) if e.size else 0.0


def assert_same_state(gpu_be, orc_be, gpu_pool, orc_pool, what=""):
    a, b = gpu_be.pool_export_state(gpu_pool), orc_be.pool_export_state(orc_pool)
    if not np.array_equal(a, b):
        sa, sb = parse(a), parse(b)
        for key in ("free", "owner"):
            assert sa[key] == sb[key], f"{what}: {key} differs"
        for m in sb["models"]:
            for key in ("frames", "bits", "rows"):
                assert sa["models"][m][key] == sb["models"][m][key], f"{what}: model {m} {key} differs"
        raise AssertionError(f"{what}: state images differ")
    return a


def run_pair(gpu_be, orc_be, cfg, attn_steps=None, check_every_step=True):
    """Drive both backends through the scenario; bookkeeping must agree bit for bit
    after every step, attention within tolerance on the steps in attn_steps
    (None = all).  Returns the worst relative error."""
    rg = Runner(gpu_be, cfg).setup()
    ro = Runner(orc_be, cfg).setup()
    worst = 0.0
    try:
        assert rg.log == ro.log
        for t in range(cfg.steps):
            rg.step(t)
            ro.step(t)
            assert rg.log == ro.log, f"step {t}: return codes differ"
            if check_every_step:
                img = assert_same_state(gpu_be, orc_be, rg.pool, ro.pool, f"step {t}")
                check_invariants(parse(img))
            if attn_steps is not None and t not in attn_steps:
                continue
            for mi in rg.active_models():
                q = rg.queries(t, mi)
                rc_g, out_g = gpu_be.decode_attention(rg.models[mi], q, rg.ctx[mi])
                rc_o, out_o = orc_be.decode_attention(ro.models[mi], q, ro.ctx[mi])
                assert rc_g == 0 and rc_o == 0
                err = row_rel_err(out_g, out_o)
                tol = TOL[cfg.models[mi].dtype]
                assert err <= tol, f"step {t} model {mi}: rel err {err:.3e} > {tol}"
                worst = max(worst, err)
        assert gpu_be.device_errors() == 0
    finally:
        rg.teardown()
        ro.teardown()
    return worst
