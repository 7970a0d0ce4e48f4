"""A request-level serving loop in which the slack-aware arbitration (paper Sec. 5.2, Alg. 2)
decides who is admitted: the library's arbitrate_requests drives the GPU side, the plain
definition in oracle/policy_oracle.py the oracle side.  Admission is balloon_resize +
seq_reserve + kv_append_chunk, running sequences grow by a token per step, finished ones are
released and their model's balloon shrinks as far as it can.  Decisions, return values and the
pool state must agree after every step; decode attention of the running sequences within
tolerance on every fifth step."""
import numpy as np
import pytest

from parity import TOL, assert_same_state, row_rel_err
from state_image import check_invariants, parse
from workloads.requests import RequestConfig, RequestRunner

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


def test_arbitration_drives_the_balloons(gpu, oracle):
    cfg = RequestConfig()
    rg, ro = RequestRunner(gpu, cfg).setup(), RequestRunner(oracle, cfg).setup()
    worst = {0: 0.0, 1: 0.0}
    steps_with_drop = 0
    try:
        for t in range(cfg.steps):
            print(f"step {t}", flush=True) if t % 50 == 0 else None
            dropped_before = len(ro.dropped)
            rg.step(t)
            ro.step(t)
            assert rg.decisions == ro.decisions, f"step {t}: the arbitration decided differently"
            assert rg.log == ro.log, f"step {t}: return values differ"
            steps_with_drop += len(ro.dropped) > dropped_before
            if t % 5 == 0:
                for mi in ro.running_models():
                    q = ro.queries(t, mi)
                    rc_g, out_g = gpu.decode_attention(rg.models[mi], q, rg.ctx[mi])
                    rc_o, out_o = oracle.decode_attention(ro.models[mi], q, ro.ctx[mi])
                    assert rc_g == 0 and rc_o == 0
                    err = row_rel_err(out_g, out_o)
                    dt = cfg.models[mi].dtype
                    assert err <= TOL[dt], (t, mi, err)
                    worst[dt] = max(worst[dt], err)
            rg.retire(t)
            ro.retire(t)
            assert rg.log == ro.log, f"step {t}: return values differ after the departures"
            img = assert_same_state(gpu, oracle, rg.pool, ro.pool, f"step {t}")
            if t % 10 == 0:
                check_invariants(parse(img))
        assert gpu.device_errors() == 0
        # the run must have exercised what it is for
        assert steps_with_drop >= 1 and len(ro.dropped) >= 1, "no request was ever dropped"
        assert ro.clamped_deflates >= 1, "no deflate ever clamped"
        assert ro.refused_inflates >= 1, "the pool never ran out of frames"
        assert len(ro.finished) >= 50 and rg.finished == ro.finished and rg.dropped == ro.dropped
        print(f"{ro.next_rid} requests: {len(ro.admitted)} admitted, {len(ro.dropped)} dropped by the arbitration "
              f"({steps_with_drop} steps with a drop), {len(ro.finished)} finished; {ro.clamped_deflates} deflates clamped, "
              f"{ro.refused_inflates} inflates refused; {len(ro.log)} calls; worst rel err bf16 {worst[0]:.2e}, e4m3 {worst[1]:.2e}")
    finally:
        rg.teardown()
        ro.teardown()
