"""The library enqueues on the caller's stream: a side stream, and a captured HIP graph that is
replayed several times with eager work in between (every replay must equal the eager result)."""
import numpy as np
import pytest
import torch

from workloads.scenarios import Runner, make_config

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    from paper_2505_04021_amd import PrismKV
    return PrismKV()


def setup(gpu):
    cfg = make_config(2, "small")
    r = Runner(gpu, cfg).setup()
    mids = r.active_models()
    qs = [torch.from_numpy(r.queries(0, mi).view(np.int16)).cuda() for mi in mids]
    ctxs = [torch.from_numpy(r.ctx[mi]).cuda() for mi in mids]
    outs = [torch.zeros((cfg.models[mi].batch, cfg.models[mi].q_heads, cfg.models[mi].head_dim), dtype=torch.float32, device="cuda")
            for mi in mids]
    return r, [r.models[mi] for mi in mids], qs, ctxs, outs


def test_side_stream(gpu):
    r, models, qs, ctxs, outs = setup(gpu)
    assert gpu.decode_attention_multi_dev(models, qs, ctxs, outs) == 0
    torch.cuda.synchronize()
    want = [o.clone() for o in outs]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu.use_current_stream()
        for o in outs:
            o.zero_()
        assert gpu.decode_attention_multi_dev(models, qs, ctxs, outs) == 0
    side.synchronize()
    gpu.use_current_stream()
    for a, b in zip(outs, want):
        assert torch.equal(a, b)
    assert gpu.device_errors() == 0
    r.teardown()


def test_graph_replays_equal_eager(gpu):
    """The very first attention call on freshly registered models is the captured one: the library
    sized its workspaces at registration, so the capture meets no allocation and no wait."""
    r, models, qs, ctxs, outs = setup(gpu)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        gpu.use_current_stream()
        graph.capture_begin()
        rc = gpu.decode_attention_multi_dev(models, qs, ctxs, outs)
        graph.capture_end()
    gpu.use_current_stream()
    assert rc == 0
    want = [torch.empty_like(o) for o in outs]
    assert gpu.decode_attention_multi_dev(models, qs, ctxs, want) == 0        # the eager result
    torch.cuda.synchronize()
    for rep in range(4):
        for o in outs:
            o.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(outs, want):
            assert torch.equal(a, b), rep
        # eager work of the library between the replays, on new queries, then back
        q2 = [torch.roll(q, 1, dims=0) for q in qs]
        o2 = [torch.empty_like(o) for o in outs]
        assert gpu.decode_attention_multi_dev(models, q2, ctxs, o2) == 0
        torch.cuda.synchronize()
    assert gpu.device_errors() == 0
    r.teardown()
