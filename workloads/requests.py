"""A request-level serving loop over one shared pool, with the slack-aware arbitration
of the paper (Sec. 5.2, Alg. 2) deciding who is admitted.

Like `scenarios.py`, this module only decides *which calls to make with which seeded
inputs*; the arbitration, the bookkeeping and the attention are the backend's.  A backend
is the GPU binding or the oracle wrapper; both are driven through the same code, every
call's return value goes to `log`, and the decisions of the arbitration go to `decisions`,
so two backends can be compared call by call.

The loop (synthetic stand-in for the paper's traces: bursty arrivals per model, Sec. 3.1;
one queue per GPU, Sec. 5.2):

  each step of `dt` seconds
    1. requests arrive: per model a two-state burst chain; while a model bursts, a few
       requests arrive (prompt length lognormal, TTFT SLO of the model, output length uniform);
    2. the queue (every request not yet admitted or dropped) goes to arbitrate_requests with
       the current time; requests it leaves out would miss their deadline whatever is done
       and are dropped;
    3. accepted requests are dispatched in schedule order while the step's prefill budget
       lasts and their model has a free row: the model's balloon is inflated if its free
       slots do not cover the prompt (a refused inflate leaves the request queued), the
       row's blocks are reserved, the prompt's KV is appended as one chunk;
    4. every running sequence grows by one token (one more block where needed, KV appended)
       and the models decode; a sequence that has produced its output is released;
    5. a model whose sequences ended shrinks its balloon to what the rest needs — the call
       clamps where frames still hold blocks.
"""
from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

from . import gen


@dataclass
class ServedModel:
    q_heads: int
    kv_heads: int
    head_dim: int
    dtype: int
    rows: int                  # sequences the model can run at once
    ttft_slo: float            # seconds
    prefill_speed: float       # prompt tokens per second of chunked prefill
    p_on: float = 0.15         # burst chain
    p_off: float = 0.35
    burst_arrivals: int = 3    # requests per step while bursting: uniform 1..burst_arrivals


@dataclass
class RequestConfig:
    seed: int = 6000
    steps: int = 200
    dt: float = 0.02
    page_tokens: int = 16
    frame_bytes: int = 256 << 10
    pool_bytes: int = 12 << 20
    prompt_median: float = 220.0
    prompt_sigma: float = 0.7
    prompt_cap: int = 900
    out_lo: int = 4
    out_hi: int = 40
    prefill_budget: int = 1200          # prompt tokens dispatched per step
    max_blocks: int = 64
    models: List[ServedModel] = field(default_factory=lambda: [
        ServedModel(32, 8, 128, gen.BF16, 6, 0.10, 9000.0),
        ServedModel(32, 8, 64, gen.BF16, 8, 0.25, 12000.0),
        ServedModel(16, 4, 128, gen.E4M3, 6, 0.15, 10000.0),
        ServedModel(8, 2, 64, gen.BF16, 8, 0.40, 16000.0),
    ])


def block_bytes(m: ServedModel, page_tokens: int) -> int:
    e = 2 if m.dtype == gen.BF16 else 1
    return 2 * page_tokens * m.kv_heads * m.head_dim * e + (128 if m.dtype == gen.E4M3 else 0)


@dataclass
class Request:
    rid: int
    model: int
    arrival: float
    prompt: int
    out_len: int


class RequestRunner:
    def __init__(self, be, cfg: RequestConfig):
        self.be, self.cfg = be, cfg
        self.log, self.decisions = [], []
        self.queue: List[Request] = []
        self.dropped, self.admitted, self.finished = [], [], []
        self.clamped_deflates = 0
        self.refused_inflates = 0
        self.pool = None
        self.models: List[int] = []
        n = len(cfg.models)
        self.slots = [cfg.frame_bytes // block_bytes(m, cfg.page_tokens) for m in cfg.models]
        self.owned = [0] * n
        self.ctx = [np.zeros(m.rows, dtype=np.int32) for m in cfg.models]       # tokens in each row's cache
        self.left = [np.zeros(m.rows, dtype=np.int32) for m in cfg.models]      # output tokens still to produce
        self.rid = [np.full(m.rows, -1, dtype=np.int64) for m in cfg.models]
        self.bursting = [False] * n
        self.next_rid = 0
        self._arrival_rng = gen.generator(cfg.seed, 1)

    # ------------------------------------------------------------ helpers
    def _rc(self, what, rc):
        self.log.append((what, int(rc)))
        return int(rc)

    def _blocks(self, tokens):
        t = self.cfg.page_tokens
        return (int(tokens) + t - 1) // t

    def _used_blocks(self, mi):
        return int(sum(self._blocks(c) for c in self.ctx[mi]))

    def _u(self):
        return float(torch.rand((), generator=self._arrival_rng))

    # -------------------------------------------------------------- setup
    def setup(self):
        c, be = self.cfg, self.be
        self.pool = self._rc("pool_create", be.pool_create(c.pool_bytes, c.page_tokens, c.frame_bytes))
        assert self.pool >= 0
        perm = gen.free_order(c.pool_bytes // c.frame_bytes, gen.generator(c.seed, 2))
        assert self._rc("pool_seed_free_order", be.pool_seed_free_order(self.pool, perm)) == 0
        for m in c.models:
            mid = self._rc("model_register", be.model_register(self.pool, m.q_heads, m.kv_heads, m.head_dim, m.dtype,
                                                              m.rows, c.max_blocks))
            assert mid >= 0
            self.models.append(mid)
        return self

    # ------------------------------------------------------------ a step
    def _arrivals(self, t):
        c = self.cfg
        for mi, m in enumerate(c.models):
            u = self._u()
            self.bursting[mi] = (u >= m.p_off) if self.bursting[mi] else (u < m.p_on)
            if not self.bursting[mi]:
                continue
            for _ in range(1 + int(self._u() * m.burst_arrivals)):
                z = float(torch.randn((), generator=self._arrival_rng, dtype=torch.float64))
                prompt = int(min(max(round(np.exp(np.log(c.prompt_median) + c.prompt_sigma * z)), 1), c.prompt_cap))
                out_len = c.out_lo + int(self._u() * (c.out_hi - c.out_lo + 1))
                self.queue.append(Request(self.next_rid, mi, t * c.dt + self._u() * c.dt * 0.5, prompt, out_len))
                self.next_rid += 1

    def _arbitrate(self, now):
        c = self.cfg
        q = self.queue
        accepted = self.be.arbitrate_requests([r.arrival for r in q], [c.models[r.model].ttft_slo for r in q],
                                              [float(r.prompt) for r in q], [c.models[r.model].prefill_speed for r in q], now)
        accepted = [int(i) for i in accepted]
        self.decisions.append((len(q), tuple(q[i].rid for i in accepted)))
        keep = set(accepted)
        self.dropped += [r.rid for i, r in enumerate(q) if i not in keep]
        return [q[i] for i in accepted]

    def _admit(self, t, schedule):
        """Dispatch in schedule order within the step's prefill budget; returns the requests still queued."""
        c, be = self.cfg, self.be
        budget, waiting = c.prefill_budget, []
        chunks = {}                      # model index -> [(row, request)]
        for r in schedule:
            mi = r.model
            free_rows = [s for s in range(c.models[mi].rows) if self.rid[mi][s] < 0]
            if r.prompt > budget or not free_rows:
                waiting.append(r)
                continue
            need = self._blocks(r.prompt + 1)          # the prompt and the first token it produces
            have = self.owned[mi] * self.slots[mi] - self._used_blocks(mi)
            if need > have:
                frames = self.owned[mi] + (need - have + self.slots[mi] - 1) // self.slots[mi]
                got = self._rc("balloon_resize", be.balloon_resize(self.models[mi], frames))
                if got < 0:                            # the pool has no frame left: stays queued
                    self.refused_inflates += 1
                    waiting.append(r)
                    continue
                self.owned[mi] = got
            s = free_rows[0]
            assert self._rc("seq_reserve", be.seq_reserve(self.models[mi], s, r.prompt)) >= 0
            self.rid[mi][s], self.ctx[mi][s], self.left[mi][s] = r.rid, r.prompt, r.out_len
            chunks.setdefault(mi, []).append((s, r))
            budget -= r.prompt
            self.admitted.append(r.rid)
        for mi, items in chunks.items():               # the prompts' KV: one chunk per admitted row
            m = c.models[mi]
            q_lens = np.zeros(m.rows, dtype=np.int32)
            parts_k, parts_v = [], []
            for s, r in sorted(items):
                q_lens[s] = r.prompt
                g = gen.generator(c.seed, 3, r.rid)
                parts_k.append(gen.randn_bf16((r.prompt, m.kv_heads, m.head_dim), g))
                parts_v.append(gen.randn_bf16((r.prompt, m.kv_heads, m.head_dim), g))
            rc = be.kv_append_chunk(self.models[mi], np.concatenate(parts_k), np.concatenate(parts_v), q_lens, self.ctx[mi])
            assert self._rc("kv_append_chunk", rc) == int(q_lens.sum())
        return waiting

    def _grow(self, t):
        """Every running sequence takes its next token: a block where needed, the token's KV."""
        c, be = self.cfg, self.be
        for mi, m in enumerate(c.models):
            live = [s for s in range(m.rows) if self.rid[mi][s] >= 0]
            if not live:
                continue
            want = [int(self.ctx[mi][s]) + 1 for s in live]
            need = sum(self._blocks(w) - self._blocks(w - 1) for w in want)
            have = self.owned[mi] * self.slots[mi] - self._used_blocks(mi)
            if need > have:
                got = self._rc("balloon_resize", be.balloon_resize(self.models[mi], self.owned[mi] + 1))
                if got < 0:            # no frame left: the sequences that need a block wait for the next step
                    self.refused_inflates += 1
                    live = [s for s, w in zip(live, want) if self._blocks(w) == self._blocks(w - 1)]
                    want = [int(self.ctx[mi][s]) + 1 for s in live]
                    if not live:
                        continue
                else:
                    self.owned[mi] = got
            assert self._rc("seq_reserve_batch", be.seq_reserve_batch(self.models[mi], live, want)) >= 0
            q_lens = np.zeros(m.rows, dtype=np.int32)
            for s, w in zip(live, want):
                self.ctx[mi][s] = w
                q_lens[s] = 1
            g = gen.generator(c.seed, 4, t, mi)
            k = gen.randn_bf16((len(live), m.kv_heads, m.head_dim), g)
            v = gen.randn_bf16((len(live), m.kv_heads, m.head_dim), g)
            assert self._rc("kv_append_chunk", be.kv_append_chunk(self.models[mi], k, v, q_lens, self.ctx[mi])) == len(live)
            for s in live:
                self.left[mi][s] -= 1

    def _retire(self, t):
        """Sequences that have produced their output leave; their model gives back what it can."""
        be = self.be
        for mi, m in enumerate(self.cfg.models):
            done = [s for s in range(m.rows) if self.rid[mi][s] >= 0 and self.left[mi][s] <= 0]
            if not done:
                continue
            assert self._rc("seq_release_batch", be.seq_release_batch(self.models[mi], done)) > 0
            for s in done:
                self.finished.append(int(self.rid[mi][s]))
                self.rid[mi][s], self.ctx[mi][s], self.left[mi][s] = -1, 0, 0
            target = (self._used_blocks(mi) + self.slots[mi] - 1) // self.slots[mi]
            got = self._rc("balloon_resize", be.balloon_resize(self.models[mi], target))
            assert got >= target
            self.clamped_deflates += got > target
            self.owned[mi] = got

    def step(self, t):
        """Bookkeeping and KV writes of step t; the caller decodes the running sequences afterwards
        (decode_inputs) and then calls retire(t)."""
        now = t * self.cfg.dt
        self._arrivals(t)
        schedule = self._arbitrate(now) if self.queue else []
        self.queue = self._admit(t, schedule)
        self._grow(t)
        return self

    def retire(self, t):
        self._retire(t)
        return self

    def running_models(self):
        return [mi for mi in range(len(self.cfg.models)) if (self.rid[mi] >= 0).any()]

    def queries(self, t, mi):
        m = self.cfg.models[mi]
        return gen.queries((self.cfg.seed, 5, t, mi), m.rows, m.q_heads, m.head_dim)

    # ------------------------------------------------------------ teardown
    def teardown(self):
        be = self.be
        for mi, mid in enumerate(self.models):
            be.seq_release_batch(mid, list(range(self.cfg.models[mi].rows)))
            be.balloon_resize(mid, 0)
            be.model_unregister(mid)
        self.models = []
        if self.pool is not None:
            be.pool_destroy(self.pool)
            self.pool = None
