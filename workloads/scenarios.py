"""The five benchmark workloads as seeded call sequences against a backend.

A backend is any object with the library's call names (the oracle wrapper and the
GPU binding both qualify).  This module only decides *which calls to make with
which seeded inputs*; it performs none of the method's work itself.  Every call's
return code is appended to `Runner.log`, so two backends driven by the same
scenario can be compared call by call.

Workload recipe (synthetic stand-in for the paper's traces and model zoo):
  cfg 1  one small model, 4 sequences, one block per frame (plain paged attention)
  cfg 2  two co-located models (head dim 128 and 64) sharing one pool, lognormal
         context lengths, frames taken alternately so the balloons interleave
  cfg 3  eight models of mixed shape switching on and off by a two-state Markov
         chain; idle models deflate to zero, active models inflate and admit a batch
  cfg 4  one model, long equal contexts, 1 % of key rows scaled by 8
  cfg 5  four e4m3 models, one release/deflate/inflate/admit cycle every 10 steps
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np

from . import gen

MiB = 1 << 20
GiB = 1 << 30
MAX_RESERVE_LIST = 4096       # entries one seq_reserve_batch call takes


@dataclass
class ModelSpec:
    q_heads: int
    kv_heads: int
    head_dim: int
    dtype: int
    batch: int
    layers: int = 1               # layers sharing the model's block table (one block holds them all)


@dataclass
class Config:
    cfg: int
    name: str
    seed: int
    page_tokens: int
    frame_bytes: int
    pool_bytes: int
    models: List[ModelSpec]
    ctx_kind: str                 # "uniform" | "lognormal" | "fixed"
    ctx_a: float = 0              # lo / median / value
    ctx_b: float = 0              # hi / sigma
    ctx_cap: int = 0
    peak_frac: float = 0.0
    steps: int = 1
    inflate_chunk: int = 8        # frames per alternating inflate call
    grow_tokens: int = 64         # tokens per sequence per interleaved reserve round
    p_on: float = 0.2
    p_off: float = 0.3
    cycle_every: int = 10
    max_seqs: int = 256
    max_blocks: int = 2048
    extra: dict = field(default_factory=dict)


def block_bytes(spec: ModelSpec, page_tokens: int) -> int:
    e = 2 if spec.dtype == gen.BF16 else 1
    return spec.layers * (2 * page_tokens * spec.kv_heads * spec.head_dim * e + (128 if spec.dtype == gen.E4M3 else 0))


def make_config(cfg: int, size: str = "full") -> Config:
    """size: "full" = the sizes the benchmark names; "small" = same structure, sized
    so the CPU oracle finishes in seconds while still spanning several tiles,
    several split-K chunks and ragged tails."""
    small = size == "small"
    B16 = gen.BF16
    if cfg == 1:
        return Config(1, "cfg1_single_small", 1000, 16, 8192, 2 * MiB,
                      [ModelSpec(8, 2, 64, B16, 4)], "uniform", 16, 256, max_seqs=8, max_blocks=16)
    if cfg == 2:
        if small:
            return Config(2, "cfg2_two_models_small", 2000, 16, 2 * MiB, 1 * GiB,
                          [ModelSpec(32, 8, 128, B16, 6), ModelSpec(32, 8, 64, B16, 6)],
                          "lognormal", 200, 0.8, 1500, max_seqs=8, max_blocks=96)
        return Config(2, "cfg2_two_models", 2000, 16, 2 * MiB, 32 * GiB,
                      [ModelSpec(32, 8, 128, B16, 64), ModelSpec(32, 8, 64, B16, 64)],
                      "lognormal", 1024, 0.8, 8192, max_seqs=64, max_blocks=512)
    if cfg == 3:
        shapes = [(32, 8, 128), (64, 8, 128), (32, 8, 64), (64, 8, 64)] * 2
        if small:
            return Config(3, "cfg3_bursty_small", 3000, 16, 2 * MiB, 2 * GiB,
                          [ModelSpec(a, b, c, B16, 4) for a, b, c in shapes],
                          "lognormal", 150, 0.8, 600, steps=40, max_seqs=4, max_blocks=40)
        return Config(3, "cfg3_bursty", 3000, 16, 2 * MiB, 160 * 10**9,
                      [ModelSpec(a, b, c, B16, 32) for a, b, c in shapes],
                      "lognormal", 2048, 0.8, 8192, steps=1000, max_seqs=32, max_blocks=512)
    if cfg == 4:
        if small:
            return Config(4, "cfg4_long_small", 4000, 16, 2 * MiB, 1 * GiB,
                          [ModelSpec(64, 8, 128, B16, 2)], "fixed", 3003, peak_frac=0.01,
                          max_seqs=2, max_blocks=192)
        return Config(4, "cfg4_long", 4000, 16, 2 * MiB, 16 * GiB,
                      [ModelSpec(64, 8, 128, B16, 16)], "fixed", 32768, peak_frac=0.01,
                      max_seqs=16, max_blocks=2048)
    if cfg == 5:
        E = gen.E4M3
        if small:
            return Config(5, "cfg5_fp8_small", 5000, 16, 2 * MiB, 256 * MiB,
                          [ModelSpec(32, 8, 128, E, b) for b in (8, 4, 2, 2)],
                          "uniform", 40, 300, steps=21, max_seqs=8, max_blocks=24)
        return Config(5, "cfg5_fp8", 5000, 16, 2 * MiB, 8 * GiB,
                      [ModelSpec(32, 8, 128, E, b) for b in (128, 64, 32, 32)],
                      "uniform", 512, 4096, steps=21, max_seqs=128, max_blocks=256)
    raise ValueError(cfg)


def kv_bytes(cfg: Config, spec: ModelSpec, ctx_lens) -> int:
    """Algorithmic KV bytes one decode step must read for these sequences:
    exact context lengths, K and V, plus the per-block scale pairs for e4m3."""
    e = 2 if spec.dtype == gen.BF16 else 1
    n = int(np.sum(ctx_lens.astype(np.int64))) * spec.kv_heads * spec.head_dim * 2 * e
    if spec.dtype == gen.E4M3:
        blocks = int(np.sum((ctx_lens.astype(np.int64) + cfg.page_tokens - 1) // cfg.page_tokens))
        n += blocks * spec.kv_heads * 2 * 4
    return n


class Runner:
    """Drives one backend through a scenario.  `fill` selects which sequences get
    their KV written: None = all, a set of (model index, sequence uid), or a
    predicate fill(model index, uid)."""

    def __init__(self, be, cfg: Config, fill=None, write_kv: bool = True, mode: str = "calls"):
        """mode: how the bookkeeping of an admission / a departure is issued —
        "calls"   one seq_reserve_batch per growth round and one seq_release per sequence, each waited for;
        "batched" the growth rounds of an admission in ONE seq_reserve_batch, the departures in ONE
                  seq_release_batch (the same state by definition of the batched calls), each waited for;
        "enqueue" as "batched" through the enqueue-only forms: nothing waits, the return values are
                  fetched by flush(), which whoever drives the scenario calls when it wants them."""
        assert mode in ("calls", "batched", "enqueue")
        self.be, self.cfg = be, cfg
        self.fill = fill
        self.write_kv = write_kv
        self.mode = mode
        self._pending = []            # (index into log, ticket) of enqueued calls whose result is still out
        self._tape = None             # plan(): the enqueue-only calls are listed here instead of being made
        self.log = []
        self.pool = None
        self.models: List[int] = []
        n = len(cfg.models)
        self.ctx = [np.zeros(s.batch, dtype=np.int32) for s in cfg.models]
        self.uid = [np.full(s.batch, -1, dtype=np.int64) for s in cfg.models]
        self.next_uid = [0] * n
        self.active = [False] * n
        self.blocks = [0] * n         # blocks currently reserved per model
        self.layer = [0] * n          # current layer per model
        self.slots: List[int] = []
        self.activity = None

    # ------------------------------------------------------------ helpers
    def _rc(self, what, rc):
        self.log.append((what, int(rc)))
        return rc

    def _need(self, what, rc):
        self._rc(what, rc)
        if rc < 0:
            raise RuntimeError(f"{self.be.name}: {what} returned {rc}")
        return rc

    def _enqueue(self, what, mi, *args):
        """An enqueue-only bookkeeping call on model index mi (or its entry on the tape while planning)."""
        if self._tape is not None:
            self._tape.append((what + "_enqueue", mi, args))
            return
        self._later(what, getattr(self.be, what + "_enqueue")(self.models[mi], *args))

    def plan(self, t0, t1):
        """Steps t0 .. t1-1 of an enqueue-mode scenario as data, for a driver that wants to issue the
        calls itself without this module's Python in its timed loop.  Returns one entry per step:
        (calls, active model indices, {model index: context lengths of a batch admitted in this step},
        KV bytes a decode of the active models reads); calls = [(method name, model index, args)].
        The runner's own view (active, ctx, uid) moves on as if the calls had been made."""
        assert self.mode == "enqueue" and not self.write_kv
        steps = []
        for t in range(t0, t1):
            self._tape = []
            before = [u.copy() for u in self.uid]
            self.step(t)
            admitted = {mi: self.ctx[mi].copy() for mi in self.active_models() if not np.array_equal(before[mi], self.uid[mi])}
            steps.append((self._tape, self.active_models(), admitted, self.kv_bytes_step()))
            self._tape = None
        return steps

    def _later(self, what, ticket):
        """An enqueue-only call: its place in the log is kept, the value follows in flush()."""
        if ticket < 0:
            raise RuntimeError(f"{self.be.name}: {what} was refused at once with {ticket}")
        self._pending.append((len(self.log), ticket))
        self.log.append((what, None))

    def flush(self, n=None):
        """Fetch the results of the first n enqueued calls still out (all of them by default); waits
        for those calls only."""
        n = len(self._pending) if n is None else min(n, len(self._pending))
        for at, ticket in self._pending[:n]:
            rc = int(self.be.ticket_result(ticket))
            self.log[at] = (self.log[at][0], rc)
            if rc < 0:
                raise RuntimeError(f"{self.be.name}: {self.log[at][0]} returned {rc}")
        self._pending = self._pending[n:]
        return self

    def _resize(self, mi, frames):
        if self.mode == "enqueue":
            return self._enqueue("balloon_resize", mi, frames)
        return self._need("balloon_resize", self.be.balloon_resize(self.models[mi], frames))

    def _wants(self, mi, uid):
        if self.fill is None:
            return True
        if callable(self.fill):
            return bool(self.fill(mi, int(uid)))
        return (mi, int(uid)) in self.fill

    def filled_rows(self, mi):
        """Sequence slots of model mi whose KV has been written."""
        return [s for s in range(self.cfg.models[mi].batch)
                if self.uid[mi][s] >= 0 and self._wants(mi, self.uid[mi][s])]

    def _draw_ctx(self, n, key):
        c, g = self.cfg, gen.generator(self.cfg.seed, 11, *key)
        if c.ctx_kind == "uniform":
            return gen.ctx_uniform(n, int(c.ctx_a), int(c.ctx_b), g)
        if c.ctx_kind == "lognormal":
            return gen.ctx_lognormal(n, c.ctx_a, c.ctx_b, c.ctx_cap, g)
        return np.full(n, int(c.ctx_a), dtype=np.int32)

    def _blocks(self, ctx):
        t = self.cfg.page_tokens
        return (np.asarray(ctx, dtype=np.int64) + t - 1) // t

    def _admit(self, mi, seqs, ctx_lens, key):
        """Reserve blocks for new sequences in interleaved rounds (so that their
        blocks mix inside the model's frames as they would under concurrent
        decoding), then write their KV."""
        c, spec, m = self.cfg, self.cfg.models[mi], self.models[mi]
        seqs = np.asarray(seqs, dtype=np.int32)
        ctx_lens = np.asarray(ctx_lens, dtype=np.int32)
        g = gen.generator(c.seed, 12, mi, *key)
        rounds = int((int(ctx_lens.max()) + c.grow_tokens - 1) // c.grow_tokens) if len(seqs) else 0
        import torch
        all_seqs, all_ctx = [], []
        for r in range(rounds):
            cur = np.minimum(ctx_lens, (r + 1) * c.grow_tokens)
            live = np.nonzero(ctx_lens > r * c.grow_tokens)[0]
            order = live[torch.randperm(len(live), generator=g).numpy()]
            if self.mode == "calls":
                self._need("seq_reserve_batch", self.be.seq_reserve_batch(m, seqs[order], cur[order]))
            else:
                all_seqs.append(seqs[order])
                all_ctx.append(cur[order])
        if all_seqs:
            a, b = np.concatenate(all_seqs), np.concatenate(all_ctx)
            for lo in range(0, len(a), MAX_RESERVE_LIST):          # (a list longer than one call takes: several calls)
                part = slice(lo, lo + MAX_RESERVE_LIST)
                if self.mode == "enqueue":
                    self._enqueue("seq_reserve_batch", mi, a[part], b[part])
                else:
                    self._need("seq_reserve_batch", self.be.seq_reserve_batch(m, a[part], b[part]))
        for s, n_tok in zip(seqs, ctx_lens):
            u = self.next_uid[mi]
            self.next_uid[mi] += 1
            self.uid[mi][s] = u
            self.ctx[mi][s] = n_tok
            self.blocks[mi] += int(self._blocks(n_tok))
            if self.write_kv and self._wants(mi, u):
                for layer in range(spec.layers):
                    kv = gen.seq_kv(self.kv_key(mi, u, layer), int(n_tok), spec.kv_heads, spec.head_dim,
                                    spec.dtype, c.page_tokens, c.peak_frac)
                    if spec.layers > 1:
                        self._need("set_layer", self.be.set_layer(m, layer))
                    self._need("kv_write", self.be.kv_write(m, int(s), 0, kv["k"], kv["v"],
                                                            kv["k_scale"], kv["v_scale"]))
        if spec.layers > 1:
            self.set_layer(mi, self.layer[mi])

    def kv_key(self, mi, uid, layer=0):
        """Seed key of the KV of sequence uid of model mi at a layer."""
        return (self.cfg.seed, 13, mi, int(uid)) + ((layer,) if layer else ())

    def set_layer(self, mi, layer):
        """The layer of model mi that attention and KV calls address from now on."""
        self.layer[mi] = layer
        return self._need("set_layer", self.be.set_layer(self.models[mi], layer))

    def _release(self, mi, seqs):
        if self.mode == "enqueue":
            self._enqueue("seq_release_batch", mi, np.asarray(seqs, dtype=np.int32))
        elif self.mode == "batched":
            self._need("seq_release_batch", self.be.seq_release_batch(self.models[mi], np.asarray(seqs, dtype=np.int32)))
        for s in seqs:
            if self.mode == "calls":
                self._need("seq_release", self.be.seq_release(self.models[mi], int(s)))
            self.blocks[mi] -= int(self._blocks(self.ctx[mi][s]))
            self.ctx[mi][s] = 0
            self.uid[mi][s] = -1

    def _frames_for(self, mi, n_blocks):
        return (n_blocks + self.slots[mi] - 1) // self.slots[mi]

    # -------------------------------------------------------------- setup
    def setup(self):
        c, be = self.cfg, self.be
        self.pool = self._need("pool_create", be.pool_create(c.pool_bytes, c.page_tokens, c.frame_bytes))
        n_frames = c.pool_bytes // c.frame_bytes
        perm = gen.free_order(n_frames, gen.generator(c.seed, 1))
        self._need("pool_seed_free_order", be.pool_seed_free_order(self.pool, perm))
        for spec in c.models:
            more = {"n_layers": spec.layers} if spec.layers > 1 else {}
            m = self._need("model_register", be.model_register(
                self.pool, spec.q_heads, spec.kv_heads, spec.head_dim, spec.dtype,
                c.max_seqs, c.max_blocks, **more))
            self.models.append(m)
            self.slots.append(c.frame_bytes // block_bytes(spec, c.page_tokens))
        if c.cfg == 3:
            self.activity = gen.markov_activity(len(c.models), c.steps, c.p_on, c.p_off,
                                                gen.generator(c.seed, 2))
            return self
        # static start: every model active with a full batch
        ctxs = [self._draw_ctx(spec.batch, (mi, 0)) for mi, spec in enumerate(c.models)]
        want = [self._frames_for(mi, int(self._blocks(ctxs[mi]).sum())) for mi in range(len(c.models))]
        have = [0] * len(c.models)
        while any(h < w for h, w in zip(have, want)):     # alternate so the balloons interleave
            for mi in range(len(c.models)):
                if have[mi] < want[mi]:
                    have[mi] = min(want[mi], have[mi] + c.inflate_chunk)
                    self._need("balloon_resize", be.balloon_resize(self.models[mi], have[mi]))
        for mi, spec in enumerate(c.models):
            self._admit(mi, np.arange(spec.batch), ctxs[mi], (0,))
            self.active[mi] = True
        return self

    # --------------------------------------------------------------- step
    def step(self, t):
        """Bookkeeping events of step t (before its decode)."""
        c, be = self.cfg, self.be
        if c.cfg == 3:
            for mi, spec in enumerate(c.models):
                on = bool(self.activity[t][mi])
                if self.active[mi] and not on:       # burst over: give everything back
                    self._release(mi, np.arange(spec.batch))
                    self._resize(mi, 0)
                    self.active[mi] = False
                elif on and not self.active[mi]:      # burst starts: inflate, admit a batch
                    ctx = self._draw_ctx(spec.batch, (mi, t + 1))
                    frames = self._frames_for(mi, int(self._blocks(ctx).sum()))
                    self._resize(mi, frames)
                    self._admit(mi, np.arange(spec.batch), ctx, (t + 1,))
                    self.active[mi] = True
        elif c.cfg == 5 and t > 0 and t % c.cycle_every == 0:
            import torch
            mi = (t // c.cycle_every) % len(c.models)
            spec, m = c.models[mi], self.models[mi]
            g = gen.generator(c.seed, 3, t)
            quarter = max(1, spec.batch // 4)
            out = np.sort(torch.randperm(spec.batch, generator=g).numpy()[:quarter])
            self._release(mi, out)
            # ask for exactly what the remaining blocks need; frames that still
            # hold blocks cannot be taken back, so the call may clamp
            owned = self._need("balloon_resize", be.balloon_resize(m, self._frames_for(mi, self.blocks[mi])))
            ctx = self._draw_ctx(quarter, (mi, t + 1))
            short = int(self._blocks(ctx).sum()) - (owned * self.slots[mi] - self.blocks[mi])
            if short > 0:
                self._need("balloon_resize", be.balloon_resize(m, owned + self._frames_for(mi, short)))
            self._admit(mi, out, ctx, (t + 1,))
        return self

    def active_models(self):
        return [mi for mi in range(len(self.cfg.models)) if self.active[mi]]

    def queries(self, t, mi):
        spec = self.cfg.models[mi]
        return gen.queries((self.cfg.seed, 14, t, mi), spec.batch, spec.q_heads, spec.head_dim)

    def kv_bytes_step(self):
        return sum(kv_bytes(self.cfg, self.cfg.models[mi], self.ctx[mi]) for mi in self.active_models())

    # ------------------------------------------------------------ teardown
    def teardown(self):
        be = self.be
        self.flush()
        for mi, m in enumerate(self.models):
            for s in range(self.cfg.models[mi].batch):
                be.seq_release(m, s)
            be.balloon_resize(m, 0)
            be.model_unregister(m)
        self.models = []
        if self.pool is not None:
            be.pool_destroy(self.pool)
            self.pool = None
