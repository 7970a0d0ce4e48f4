"""ctypes binding of libprismkv.so: argument marshalling only.

Every method has the name of the C entry point it calls.  Device buffers are torch
tensors on the GPU (torch is used for device memory and streams, nothing else);
numpy inputs are copied to the device first.  No step of the path runs in Python.
"""
import ctypes as C
import os

import numpy as np

PKV_BF16, PKV_E4M3 = 0, 1

_HERE = os.path.dirname(os.path.abspath(__file__))


def lib_path():
    # PRISMKV_LIB selects another build of the same library (kernel tuning experiments)
    return os.environ.get("PRISMKV_LIB") or os.path.join(_HERE, "libprismkv.so")


def _load():
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is missing: build it with paper_2505_04021_amd/build.py (no CPU fallback exists)")
    lib = C.CDLL(path)
    i, l, sz, vp, u32 = C.c_int, C.c_long, C.c_size_t, C.c_void_p, C.c_uint32
    sig = {
        "pkv_set_stream": (i, [vp]),
        "pkv_last_error": (C.c_char_p, []),
        "pkv_device_errors": (i, []),
        "pkv_set_split": (i, [i, i]),
        "pkv_set_page_cost": (i, [i]),
        "pkv_debug_fastdiv": (u32, [u32, u32]),
        "pkv_debug_fail_frame_map": (i, [i]),
        "pkv_set_xcd_weights": (i, [C.POINTER(C.c_float)]),
        "pkv_get_xcd_weights": (i, [C.POINTER(C.c_float)]),
        "pkv_tune_xcd": (i, [i]),
        "pkv_set_segment_cost": (i, [i]),
        "pkv_set_kernel_form": (i, [i]),
        "pkv_last_kernel_form": (i, []),
        "pkv_last_launch_items": (i, []),
        "pkv_stream_read_probe": (i, [sz, sz, i, C.POINTER(C.c_double)]),
        "pkv_timing_enable": (i, [i]),
        "pkv_timing_read": (l, [C.POINTER(C.c_double)]),
        "pool_create": (i, [sz, i]),
        "pool_create_ex": (i, [sz, i, sz, vp]),
        "pool_destroy": (i, [i]),
        "pool_seed_free_order": (i, [i, vp, sz]),
        "model_register": (i, [i, i, i, i]),
        "model_register_ex": (i, [i, i, i, i, i, i, i]),
        "model_register_layers": (i, [i, i, i, i, i, i, i, i]),
        "pkv_set_layer": (i, [i, i]),
        "model_unregister": (i, [i]),
        "balloon_resize": (l, [i, l]),
        "seq_reserve": (i, [i, i, i]),
        "seq_reserve_batch": (i, [i, i, vp, vp]),
        "seq_release": (i, [i, i]),
        "seq_release_batch": (i, [i, i, vp]),
        "balloon_resize_enqueue": (i, [i, l]),
        "seq_reserve_batch_enqueue": (i, [i, i, vp, vp]),
        "seq_release_batch_enqueue": (i, [i, i, vp]),
        "pkv_ticket_result": (l, [i]),
        "model_block_table": (vp, [i, C.POINTER(i)]),
        "kv_write": (i, [i, i, i, i, vp, vp, vp, vp]),
        "kv_append": (i, [i, i, vp, vp, vp]),
        "kv_append_chunk": (i, [i, i, vp, vp, vp, vp]),
        "kv_read": (i, [i, i, i, i, vp, vp, vp, vp]),
        "model_set_batch": (i, [i, i, i]),
        "decode_attention": (i, [i, vp, vp, vp, vp]),
        "decode_attention_ex": (i, [i, i, vp, vp, i, vp, vp]),
        "decode_attention_static": (i, [i, i, vp, vp, i, vp, vp]),
        "decode_attention_multi": (i, [i, vp, vp, vp, vp, vp]),
        "prefill_attention": (i, [i, i, vp, vp, vp, vp]),
        "pool_export_state": (l, [i, vp, sz]),
        "pool_stats": (i, [i, vp]),
        "pool_create_elastic": (i, [sz, i, sz]),
        "arbitrate_requests": (i, [i, vp, vp, vp, vp, C.c_double, vp]),
        "place_models": (i, [i, C.c_double, C.c_double, i, vp, vp, vp, vp, vp, vp, vp]),
        "pool_set_prealloc": (i, [i, l]),
        "pool_prealloc_wait": (i, [i]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


EXPORTS = ["pkv_set_stream", "pkv_last_error", "pkv_device_errors", "pkv_set_split", "pkv_set_page_cost", "pkv_debug_fastdiv", "pkv_debug_fail_frame_map",
           "pkv_set_xcd_weights", "pkv_get_xcd_weights", "pkv_tune_xcd", "pkv_set_segment_cost", "pkv_set_kernel_form", "pkv_last_kernel_form", "pkv_last_launch_items",
           "pkv_timing_enable", "pkv_timing_read", "pkv_stream_read_probe",
           "pool_create", "pool_create_ex", "pool_create_elastic", "pool_set_prealloc", "pool_prealloc_wait", "pool_destroy", "pool_seed_free_order", "model_register",
           "model_register_ex", "model_register_layers", "pkv_set_layer", "model_unregister", "balloon_resize", "seq_reserve", "seq_reserve_batch",
           "seq_release", "seq_release_batch", "balloon_resize_enqueue", "seq_reserve_batch_enqueue", "seq_release_batch_enqueue",
           "pkv_ticket_result", "model_block_table", "kv_write", "kv_append", "kv_append_chunk", "kv_read", "model_set_batch", "decode_attention",
           "decode_attention_ex", "decode_attention_static", "decode_attention_multi", "prefill_attention", "pool_export_state", "pool_stats",
           "arbitrate_requests", "place_models"]


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def arbitrate_requests(arrival, ttft_slo, prompt_len, prefill_speed, now, lib=None):
    """Host-only policy call (needs no GPU): -> list of accepted request indices in dispatch order."""
    lib = lib or _load()
    a, s, p, c = _f64(arrival), _f64(ttft_slo), _f64(prompt_len), _f64(prefill_speed)
    out = np.zeros(max(a.size, 1), dtype=np.int32)
    ptr = lambda x: x.ctypes.data_as(C.c_void_p)
    m = lib.arbitrate_requests(a.size, ptr(a), ptr(s), ptr(p), ptr(c), float(now), ptr(out))
    if m < 0:
        raise ValueError(f"arbitrate_requests: {m}")
    return out[:m].tolist()


def place_models(n_gpus, capacity, tau, token_rate, token_size, slo, weight, current_gpu=None, tp_group=None, lib=None):
    """Host-only policy call (needs no GPU): -> list of GPU indices, one per model."""
    lib = lib or _load()
    t, z, s, w = _f64(token_rate), _f64(token_size), _f64(slo), _f64(weight)
    ptr = lambda x: None if x is None else x.ctypes.data_as(C.c_void_p)
    cur = None if current_gpu is None else np.ascontiguousarray(current_gpu, dtype=np.int32)
    tp = None if tp_group is None else np.ascontiguousarray(tp_group, dtype=np.int32)
    out = np.full(max(t.size, 1), -1, dtype=np.int32)
    rc = lib.place_models(int(n_gpus), float(capacity), float(tau), t.size, ptr(t), ptr(z), ptr(s), ptr(w), ptr(cur), ptr(tp), ptr(out))
    if rc < 0:
        raise ValueError(f"place_models: {rc}")
    return out[:t.size].tolist()


class PrismKV:
    """One per process; the library holds global pool / model tables."""

    name = "gpu"

    def __init__(self, device="cuda:0"):
        import torch
        if not torch.cuda.is_available():
            raise RuntimeError("PrismKV needs a GPU: the HIP path has no CPU fallback")
        self.torch = torch
        self.device = torch.device(device)
        self.lib = _load()
        self._shape = {}
        self._keep = {}
        self.use_current_stream()

    # ---- host policies (no GPU work)
    def arbitrate_requests(self, arrival, ttft_slo, prompt_len, prefill_speed, now):
        return arbitrate_requests(arrival, ttft_slo, prompt_len, prefill_speed, now, lib=self.lib)

    def place_models(self, *args, **kw):
        return place_models(*args, lib=self.lib, **kw)

    # ---- plumbing
    def use_current_stream(self):
        s = self.torch.cuda.current_stream(self.device)
        return self.lib.pkv_set_stream(C.c_void_p(s.cuda_stream))

    def last_error(self):
        return self.lib.pkv_last_error().decode()

    def device_errors(self):
        return self.lib.pkv_device_errors()

    def set_page_cost(self, per_mille=-1):
        return self.lib.pkv_set_page_cost(per_mille)

    def set_xcd_weights(self, w=None):
        if w is None:
            return self.lib.pkv_set_xcd_weights(None)
        arr = (C.c_float * 8)(*[float(x) for x in w])
        return self.lib.pkv_set_xcd_weights(arr)

    def get_xcd_weights(self):
        arr = (C.c_float * 8)()
        rc = self.lib.pkv_get_xcd_weights(arr)
        if rc:
            raise RuntimeError(f"pkv_get_xcd_weights: {rc}")
        return [float(x) for x in arr]

    def tune_xcd(self, launches):
        return self.lib.pkv_tune_xcd(int(launches))

    def set_kernel_form(self, form=-1):
        return self.lib.pkv_set_kernel_form(form)

    def debug_fail_frame_map(self, after=-1):
        return self.lib.pkv_debug_fail_frame_map(int(after))

    def last_kernel_form(self):
        return self.lib.pkv_last_kernel_form()

    def last_launch_items(self):
        return self.lib.pkv_last_launch_items()

    def set_segment_cost(self, pages=-1):
        return self.lib.pkv_set_segment_cost(int(pages))

    def set_split(self, items=0, min_share=0):
        return self.lib.pkv_set_split(items, min_share)

    def stream_read_probe(self, nbytes=4 << 30, granule_bytes=0, iters=10):
        g = C.c_double(0)
        rc = self.lib.pkv_stream_read_probe(nbytes, granule_bytes, iters, C.byref(g))
        if rc != 0:
            raise RuntimeError(f"pkv_stream_read_probe failed: {rc} {self.last_error()}")
        return g.value

    def timing_enable(self, every=1):
        """every = n: bracket every n-th attention launch with events; 0 / False = off."""
        return self.lib.pkv_timing_enable(int(every))

    def timing_read(self):
        """(recorded calls, attention kernel ms summed since the last read)."""
        a = C.c_double(0)
        n = self.lib.pkv_timing_read(C.byref(a))
        return n, a.value

    def _dev(self, a, dtype=None):
        """torch device tensor for a numpy array / tensor; dtype is a torch dtype to view as."""
        t = self.torch
        if a is None:
            return None
        if isinstance(a, np.ndarray):
            if a.dtype == np.uint16:
                a = t.from_numpy(np.ascontiguousarray(a).view(np.int16))
            else:
                a = t.from_numpy(np.ascontiguousarray(a))
        a = a.to(self.device).contiguous()
        return a

    @staticmethod
    def _p(tensor):
        return None if tensor is None else C.c_void_p(tensor.data_ptr())

    # ---- pool
    def pool_create(self, nbytes, page_tokens, frame_bytes=None, storage=None):
        """storage: optional torch uint8 device tensor to use as the pool memory."""
        if frame_bytes is None and storage is None:
            return self.lib.pool_create(nbytes, page_tokens)
        base = None
        if storage is not None:
            assert storage.is_cuda and storage.numel() * storage.element_size() >= nbytes
            base = C.c_void_p(storage.data_ptr())
        pool = self.lib.pool_create_ex(nbytes, page_tokens, frame_bytes or (2 << 20), base)
        if pool >= 0 and storage is not None:
            self._keep[("pool", pool)] = storage
        return pool

    def pool_destroy(self, pool):
        rc = self.lib.pool_destroy(pool)
        if rc == 0:
            self._keep.pop(("pool", pool), None)
        return rc

    def pool_seed_free_order(self, pool, perm):
        perm = np.ascontiguousarray(perm, dtype=np.uint32)
        return self.lib.pool_seed_free_order(pool, perm.ctypes.data_as(C.c_void_p), perm.size)

    # ---- models
    def model_register(self, pool, q_heads, kv_heads, head_dim, dtype, max_seqs=None, max_blocks=None, n_layers=1):
        m = self.lib.model_register_layers(pool, q_heads, kv_heads, head_dim, dtype, max_seqs or 256,
                                           max_blocks or 2048, n_layers)
        if m >= 0:
            self._shape[m] = (q_heads, kv_heads, head_dim, dtype)
        return m

    def set_layer(self, model, layer):
        return self.lib.pkv_set_layer(model, layer)

    def model_unregister(self, model):
        return self.lib.model_unregister(model)

    def balloon_resize(self, model, frames):
        return self.lib.balloon_resize(model, frames)

    def seq_reserve(self, model, seq, ctx_len):
        return self.lib.seq_reserve(model, seq, ctx_len)

    def seq_reserve_batch(self, model, seqs, ctx_lens):
        seqs = np.ascontiguousarray(seqs, dtype=np.int32)
        ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        assert seqs.size == ctx_lens.size
        return self.lib.seq_reserve_batch(model, seqs.size, seqs.ctypes.data_as(C.c_void_p),
                                          ctx_lens.ctypes.data_as(C.c_void_p))

    def seq_release(self, model, seq):
        return self.lib.seq_release(model, seq)

    def seq_release_batch(self, model, seqs):
        seqs = np.ascontiguousarray(seqs, dtype=np.int32)
        return self.lib.seq_release_batch(model, seqs.size, seqs.ctypes.data_as(C.c_void_p))

    # ---- the same bookkeeping, enqueue-only: each returns a ticket (or a negative code at once)
    def balloon_resize_enqueue(self, model, frames):
        return self.lib.balloon_resize_enqueue(model, frames)

    def seq_reserve_batch_enqueue(self, model, seqs, ctx_lens):
        seqs = np.ascontiguousarray(seqs, dtype=np.int32)
        ctx_lens = np.ascontiguousarray(ctx_lens, dtype=np.int32)
        assert seqs.size == ctx_lens.size
        return self.lib.seq_reserve_batch_enqueue(model, seqs.size, seqs.ctypes.data_as(C.c_void_p),
                                                  ctx_lens.ctypes.data_as(C.c_void_p))

    def seq_release_batch_enqueue(self, model, seqs):
        seqs = np.ascontiguousarray(seqs, dtype=np.int32)
        return self.lib.seq_release_batch_enqueue(model, seqs.size, seqs.ctypes.data_as(C.c_void_p))

    def ticket_result(self, ticket):
        return self.lib.pkv_ticket_result(ticket)

    def model_block_table(self, model):
        """(device pointer, row stride) of the library-owned block table."""
        stride = C.c_int(0)
        p = self.lib.model_block_table(model, C.byref(stride))
        return p, stride.value

    # ---- data
    def kv_write(self, model, seq, tok_begin, k, v, k_scale=None, v_scale=None):
        _, hkv, d, _ = self._shape[model]
        k, v = self._dev(k), self._dev(v)
        assert tuple(k.shape[1:]) == (hkv, d) and k.shape == v.shape
        ks, vs = self._dev(k_scale), self._dev(v_scale)
        rc = self.lib.kv_write(model, seq, tok_begin, k.shape[0], self._p(k), self._p(v), self._p(ks), self._p(vs))
        # the call only enqueues: keep the staging tensors alive until the stream has used them
        self.torch.cuda.current_stream(self.device).synchronize()
        return rc

    def kv_append_dev(self, model, k_new, v_new, ctx_lens):
        """Device tensors (bf16 bits [B][Hkv][D], int32 [B]); only enqueues."""
        return self.lib.kv_append(model, ctx_lens.numel(), self._p(k_new), self._p(v_new), self._p(ctx_lens))

    def kv_append(self, model, k_new, v_new, ctx_lens):
        _, hkv, d, _ = self._shape[model]
        k_new, v_new = self._dev(np.ascontiguousarray(k_new)), self._dev(np.ascontiguousarray(v_new))
        ctx = self._dev(np.ascontiguousarray(ctx_lens, dtype=np.int32))
        assert tuple(k_new.shape) == (ctx.numel(), hkv, d) and k_new.shape == v_new.shape
        rc = self.kv_append_dev(model, k_new, v_new, ctx)
        self.torch.cuda.current_stream(self.device).synchronize()
        return rc

    def kv_append_chunk_dev(self, model, k_new, v_new, q_lens, ctx_lens):
        """k_new, v_new, ctx_lens: device tensors; q_lens: host int32 numpy array.  Only enqueues."""
        q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
        return self.lib.kv_append_chunk(model, q_lens.size, self._p(k_new), self._p(v_new),
                                        q_lens.ctypes.data_as(C.c_void_p), self._p(ctx_lens))

    def kv_append_chunk(self, model, k_new, v_new, q_lens, ctx_lens):
        _, hkv, d, _ = self._shape[model]
        q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
        k_new, v_new = self._dev(np.ascontiguousarray(k_new)), self._dev(np.ascontiguousarray(v_new))
        ctx = self._dev(np.ascontiguousarray(ctx_lens, dtype=np.int32))
        assert tuple(k_new.shape) == (int(q_lens.sum()), hkv, d) and k_new.shape == v_new.shape
        rc = self.kv_append_chunk_dev(model, k_new, v_new, q_lens, ctx)
        self.torch.cuda.current_stream(self.device).synchronize()
        return rc

    def kv_read(self, model, seq, tok_begin, n_tok):
        """-> (code, k, v, k_scale, v_scale) as numpy: elements [n_tok][Hkv][D], scales [n_tok][Hkv] (None for bf16)."""
        t = self.torch
        _, hkv, d, dtype = self._shape[model]
        et = t.int16 if dtype == 0 else t.uint8
        k = t.zeros((n_tok, hkv, d), dtype=et, device=self.device)
        v = t.zeros((n_tok, hkv, d), dtype=et, device=self.device)
        ks = vs = None
        if dtype != 0:
            ks = t.zeros((n_tok, hkv), dtype=t.float32, device=self.device)
            vs = t.zeros((n_tok, hkv), dtype=t.float32, device=self.device)
        rc = self.lib.kv_read(model, seq, tok_begin, n_tok, self._p(k), self._p(v), self._p(ks), self._p(vs))
        t.cuda.current_stream(self.device).synchronize()
        kn, vn = k.cpu().numpy(), v.cpu().numpy()
        if dtype == 0:
            kn, vn = kn.view(np.uint16), vn.view(np.uint16)
        return rc, kn, vn, (None if ks is None else ks.cpu().numpy()), (None if vs is None else vs.cpu().numpy())

    def model_set_batch(self, model, batch, row_stride):
        return self.lib.model_set_batch(model, batch, row_stride)

    def decode_attention_dev(self, model, q, ctx_lens, out, block_table=None):
        """All arguments are device tensors; only enqueues.  Returns the library's code."""
        b = ctx_lens.numel()
        if block_table is None:
            return self.lib.decode_attention_ex(model, b, self._p(q), None, 0, self._p(ctx_lens), self._p(out))
        return self.lib.decode_attention_ex(model, b, self._p(q), self._p(block_table), block_table.shape[1],
                                            self._p(ctx_lens), self._p(out))

    def decode_attention_static_dev(self, model, q, ctx_lens, out, block_table=None):
        """decode_attention_dev through the entry point that allocates nothing; only enqueues."""
        b = ctx_lens.numel()
        if block_table is None:
            return self.lib.decode_attention_static(model, b, self._p(q), None, 0, self._p(ctx_lens), self._p(out))
        return self.lib.decode_attention_static(model, b, self._p(q), self._p(block_table), block_table.shape[1],
                                                self._p(ctx_lens), self._p(out))

    def decode_attention(self, model, q, ctx_lens, block_table=None):
        """Convenience for tests: host or device inputs -> (code, out as numpy fp32 [B][Hq][D])."""
        t = self.torch
        hq, _, d, _ = self._shape[model]
        q = self._dev(q)
        ctx = self._dev(np.ascontiguousarray(ctx_lens, dtype=np.int32) if isinstance(ctx_lens, np.ndarray) else ctx_lens)
        bt = None
        if block_table is not None:
            bt = self._dev(np.ascontiguousarray(block_table, dtype=np.int32)
                           if isinstance(block_table, np.ndarray) else block_table)
        out = t.empty((ctx.numel(), hq, d), dtype=t.float32, device=self.device)
        rc = self.decode_attention_dev(model, q, ctx, out, bt)
        t.cuda.current_stream(self.device).synchronize()
        return rc, out.cpu().numpy()

    def prefill_attention_dev(self, model, q, q_lens, ctx_lens, out):
        """q, ctx_lens, out: device tensors; q_lens: host int32 numpy array.  Only enqueues."""
        q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
        return self.lib.prefill_attention(model, q_lens.size, self._p(q), q_lens.ctypes.data_as(C.c_void_p),
                                          self._p(ctx_lens), self._p(out))

    def prefill_attention(self, model, q, q_lens, ctx_lens):
        """Convenience for tests: -> (code, out as numpy fp32 [sum q_lens][Hq][D])."""
        t = self.torch
        hq, _, d, _ = self._shape[model]
        q = self._dev(q)
        ctx = self._dev(np.ascontiguousarray(ctx_lens, dtype=np.int32))
        q_lens = np.ascontiguousarray(q_lens, dtype=np.int32)
        assert tuple(q.shape) == (int(q_lens.sum()), hq, d)
        out = t.empty((int(q_lens.sum()), hq, d), dtype=t.float32, device=self.device)
        rc = self.prefill_attention_dev(model, q, q_lens, ctx, out)
        t.cuda.current_stream(self.device).synchronize()
        return rc, out.cpu().numpy()

    def decode_attention_multi_dev(self, models, qs, ctxs, outs):
        """One grouped launch; lists of device tensors.  Only enqueues."""
        n = len(models)
        ids = (C.c_int * n)(*models)
        bs = (C.c_int * n)(*[c.numel() for c in ctxs])
        qp = (C.c_void_p * n)(*[q.data_ptr() for q in qs])
        cp = (C.c_void_p * n)(*[c.data_ptr() for c in ctxs])
        op = (C.c_void_p * n)(*[o.data_ptr() for o in outs])
        return self.lib.decode_attention_multi(n, ids, bs, qp, cp, op)

    def pool_create_elastic(self, nbytes, page_tokens, frame_bytes=2 << 20):
        return self.lib.pool_create_elastic(nbytes, page_tokens, frame_bytes)

    def pool_set_prealloc(self, pool, frames):
        return self.lib.pool_set_prealloc(pool, frames)

    def pool_prealloc_wait(self, pool):
        return self.lib.pool_prealloc_wait(pool)

    def pool_stats(self, pool):
        """-> dict(n_frames, n_free, owned[64], used_blocks[64], mapped_bytes, spare_frames, idle_frames)"""
        buf = (C.c_int64 * (2 + 64 + 64 + 3))()
        rc = self.lib.pool_stats(pool, C.cast(buf, C.c_void_p))
        if rc:
            raise RuntimeError(f"pool_stats: {rc} {self.last_error()}")
        v = list(buf)
        return {"n_frames": v[0], "n_free": v[1], "owned": v[2:66], "used_blocks": v[66:130], "mapped_bytes": v[130],
                "spare_frames": v[131], "idle_frames": v[132]}

    # ---- state
    def pool_export_state(self, pool):
        n = self.lib.pool_export_state(pool, None, 0)
        if n < 0:
            raise RuntimeError(f"pool_export_state failed: {n} {self.last_error()}")
        buf = np.empty(n // 4, dtype=np.int32)
        n2 = self.lib.pool_export_state(pool, buf.ctypes.data_as(C.c_void_p), buf.nbytes)
        assert n2 == n
        return buf
