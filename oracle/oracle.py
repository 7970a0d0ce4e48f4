"""ctypes face of the CPU oracle (oracle/prism_oracle.c).  TEST INFRASTRUCTURE ONLY.

Marshals numpy arrays to the C functions; holds no arithmetic of its own.
bf16 data travels as uint16 bit patterns, e4m3 data as uint8 codes.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

ORC_BF16, ORC_E4M3 = 0, 1

E_ARG, E_HANDLE, E_NOMEM, E_BALLOON, E_SHAPE, E_RANGE, E_BUSY, E_INTERNAL = range(-1, -9, -1)


class OracleError(RuntimeError):
    def __init__(self, code, what):
        super().__init__(f"oracle call {what} failed with code {code}")
        self.code = code


def _load():
    lib_path = _build.LIB
    if not os.path.exists(lib_path):
        _build.build()
    lib = C.CDLL(lib_path)
    i, l, sz, vp = C.c_int, C.c_long, C.c_size_t, C.c_void_p
    sig = {
        "orc_pool_create": (i, [sz, i]),
        "orc_pool_create_ex": (i, [sz, i, sz]),
        "orc_pool_destroy": (i, [i]),
        "orc_pool_seed_free_order": (i, [i, vp, sz]),
        "orc_model_register": (i, [i, i, i, i, i]),
        "orc_model_register_ex": (i, [i, i, i, i, i, i, i]),
        "orc_model_register_layers": (i, [i, i, i, i, i, i, i, i]),
        "orc_set_layer": (i, [i, i]),
        "orc_model_layers": (i, [i]),
        "orc_model_unregister": (i, [i]),
        "orc_balloon_resize": (l, [i, l]),
        "orc_seq_reserve": (i, [i, i, i]),
        "orc_seq_reserve_batch": (i, [i, i, vp, vp]),
        "orc_seq_release": (i, [i, i]),
        "orc_kv_write": (i, [i, i, i, i, vp, vp, vp, vp]),
        "orc_decode_attention": (i, [i, i, vp, vp, i, vp, vp]),
        "orc_attention_probs": (i, [i, vp, vp, i, i, vp]),
        "orc_pool_export_state": (l, [i, vp, sz]),
        "orc_pool_n_frames": (l, [i]),
        "orc_pool_n_free": (l, [i]),
        "orc_model_owned": (l, [i]),
        "orc_model_slots": (i, [i]),
        "orc_model_block_bytes": (l, [i]),
        "orc_block_address": (l, [i, i]),
        "orc_model_block_table": (C.POINTER(C.c_int32), [i, C.POINTER(i)]),
        "orc_model_row_len": (i, [i, i]),
        "orc_e4m3_decode": (C.c_double, [C.c_uint8]),
        "orc_e4m3_encode": (C.c_uint8, [C.c_float]),
        "orc_kv_append": (i, [i, i, vp, vp, vp]),
        "orc_kv_append_chunk": (i, [i, i, vp, vp, vp, vp]),
        "orc_kv_read": (i, [i, i, i, i, vp, vp, vp, vp]),
        "orc_prefill_attention": (i, [i, i, vp, vp, vp, i, vp, vp]),
        "orc_num_threads": (i, []),
        "orc_set_num_threads": (None, [i]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


class Oracle:
    """Same call names as the product binding; host (numpy) arguments."""

    name = "oracle"

    def __init__(self):
        self.lib = _load()
        self._shape = {}

    # ---- pool
    def pool_create(self, nbytes, page_tokens, frame_bytes=None):
        if frame_bytes is None:
            return self.lib.orc_pool_create(nbytes, page_tokens)
        return self.lib.orc_pool_create_ex(nbytes, page_tokens, frame_bytes)

    def pool_destroy(self, pool):
        return self.lib.orc_pool_destroy(pool)

    def pool_seed_free_order(self, pool, perm):
        perm = _arr(perm, np.uint32)
        return self.lib.orc_pool_seed_free_order(pool, _ptr(perm), perm.size)

    # ---- models
    def model_register(self, pool, q_heads, kv_heads, head_dim, dtype, max_seqs=None, max_blocks=None, n_layers=1):
        if n_layers != 1:
            m = self.lib.orc_model_register_layers(pool, q_heads, kv_heads, head_dim, dtype,
                                                   max_seqs or 256, max_blocks or 2048, n_layers)
        elif max_seqs is None and max_blocks is None:
            m = self.lib.orc_model_register(pool, q_heads, kv_heads, head_dim, dtype)
        else:
            m = self.lib.orc_model_register_ex(pool, q_heads, kv_heads, head_dim, dtype,
                                               max_seqs or 256, max_blocks or 2048)
        if m >= 0:
            self._shape[m] = (q_heads, kv_heads, head_dim, dtype)
        return m

    def set_layer(self, model, layer):
        return self.lib.orc_set_layer(model, layer)

    def model_unregister(self, model):
        return self.lib.orc_model_unregister(model)

    def balloon_resize(self, model, frames):
        return self.lib.orc_balloon_resize(model, frames)

    def seq_reserve(self, model, seq, ctx_len):
        return self.lib.orc_seq_reserve(model, seq, ctx_len)

    def seq_reserve_batch(self, model, seqs, ctx_lens):
        seqs = _arr(seqs, np.int32)
        ctx_lens = _arr(ctx_lens, np.int32)
        assert seqs.size == ctx_lens.size
        return self.lib.orc_seq_reserve_batch(model, seqs.size, _ptr(seqs), _ptr(ctx_lens))

    def seq_release(self, model, seq):
        return self.lib.orc_seq_release(model, seq)

    def seq_release_batch(self, model, seqs):
        """The batched release is defined as the single releases in order (paper Sec. 4.2, D2: blocks go
        back to the slots of the model's pages); a list with an invalid sequence is refused as a whole."""
        seqs = [int(x) for x in np.asarray(seqs).ravel()]
        for sq in seqs:
            if self.lib.orc_model_row_len(model, sq) < 0:
                return self.lib.orc_model_row_len(model, sq)
        total = 0
        for sq in seqs:
            total += self.lib.orc_seq_release(model, sq)
        return total

    # The product has enqueue-only forms of the bookkeeping calls (the result is fetched later through a
    # ticket).  The oracle knows no streams: it runs the call at once and keeps the result for the ticket.
    def _ticket(self, value):
        if not hasattr(self, "_tickets"):
            self._tickets = []
        self._tickets.append(int(value))
        return len(self._tickets) - 1

    def balloon_resize_enqueue(self, model, frames):
        return self._ticket(self.balloon_resize(model, frames))

    def seq_reserve_batch_enqueue(self, model, seqs, ctx_lens):
        return self._ticket(self.seq_reserve_batch(model, seqs, ctx_lens))

    def seq_release_batch_enqueue(self, model, seqs):
        return self._ticket(self.seq_release_batch(model, seqs))

    def ticket_result(self, ticket):
        return self._tickets[ticket]

    # ---- host policies: the plain definitions of oracle/policy_oracle.py under the product's call names
    def arbitrate_requests(self, arrival, ttft_slo, prompt_len, prefill_speed, now):
        from . import policy_oracle
        return policy_oracle.arbitrate(list(arrival), list(ttft_slo), list(prompt_len), list(prefill_speed), now)

    # ---- data
    def kv_write(self, model, seq, tok_begin, k, v, k_scale=None, v_scale=None):
        _, hkv, d, dtype = self._shape[model]
        et = np.uint16 if dtype == ORC_BF16 else np.uint8
        k = _arr(k, et)
        v = _arr(v, et)
        assert k.shape == v.shape and k.shape[1:] == (hkv, d), (k.shape, hkv, d)
        ks = _arr(k_scale, np.float32)
        vs = _arr(v_scale, np.float32)
        return self.lib.orc_kv_write(model, seq, tok_begin, k.shape[0], _ptr(k), _ptr(v), _ptr(ks), _ptr(vs))

    def kv_append(self, model, k_new, v_new, ctx_lens):
        """k_new, v_new: uint16 (bf16 bits) [B][Hkv][D]; writes token ctx_lens[s] - 1 of every sequence."""
        _, hkv, d, _ = self._shape[model]
        k_new = _arr(k_new, np.uint16)
        v_new = _arr(v_new, np.uint16)
        ctx_lens = _arr(ctx_lens, np.int32)
        assert k_new.shape == v_new.shape == (ctx_lens.size, hkv, d)
        return self.lib.orc_kv_append(model, ctx_lens.size, _ptr(k_new), _ptr(v_new), _ptr(ctx_lens))

    def kv_append_chunk(self, model, k_new, v_new, q_lens, ctx_lens):
        """k_new, v_new: uint16 [sum q_lens][Hkv][D]; sequence s writes tokens ctx_lens[s] - q_lens[s] .. ctx_lens[s] - 1."""
        _, hkv, d, _ = self._shape[model]
        k_new, v_new = _arr(k_new, np.uint16), _arr(v_new, np.uint16)
        q_lens, ctx_lens = _arr(q_lens, np.int32), _arr(ctx_lens, np.int32)
        assert k_new.shape == v_new.shape == (int(q_lens.sum()), hkv, d)
        return self.lib.orc_kv_append_chunk(model, ctx_lens.size, _ptr(k_new), _ptr(v_new), _ptr(q_lens), _ptr(ctx_lens))

    def kv_read(self, model, seq, tok_begin, n_tok):
        """-> (code, k, v, k_scale, v_scale): elements [n_tok][Hkv][D], scales [n_tok][Hkv] (None for bf16)."""
        _, hkv, d, dtype = self._shape[model]
        et = np.uint16 if dtype == ORC_BF16 else np.uint8
        k = np.zeros((n_tok, hkv, d), dtype=et)
        v = np.zeros((n_tok, hkv, d), dtype=et)
        ks = vs = None
        if dtype != ORC_BF16:
            ks = np.zeros((n_tok, hkv), dtype=np.float32)
            vs = np.zeros((n_tok, hkv), dtype=np.float32)
        rc = self.lib.orc_kv_read(model, seq, tok_begin, n_tok, _ptr(k), _ptr(v), _ptr(ks), _ptr(vs))
        return rc, k, v, ks, vs

    def prefill_attention(self, model, q, q_lens, ctx_lens, block_table=None):
        """q: uint16 [sum q_lens][Hq][D]; returns (code, out fp32 [sum q_lens][Hq][D])."""
        hq, _, d, _ = self._shape[model]
        q = _arr(q, np.uint16)
        q_lens = _arr(q_lens, np.int32)
        ctx_lens = _arr(ctx_lens, np.int32)
        assert q.shape == (int(q_lens.sum()), hq, d), (q.shape, q_lens.sum(), hq, d)
        out = np.empty(q.shape, dtype=np.float32)
        stride = 0
        if block_table is not None:
            block_table = _arr(block_table, np.int32)
            stride = block_table.shape[1]
        rc = self.lib.orc_prefill_attention(model, ctx_lens.size, _ptr(q), _ptr(q_lens), _ptr(block_table), stride,
                                            _ptr(ctx_lens), _ptr(out))
        return rc, out

    def e4m3_encode(self, y):
        return int(self.lib.orc_e4m3_encode(float(y)))

    def decode_attention(self, model, q, ctx_lens, block_table=None):
        """q: uint16 [B][Hq][D]; returns (code, out fp32 [B][Hq][D])."""
        hq, _, d, _ = self._shape[model]
        q = _arr(q, np.uint16)
        ctx_lens = _arr(ctx_lens, np.int32)
        b = ctx_lens.size
        assert q.shape == (b, hq, d), (q.shape, b, hq, d)
        out = np.empty((b, hq, d), dtype=np.float32)
        stride = 0
        if block_table is not None:
            block_table = _arr(block_table, np.int32)
            assert block_table.ndim == 2 and block_table.shape[0] == b
            stride = block_table.shape[1]
        rc = self.lib.orc_decode_attention(model, b, _ptr(q), _ptr(block_table), stride, _ptr(ctx_lens), _ptr(out))
        return rc, out

    def attention_probs(self, model, q_row, table_row, ctx_len, q_head):
        q_row = _arr(q_row, np.uint16)
        table_row = _arr(table_row, np.int32)
        p = np.empty(ctx_len, dtype=np.float64)
        rc = self.lib.orc_attention_probs(model, _ptr(q_row), _ptr(table_row), ctx_len, q_head, _ptr(p))
        return rc, p

    # ---- state
    def pool_export_state(self, pool):
        n = self.lib.orc_pool_export_state(pool, None, 0)
        if n < 0:
            raise OracleError(n, "pool_export_state")
        buf = np.empty(n // 4, dtype=np.int32)
        n2 = self.lib.orc_pool_export_state(pool, _ptr(buf), buf.nbytes)
        assert n2 == n
        return buf

    def block_table(self, model):
        stride = C.c_int(0)
        p = self.lib.orc_model_block_table(model, C.byref(stride))
        return p, stride.value

    def block_table_rows(self, model, n_rows):
        """Copy of the model's first n_rows block-table rows as int32 [n_rows][max_blocks]."""
        p, stride = self.block_table(model)
        return np.ctypeslib.as_array(p, shape=(n_rows, stride)).copy()

    def row_len(self, model, seq):
        return self.lib.orc_model_row_len(model, seq)

    def n_frames(self, pool):
        return self.lib.orc_pool_n_frames(pool)

    def n_free(self, pool):
        return self.lib.orc_pool_n_free(pool)

    def owned(self, model):
        return self.lib.orc_model_owned(model)

    def slots(self, model):
        return self.lib.orc_model_slots(model)

    def block_bytes(self, model):
        return self.lib.orc_model_block_bytes(model)

    def block_address(self, model, block_id):
        return self.lib.orc_block_address(model, block_id)

    def e4m3_decode(self, code):
        return self.lib.orc_e4m3_decode(code)

    def num_threads(self):
        return self.lib.orc_num_threads()

    def set_num_threads(self, n):
        self.lib.orc_set_num_threads(n)
