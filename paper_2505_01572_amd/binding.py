"""ctypes binding of include/pipeverify.h.  Argument marshalling only."""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpipeverify.so")

PV_F32, PV_BF16 = 0, 1
PROF = {"none": 0, "qkv": 1, "attention": 2, "oproj": 3, "gateup": 4, "down": 5, "lmhead": 6}
PATH_AUTO, PATH_VECTOR, PATH_MATRIX = 0, 1, 2
KINDS = {"embed": 0, "attn_norm": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5,
         "ffn_norm": 6, "wg": 7, "wu": 8, "wd": 9, "final_norm": 10, "lm_head": 11}
_GLOBAL = ("embed", "final_norm", "lm_head")


class PVError(RuntimeError):
    def __init__(self, status, where, detail):
        super().__init__(f"{where}: {detail} (status {status})")
        self.status = status


class pv_model_config(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rms_eps", ctypes.c_double), ("rope_base", ctypes.c_double)] + \
               [(n, ctypes.c_int32) for n in ("dtype", "page_tokens", "max_gamma", "kernel_path", "weight_bits")]


EXPORTS = [
    "pv_model_bytes", "pv_cache_bytes", "pv_model_create", "pv_model_destroy", "pv_load_weights",
    "pv_cache_create", "pv_cache_destroy", "pv_cache_set_page_table", "pv_prefill", "pv_verify",
    "pv_verify_async", "pv_verify_wait", "pv_rollback", "pv_cache_len", "pv_cache_set_pending",
    "pv_debug_logits", "pv_debug_pred", "pv_cache_export", "pv_step_bytes", "pv_strerror", "pv_last_error",
    "pv_profile_select", "pv_profile_read", "pv_cache_readmit", "pv_calib_copy", "pv_calib_read", "pv_verify_async_static", "pv_verify_batch", "pv_verify_tree", "pv_cache_use_graphs", "pv_load_weights_q4",
]

_lib = None


def lib():
    """The loaded shared library.  There is no fallback: a missing build is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2505_01572_amd.build`")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        P = ctypes.POINTER
        cfgp = P(pv_model_config)
        L.pv_model_bytes.argtypes = [cfgp, P(sz), P(sz)]
        L.pv_cache_bytes.argtypes = [vp, i32, P(sz), P(sz)]
        L.pv_model_create.argtypes = [cfgp, vp, sz, vp, sz, P(vp)]
        L.pv_model_destroy.argtypes = [vp]; L.pv_model_destroy.restype = None
        L.pv_load_weights.argtypes = [vp, i32, i32, i64, i64, vp, vp]
        L.pv_load_weights_q4.argtypes = [vp, i32, i32, i64, i64, vp, vp, vp]
        L.pv_cache_create.argtypes = [vp, vp, sz, vp, sz, i32, P(vp)]
        L.pv_cache_destroy.argtypes = [vp]; L.pv_cache_destroy.restype = None
        L.pv_cache_set_page_table.argtypes = [vp, vp, i32, vp]
        L.pv_prefill.argtypes = [vp, vp, i32, vp]
        L.pv_verify.argtypes = [vp, i32, vp, i32, P(i32), P(i32), vp]
        L.pv_verify_async.argtypes = [vp, i32, vp, i32, vp]
        L.pv_verify_async_static.argtypes = [vp, i32, vp, i32, vp]
        L.pv_verify_wait.argtypes = [vp, P(i32), P(i32)]
        L.pv_verify_batch.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp]
        L.pv_verify_tree.argtypes = [vp, i32, vp, vp, i32, P(i32), P(i32), vp, vp]
        L.pv_rollback.argtypes = [vp, i32, vp]
        L.pv_cache_readmit.argtypes = [vp, i32, i32, vp]
        L.pv_cache_len.argtypes = [vp, P(i32), P(i32)]
        L.pv_cache_set_pending.argtypes = [vp, i32, vp]
        L.pv_debug_logits.argtypes = [vp, vp, P(i32), vp]
        L.pv_debug_pred.argtypes = [vp, vp, P(i32), vp]
        L.pv_cache_export.argtypes = [vp, vp, sz, vp]
        L.pv_step_bytes.argtypes = [vp, i32, P(ctypes.c_uint64)]
        L.pv_profile_select.argtypes = [vp, i32]
        L.pv_profile_read.argtypes = [vp, P(ctypes.c_double), P(i64), P(ctypes.c_uint64)]
        L.pv_calib_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.pv_calib_read.argtypes = [vp, ctypes.c_size_t, vp, vp]
        L.pv_cache_use_graphs.argtypes = [vp, i32]
        L.pv_strerror.argtypes = [ctypes.c_int]; L.pv_strerror.restype = ctypes.c_char_p
        L.pv_last_error.argtypes = []; L.pv_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(status, where):
    if status != 0:
        L = lib()
        raise PVError(status, where, f"{L.pv_strerror(status).decode()}: {L.pv_last_error().decode()}")


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dev_bytes(n, device):
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=device)


def calib_copy(dst, src, stream=None):
    """Plain copy kernel of known size between two device tensors (counter calibration)."""
    n = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == n and dst.is_cuda and src.is_cuda
    _check(lib().pv_calib_copy(ctypes.c_void_p(dst.data_ptr()), ctypes.c_void_p(src.data_ptr()), n, _stream_ptr(stream)),
           "pv_calib_copy")


def calib_read(src, nbytes=None, offset=0, sink=None, stream=None):
    """Plain read-only stream over `nbytes` bytes of a device tensor, starting `offset` bytes in."""
    total = src.numel() * src.element_size()
    nbytes = total - offset if nbytes is None else nbytes
    assert src.is_cuda and offset % 16 == 0 and nbytes % 16 == 0 and offset + nbytes <= total
    if sink is None:
        sink = torch.zeros(16, dtype=torch.uint8, device=src.device)
    _check(lib().pv_calib_read(ctypes.c_void_p(src.data_ptr() + offset), nbytes, ctypes.c_void_p(sink.data_ptr()),
                               _stream_ptr(stream)), "pv_calib_read")
    return sink


def verify_batch(caches, drafts, stream=None):
    """Blocks of several sequences in one pass over the weights.  caches: Cache objects of one model,
    drafts: one token list per cache.  Returns [(accepted_len, next_token), ...]."""
    n = len(caches)
    assert n == len(drafts) and n >= 1
    ptrs = (ctypes.c_void_p * n)(*[c.h for c in caches])
    gam = np.array([len(d) for d in drafts], dtype=np.int32)
    flat = np.ascontiguousarray(np.concatenate([np.asarray(d, dtype=np.int32) for d in drafts]), dtype=np.int32)
    pre = np.array([len(c) for c in caches], dtype=np.int32)
    acc, nxt = np.empty(n, dtype=np.int32), np.empty(n, dtype=np.int32)
    with caches[0]._dev():
        _check(lib().pv_verify_batch(ptrs, n, pre.ctypes.data, flat.ctypes.data, gam.ctypes.data, acc.ctypes.data, nxt.ctypes.data,
                                     _stream_ptr(stream)), "pv_verify_batch")
    return [(int(a), int(t)) for a, t in zip(acc, nxt)]


class Model:
    """pv_model plus the torch-owned device arena behind it."""

    def __init__(self, shape, max_gamma=16, kernel_path=PATH_AUTO, device="cuda:0"):
        """shape: object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab,
        rms_eps, rope_base, dtype ("f32"|"bf16"), page_tokens and optionally weight_bits (16 | 4)."""
        self.L, self.shape, self.device = lib(), shape, torch.device(device)
        self.cfg = pv_model_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads,
                                   shape.head_dim, shape.ffn_dim, shape.vocab, shape.rms_eps, shape.rope_base,
                                   PV_BF16 if shape.dtype == "bf16" else PV_F32, shape.page_tokens,
                                   max_gamma, kernel_path, 4 if getattr(shape, "weight_bits", 16) == 4 else 16)
        self.weight_bits = self.cfg.weight_bits
        wb, sb = ctypes.c_size_t(), ctypes.c_size_t()
        _check(self.L.pv_model_bytes(ctypes.byref(self.cfg), ctypes.byref(wb), ctypes.byref(sb)), "pv_model_bytes")
        with torch.cuda.device(self.device):
            self.arena = _dev_bytes(wb.value, self.device)
            self.staging = _dev_bytes(sb.value, self.device)
            self.h = ctypes.c_void_p()
            _check(self.L.pv_model_create(ctypes.byref(self.cfg), self.arena.data_ptr(), self.arena.numel(),
                                          self.staging.data_ptr(), self.staging.numel(), ctypes.byref(self.h)),
                   "pv_model_create")
        self.weight_bytes, self.staging_bytes = wb.value, sb.value
        self.np_dtype = np.uint16 if shape.dtype == "bf16" else np.float32

    def load_weights(self, kind, layer, row_begin, rows, stream=None):
        """rows: numpy array [row_count, in_features] (float32, or uint16 bf16 bits) on the host."""
        rows = np.ascontiguousarray(rows)
        assert rows.dtype == self.np_dtype and rows.ndim == 2
        with torch.cuda.device(self.device):
            _check(self.L.pv_load_weights(self.h, KINDS[kind], layer, row_begin, rows.shape[0],
                                          rows.ctypes.data, _stream_ptr(stream)), f"pv_load_weights({kind},{layer})")

    def load_weights_q4(self, kind, layer, row_begin, codes, scales, stream=None):
        """Rows of a matrix of a 4-bit model: codes uint8 [row_count, in_features / 2] (even feature in
        the low nibble), scales uint16 = bf16 bits [row_count, in_features / 32]."""
        codes, scales = np.ascontiguousarray(codes), np.ascontiguousarray(scales)
        assert codes.dtype == np.uint8 and scales.dtype == np.uint16 and codes.shape[0] == scales.shape[0]
        assert codes.shape[1] * 2 == scales.shape[1] * 32
        with torch.cuda.device(self.device):
            _check(self.L.pv_load_weights_q4(self.h, KINDS[kind], layer, row_begin, codes.shape[0], codes.ctypes.data,
                                             scales.ctypes.data, _stream_ptr(stream)), f"pv_load_weights_q4({kind},{layer})")

    def chunk_rows(self, in_features):
        """Largest row count (multiple of 16) whose chunk fits the staging buffer."""
        per_row = in_features * self.np_dtype().itemsize
        return max(16, (self.staging_bytes // per_row) // 16 * 16)

    def close(self):
        if getattr(self, "h", None):
            self.L.pv_model_destroy(self.h); self.h = None

    def __del__(self):
        self.close()


class Cache:
    """pv_cache plus the torch-owned page pool and workspace."""

    def __init__(self, model, max_tokens):
        self.L, self.m = model.L, model
        pb, wb = ctypes.c_size_t(), ctypes.c_size_t()
        _check(self.L.pv_cache_bytes(model.h, max_tokens, ctypes.byref(pb), ctypes.byref(wb)), "pv_cache_bytes")
        with torch.cuda.device(model.device):
            self.pool = _dev_bytes(pb.value, model.device)
            self.ws = _dev_bytes(wb.value, model.device)
            self.h = ctypes.c_void_p()
            _check(self.L.pv_cache_create(model.h, self.pool.data_ptr(), self.pool.numel(), self.ws.data_ptr(),
                                          self.ws.numel(), max_tokens, ctypes.byref(self.h)), "pv_cache_create")
        self.max_tokens = max_tokens

    def _dev(self):
        return torch.cuda.device(self.m.device)

    def set_page_table(self, phys, stream=None):
        a = np.ascontiguousarray(phys, dtype=np.int32)
        with self._dev():
            _check(self.L.pv_cache_set_page_table(self.h, a.ctypes.data, len(a), _stream_ptr(stream)), "pv_cache_set_page_table")

    def prefill(self, tokens, stream=None):
        a = np.ascontiguousarray(tokens, dtype=np.int32)
        with self._dev():
            _check(self.L.pv_prefill(self.h, a.ctypes.data, len(a), _stream_ptr(stream)), "pv_prefill")

    def verify(self, prefix_len, draft, stream=None):
        a = np.ascontiguousarray(draft, dtype=np.int32)
        n, t = ctypes.c_int32(), ctypes.c_int32()
        with self._dev():
            _check(self.L.pv_verify(self.h, prefix_len, a.ctypes.data, len(a), ctypes.byref(n), ctypes.byref(t),
                                    _stream_ptr(stream)), "pv_verify")
        return n.value, t.value

    def verify_async(self, prefix_len, draft, stream=None):
        a = np.ascontiguousarray(draft, dtype=np.int32)
        with self._dev():
            _check(self.L.pv_verify_async(self.h, prefix_len, a.ctypes.data, len(a), _stream_ptr(stream)), "pv_verify_async")

    def verify_tree(self, prefix_len, tokens, parents, stream=None):
        """A draft tree: tokens[i] hangs under node parents[i] (-1: under the prefix).  Returns
        (accepted_len, next_token, path) with path = the accepted nodes in order."""
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        p = np.ascontiguousarray(parents, dtype=np.int32)
        assert len(t) == len(p)
        n, nxt = ctypes.c_int32(), ctypes.c_int32()
        path = np.full(len(t), -1, dtype=np.int32)
        with self._dev():
            _check(self.L.pv_verify_tree(self.h, prefix_len, t.ctypes.data, p.ctypes.data, len(t), ctypes.byref(n), ctypes.byref(nxt),
                                         path.ctypes.data, _stream_ptr(stream)), "pv_verify_tree")
        return n.value, nxt.value, path[:n.value].copy()

    def verify_async_static(self, prefix_len, draft, stream=None):
        """The step without any allocation: per-step buffers in the library's fixed device array."""
        a = np.ascontiguousarray(draft, dtype=np.int32)
        with self._dev():
            _check(self.L.pv_verify_async_static(self.h, prefix_len, a.ctypes.data, len(a), _stream_ptr(stream)), "pv_verify_async_static")

    def verify_wait(self):
        n, t = ctypes.c_int32(), ctypes.c_int32()
        with self._dev():
            _check(self.L.pv_verify_wait(self.h, ctypes.byref(n), ctypes.byref(t)), "pv_verify_wait")
        return n.value, t.value

    def rollback(self, new_len, stream=None):
        with self._dev():
            _check(self.L.pv_rollback(self.h, new_len, _stream_ptr(stream)), "pv_rollback")

    def readmit(self, new_len, pending=-1, stream=None):
        with self._dev():
            _check(self.L.pv_cache_readmit(self.h, new_len, pending, _stream_ptr(stream)), "pv_cache_readmit")

    def set_pending(self, token, stream=None):
        with self._dev():
            _check(self.L.pv_cache_set_pending(self.h, token, _stream_ptr(stream)), "pv_cache_set_pending")

    def state(self):
        n, p = ctypes.c_int32(), ctypes.c_int32()
        _check(self.L.pv_cache_len(self.h, ctypes.byref(n), ctypes.byref(p)), "pv_cache_len")
        return n.value, p.value

    def __len__(self):
        return self.state()[0]

    @property
    def pending(self):
        return self.state()[1]

    def debug_logits(self, stream=None):
        r = ctypes.c_int32()
        with self._dev():
            _check(self.L.pv_debug_logits(self.h, None, ctypes.byref(r), _stream_ptr(stream)), "pv_debug_logits")
            out = np.empty((r.value, self.m.shape.vocab), dtype=np.float32)
            if r.value:
                _check(self.L.pv_debug_logits(self.h, out.ctypes.data, None, _stream_ptr(stream)), "pv_debug_logits")
        return out

    def debug_pred(self, stream=None):
        r = ctypes.c_int32()
        with self._dev():
            _check(self.L.pv_debug_pred(self.h, None, ctypes.byref(r), _stream_ptr(stream)), "pv_debug_pred")
            out = np.empty(r.value, dtype=np.int32)
            if r.value:
                _check(self.L.pv_debug_pred(self.h, out.ctypes.data, None, _stream_ptr(stream)), "pv_debug_pred")
        return out

    def export(self, stream=None):
        s = self.m.shape
        out = np.empty((s.n_layers, 2, len(self), s.n_kv_heads * s.head_dim), dtype=self.m.np_dtype)
        if out.size:
            with self._dev():
                _check(self.L.pv_cache_export(self.h, out.ctypes.data, out.nbytes, _stream_ptr(stream)), "pv_cache_export")
        return out

    def step_bytes(self, gamma):
        b = ctypes.c_uint64()
        _check(self.L.pv_step_bytes(self.h, gamma, ctypes.byref(b)), "pv_step_bytes")
        return b.value

    def profile_select(self, which):
        _check(self.L.pv_profile_select(self.h, which), "pv_profile_select")

    def use_graphs(self, enable):
        _check(self.L.pv_cache_use_graphs(self.h, 1 if enable else 0), "pv_cache_use_graphs")

    def profile_read(self):
        ms, n, b = ctypes.c_double(), ctypes.c_int64(), ctypes.c_uint64()
        _check(self.L.pv_profile_read(self.h, ctypes.byref(ms), ctypes.byref(n), ctypes.byref(b)), "pv_profile_read")
        return ms.value, n.value, b.value

    def close(self):
        if self.h:
            self.L.pv_cache_destroy(self.h); self.h = None

    def __del__(self):
        self.close()
