"""ctypes wrapper around the C oracle (ref_decoder.c).  Test infrastructure only.

RefModel borrows numpy arrays (float32, or uint16 bfloat16 bit patterns) as weights;
RefCache is one sequence's key/value cache plus the carried `pending` token.
"""
import ctypes
import os
import numpy as np

from . import build as _build

KINDS = {"embed": 0, "attn_norm": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5,
         "ffn_norm": 6, "wg": 7, "wu": 8, "wd": 9, "final_norm": 10, "lm_head": 11}
KV_REAL, KV_BF16, KV_F32 = 0, 1, 2


class _Cfg(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "ffn_dim", "vocab")] + \
               [("rms_eps", ctypes.c_double), ("rope_base", ctypes.c_double)]


_libs = {}


def load(real="f64"):
    if real not in _libs:
        path = _build.lib_path(real)
        if not os.path.exists(path):
            _build.build(force=False)
        lib = ctypes.CDLL(path)
        vp, i32, ip = ctypes.c_void_p, ctypes.c_int, ctypes.POINTER(ctypes.c_int32)
        lib.ref_model_new.restype = vp
        lib.ref_model_new.argtypes = [ctypes.POINTER(_Cfg)]
        lib.ref_model_free.argtypes = [vp]
        lib.ref_model_set_tensor.argtypes = [vp, i32, i32, vp, i32]
        lib.ref_cache_new.restype = vp
        lib.ref_cache_new.argtypes = [vp, i32, i32]
        lib.ref_cache_free.argtypes = [vp]
        lib.ref_cache_len.argtypes = [vp]
        lib.ref_truncate.argtypes = [vp, i32]
        lib.ref_cache_export.argtypes = [vp, vp]
        lib.ref_decode_one.argtypes = [vp, i32, vp]
        lib.ref_forward_block.argtypes = [vp, vp, i32, vp, i32]
        lib.ref_verify.argtypes = [vp, i32, vp, i32, ip, ip, ip, vp, vp]
        lib.ref_embed_block.argtypes = [vp, vp, i32, vp]
        lib.ref_layer_block.argtypes = [vp, i32, i32, vp, i32]
        lib.ref_head_block.argtypes = [vp, vp, i32, vp]
        lib.ref_cache_set_len.argtypes = [vp, i32]
        lib.ref_rmsnorm.argtypes = [vp, vp, i32, ctypes.c_double, vp]
        lib.ref_linear.argtypes = [vp, i32, vp, i32, i32, vp]
        lib.ref_rope.argtypes = [vp, i32, i32, ctypes.c_double]
        rt = ctypes.c_double if real == "f64" else ctypes.c_float
        lib.ref_silu.argtypes = [rt]
        lib.ref_silu.restype = rt
        lib.ref_store_round.argtypes = [rt, i32]
        lib.ref_store_round.restype = rt
        _libs[real] = lib
    return _libs[real]


class _Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("dtype", ctypes.c_int)]


def _np_real(real):
    return np.float64 if real == "f64" else np.float32


def _as_tensor(arr):
    arr = np.ascontiguousarray(arr)
    assert arr.dtype in (np.float32, np.uint16)
    return arr, _Tensor(arr.ctypes.data, 1 if arr.dtype == np.uint16 else 0)


# ---- single pieces, for pin tests ----
def rmsnorm(x, g, eps, real="f64"):
    lib, rt = load(real), _np_real(real)
    x = np.ascontiguousarray(x, dtype=rt); y = np.empty_like(x)
    ga, gt = _as_tensor(g)
    lib.ref_rmsnorm(x.ctypes.data, ctypes.addressof(gt), x.shape[-1], eps, y.ctypes.data)
    return y


def linear(x, W, real="f64"):
    lib, rt = load(real), _np_real(real)
    x = np.ascontiguousarray(np.atleast_2d(x), dtype=rt)
    Wa, Wt = _as_tensor(W)
    y = np.empty((x.shape[0], Wa.shape[0]), dtype=rt)
    lib.ref_linear(x.ctypes.data, x.shape[0], ctypes.addressof(Wt), Wa.shape[0], Wa.shape[1], y.ctypes.data)
    return y


def rope(v, pos, base, real="f64"):
    lib, rt = load(real), _np_real(real)
    v = np.array(v, dtype=rt, copy=True)
    lib.ref_rope(v.ctypes.data, v.shape[0], pos, base)
    return v


def silu(z, real="f64"):
    return load(real).ref_silu(z)


def store_round(v, kv_store, real="f64"):
    """What the cache keeps of a key/value element v under storage mode kv_store."""
    return load(real).ref_store_round(v, kv_store)


def dequant_q4(codes, scales):
    """Weights of a 4-bit matrix as float32 (exact): w[r, k] = (code[r, k] - 8) * scale[r, k // 32].
    codes: uint8 [rows, cols/2], two codes per byte, the even input feature in the low nibble;
    scales: bf16 bit patterns [rows, cols/32].  (The paper runs its 70B model in 4 bit, Sec. 4.1,
    without naming a format; this is the group-wise symmetric one the build settled on.)"""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    rows, half = codes.shape
    c = np.empty((rows, 2 * half), dtype=np.int32)
    c[:, 0::2] = codes & 15
    c[:, 1::2] = codes >> 4
    s = (np.ascontiguousarray(scales, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)
    assert s.shape == (rows, 2 * half // 32)
    w = (c - 8).astype(np.float32).reshape(rows, -1, 32) * s[:, :, None]
    return np.ascontiguousarray(w.reshape(rows, 2 * half))


class RefModel:
    def __init__(self, shape, real="f64"):
        """shape: any object with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, ffn_dim, vocab,
        rms_eps, rope_base attributes."""
        self.lib, self.real, self.shape = load(real), real, shape
        cfg = _Cfg(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                   shape.ffn_dim, shape.vocab, shape.rms_eps, shape.rope_base)
        self.h = self.lib.ref_model_new(ctypes.byref(cfg))
        self._keep = {}

    def set_tensor(self, kind, layer, arr):
        arr = np.ascontiguousarray(arr)
        assert arr.dtype in (np.float32, np.uint16)
        self._keep[(kind, layer)] = arr
        rc = self.lib.ref_model_set_tensor(self.h, KINDS[kind], layer, arr.ctypes.data,
                                           1 if arr.dtype == np.uint16 else 0)
        assert rc == 0

    def drop_tensor(self, kind, layer):
        """Forget a borrowed array (the model must not be asked for that tensor again)."""
        self._keep.pop((kind, layer), None)
        self.lib.ref_model_set_tensor(self.h, KINDS[kind], layer, None, 0)

    def embed_block(self, tokens):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        X = np.empty((len(t), self.shape.d_model), dtype=_np_real(self.real))
        assert self.lib.ref_embed_block(self.h, t.ctypes.data, len(t), X.ctypes.data) == 0
        return X

    def head_block(self, X):
        X = np.ascontiguousarray(X, dtype=_np_real(self.real))
        logits = np.empty((X.shape[0], self.shape.vocab), dtype=X.dtype)
        assert self.lib.ref_head_block(self.h, X.ctypes.data, X.shape[0], logits.ctypes.data) == 0
        return logits

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.ref_model_free(self.h); self.h = None


class RefCache:
    def __init__(self, model, max_tokens, kv_store=KV_REAL):
        self.m, self.lib, self.max_tokens = model, model.lib, max_tokens
        self.rt = _np_real(model.real)
        self.h = self.lib.ref_cache_new(model.h, max_tokens, kv_store)
        self.pending = -1

    def __len__(self):
        return self.lib.ref_cache_len(self.h)

    def decode_one(self, token):
        logits = np.empty(self.m.shape.vocab, dtype=self.rt)
        assert self.lib.ref_decode_one(self.h, int(token), logits.ctypes.data) == 0
        self.pending = -1
        return logits

    def forward_block(self, tokens, only_last=False, want_logits=True):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        logits = None
        if want_logits:
            logits = np.empty((1 if only_last else len(t), self.m.shape.vocab), dtype=self.rt)
        rc = self.lib.ref_forward_block(self.h, t.ctypes.data, len(t),
                                        logits.ctypes.data if want_logits else None, int(only_last))
        assert rc == 0
        self.pending = -1
        return logits

    def layer_block(self, layer, T, X):
        """Layer `layer` over the rows X (in place) at positions T .. T+len(X)-1; length untouched."""
        assert X.dtype == self.rt and X.flags.c_contiguous and X.ndim == 2
        assert self.lib.ref_layer_block(self.h, layer, T, X.ctypes.data, X.shape[0]) == 0

    def set_len(self, n):
        assert self.lib.ref_cache_set_len(self.h, n) == 0
        self.pending = -1

    def prefill(self, tokens, chunk=64):
        """Append the prompt; sets pending = greedy token after the prompt. Returns last-row logits."""
        tokens = np.asarray(tokens, dtype=np.int32)
        last = None
        for s in range(0, len(tokens), chunk):
            blk = tokens[s:s + chunk]
            is_last = s + chunk >= len(tokens)
            last = self.forward_block(blk, only_last=True, want_logits=is_last)
        self.pending = int(np.argmax(last[0]))
        return last[0]

    def verify(self, prefix_len, draft, want_logits=False):
        d = np.ascontiguousarray(draft, dtype=np.int32)
        g = len(d)
        pend, acc, nxt = ctypes.c_int32(self.pending), ctypes.c_int32(), ctypes.c_int32()
        pred = np.empty(g, dtype=np.int32)
        logits = np.empty((g, self.m.shape.vocab), dtype=self.rt) if want_logits else None
        rc = self.lib.ref_verify(self.h, prefix_len, d.ctypes.data, g, ctypes.byref(pend), ctypes.byref(acc),
                                 ctypes.byref(nxt), pred.ctypes.data,
                                 logits.ctypes.data if want_logits else None)
        if rc != 0:
            raise ValueError("ref_verify: bad argument or prefix_len != cache length")
        self.pending = pend.value
        return acc.value, nxt.value, pred, logits

    def rollback(self, new_len):
        if self.lib.ref_truncate(self.h, new_len) != 0:
            raise ValueError("rollback: new_len out of range")
        self.pending = -1

    def export(self):
        s = self.m.shape
        out = np.empty((s.n_layers, 2, len(self), s.n_kv_heads * s.head_dim), dtype=self.rt)
        self.lib.ref_cache_export(self.h, out.ctypes.data)
        return out

    def __del__(self):
        if getattr(self, "h", None):
            self.lib.ref_cache_free(self.h); self.h = None
