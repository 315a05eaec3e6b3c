"""Counter-based seeded draws: weight tensors, prompt tokens, draft perturbations.

value(seed, tensor, i) = table[h >> 48] with h a two-round splitmix64 hash of
(seed, tensor, i) and `table` 65536 quantiles of N(0, sigma^2) taken at
(k + 1/2) / 65536 in double precision and then rounded to the storage type.
Tensors are produced piece by piece, so neither consumer ever needs a whole
model in host memory.  A small C library does the bulk fill; a numpy fallback
computes the same bits.
"""
import ctypes
import os
import subprocess
import numpy as np

from .configs import ModelShape, PER_LAYER, GLOBAL, tensor_shape, tensor_id

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpvsynth.so")
_lib = None
_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)


def build(force=True):
    """Compile synth.c into libpvsynth.so (gcc, OpenMP)."""
    global _lib
    if force or not os.path.exists(_LIB_PATH):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH,
                               os.path.join(_HERE, "synth.c")])
    _lib = None
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None and os.path.exists(_LIB_PATH):
        lib = ctypes.CDLL(_LIB_PATH)
        u64, vp = ctypes.c_uint64, ctypes.c_void_p
        lib.pvs_fill_table.argtypes = [u64, u64, u64, u64, vp, ctypes.c_int, vp]
        lib.pvs_fill_table.restype = ctypes.c_int
        lib.pvs_quantize_q4.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, vp, vp]
        lib.pvs_quantize_q4.restype = ctypes.c_int
        _lib = lib
    return _lib


def _mix64(z):
    z = z ^ (z >> np.uint64(30)); z = z * _M1
    z = z ^ (z >> np.uint64(27)); z = z * _M2
    return z ^ (z >> np.uint64(31))


def _stream_key(seed, stream):
    with np.errstate(over="ignore"):
        s = np.array([stream], dtype=np.uint64)
        return _mix64(np.uint64(seed) ^ _mix64(s + _GOLDEN))[0]


def _draw(seed, stream, start, count):
    with np.errstate(over="ignore"):
        key = _stream_key(seed, stream)
        i = np.arange(start, start + count, dtype=np.uint64)
        return _mix64(key + i * _GOLDEN)


def bf16_round_f32(x):
    """Round float32 array to the nearest bfloat16 (ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


_tables = {}


def quantile_table(dtype: str, sigma: float = 0.02):
    """65536 N(0, sigma^2) quantiles in the storage type: float32 array or bf16 bit patterns (uint16)."""
    key = (dtype, sigma)
    if key not in _tables:
        from scipy.special import ndtri
        q = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0) * sigma
        f = q.astype(np.float32)
        _tables[key] = bf16_round_f32(f) if dtype == "bf16" else f
    return _tables[key]


def fill_tensor(m: ModelShape, kind: str, layer: int, start: int = 0, count: int = None,
                gains: str = "ones", use_c: bool = True, out=None):
    """Flat slice [start, start+count) of one tensor in storage type (uint16 bf16 bits or float32).

    Norm gains are 1.0 ("ones") or 1 + N(0, 0.02^2) draws ("perturbed", used by tests so that a
    dropped gain is visible); every matrix is N(0, 0.02^2).
    """
    shape = tensor_shape(m, kind)
    n = int(np.prod(shape))
    if count is None:
        count = n - start
    assert 0 <= start and start + count <= n
    table = quantile_table(m.dtype)
    is_gain = len(shape) == 1
    if is_gain and gains == "ones":
        one = np.float32(1.0)
        return (np.full(count, bf16_round_f32(np.array([one]))[0], dtype=np.uint16)
                if m.dtype == "bf16" else np.full(count, one, dtype=np.float32))
    if out is None:
        out = np.empty(count, dtype=table.dtype)
    else:                       # caller-owned scratch (reused between calls: no fresh page faults)
        assert out.dtype == table.dtype and out.size >= count and out.flags.c_contiguous
        out = out.reshape(-1)[:count]
    lib = _load() if use_c else None
    if lib is not None:
        rc = lib.pvs_fill_table(m.seed, tensor_id(kind, layer), start, count,
                                table.ctypes.data, table.itemsize, out.ctypes.data)
        assert rc == 0
    else:
        out[:] = table[(_draw(m.seed, tensor_id(kind, layer), start, count) >> np.uint64(48)).astype(np.int64)]
    if is_gain:  # perturbed gains: 1 + draw
        f = bf16_bits_to_f32(out) if m.dtype == "bf16" else out
        f = (np.float32(1.0) + f).astype(np.float32)
        out = bf16_round_f32(f) if m.dtype == "bf16" else f
    return out


def iter_tensors(m: ModelShape):
    """Yield (kind, layer) for every tensor of the model; layer = -1 for the three global ones."""
    yield "embed", -1
    for l in range(m.n_layers):
        for k in PER_LAYER:
            yield k, l
    yield "final_norm", -1
    yield "lm_head", -1


def uniform_tokens(seed: int, n: int, vocab: int, stream: int = 0):
    """n uniform token ids in [0, vocab)."""
    return (_draw(seed, stream, 0, n) % np.uint64(vocab)).astype(np.int32)


def unit_draws(seed: int, n: int, stream: int = 0, start: int = 0):
    """n doubles uniform in [0, 1)."""
    return (_draw(seed, stream, start, n) >> np.uint64(11)).astype(np.float64) / 9007199254740992.0


def perturb_drafts(tokens, alpha: float, vocab: int, seed: int, step: int):
    """Replace each position independently, with probability 1 - alpha, by a uniform token id.

    `tokens` is the block the verifier itself would produce; the result is the synthetic
    draft block.  Draw streams are keyed by the step index so any step can be regenerated.
    """
    tokens = np.asarray(tokens, dtype=np.int32)
    n = len(tokens)
    u = unit_draws(seed, n, stream=2 * step + 1)
    r = uniform_tokens(seed, n, vocab, stream=2 * step + 2)
    return np.where(u < (1.0 - alpha), r, tokens).astype(np.int32)


def iter_row_chunks(m: ModelShape, kind: str, layer: int, max_rows: int, gains: str = "ones", scratch=None):
    """Yield (row_begin, rows[row_count, in_features]) pieces of one tensor, at most max_rows rows each.

    With `scratch` (a flat array of the storage type, >= max_rows * in_features elements) every
    piece is written into that same buffer, so a piece is only valid until the next one is drawn."""
    shape = tensor_shape(m, kind)
    rows, cols = (1, shape[0]) if len(shape) == 1 else shape
    is_gain = len(shape) == 1
    for r0 in range(0, rows, max_rows):
        n = min(max_rows, rows - r0)
        buf = None if (scratch is None or is_gain) else scratch
        yield r0, fill_tensor(m, kind, layer, start=r0 * cols, count=n * cols, gains=gains, out=buf).reshape(n, cols)


# ---- 4-bit weight format: input preparation (the stand-in for a 4-bit checkpoint) ----

Q4_GROUP = 32


def quantize_q4(w_bits, use_native=True):
    """bf16 bit patterns [rows, cols] (cols % 32 == 0) -> (codes uint8 [rows, cols/2], scales
    uint16 = bf16 bits [rows, cols/32]).  Per group of 32 input features: scale = bf16(max|w| / 7)
    (1.0 for an all-zero group), code = clamp(rint(w / scale) + 8, 0, 15), two codes per byte with
    the even feature in the low nibble.  The weight a 4-bit model uses is (code - 8) * scale."""
    w_bits = np.ascontiguousarray(w_bits, dtype=np.uint16)
    rows, cols = w_bits.shape
    assert cols % Q4_GROUP == 0
    lib = _load() if use_native else None
    codes = np.empty((rows, cols // 2), dtype=np.uint8)
    scales = np.empty((rows, cols // Q4_GROUP), dtype=np.uint16)
    if lib is not None:
        rc = lib.pvs_quantize_q4(w_bits.ctypes.data, rows, cols, codes.ctypes.data, scales.ctypes.data)
        assert rc == 0
        return codes, scales
    v = bf16_bits_to_f32(w_bits).reshape(rows, cols // Q4_GROUP, Q4_GROUP)
    m = np.abs(v).max(axis=2)
    sbits = bf16_round_f32((m / np.float32(7.0)).astype(np.float32))
    sb = bf16_bits_to_f32(sbits)
    dead = ~(sb > 0)
    sbits = np.where(dead, np.uint16(0x3F80), sbits).astype(np.uint16)
    sb = np.where(dead, np.float32(1.0), sb).astype(np.float32)
    c = np.clip(np.rint(v / sb[:, :, None]).astype(np.int32) + 8, 0, 15).astype(np.uint8).reshape(rows, cols)
    codes[:] = c[:, 0::2] | (c[:, 1::2] << 4)
    scales[:] = sbits
    return codes, scales


Q4_KINDS = ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "lm_head")      # matrices a 4-bit model stores as codes + scales


def iter_row_chunks_q4(m: ModelShape, kind: str, layer: int, max_rows: int, scratch=None):
    """Like iter_row_chunks for a matrix of a 4-bit model: yields (row_begin, codes, scales)."""
    assert kind in Q4_KINDS
    for r0, rows in iter_row_chunks(m, kind, layer, max_rows, scratch=scratch):
        codes, scales = quantize_q4(rows)
        yield r0, codes, scales
