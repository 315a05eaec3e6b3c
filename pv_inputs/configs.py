"""Workload shape tables: the synthetic LLaMA-shaped verifiers the benchmarks and tests use.

The paper evaluates LLaMA-2 / LLaMA-3 checkpoints on public summarisation and code
prompts (Sec. 4.1); neither is available offline, so random weights of the same
public shapes and uniform-random prompts stand in for them.
"""
from dataclasses import dataclass, asdict

# tensor kinds: numbering is part of the library boundary (pv_tensor_kind)
TENSOR_KINDS = {
    "embed": 0, "attn_norm": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5,
    "ffn_norm": 6, "wg": 7, "wu": 8, "wd": 9, "final_norm": 10, "lm_head": 11,
}
PER_LAYER = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd")
GLOBAL = ("embed", "final_norm", "lm_head")


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn_dim: int
    vocab: int
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    dtype: str = "bf16"          # storage type of weights and KV cache: "f32" | "bf16"
    page_tokens: int = 16
    seed: int = 1000
    weight_bits: int = 16        # 16: matrices stored in `dtype`; 4: projection matrices and LM head as 4-bit codes + bf16 group scales

    def replace(self, **kw):
        d = asdict(self)
        d.update(kw)
        return ModelShape(**d)

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def n_params(self):
        per_layer = sum(_numel(tensor_shape(self, k)) for k in PER_LAYER)
        return self.n_layers * per_layer + sum(_numel(tensor_shape(self, k)) for k in GLOBAL)

    def streamed_bytes(self):
        """Bytes of weights one verify step must read: everything except the embedding table."""
        eb = 2 if self.dtype == "bf16" else 4
        if self.weight_bits == 4:
            mats = sum(_numel(tensor_shape(self, k)) for k in PER_LAYER if len(tensor_shape(self, k)) == 2) * self.n_layers
            mats += _numel(tensor_shape(self, "lm_head"))
            gains = self.n_params() - _numel(tensor_shape(self, "embed")) - mats
            return mats * 9 // 16 + gains * eb           # 4 bits + one bf16 scale per 32 weights = 4.5 bits
        return (self.n_params() - _numel(tensor_shape(self, "embed"))) * eb

    def kv_bytes_per_token(self):
        eb = 2 if self.dtype == "bf16" else 4
        return self.n_layers * 2 * self.kv_dim * eb


def _numel(shape):
    n = 1
    for s in shape:
        n *= s
    return n


def tensor_shape(m: ModelShape, kind: str):
    """Logical shape, [out_features, in_features] row-major for matrices (y = x @ W.T)."""
    d, F, V = m.d_model, m.ffn_dim, m.vocab
    return {
        "embed": (V, d), "attn_norm": (d,), "wq": (m.q_dim, d), "wk": (m.kv_dim, d),
        "wv": (m.kv_dim, d), "wo": (d, m.q_dim), "ffn_norm": (d,), "wg": (F, d),
        "wu": (F, d), "wd": (d, F), "final_norm": (d,), "lm_head": (V, d),
    }[kind]


def tensor_id(kind: str, layer: int) -> int:
    """Stream id of one tensor for the counter-based generator (layer = -1 for globals)."""
    return (layer + 1) * 16 + TENSOR_KINDS[kind]


# The five benchmark configurations (index = position in the baseline's config list).
CONFIGS = {
    "tiny": ModelShape("tiny", 2, 256, 4, 4, 64, 688, 1024, dtype="f32", seed=1000),
    "7b": ModelShape("7b", 32, 4096, 32, 32, 128, 11008, 32000, seed=1001),
    "8b": ModelShape("8b", 32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0, seed=1002),
    "70b": ModelShape("70b", 80, 8192, 64, 8, 128, 28672, 32000, seed=1003),
    "1b": ModelShape("1b", 16, 2048, 32, 8, 64, 8192, 128256, rope_base=500000.0, seed=1004),
    "70b_v128k": ModelShape("70b_v128k", 80, 8192, 64, 8, 128, 28672, 128256,
                            rope_base=500000.0, seed=1005),
    # 4-bit variants of the verifier shapes (the paper runs its 70B model in 4 bit, Sec. 4.1)
    "70b_q4": ModelShape("70b_q4", 80, 8192, 64, 8, 128, 28672, 32000, seed=1003, weight_bits=4),
    "8b_q4": ModelShape("8b_q4", 32, 4096, 32, 8, 128, 14336, 128256, rope_base=500000.0, seed=1002, weight_bits=4),
    "70b_v128k_q4": ModelShape("70b_v128k_q4", 80, 8192, 64, 8, 128, 28672, 128256, rope_base=500000.0, seed=1005, weight_bits=4),
}
