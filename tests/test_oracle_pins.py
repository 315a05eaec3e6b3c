"""Pins for the CPU oracle: closed forms, library routines, special cases, invariants.

The oracle is the yardstick for the GPU path, so it is itself checked here against things
it does not define: closed-form values, torch/numpy library routines, degenerate models
whose output has a one-line formula, brute force (block forward == sequential decodes),
and the invariants the method guarantees (greedy acceptance is lossless, rollback restores
the cache, accepted lengths of i.i.d. perturbed drafts are truncated-geometric).
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import pv_inputs
from pv_inputs import CONFIGS
from oracle import ref, ratecheck
from helpers import ref_model, tensors_f64, greedy_continuation, draft_block

TINY = CONFIGS["tiny"]
# a small grouped-query shape with bf16 storage, odd sizes on purpose
GQA = pv_inputs.ModelShape("gqa_small", 3, 128, 8, 2, 32, 176, 512, rope_base=500000.0,
                           dtype="bf16", seed=4242)


# ---------------- single pieces ----------------

def test_rmsnorm_constant_vector_closed_form():
    d, c, eps = 256, 3.0, 1e-5
    g = np.linspace(0.5, 1.5, d).astype(np.float32)
    y = ref.rmsnorm(np.full(d, c), g, eps)
    assert np.allclose(y, g.astype(np.float64) * c / math.sqrt(c * c + eps), rtol=1e-14)


def test_rmsnorm_matches_library_routine():
    rng = np.random.default_rng(0)
    x = rng.normal(size=300)
    g = rng.normal(size=300).astype(np.float32)
    want = F.rms_norm(torch.tensor(x), (300,), torch.tensor(g, dtype=torch.float64), eps=1e-5).numpy()
    assert np.allclose(ref.rmsnorm(x, g, 1e-5), want, rtol=1e-13, atol=1e-15)


def test_linear_is_x_times_w_transposed():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(3, 70))
    W = rng.normal(size=(11, 70)).astype(np.float32)
    assert np.allclose(ref.linear(x, W), x @ W.astype(np.float64).T, rtol=1e-13)
    Wb = pv_inputs.bf16_round_f32(W)
    assert np.allclose(ref.linear(x, Wb), x @ pv_inputs.bf16_bits_to_f32(Wb).astype(np.float64).T, rtol=1e-13)


def test_rope_closed_forms():
    hd, base = 64, 10000.0
    rng = np.random.default_rng(2)
    v = rng.normal(size=hd)
    assert np.array_equal(ref.rope(v, 0, base), v)                      # position 0: identity
    for pos in (1, 17, 2055):
        r = ref.rope(v, pos, base)
        # each (i, i + hd/2) pair is rotated: its norm is unchanged
        assert np.allclose(r[:32] ** 2 + r[32:] ** 2, v[:32] ** 2 + v[32:] ** 2, rtol=1e-12)
    # unit vector on coordinate i turns into (cos, sin) of pos * base^(-2i/hd) on coordinates (i, i+hd/2)
    for i in (0, 5, 31):
        e = np.zeros(hd); e[i] = 1.0
        r = ref.rope(e, 7, base)
        ang = 7 * base ** (-2.0 * i / hd)
        want = np.zeros(hd); want[i] = math.cos(ang); want[i + 32] = math.sin(ang)
        assert np.allclose(r, want, atol=1e-15)
    # scores depend on the position difference only
    q, k = rng.normal(size=hd), rng.normal(size=hd)
    s1 = ref.rope(q, 40, base) @ ref.rope(k, 33, base)
    s2 = ref.rope(q, 1007, base) @ ref.rope(k, 1000, base)
    assert abs(s1 - s2) < 1e-10


def test_silu_values():
    assert ref.silu(0.0) == 0.0
    for z in (-4.0, -0.3, 0.7, 5.5):
        assert abs(ref.silu(z) - float(F.silu(torch.tensor(z, dtype=torch.float64)))) < 1e-15
    assert abs(ref.silu(30.0) - 30.0) < 1e-10 and abs(ref.silu(-30.0)) < 1e-10


# ---------------- whole decoder ----------------

def _torch_forward(shape, W, tokens):
    """The decoder written with library routines (fp64): rms_norm, matmul, SDPA, silu."""
    t = lambda a: torch.tensor(a, dtype=torch.float64)
    n, hd, Hq, Hkv = len(tokens), shape.head_dim, shape.n_q_heads, shape.n_kv_heads
    x = t(W[("embed", -1)])[torch.tensor(tokens, dtype=torch.long)]
    pos = torch.arange(n, dtype=torch.float64)
    inv = torch.tensor([shape.rope_base ** (-2.0 * i / hd) for i in range(hd // 2)], dtype=torch.float64)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[None], torch.sin(ang)[None]          # [1, n, hd/2]

    def rot(v):                                                    # v: [H, n, hd]
        a, b = v[..., : hd // 2], v[..., hd // 2:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], dim=-1)

    for l in range(shape.n_layers):
        h = F.rms_norm(x, (shape.d_model,), t(W[("attn_norm", l)]), eps=shape.rms_eps)
        q = (h @ t(W[("wq", l)]).T).view(n, Hq, hd).transpose(0, 1)
        k = (h @ t(W[("wk", l)]).T).view(n, Hkv, hd).transpose(0, 1)
        v = (h @ t(W[("wv", l)]).T).view(n, Hkv, hd).transpose(0, 1)
        q, k = rot(q), rot(k)
        k = k.repeat_interleave(Hq // Hkv, dim=0)
        v = v.repeat_interleave(Hq // Hkv, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        x = x + o.transpose(0, 1).reshape(n, Hq * hd) @ t(W[("wo", l)]).T
        h = F.rms_norm(x, (shape.d_model,), t(W[("ffn_norm", l)]), eps=shape.rms_eps)
        x = x + (F.silu(h @ t(W[("wg", l)]).T) * (h @ t(W[("wu", l)]).T)) @ t(W[("wd", l)]).T
    h = F.rms_norm(x, (shape.d_model,), t(W[("final_norm", -1)]), eps=shape.rms_eps)
    return (h @ t(W[("lm_head", -1)]).T).numpy()


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["tiny_mha_f32", "gqa_bf16"])
def test_block_forward_matches_library_routines(shape):
    toks = pv_inputs.uniform_tokens(7, 21, shape.vocab)
    m = ref_model(shape, gains="perturbed")
    c = ref.RefCache(m, 64)
    got = c.forward_block(toks)
    want = _torch_forward(shape, tensors_f64(shape, gains="perturbed"), toks)
    assert np.abs(got - want).max() < 1e-11


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["tiny_mha_f32", "gqa_bf16"])
@pytest.mark.parametrize("kv_store", [ref.KV_REAL, ref.KV_BF16])
def test_block_equals_sequential_decodes(shape, kv_store):
    """A gamma-row block forward equals gamma one-token decodes (brute force)."""
    m = ref_model(shape, gains="perturbed")
    toks = pv_inputs.uniform_tokens(11, 30, shape.vocab)
    a, b = ref.RefCache(m, 64, kv_store), ref.RefCache(m, 64, kv_store)
    seq = np.stack([a.decode_one(t) for t in toks])
    b.forward_block(toks[:19], want_logits=False)
    blk = b.forward_block(toks[19:])                 # 11 rows on top of a 19-token cache
    assert np.abs(seq[19:] - blk).max() < 1e-11
    assert np.array_equal(a.export(), b.export()) or np.abs(a.export() - b.export()).max() < 1e-12


def test_cache_store_rounding_is_round_to_nearest_even():
    """The oracle rounds K/V on store to the cache's storage type; every bf16 comparison with the
    GPU rests on that rounding, so it is pinned to torch's own float32 -> bfloat16 conversion
    (round to nearest, ties to even), bit for bit: hand-picked ties, neighbours of ties, signs,
    tiny and huge magnitudes, and a large random set.  A truncating store fails on the first tie."""
    def want_bf16(vals):
        t = torch.tensor(np.asarray(vals, dtype=np.float64)).to(torch.float32).to(torch.bfloat16)
        return t.to(torch.float64).numpy()

    def want_f32(vals):
        return np.asarray(vals, dtype=np.float64).astype(np.float32).astype(np.float64)

    u = 2.0 ** -7                                   # spacing of bfloat16 in [1, 2)
    ties = [1 + u / 2, 1 + 3 * u / 2, 1 + 5 * u / 2, -(1 + u / 2), -(1 + 3 * u / 2),      # exact halves: to even
            1 + u / 2 + 2.0 ** -23, 1 + u / 2 - 2.0 ** -23, 1 + 3 * u / 2 - 2.0 ** -23,   # float32 neighbours of a half
            2 - u / 2, 0.0, -0.0, 1.0, 0.02, -0.02, 3.0e-39, 1e-30, 6.5e4, 3.0e38, float("inf"), -float("inf")]
    rng = np.random.default_rng(11)
    rand = np.concatenate([rng.normal(size=20000) * 0.5, rng.normal(size=2000) * 1e-3,
                           (rng.integers(0, 2 ** 31 - 2 ** 24, size=20000, dtype=np.int64).astype(np.uint32)).view(np.float32).astype(np.float64)])
    vals = np.concatenate([np.array(ties), rand])
    got = np.array([ref.store_round(float(v), ref.KV_BF16) for v in vals])
    assert np.array_equal(got.view(np.uint64), want_bf16(vals).view(np.uint64))
    assert got[0] == 1.0 and got[1] == 1 + 2 * u and got[2] == 1 + 2 * u       # the ties went to the even neighbour
    got32 = np.array([ref.store_round(float(v), ref.KV_F32) for v in vals])
    assert np.array_equal(got32.view(np.uint64), want_f32(vals).view(np.uint64))
    assert all(ref.store_round(float(v), ref.KV_REAL) == v for v in vals[:200])
    assert math.isnan(ref.store_round(float("nan"), ref.KV_BF16))


@pytest.mark.parametrize("shape", [TINY, GQA], ids=["tiny_mha_f32", "gqa_bf16"])
def test_stored_kv_is_the_rounded_exact_kv(shape):
    """Layer 0's keys and values depend on nothing that was stored before, so what a rounding cache
    exports for layer 0 must be torch's conversion of what the exact cache exports, bit for bit;
    the layers above see the rounded keys and values and may differ, but only by rounding."""
    toks = pv_inputs.uniform_tokens(31, 24, shape.vocab)
    rm = ref_model(shape, gains="perturbed")
    exact = ref.RefCache(rm, 32, ref.KV_REAL); exact.forward_block(toks, want_logits=False)
    e = exact.export()
    for mode, conv in ((ref.KV_BF16, torch.bfloat16), (ref.KV_F32, torch.float32)):
        c = ref.RefCache(rm, 32, mode); c.forward_block(toks[:10], want_logits=False)
        for t in toks[10:]:
            c.decode_one(t)                                   # both forward routines store through the same rounding
        got = c.export()
        want0 = torch.tensor(e[0]).to(torch.float32).to(conv).to(torch.float64).numpy()
        assert np.array_equal(got[0], want0)
        assert np.array_equal(got, torch.tensor(got).to(torch.float32).to(conv).to(torch.float64).numpy())   # every stored value is representable
        assert np.abs(got - e).max() < (2.0 ** -6 if mode == ref.KV_BF16 else 1e-6) * np.abs(e).max()


def test_f32_oracle_build_close_to_f64():
    m64, m32 = ref_model(TINY, real="f64"), ref_model(TINY, real="f32")
    toks = pv_inputs.uniform_tokens(5, 40, TINY.vocab)
    l64 = ref.RefCache(m64, 64).forward_block(toks)
    l32 = ref.RefCache(m32, 64).forward_block(toks)
    assert np.abs(l64 - l32).max() < 1e-5           # block == sequential bar of the fp32 decoder
    seq32 = ref.RefCache(m32, 64)
    s = np.stack([seq32.decode_one(t) for t in toks])
    assert np.abs(s - l32).max() < 1e-5


def test_bf16_cache_amplifies_arithmetic_differences_with_depth():
    """Two runs of a deep model that differ only in rounding (the oracle in fp32 and in fp64) stay within fp32 rounding
    of each other with an unrounded cache, but not with the bf16 one: a K/V element whose two values fall on different
    sides of a rounding boundary is stored one bf16 step (0.4 %) apart, and that is noise on the layers above.  The
    flip rate grows with the layer and the logits end up two orders of magnitude further apart: the reason why the
    end-to-end bars of the deep shapes are wider than the arithmetic of either side, and grow with depth."""
    deep = pv_inputs.ModelShape("deep_narrow", 40, 256, 4, 2, 64, 704, 2048, rope_base=500000.0, dtype="bf16", seed=4242)
    T = 64
    toks = pv_inputs.uniform_tokens(9, T + 8, deep.vocab)
    out = {}
    for store in (ref.KV_BF16, ref.KV_REAL):
        for real in ("f64", "f32"):
            c = ref.RefCache(ref_model(deep, real=real), T + 16, kv_store=store)
            c.prefill(toks[:T])
            out[(store, real)] = (c.export().astype(np.float64), c.forward_block(toks[T:]).astype(np.float64))
    rms = np.sqrt((out[(ref.KV_REAL, "f64")][1] ** 2).mean(axis=1, keepdims=True))
    plain = (np.abs(out[(ref.KV_REAL, "f64")][1] - out[(ref.KV_REAL, "f32")][1]) / rms).max()
    bf = (np.abs(out[(ref.KV_BF16, "f64")][1] - out[(ref.KV_BF16, "f32")][1]) / rms).max()
    flips = (out[(ref.KV_BF16, "f64")][0] != out[(ref.KV_BF16, "f32")][0]).mean(axis=(1, 2, 3))
    assert plain < 1e-5 and 10 * plain < bf < 3e-2
    assert flips[0] < 1e-3 and flips[:8].mean() < flips[16:24].mean() < flips[32:].mean() < 0.2


def test_degenerate_model_without_mixing_is_a_bigram_table():
    """W_o = 0 and W_d = 0: logits = lm_head . rmsnorm(E[token]) regardless of context."""
    shape = GQA
    zo = {("wo", l): np.zeros(pv_inputs.tensor_shape(shape, "wo"), np.float32) for l in range(shape.n_layers)}
    zd = {("wd", l): np.zeros(pv_inputs.tensor_shape(shape, "wd"), np.float32) for l in range(shape.n_layers)}
    m = ref_model(shape, gains="perturbed", overrides={**zo, **zd})
    W = tensors_f64(shape, gains="perturbed")
    toks = pv_inputs.uniform_tokens(3, 9, shape.vocab)
    got = ref.RefCache(m, 16).forward_block(toks)
    x = W[("embed", -1)][toks]
    h = x / np.sqrt((x * x).mean(-1, keepdims=True) + shape.rms_eps) * W[("final_norm", -1)]
    assert np.abs(got - h @ W[("lm_head", -1)].T).max() < 1e-12


def test_single_key_attention_returns_v_of_the_mapped_kv_head():
    """One token, one layer, W_d = 0: softmax over one key is 1, so each query head outputs the
    value vector of kv head (q_head // group): logits follow from three matmuls."""
    shape = GQA.replace(n_layers=1)
    m = ref_model(shape, gains="perturbed",
                  overrides={("wd", 0): np.zeros(pv_inputs.tensor_shape(shape, "wd"), np.float32)})
    W = tensors_f64(shape, gains="perturbed")
    tok = 77
    norm = lambda x, g: x / np.sqrt((x * x).mean() + shape.rms_eps) * g
    x0 = W[("embed", -1)][tok]
    v = W[("wv", 0)] @ norm(x0, W[("attn_norm", 0)])                          # [Hkv*hd]
    group = shape.n_q_heads // shape.n_kv_heads
    o = np.concatenate([v[(a // group) * shape.head_dim:(a // group + 1) * shape.head_dim]
                        for a in range(shape.n_q_heads)])
    x1 = x0 + W[("wo", 0)] @ o
    want = W[("lm_head", -1)] @ norm(x1, W[("final_norm", -1)])
    got = ref.RefCache(m, 4).decode_one(tok)
    assert np.abs(got - want).max() < 1e-12


def test_gqa_equals_mha_with_replicated_kv_heads():
    shape = GQA
    group = shape.n_q_heads // shape.n_kv_heads
    mha = shape.replace(n_kv_heads=shape.n_q_heads)
    over = {}
    for l in range(shape.n_layers):
        for kind in ("wk", "wv"):
            w = pv_inputs.fill_tensor(shape, kind, l).reshape(shape.n_kv_heads, shape.head_dim, shape.d_model)
            over[(kind, l)] = np.repeat(w, group, axis=0).reshape(shape.n_q_heads * shape.head_dim, shape.d_model)
    toks = pv_inputs.uniform_tokens(13, 12, shape.vocab)
    a = ref.RefCache(ref_model(shape), 16).forward_block(toks)
    b = ref.RefCache(ref_model(mha, overrides=over), 16).forward_block(toks)
    assert np.abs(a - b).max() < 1e-12


# ---------------- the verification rule ----------------

def _run_config1(shape, steps, gamma, alpha, kv_store=ref.KV_REAL, seed=3000):
    m = ref_model(shape)
    T0 = 64
    prompt = pv_inputs.uniform_tokens(2000, T0, shape.vocab)
    ar = ref.RefCache(m, T0 + steps * gamma + gamma + 2, kv_store)
    ar.prefill(prompt)
    G = greedy_continuation(ar, steps * gamma + gamma + 1)       # the verifier's own greedy output
    c = ref.RefCache(m, T0 + steps * gamma + gamma + 2, kv_store)
    c.prefill(prompt)
    assert c.pending == G[0]
    committed, accepted, trust = [], [], False
    for s in range(steps):
        T = len(c)
        d = draft_block(G, T0, T, gamma, alpha, shape.vocab, seed, s, trust)
        n, nxt, pred, _ = c.verify(T, d)
        assert len(c) == T + n and c.pending == nxt
        committed += list(d[:n])
        accepted.append(n)
        trust = (n == 0)
    return np.array(committed), np.array(accepted), G


def test_greedy_acceptance_is_lossless_config1():
    """Config 1 workload: everything committed over 100 verify steps is the verifier's own greedy
    output, and each step's correction token is the next greedy token."""
    committed, accepted, G = _run_config1(TINY, 100, 4, 0.7)
    assert len(committed) == accepted.sum() > 100
    assert np.array_equal(committed, G[: len(committed)])


def test_accepted_lengths_are_truncated_geometric():
    steps, gamma, alpha = 600, 4, 0.7
    _, accepted, _ = _run_config1(TINY, steps, gamma, alpha)
    # position 0 is trusted right after a zero-accept step; drop those steps from the statistic
    keep = np.concatenate([[True], accepted[:-1] != 0])
    a_eff = alpha + (1 - alpha) / TINY.vocab
    pmf = ratecheck.accepted_length_pmf(a_eff, gamma)
    obs = np.bincount(accepted[keep], minlength=gamma + 1)
    n = keep.sum()
    chi2 = ((obs - n * pmf) ** 2 / (n * pmf)).sum()
    assert chi2 < 18.5        # chi-square, 4 dof, p ~ 0.001


def test_rollback_restores_cache_and_outputs():
    m = ref_model(GQA, gains="perturbed")
    c = ref.RefCache(m, 64, ref.KV_BF16)
    c.prefill(pv_inputs.uniform_tokens(1, 20, GQA.vocab))
    before, pend = c.export().copy(), c.pending
    d = pv_inputs.uniform_tokens(2, 8, GQA.vocab)
    d[0] = pend
    n1, nx1, pred1, lg1 = c.verify(20, d, want_logits=True)
    assert n1 >= 1
    c.rollback(20)
    assert len(c) == 20 and np.array_equal(c.export(), before)
    c.pending = pend
    n2, nx2, pred2, lg2 = c.verify(20, d, want_logits=True)
    assert (n1, nx1) == (n2, nx2) and np.array_equal(pred1, pred2) and np.array_equal(lg1, lg2)
    with pytest.raises(ValueError):
        c.rollback(len(c) + 1)
    with pytest.raises(ValueError):
        c.verify(len(c) + 3, d)


def test_gamma1_trusted_is_one_greedy_decode_step():
    m = ref_model(TINY)
    prompt = pv_inputs.uniform_tokens(9, 16, TINY.vocab)
    a, b = ref.RefCache(m, 40), ref.RefCache(m, 40)
    a.prefill(prompt); b.prefill(prompt)
    tok = a.pending
    for _ in range(6):
        nxt_ref = int(np.argmax(a.decode_one(tok)))
        b.pending = -1                              # unknown -> draft[0] is trusted
        n, nxt, _, _ = b.verify(len(b), [tok])
        assert n == 1 and nxt == nxt_ref and len(b) == len(a)
        tok = nxt


def test_acceptance_rule_cases():
    """All-accept, reject at each position, reject at 0 (cache untouched), argmax tie -> lowest id."""
    m = ref_model(TINY)
    c = ref.RefCache(m, 64)
    c.prefill(pv_inputs.uniform_tokens(21, 10, TINY.vocab))
    G = greedy_continuation(ref_clone(m, 10, 64), 6)
    assert c.pending == G[0]
    for k in range(5):                               # first mismatch at position k
        d = G[:4].copy()
        if k < 4:
            d[k] = (d[k] + 1) % TINY.vocab
        n, nxt, pred, _ = c.verify(10, d)
        assert n == k if k < 4 else n == 4
        assert nxt == G[n]                           # correction token = verifier's own next token
        assert len(c) == 10 + n
        c.rollback(10); c.pending = G[0]
    # tie: duplicate the winning LM-head row at a lower id -> lower id wins
    Wl = pv_inputs.fill_tensor(TINY, "lm_head", -1).reshape(TINY.vocab, TINY.d_model).copy()
    lo, hi = sorted((int(G[1]), (int(G[1]) + 7) % TINY.vocab))
    Wl[hi] = Wl[lo] = Wl[int(G[1])]
    m2 = ref_model(TINY, overrides={("lm_head", -1): Wl})
    c2 = ref.RefCache(m2, 64)
    c2.prefill(pv_inputs.uniform_tokens(21, 10, TINY.vocab))
    _, _, pred, lg = c2.verify(10, [G[0]], want_logits=True)
    assert lg[0, lo] == lg[0, hi] == lg[0].max() and pred[0] == lo


def ref_clone(m, prompt_len, max_tokens):
    c = ref.RefCache(m, max_tokens)
    c.prefill(pv_inputs.uniform_tokens(21, prompt_len, TINY.vocab))
    return c


# ---- 4-bit weights: the dequantisation rule and the input-side quantiser ----

def test_q4_dequant_closed_forms_and_nibble_order():
    # one row, two groups; scale bits 0x3F00 = 0.5 and 0x4000 = 2.0
    codes = np.zeros((1, 32), dtype=np.uint8)
    k = np.arange(64)
    c = (k * 7 + 3) % 16                                   # every code value occurs
    codes[0] = (c[0::2] | (c[1::2] << 4)).astype(np.uint8)  # even feature in the low nibble
    scales = np.array([[0x3F00, 0x4000]], dtype=np.uint16)
    w = ref.dequant_q4(codes, scales)
    expect = (c - 8) * np.where(k < 32, 0.5, 2.0)
    assert w.dtype == np.float32 and np.array_equal(w[0], expect.astype(np.float32))
    assert w[0][c == 8].tolist() == [0.0] * int((c == 8).sum())      # code 8 is zero whatever the scale
    assert w[0].min() == -8 * 2.0 and w[0].max() == 7 * 2.0


def test_q4_quantiser_roundtrip_properties():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((48, 256)) * 0.02).astype(np.float32)
    bits = pv_inputs.bf16_round_f32(w)
    bits[7, 64:96] = 0                                     # an all-zero group
    wf = pv_inputs.bf16_bits_to_f32(bits)
    codes, scales = pv_inputs.quantize_q4(bits)
    c2, s2 = pv_inputs.quantize_q4(bits, use_native=False)  # the C routine and its numpy twin agree
    assert np.array_equal(codes, c2) and np.array_equal(scales, s2)
    dq = ref.dequant_q4(codes, scales)
    s = pv_inputs.bf16_bits_to_f32(scales)
    # error at most half a step, except where +max clips to code 15 = 7 steps (max / 7 rounded down to bf16)
    err = np.abs(dq - wf).reshape(48, 8, 32)
    assert (err <= 0.5 * s[:, :, None] * (1 + 2.0 ** -7) + np.abs(wf).reshape(48, 8, 32) * 2.0 ** -7).all()
    assert np.array_equal(dq[7, 64:96], np.zeros(32, dtype=np.float32)) and scales[7, 2] == 0x3F80
    # weights that are integer multiples of a bf16 step survive exactly
    step = np.float32(0.015625)
    ints = rng.integers(-7, 8, size=(4, 64)); ints[:, 0] = 7; ints[:, 32] = -7
    exact = (ints * step).astype(np.float32)
    codes, scales = pv_inputs.quantize_q4(pv_inputs.bf16_round_f32(exact))
    assert np.array_equal(ref.dequant_q4(codes, scales), exact)


def test_q4_linear_equals_integer_arithmetic():
    """A projection with 4-bit weights, by brute force in exact integer arithmetic: with small
    integer activations, y[n] = sum_g scale[n, g] * sum_{k in g} (code - 8) * x[k]."""
    rng = np.random.default_rng(6)
    N, K = 16, 96
    c = rng.integers(0, 16, size=(N, K))
    codes = (c[:, 0::2] | (c[:, 1::2] << 4)).astype(np.uint8)
    sc = np.array([0.25, 1.0, 8.0, 0.5, 2.0, 0.125])
    sidx = rng.integers(0, len(sc), size=(N, K // 32))
    scales = pv_inputs.bf16_round_f32(sc[sidx].astype(np.float32))
    x = rng.integers(-5, 6, size=(3, K)).astype(np.float64)
    want = np.zeros((3, N))
    for j in range(3):
        for n in range(N):
            for g in range(K // 32):
                want[j, n] += sc[sidx[n, g]] * sum((int(c[n, k]) - 8) * int(x[j, k]) for k in range(32 * g, 32 * g + 32))
    got = ref.linear(x, ref.dequant_q4(codes, scales))     # float32 weights (exact), fp64 arithmetic
    assert np.array_equal(got, want)
