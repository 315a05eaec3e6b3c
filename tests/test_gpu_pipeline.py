"""Three-stage asynchronous drive on the GPU with small real models on separate streams, and the
pv_cache_readmit hook it relies on."""
import numpy as np
import pytest

import pv_inputs

pytestmark = pytest.mark.gpu

S0 = pv_inputs.ModelShape("p0", 1, 128, 4, 2, 32, 352, 512, dtype="bf16", seed=6060)
S1 = pv_inputs.ModelShape("p1", 2, 256, 8, 2, 32, 704, 512, dtype="bf16", seed=6161)
S2 = pv_inputs.ModelShape("p2", 3, 512, 8, 2, 64, 1280, 512, rope_base=500000.0, dtype="bf16", seed=6262)


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available()
    import paper_2505_01572_amd as pv
    return pv


def test_readmit_keeps_the_blocks_kv(pvlib):
    from gpu_helpers import gpu_model
    gm = gpu_model(S2, gains="perturbed")
    toks = pv_inputs.uniform_tokens(1, 40, S2.vocab)
    a, b = pvlib.Cache(gm, 64), pvlib.Cache(gm, 64)
    a.prefill(toks[:21]); b.prefill(toks[:21])
    n, _ = a.verify(21, toks[21:29])                       # random drafts: almost nothing is accepted by the model
    assert n <= 1
    with pytest.raises(pvlib.PVError):
        a.readmit(21 + 9)                                  # beyond the block
    a.readmit(21 + 5, pending=7)
    assert a.state() == (26, 7)
    b.prefill(toks[21:26])
    assert np.array_equal(a.export(), b.export())          # the re-admitted positions hold exactly those tokens' K/V
    with pytest.raises(pvlib.PVError):
        a.readmit(27)                                      # export forgot the block
    # and the cache continues normally from there
    b.set_pending(7)
    d = toks[26:34].copy(); d[0] = 7
    assert a.verify(26, d) == b.verify(26, d)
    assert np.array_equal(a.debug_logits(), b.debug_logits())


def test_three_stage_pipeline_is_lossless(pvlib):
    import torch
    from gpu_helpers import gpu_model
    from paper_2505_01572_amd import pipeline as pl
    T0, gamma, n_tokens = 48, 8, 60
    prompt = pv_inputs.uniform_tokens(2, T0, 512)
    stages = []
    for i, (shp, level) in enumerate(((S0, 0.6), (S1, 0.8), (S2, 1.0))):
        c = pvlib.Cache(gpu_model(shp), T0 + n_tokens + 64)
        c.prefill(prompt)
        stages.append(pl.Stage(i, c, level, 1 if i == 0 else gamma, torch.cuda.Stream()))
    last = stages[-1].cache
    target = [last.pending]
    for k in range(n_tokens + 3 * gamma):
        n, nxt = last.verify(T0 + k, [target[-1]]); assert n == 1
        target.append(nxt)
    last.rollback(T0)
    u = pv_inputs.unit_draws(3, len(target), stream=9)
    res = pl.run_pipeline(stages, T0, np.array(target), u, 512, n_tokens, timeout_s=60.0)
    assert res["tokens"] >= n_tokens
    assert res["output"] == [int(t) for t in target[: res["tokens"]]]
    assert res["stages"][0]["steps"] >= res["tokens"] and res["stages"][2]["steps"] > 0
    assert 0.4 < res["stages"][2]["alpha_measured"] <= 1.0
    # the last stage's cache really holds the committed sequence: decoding on from it reproduces the target
    fin = stages[-1]
    if fin.rb is None:
        fin.cache.rollback(T0 + fin.m)
        n, nxt = fin.cache.verify(T0 + fin.m, [target[fin.m]])
        assert (n, nxt) == (1, target[fin.m + 1])


def test_sync_speculative_decoding_on_real_caches(pvlib):
    """Draft-then-verify with two small real models: the output is the target model's own greedy
    decoding, and afterwards the target cache holds exactly the K/V of prompt + output (compared
    with a fresh cache that prefilled that sequence), i.e. readmit / rollback left no trace."""
    from gpu_helpers import gpu_model
    from paper_2505_01572_amd import drivers as dr, pipeline as pl
    T0, n_draft, n_tokens = 48, 7, 50
    prompt = pv_inputs.uniform_tokens(2, T0, 512)
    gm_t = gpu_model(S2)
    cd, ct = pvlib.Cache(gpu_model(S0), T0 + n_tokens + 64), pvlib.Cache(gm_t, T0 + n_tokens + 64)
    cd.prefill(prompt); ct.prefill(prompt)
    target, _, _ = dr.autoregressive(ct, T0, ct.pending, n_tokens + 4 * (n_draft + 1))
    u = pv_inputs.unit_draws(4, len(target), stream=11)
    res = dr.speculative_sync(pl.Stage(0, cd, 0.7, 1), ct, T0, np.array(target), u, 512, n_tokens, n_draft)
    m = res["tokens"]
    assert m >= n_tokens and res["output"] == [int(t) for t in target[:m]]
    assert 1.0 < res["tokens_per_round"] <= n_draft + 1 and 0.4 < res["alpha_trials"] < 0.95
    assert ct.state() == (T0 + m, int(target[m]))
    fresh = pvlib.Cache(gm_t, T0 + m + 16)
    fresh.prefill(np.concatenate([prompt, np.array(target[:m], dtype=np.int32)]))
    a, b = ct.export(), fresh.export()
    # same tokens at the same positions; block shapes differ between the two runs (rows per step),
    # so equality is up to the 1-ulp bf16 flips of a different summation order
    assert a.shape == b.shape
    fa, fb = pv_inputs.bf16_bits_to_f32(a), pv_inputs.bf16_bits_to_f32(b)
    assert np.mean(fa != fb) < 0.05 and np.abs(fa - fb).max() <= 2.0 ** -6 * np.abs(fb).max()
    # decoding on from the speculative run's cache reproduces the reference continuation
    n, nxt = ct.verify(T0 + m, [target[m]])
    assert (n, nxt) == (1, target[m + 1])
