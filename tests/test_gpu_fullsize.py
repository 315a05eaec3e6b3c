"""Parity at the benchmark shapes (bf16, matrix-core path), in the launch configuration bench.py times.

The oracle cannot prefill a 2048-token prompt through 32 full-width layers in test time, so each
shape is covered by two element-by-element comparisons that together span every dimension at
full size - (a) every layer at full width on a short prompt, (b) the full prompt length and
every gamma on the first two layers - plus properties that hold at any size on the complete
configuration (block forward == single-token steps, bit-exact rollback, lossless acceptance
against the library's own greedy decoding).
Bars: |dlogit| <= 3e-2 x RMS(logits of the row) (stated for bf16 storage; the split-bf16
activations are expected near 1e-3, asserted at 5e-3); argmax / accepted_len / next_token
bit-exact wherever the oracle's top-2 margin exceeds 0.05.
"""
import time

import numpy as np
import pytest

import pv_inputs
from pv_inputs import CONFIGS
from oracle import ref

pytestmark = pytest.mark.gpu
FLIP_BOUND_L0, FLIP_BOUND = 1e-3, 0.08


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available()
    import paper_2505_01572_amd as pv
    return pv


def _compare_steps(pvlib, gm, rm, shape, T0, gammas, alpha, seed, expect=5e-3):
    from gpu_helpers import logit_scale, top2_margin
    prompt = pv_inputs.uniform_tokens(2000 + shape.seed, T0, shape.vocab)
    span = sum(gammas) + 8
    gc, rc = pvlib.Cache(gm, T0 + span), ref.RefCache(rm, T0 + span, ref.KV_BF16)
    t0 = time.time(); gc.prefill(prompt); t1 = time.time(); rc.prefill(prompt); t2 = time.time()
    print(f"[{shape.name} L={shape.n_layers} T={T0}] prefill gpu {t1 - t0:.2f}s oracle {t2 - t1:.2f}s", flush=True)
    assert gc.state()[0] == T0
    worst = 0.0
    for step, gamma in enumerate(gammas):
        T = len(rc)
        # draft: the oracle's own greedy tokens (teacher: previous preds), perturbed at rate 1-alpha
        d = pv_inputs.uniform_tokens(seed + step, gamma, shape.vocab)
        d[0] = rc.pending
        n_r, t_r, pred_r, lg_r = rc.verify(T, d, want_logits=True)
        # second pass with a draft that follows the oracle's predictions, perturbed: exercises accepts
        rc.rollback(T); rc.pending = int(d[0])
        d2 = np.concatenate([[d[0]], pred_r[:-1]]).astype(np.int32)
        d2 = pv_inputs.perturb_drafts(d2, alpha, shape.vocab, seed, step); d2[0] = d[0]
        n_r, t_r, pred_r, lg_r = rc.verify(T, d2, want_logits=True)
        if gc.pending != d2[0]:
            gc.set_pending(int(d2[0]))
        n_g, t_g = gc.verify(T, d2)
        lg_g = gc.debug_logits()
        err = (np.abs(lg_g - lg_r) / logit_scale(lg_r)).max()
        worst = max(worst, err)
        assert err < 3e-2, f"gamma {gamma}: rel logit error {err}"
        safe = top2_margin(lg_r) > 0.05
        assert np.array_equal(gc.debug_pred()[safe], pred_r[safe])
        if safe[: max(n_r, 1)].all():
            assert (n_g, t_g) == (n_r, t_r), f"gamma {gamma}"
            assert gc.state() == (len(rc), rc.pending)
        else:
            gc.rollback(T); rc.rollback(T)
            gc.set_pending(int(d2[0])); rc.pending = int(d2[0])
        print(f"  gamma {gamma}: accepted {n_r}, rel err {err:.2e}, safe rows {int(safe.sum())}/{gamma}", flush=True)
    assert worst < expect, worst
    return gc, rc


@pytest.mark.parametrize("name,T0", [("8b", 2048), ("7b", 512), ("70b", 1024), ("1b", 1024), ("70b_q4", 1024), ("8b_q4", 512)])
def test_full_prefix_two_layers(pvlib, name, T0):
    """Full width, full prompt length, gamma in {1,4,8,16}; first two layers (+ final norm and LM head)."""
    from gpu_helpers import paired_models
    shape = CONFIGS[name].replace(n_layers=2)
    gm, rm = paired_models(shape)
    gc, rc = _compare_steps(pvlib, gm, rm, shape, T0, (1, 4, 8, 16), 0.7, 7000)
    ge = pv_inputs.bf16_bits_to_f32(gc.export()).astype(np.float64)
    re_ = rc.export()
    assert ge.shape == re_.shape
    flips = (ge != re_).mean(axis=(1, 2, 3))                 # per layer: stored bf16 K/V elements that rounded the other way
    print(f"  K/V elements that differ from the oracle's (1 ulp of bf16), per layer: {flips}", flush=True)
    # A stored element differs when the fp32 result falls on the other side of a bf16 rounding boundary
    # than the fp64 one: rate = (relative error of the element) / (bf16 spacing, 2^-8 .. 2^-7).  Layer 0
    # sees exact inputs, so its rate measures the projection arithmetic alone (16-bit operands: a few
    # 1e-4; operands cut to 8 bits would give tens of percent).  Every flipped element below then acts
    # as noise of 1 ulp of bf16 on a layer's inputs (rate f -> relative noise sqrt(f) * 2^-8), which is
    # what sets the rate of the layers above: a few percent, not growing with the arithmetic error.
    assert flips[0] < FLIP_BOUND_L0 and flips.max() < FLIP_BOUND
    assert np.abs(ge - re_).max() <= 2.0 ** -7 * np.abs(re_).max()


@pytest.mark.parametrize("name,T0", [("8b", 300), ("70b", 200), ("70b_q4", 200)])
def test_full_width_wide_blocks_two_layers(pvlib, name, T0):
    """Blocks of 17..64 rows at full width (shared-tile GEMM: K cut over workgroups for the
    projections with few strips, one slice for gate/up and the vocabulary projection); the prompt
    goes in as 64-row chunks plus a ragged rest."""
    from gpu_helpers import paired_models
    shape = CONFIGS[name].replace(n_layers=2)
    gm, rm = paired_models(shape, max_gamma=64)
    _compare_steps(pvlib, gm, rm, shape, T0, (64, 17, 32, 8, 40), 0.7, 7200)


@pytest.mark.parametrize("name,T0", [("8b", 300), ("70b_q4", 130)])
def test_full_width_draft_tree_two_layers(pvlib, name, T0):
    """A draft tree of 48 nodes at full width (head_dim 128, four / eight query heads per kv head): every probed node's
    logits are the oracle's block forward over its chain of ancestors, the accepted path is the oracle's greedy
    continuation as far as the tree carries it, and the compacted cache equals the oracle's after the same tokens."""
    from gpu_helpers import paired_models, logit_scale, top2_margin
    from helpers import greedy_continuation
    from test_gpu_tree import _tree, _chain
    shape = CONFIGS[name].replace(n_layers=2)
    gm, rm = paired_models(shape, max_gamma=64)
    prompt = pv_inputs.uniform_tokens(2000 + shape.seed, T0, shape.vocab)
    gc, rc, ar = pvlib.Cache(gm, T0 + 160), ref.RefCache(rm, T0 + 160, ref.KV_BF16), ref.RefCache(rm, T0 + 160, ref.KV_BF16)
    gc.prefill(prompt); rc.prefill(prompt); ar.prefill(prompt)
    assert gc.state() == (T0, rc.pending)
    G = greedy_continuation(ar, 10)
    tokens, parents, want_path = _tree(G, 48, 7300, shape.vocab, 6)
    n_g, nxt_g, path_g = gc.verify_tree(T0, tokens, parents)
    lg_g = gc.debug_logits()
    probe = sorted(set(want_path[-1:] + [47, 24, 0] + [i for i in range(48) if i not in set(parents)][:3]))
    worst = 0.0
    for i in probe:
        ch = _chain(parents, i)
        lg_r = rc.forward_block(tokens[ch]); rc.rollback(T0)
        worst = max(worst, float((np.abs(lg_g[ch] - lg_r) / logit_scale(lg_r)).max()))
    assert worst < 5e-3, worst
    m = len(want_path)
    lg_path = rc.forward_block(tokens[want_path]); rc.rollback(T0)
    if (top2_margin(lg_path) > 0.05).all():
        assert (n_g, list(path_g)) == (m, want_path) and nxt_g == G[m]
        assert gc.state() == (T0 + m, int(G[m]))
    rc.pending = int(G[0])
    if n_g:
        rc.verify(T0, tokens[list(path_g)])
    assert len(rc) == len(gc)
    ge, re_ = pv_inputs.bf16_bits_to_f32(gc.export()).astype(np.float64), rc.export()
    flips = (ge != re_).mean(axis=(1, 2, 3))
    assert flips[0] < FLIP_BOUND_L0 and flips.max() < FLIP_BOUND and np.abs(ge - re_).max() <= 2.0 ** -7 * np.abs(re_).max()
    print(f"[{name}] tree of 48 nodes: accepted {n_g} (path {[int(i) for i in path_g]}), worst relative logit error {worst:.2e}, K/V flips per layer {flips}", flush=True)


@pytest.mark.parametrize("name,T0", [("8b", 96), ("7b", 96)])
def test_full_depth_short_prefix(pvlib, name, T0):
    """Every layer at full width; the prompt is cut to what the oracle prefills in seconds."""
    from gpu_helpers import paired_models
    shape = CONFIGS[name]
    t0 = time.time()
    gm, rm = paired_models(shape)
    print(f"[{name}] models built in {time.time() - t0:.1f}s", flush=True)
    # 1-ulp differences in which way a stored bf16 K/V element rounded (about 1 % of them, see the
    # two-layer test) compound over 32 layers; the stated bar of 3e-2 still holds with margin
    _compare_steps(pvlib, gm, rm, shape, T0, (8, 8), 0.7, 7100, expect=2e-2)


@pytest.mark.parametrize("name,T0", [("8b", 2048), ("70b", 1024)])
def test_full_configuration_properties(pvlib, name, T0):
    """Configs 3 and 4 as benchmarked (every layer, full prefix, paged KV, the launch configuration
    bench.py times): properties that need no oracle."""
    import bench
    import gc
    import torch
    gc.collect(); torch.cuda.empty_cache()          # the 70B shape needs 140 GB of the card
    shape = CONFIGS[name]
    print(f"full configuration {name}: loading", flush=True)
    gm = bench.load_model(pvlib, pv_inputs, shape, 16)
    gamma = 8
    c = pvlib.Cache(gm, T0 + 96)
    c.prefill(pv_inputs.uniform_tokens(2000 + shape.seed, T0, shape.vocab))
    first = c.pending
    # greedy continuation by single-token steps, keeping each step's logits
    G, seq_logits = [first], []
    for i in range(gamma):
        n, nxt = c.verify(T0 + i, [G[-1]]); assert n == 1
        seq_logits.append(c.debug_logits()[0]); G.append(nxt)
    c.rollback(T0)
    before = c.export()
    c.set_pending(first)
    # block forward of the greedy tokens == the single-token steps; everything accepted
    n, nxt = c.verify(T0, G[:gamma])
    blk = c.debug_logits()
    scale = np.sqrt((blk ** 2).mean())
    assert np.abs(blk - np.stack(seq_logits)).max() < 2e-3 * scale
    assert (n, nxt) == (gamma, G[gamma])
    # a perturbed draft is cut at the first mismatch and corrected with the greedy token
    c.rollback(T0); c.set_pending(first)
    d = np.array(G[:gamma], dtype=np.int32); d[3] = (d[3] + 1) % shape.vocab
    assert c.verify(T0, d) == (3, G[3])
    assert c.state() == (T0 + 3, G[3])
    # rollback restores the cache bit for bit and reruns are bit-identical
    c.rollback(T0)
    assert np.array_equal(c.export(), before)
    c.set_pending(first)
    assert c.verify(T0, G[:gamma]) == (gamma, G[gamma])
    assert np.array_equal(c.debug_logits(), blk)


def test_full_configuration_batched_steps(pvlib):
    """The 8B-shaped verifier at full depth: four sequences with prompts of their own, verified as one
    stacked block (4 x gamma 8 = 32 rows, the configuration bench.py times as its batch point), against
    the same blocks verified one sequence at a time by the library itself (the oracle comparison of the
    batched path is tests/test_gpu_batch.py; the single-sequence path at this depth is checked against the
    oracle's goldens).  Logits within 1e-2 x RMS of each other (different row counts take different GEMM
    kernels; 32 layers of bf16-stored K/V), decisions identical wherever the margin is clear, K/V of the accepted rows identical up to
    bf16 rounding-boundary flips."""
    import bench
    import gc
    import torch
    gc.collect(); torch.cuda.empty_cache()
    shape = CONFIGS["8b"]
    gm = bench.load_model(pvlib, pv_inputs, shape, 16)
    T0s, gamma = (2048, 777, 1500, 64), 8
    solo, batch = [], []
    for i, T0 in enumerate(T0s):
        prompt = pv_inputs.uniform_tokens(8800 + i, T0, shape.vocab)
        a, b = pvlib.Cache(gm, 2048 + 64), pvlib.Cache(gm, 2048 + 64)
        a.prefill(prompt); b.prefill(prompt)
        assert a.state() == b.state()
        solo.append(a); batch.append(b)
    for step in range(3):
        drafts, want, rows = [], [], []
        for i, a in enumerate(solo):
            d = pv_inputs.uniform_tokens(8900 + 10 * step + i, gamma, shape.vocab)
            d[0] = a.pending
            T = len(a)
            n, nxt = a.verify(T, d)
            lg, pred = a.debug_logits(), a.debug_pred()
            drafts.append(d); want.append((T, n, nxt, pred)); rows.append(lg)
        got = pvlib.verify_batch(batch, drafts)
        lg_b, pred_b = batch[0].debug_logits(), batch[0].debug_pred()
        r0 = 0
        for i, (T, n, nxt, pred) in enumerate(want):
            lg = rows[i]
            scale = np.sqrt((lg.astype(np.float64) ** 2).mean(axis=1, keepdims=True))
            err = float((np.abs(lg_b[r0:r0 + gamma] - lg) / scale).max())
            assert err < 1e-2, (step, i, err)        # each side is within 3e-3..6e-3 of the oracle at this depth (the goldens)
            srt = np.sort(lg, axis=1)
            safe = (srt[:, -1] - srt[:, -2]) > 0.05
            assert np.array_equal(pred_b[r0:r0 + gamma][safe], pred[safe])
            if safe[: max(n, 1)].all():
                assert got[i] == (n, nxt) and batch[i].state() == solo[i].state()
            else:
                solo[i].rollback(T); batch[i].rollback(T)
                solo[i].set_pending(int(drafts[i][0])); batch[i].set_pending(int(drafts[i][0]))
            r0 += gamma
    for a, b in zip(solo, batch):
        ea, eb = pv_inputs.bf16_bits_to_f32(a.export()), pv_inputs.bf16_bits_to_f32(b.export())
        assert ea.shape == eb.shape and np.abs(ea - eb).max() <= 2.0 ** -6 * np.abs(ea).max()
