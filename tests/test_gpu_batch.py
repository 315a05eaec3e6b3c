"""Batched verification (pv_verify_batch): the blocks of several sequences stacked into one pass over
the weights (Sec. 2.2: batched verification).  Oracle rule: every sequence is verified exactly as if it
were alone, i.e. an independent ref_verify per sequence on its own cache.

Bars as for the matrix path: |dlogit| <= 3e-2 x RMS(logits of the row), asserted at 2e-3 (split-bf16
operands); arg-max / accepted_len / next_token bit-exact wherever the oracle's top-2 margin is clear of
the logit error; stored K/V equal up to bf16 rounding-boundary flips.
"""
import numpy as np
import pytest

import pv_inputs
from oracle import ref
from helpers import ref_model

pytestmark = pytest.mark.gpu

GQA4 = pv_inputs.ModelShape("batch_gqa", 3, 256, 8, 2, 64, 704, 1024, rope_base=500000.0, dtype="bf16", seed=7101)   # 4 q heads per kv head
MHA = pv_inputs.ModelShape("batch_mha", 2, 256, 4, 4, 64, 512, 1008, dtype="bf16", seed=7102)


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available()
    import paper_2505_01572_amd as pv
    return pv


def _rel_err(lg_g, lg_r):
    from gpu_helpers import logit_scale
    return float((np.abs(lg_g - lg_r) / logit_scale(lg_r)).max())


def _batch_step(pvlib, gcs, rcs, drafts, label):
    """One batched step on the library caches gcs, the same blocks one by one through the oracle caches rcs."""
    from gpu_helpers import top2_margin
    want = []
    for rc, d in zip(rcs, drafts):
        T = len(rc)
        n, t, pred, lg = rc.verify(T, d, want_logits=True)
        want.append((T, n, t, pred, lg))
    got = pvlib.verify_batch(gcs, drafts)
    lg_all, pred_all = gcs[0].debug_logits(), gcs[0].debug_pred()
    assert lg_all.shape[0] == sum(len(d) for d in drafts)
    r0, worst = 0, 0.0
    for i, (gc, rc, d) in enumerate(zip(gcs, rcs, drafts)):
        T, n, t, pred, lg = want[i]
        g = len(d)
        err = _rel_err(lg_all[r0:r0 + g], lg)
        worst = max(worst, err)
        assert err < 2e-3, f"{label} sequence {i}: {err}"
        safe = top2_margin(lg) > 4 * np.abs(lg_all[r0:r0 + g] - lg).max()
        assert np.array_equal(pred_all[r0:r0 + g][safe], pred[safe])
        if safe[: max(n, 1)].all():
            assert got[i] == (n, t), f"{label} sequence {i}"
            assert gc.state() == (T + n, t)
        else:                                   # a near-tie decided: follow the oracle
            gc.rollback(T); rc.rollback(T)
        r0 += g
    return worst


@pytest.mark.parametrize("shape", [GQA4, MHA], ids=lambda s: s.name)
def test_batched_blocks_match_independent_oracle_steps(pvlib, shape):
    from gpu_helpers import gpu_model
    gm, rm = gpu_model(shape, gains="perturbed"), ref_model(shape, gains="perturbed")
    lens = (150, 37, 290, 5)                    # different lengths: different numbers of attention chunks per sequence
    gcs, rcs = [], []
    for i, T0 in enumerate(lens):
        prompt = pv_inputs.uniform_tokens(900 + i, T0, shape.vocab)
        gc, rc = pvlib.Cache(gm, 400), ref.RefCache(rm, 400, ref.KV_BF16)
        gc.prefill(prompt); rc.prefill(prompt)
        assert gc.state() == (T0, rc.pending)
        gcs.append(gc); rcs.append(rc)

    def drafts_for(seed, gammas, idx):
        out = []
        for k, (i, g) in enumerate(zip(idx, gammas)):
            d = pv_inputs.uniform_tokens(seed + k, g, shape.vocab)
            if rcs[i].pending >= 0:
                d[0] = rcs[i].pending
            out.append(d)
        return out
    # three sequences, packed rows (8 + 3 + 5 = 16 rows: one column tile)
    idx = (0, 1, 2)
    w1 = _batch_step(pvlib, [gcs[i] for i in idx], [rcs[i] for i in idx], drafts_for(910, (8, 3, 5), idx), "16 rows")
    # another leader, another order, a single-row block among them, more than 16 rows (two column tiles)
    idx = (3, 2, 0, 1)
    w2 = _batch_step(pvlib, [gcs[i] for i in idx], [rcs[i] for i in idx], drafts_for(920, (1, 8, 8, 6), idx), "23 rows")
    # the widest block: four sequences x 16 rows
    idx = (1, 0, 3, 2)
    w3 = _batch_step(pvlib, [gcs[i] for i in idx], [rcs[i] for i in idx], drafts_for(930, (16, 16, 16, 16), idx), "64 rows")
    # one sequence alone through the batched entry point, then plain steps on former leaders
    w4 = _batch_step(pvlib, [gcs[2]], [rcs[2]], drafts_for(940, (8,), (2,)), "one sequence")
    for i in (0, 3, 1):
        T = len(rcs[i])
        d = pv_inputs.uniform_tokens(950 + i, 4, shape.vocab)
        if rcs[i].pending >= 0:
            d[0] = rcs[i].pending
        n, t, pred, lg = rcs[i].verify(T, d, want_logits=True)
        n_g, t_g = gcs[i].verify(T, d)
        assert _rel_err(gcs[i].debug_logits(), lg) < 2e-3
        if (n_g, t_g) != (n, t):
            gcs[i].rollback(T); rcs[i].rollback(T)
    # what every sequence has committed to its own pages
    for gc, rc in zip(gcs, rcs):
        assert len(gc) == len(rc)
        ge, re_ = pv_inputs.bf16_bits_to_f32(gc.export()).astype(np.float64), rc.export()
        assert ge.shape == re_.shape and np.mean(ge != re_) < 0.03
        assert np.abs(ge - re_).max() <= 2.0 ** -7 * np.abs(re_).max()
    print(f"{shape.name}: worst relative logit error per batch {w1:.2e} {w2:.2e} {w3:.2e} {w4:.2e}")


def test_batch_argument_checks(pvlib):
    from gpu_helpers import gpu_model
    gm = gpu_model(GQA4)
    a, b, c = pvlib.Cache(gm, 128), pvlib.Cache(gm, 128), pvlib.Cache(gm, 256)
    for x in (a, b, c):
        x.prefill(pv_inputs.uniform_tokens(3, 10, GQA4.vocab))
    st = [x.state() for x in (a, b, c)]
    cases = [(lambda: pvlib.verify_batch([a, a], [[1, 2], [3]]), -1),                      # the same cache twice
             (lambda: pvlib.verify_batch([a, c], [[1, 2], [3]]), -1),                      # different max_tokens
             (lambda: pvlib.verify_batch([a, b], [[1, 2], [GQA4.vocab]]), -3),             # token out of range
             (lambda: pvlib.verify_batch([a, b], [list(range(1, 18)), [3]]), -3),          # one block above max_gamma
             (lambda: pvlib.verify_batch([a, b], [[1] * 16, [2] * 16] + []), 0)]           # fine: 32 rows
    for bad, code in cases[:-1]:
        with pytest.raises(pvlib.PVError) as e:
            bad()
        assert e.value.status == code
        assert [x.state() for x in (a, b, c)] == st
    res = cases[-1][0]()
    assert len(res) == 2 and all(0 <= n <= 16 for n, _ in res)
    tiny = gpu_model(pv_inputs.CONFIGS["tiny"])
    t = pvlib.Cache(tiny, 64)
    t.prefill([1, 2, 3])
    with pytest.raises(pvlib.PVError) as e:
        pvlib.verify_batch([t], [[4, 5]])                                                   # fp32 vector path
    assert e.value.status == -1
