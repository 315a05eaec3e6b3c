"""GPU parity on the tiny fp32 configuration and a small bf16 grouped-query shape (vector path).

Every call goes through the C ABI.  Bars: fp32 logits within 1e-4 (max abs) of the fp64
oracle; accepted_len / next_token bit-exact (the oracle's top-2 margin is checked to be far
above the logit error wherever a decision is compared); integer state bit-exact.
"""
import numpy as np
import pytest

import pv_inputs
from pv_inputs import CONFIGS
from oracle import ref
from helpers import ref_model, greedy_continuation, draft_block

pytestmark = pytest.mark.gpu

TINY = CONFIGS["tiny"]
GQA = pv_inputs.ModelShape("gqa_small", 3, 128, 8, 2, 32, 176, 512, rope_base=500000.0,
                           dtype="bf16", seed=4242)


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2505_01572_amd as pv
    return pv


@pytest.fixture(scope="module")
def tiny_pair(pvlib):
    from gpu_helpers import gpu_model
    return gpu_model(TINY, gains="perturbed"), ref_model(TINY, gains="perturbed")


def test_tiny_logits_and_decisions_match_oracle(pvlib, tiny_pair):
    gm, rm = tiny_pair
    prompt = pv_inputs.uniform_tokens(2000, 64, TINY.vocab)
    gc, rc = pvlib.Cache(gm, 128), ref.RefCache(rm, 128)
    gc.prefill(prompt); last = rc.prefill(prompt)
    assert len(gc) == 64 and gc.pending == rc.pending
    assert np.abs(gc.debug_logits()[-1] - last).max() < 1e-4
    draft = pv_inputs.uniform_tokens(77, 4, TINY.vocab); draft[0] = rc.pending
    n_r, t_r, pred_r, lg_r = rc.verify(64, draft, want_logits=True)
    n_g, t_g = gc.verify(64, draft)
    lg_g = gc.debug_logits()
    assert lg_g.shape == (4, TINY.vocab)
    assert np.abs(lg_g - lg_r).max() < 1e-4
    assert np.array_equal(gc.debug_pred(), pred_r)
    assert (n_g, t_g) == (n_r, t_r) and gc.state() == (len(rc), rc.pending)


def test_tiny_config1_100_steps(pvlib):
    """Config 1: prefix 64, gamma 4, alpha 0.7, 100 verify(+rollback) steps; outputs bit-exact vs oracle,
    and everything committed equals the oracle's greedy continuation (lossless acceptance)."""
    from gpu_helpers import gpu_model, top2_margin
    gm, rm = gpu_model(TINY), ref_model(TINY)
    T0, gamma, alpha, steps = 64, 4, 0.7, 100
    prompt = pv_inputs.uniform_tokens(2000, T0, TINY.vocab)
    ar = ref.RefCache(rm, T0 + steps * gamma + 8); ar.prefill(prompt)
    G = greedy_continuation(ar, steps * gamma + gamma + 1)
    gc, rc = pvlib.Cache(gm, T0 + steps * gamma + 8), ref.RefCache(rm, T0 + steps * gamma + 8)
    gc.prefill(prompt); rc.prefill(prompt)
    committed, trust, worst = [], False, 0.0
    for s in range(steps):
        T = len(rc)
        d = draft_block(G, T0, T, gamma, alpha, TINY.vocab, 3000, s, trust)
        n_r, t_r, _, lg_r = rc.verify(T, d, want_logits=True)
        n_g, t_g = gc.verify(T, d)
        err = np.abs(gc.debug_logits() - lg_r).max()
        worst = max(worst, err)
        # an argmax can only flip where the oracle's top-2 margin is within twice the logit error
        assert top2_margin(lg_r[: max(n_r, 1)]).min() > 2 * err + 1e-7, f"step {s}: near-tie, pick another seed"
        assert (n_g, t_g) == (n_r, t_r), f"step {s}"
        assert gc.state() == (T + n_r, t_r)
        committed += list(d[:n_g]); trust = n_g == 0
    assert worst < 1e-4
    assert np.array_equal(committed, G[: len(committed)]) and len(committed) > 100


def test_rollback_restores_cache_bits(pvlib, tiny_pair):
    gm, _ = tiny_pair
    gc = pvlib.Cache(gm, 64)
    gc.prefill(pv_inputs.uniform_tokens(5, 21, TINY.vocab))     # ends inside the second page
    before, pend = gc.export(), gc.pending
    d = pv_inputs.uniform_tokens(6, 16, TINY.vocab); d[0] = pend
    n1, t1 = gc.verify(21, d)
    lg1, pred1 = gc.debug_logits(), gc.debug_pred()
    assert n1 >= 1
    gc.rollback(21)
    assert gc.state() == (21, -1)
    assert np.array_equal(gc.export(), before)
    gc.set_pending(pend)
    n2, t2 = gc.verify(21, d)
    assert (n1, t1) == (n2, t2)
    assert np.array_equal(gc.debug_logits(), lg1) and np.array_equal(gc.debug_pred(), pred1)
    gc.rollback(0)
    assert gc.state() == (0, -1) and gc.export().shape[2] == 0


def test_block_equals_sequential_on_gpu(pvlib, tiny_pair):
    gm, _ = tiny_pair
    toks = pv_inputs.uniform_tokens(8, 30, TINY.vocab)
    a, b = pvlib.Cache(gm, 64), pvlib.Cache(gm, 64)
    a.prefill(toks[:19]); b.prefill(toks[:19])
    a.set_pending(-1)
    a.verify(19, toks[19:])                          # 11 rows at once (all trusted/compared; logits are what we read)
    blk = a.debug_logits()
    seq = []
    for t in toks[19:]:
        b.rollback(len(b))                           # forget pending: draft[0] trusted
        n, _ = b.verify(len(b), [t]); assert n == 1
        seq.append(b.debug_logits()[0])
    assert np.abs(blk - np.stack(seq)).max() < 1e-5


def test_result_independent_of_page_order(pvlib, tiny_pair):
    gm, _ = tiny_pair
    toks = pv_inputs.uniform_tokens(9, 50, TINY.vocab)
    a, b = pvlib.Cache(gm, 96), pvlib.Cache(gm, 96)
    perm = np.array([3, 0, 5, 1, 4, 2], dtype=np.int32)
    b.set_page_table(perm)
    for c in (a, b):
        c.prefill(toks[:40]); c.set_pending(-1); c.verify(40, toks[40:])
    assert np.array_equal(a.debug_logits(), b.debug_logits())
    assert np.array_equal(a.export(), b.export())
    with pytest.raises(pvlib.PVError):
        b.set_page_table(perm)                       # only on an empty cache


def test_gqa_bf16_vector_path_matches_oracle(pvlib):
    from gpu_helpers import gpu_model, logit_scale
    gm = gpu_model(GQA, gains="perturbed", kernel_path=pvlib.PATH_VECTOR)
    rm = ref_model(GQA, gains="perturbed")
    prompt = pv_inputs.uniform_tokens(31, 37, GQA.vocab)
    gc, rc = pvlib.Cache(gm, 64), ref.RefCache(rm, 64, ref.KV_BF16)
    gc.prefill(prompt); rc.prefill(prompt)
    assert gc.pending == rc.pending
    d = pv_inputs.uniform_tokens(32, 13, GQA.vocab); d[0] = rc.pending
    n_r, t_r, pred_r, lg_r = rc.verify(37, d, want_logits=True)
    n_g, t_g = gc.verify(37, d)
    err = np.abs(gc.debug_logits() - lg_r) / logit_scale(lg_r)
    assert err.max() < 3e-2          # bar stated for bf16 storage
    assert err.max() < 2e-3          # what fp32 arithmetic on identical stored values should reach
    assert np.array_equal(gc.debug_pred(), pred_r) and (n_g, t_g) == (n_r, t_r)
    # stored K/V: bf16 bit patterns equal to the oracle's rounded values except for rare 1-ulp flips
    ge = pv_inputs.bf16_bits_to_f32(gc.export()).astype(np.float64)
    re_ = rc.export()
    assert ge.shape == re_.shape
    assert np.abs(ge - re_).max() <= 2.0 ** -7 * np.abs(re_).max()
    assert np.mean(ge != re_) < 0.01


def test_argmax_tie_goes_to_lowest_id(pvlib):
    from gpu_helpers import gpu_model
    rm = ref_model(TINY)
    c = ref.RefCache(rm, 32); c.prefill(pv_inputs.uniform_tokens(21, 10, TINY.vocab))
    g0 = c.pending
    g1 = int(np.argmax(c.decode_one(g0)))
    Wl = pv_inputs.fill_tensor(TINY, "lm_head", -1).reshape(TINY.vocab, TINY.d_model).copy()
    lo, hi = sorted((g1, (g1 + 7) % TINY.vocab))
    row = Wl[g1].copy(); Wl[lo] = row; Wl[hi] = row
    gm = gpu_model(TINY, overrides={("lm_head", -1): Wl})
    gc = pvlib.Cache(gm, 32); gc.prefill(pv_inputs.uniform_tokens(21, 10, TINY.vocab))
    assert gc.pending == g0
    n, t = gc.verify(10, [g0])
    lg = gc.debug_logits()[0]
    assert lg[lo] == lg[hi] == lg.max() and (n, t) == (1, lo)


def test_error_paths_leave_state_untouched(pvlib, tiny_pair):
    gm, _ = tiny_pair
    gc = pvlib.Cache(gm, 40)
    gc.prefill(pv_inputs.uniform_tokens(3, 12, TINY.vocab))
    st = gc.state()
    for bad, code in ((lambda: gc.verify(11, [1, 2]), -2), (lambda: gc.verify(12, list(range(17))), -3),
                      (lambda: gc.verify(12, [1, TINY.vocab]), -3), (lambda: gc.verify(12, [1, -1]), -3),
                      (lambda: gc.rollback(13), -3), (lambda: gc.rollback(-1), -3),
                      (lambda: gc.prefill(np.zeros(29, np.int32)), -3), (lambda: gc.verify_wait(), -2)):
        with pytest.raises(pvlib.PVError) as e:
            bad()
        assert e.value.status == code
        assert gc.state() == st
    n, _ = gc.verify(12, [gc.pending])               # still usable
    assert n == 1


@pytest.mark.parametrize("path", ["vector", "matrix"])
def test_rows_without_a_finite_logit_are_reported(pvlib, path):
    """A final-norm gain of NaN makes every logit NaN: no row has an arg-max.  The step must say so
    (PV_ENUMERIC) and commit nothing, instead of returning a token id outside the vocabulary."""
    from gpu_helpers import gpu_model
    if path == "vector":
        shape = CONFIGS["tiny"]
        bad = np.full(shape.d_model, np.nan, dtype=np.float32)
    else:
        shape = pv_inputs.ModelShape("nan_small", 2, 128, 8, 2, 32, 192, 512, dtype="bf16", seed=99)
        bad = np.full(shape.d_model, 0x7FC0, dtype=np.uint16)
    m = gpu_model(shape, overrides={("final_norm", -1): bad})
    c = pvlib.Cache(m, 64)
    with pytest.raises(pvlib.PVError) as e:
        c.prefill(pv_inputs.uniform_tokens(5, 12, shape.vocab))          # (one chunk on either path)
    assert e.value.status == -6 and c.state() == (0, -1)
    good = gpu_model(shape)
    c2 = pvlib.Cache(good, 64)
    c2.prefill(pv_inputs.uniform_tokens(5, 20, shape.vocab))
    assert c2.state()[0] == 20 and 0 <= c2.pending < shape.vocab


def test_weight_chunks_must_come_in_row_order(pvlib):
    """Overlapping or skipped chunks may not add up to a 'complete' tensor: a chunk continues where
    the last one ended or starts the tensor over; a model with a hole refuses to run."""
    m = pvlib.Model(TINY)
    w = pv_inputs.fill_tensor(TINY, "wq", 0).reshape(pv_inputs.tensor_shape(TINY, "wq"))
    m.load_weights("wq", 0, 0, w[:64])
    for r0 in (32, 128):                                  # overlap, gap
        with pytest.raises(pvlib.PVError) as e:
            m.load_weights("wq", 0, r0, w[r0:r0 + 64])
        assert e.value.status == -2
    m.load_weights("wq", 0, 64, w[64:])                   # in order: completes the tensor
    m.load_weights("wq", 0, 0, w[:64])                    # starting over makes it incomplete again
    for kind, layer in pv_inputs.iter_tensors(TINY):
        if (kind, layer) != ("wq", 0):
            m.load_weights(kind, layer, 0, pv_inputs.fill_tensor(TINY, kind, layer).reshape(-1, pv_inputs.tensor_shape(TINY, kind)[-1]))
    c = pvlib.Cache(m, 32)
    with pytest.raises(pvlib.PVError) as e:
        c.prefill([1, 2, 3])
    assert e.value.status == -2
    m.load_weights("wq", 0, 64, w[64:])
    c.prefill([1, 2, 3])
    assert c.state()[0] == 3


def test_calibration_kernels_run_on_ragged_sizes(pvlib):
    """The plain copy and read-stream kernels (yardsticks for counters and for the stream ceiling) on sizes that
    do not divide into whole wave slices, and their argument checks."""
    import torch
    src = torch.arange(0, 3 * 1024 * 1024 + 48, dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    pvlib.calib_copy(dst, src)
    sink = pvlib.calib_read(src)                      # whole buffer: slices + a ragged rest
    pvlib.calib_read(src, nbytes=16 * 7, offset=32)    # smaller than one slice round: only the rest loop
    torch.cuda.synchronize()
    assert torch.equal(dst, src) and int(sink.sum()) == 0
    import ctypes
    assert pvlib.lib().pv_calib_read(ctypes.c_void_p(src.data_ptr() + 8), 32, ctypes.c_void_p(sink.data_ptr()), None) == -1    # misaligned
    assert pvlib.lib().pv_calib_read(ctypes.c_void_p(src.data_ptr()), 24, ctypes.c_void_p(sink.data_ptr()), None) == -1       # not a multiple of 16
