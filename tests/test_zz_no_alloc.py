"""The allocation-free entry point (pv_verify_async_static) against pv_verify, through the C ABI.

Same model, two caches fed the same blocks: one steps through pv_verify with its own workspace, the
other through pv_verify_async_static + pv_verify_wait with the library's fixed device array.  Results,
cache state and the K/V bits written must be identical, on two calls in a row (the second with a
smaller block), with another model's call on the shared array in between, and a step that does not
fit the array must be refused without touching anything.
"""
import numpy as np
import pytest

import pv_inputs
from pv_inputs import CONFIGS

pytestmark = pytest.mark.gpu

MAT = pv_inputs.ModelShape("na_mat", 3, 256, 8, 2, 64, 704, 1024, rope_base=500000.0, dtype="bf16", seed=6101)
SLIM = pv_inputs.ModelShape("na_slim", 1, 128, 4, 2, 32, 128, 512, dtype="bf16", seed=6102)
MAT_Q4 = pv_inputs.ModelShape("na_q4", 2, 512, 8, 2, 64, 1408, 1008, rope_base=500000.0, dtype="bf16", seed=6103, weight_bits=4)


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available()
    import paper_2505_01572_amd as pv
    return pv


def _twin_steps(pvlib, model, shape, blocks, between=None):
    prompt = pv_inputs.uniform_tokens(61, 70, shape.vocab)
    a, b = pvlib.Cache(model, 160), pvlib.Cache(model, 160)
    a.prefill(prompt); b.prefill(prompt)
    assert a.state() == b.state()
    for i, gamma in enumerate(blocks):
        T = len(a)
        d = pv_inputs.uniform_tokens(62 + i, gamma, shape.vocab)
        d[0] = a.pending if a.pending >= 0 else d[0]
        want = a.verify(T, d)
        pred = a.debug_pred()
        b.verify_async_static(T, d)
        got = b.verify_wait()
        assert got == want, (gamma, got, want)
        assert b.state() == a.state()
        assert np.array_equal(b.debug_pred(), pred) if len(b.debug_pred()) else True
        if between is not None:
            between()
        # follow the greedy token so that later blocks accept something
        d2 = np.concatenate([[a.pending], pred[:gamma - 1]]).astype(np.int32)[:gamma]
        T = len(a)
        want = a.verify(T, d2)
        b.verify_async_static(T, d2)
        assert b.verify_wait() == want
        assert np.array_equal(a.export(), b.export())
    return a, b


def test_static_scratch_step_equals_workspace_step(pvlib):
    from gpu_helpers import gpu_model
    m = gpu_model(MAT, gains="perturbed")
    tiny = gpu_model(CONFIGS["tiny"], gains="perturbed")          # fp32 vector path: another layout in the same array
    tc = pvlib.Cache(tiny, 64)
    tc.prefill(pv_inputs.uniform_tokens(5, 20, CONFIGS["tiny"].vocab))

    def other_model_call():
        T = len(tc)
        tc.verify_async_static(T, [tc.pending, 3, 4, 5])
        n, nxt = tc.verify_wait()
        assert 1 <= n <= 4
    # two calls in a row, the second smaller; then wider blocks (two column tiles) and one row
    _twin_steps(pvlib, m, MAT, (8, 3), between=other_model_call)
    _twin_steps(pvlib, m, MAT, (16, 5, 1))
    # the vector path too, against its own workspace step
    _twin_steps(pvlib, tiny, CONFIGS["tiny"], (4, 2))
    # 4-bit weights: 9..16-row blocks run the K-sliced shared-tile GEMM, whose partial sums sit in the step's buffers
    # (here: in the fixed array, laid out for 16 rows)
    q4 = gpu_model(MAT_Q4, gains="perturbed")
    _twin_steps(pvlib, q4, MAT_Q4, (12, 16, 7))


def test_static_scratch_refuses_what_does_not_fit(pvlib):
    from gpu_helpers import gpu_model
    m = gpu_model(SLIM)
    c = pvlib.Cache(m, 1 << 20)           # a million positions: the attention partials of one step outgrow the fixed array
    c.prefill(pv_inputs.uniform_tokens(7, 10, SLIM.vocab))
    st = c.state()
    with pytest.raises(pvlib.PVError) as e:
        c.verify_async_static(10, [c.pending, 1, 2, 3, 4, 5, 6, 7])
    assert e.value.status == -5 and "fixed array" in str(e.value)
    assert c.state() == st
    n, _ = c.verify(10, [c.pending, 1, 2])              # untouched and usable
    assert n >= 1
    small = pvlib.Cache(m, 256)
    small.prefill(pv_inputs.uniform_tokens(7, 10, SLIM.vocab))
    small.verify_async_static(10, [small.pending, 1, 2])
    assert small.verify_wait()[0] >= 1
