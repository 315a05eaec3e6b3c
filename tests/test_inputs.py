"""Input generator: C fill == numpy fill, distribution sanity, parameter counts."""
import numpy as np
import pv_inputs
from pv_inputs import CONFIGS


def test_c_and_numpy_fill_agree():
    for name in ("tiny", "7b"):
        m = CONFIGS[name]
        a = pv_inputs.fill_tensor(m, "wk", 1, start=12345, count=50000, use_c=True)
        b = pv_inputs.fill_tensor(m, "wk", 1, start=12345, count=50000, use_c=False)
        assert a.dtype == b.dtype and np.array_equal(a, b)


def test_slices_compose():
    m = CONFIGS["tiny"]
    whole = pv_inputs.fill_tensor(m, "wg", 0)
    part = pv_inputs.fill_tensor(m, "wg", 0, start=1000, count=777)
    assert np.array_equal(whole[1000:1777], part)


def test_distribution_and_streams_differ():
    m = CONFIGS["tiny"]
    a = pv_inputs.fill_tensor(m, "wq", 0)
    b = pv_inputs.fill_tensor(m, "wq", 1)
    assert abs(a.mean()) < 5e-4 and abs(a.std() - 0.02) < 5e-4
    assert not np.array_equal(a, b)
    g = pv_inputs.fill_tensor(m, "attn_norm", 0)
    assert np.all(g == 1.0)
    gp = pv_inputs.fill_tensor(m, "attn_norm", 0, gains="perturbed")
    assert abs(gp.mean() - 1.0) < 0.01 and gp.std() > 0.01


def test_bf16_round_trip():
    x = np.array([1.0, 1.0078125, 1.00390625, 1.01171875, -3.1415926, 0.02, 1e-30], dtype=np.float32)
    b = pv_inputs.bf16_round_f32(x)
    f = pv_inputs.bf16_bits_to_f32(b)
    assert f[0] == 1.0 and f[1] == 1.0078125
    assert f[2] == 1.0 and f[3] == 1.015625     # ties round to the even mantissa
    assert np.all(np.abs(f - x) <= np.abs(x) * 2.0 ** -8)
    assert np.array_equal(pv_inputs.bf16_round_f32(f), b)


def test_param_counts_match_public_shapes():
    assert CONFIGS["7b"].n_params() == 6_738_415_616
    assert CONFIGS["8b"].n_params() == 8_030_261_248
    assert CONFIGS["70b"].n_params() == 68_976_648_192
    assert CONFIGS["tiny"].n_params() == 2_106_624


def test_perturbation_rate():
    toks = np.zeros(20000, dtype=np.int32)
    d = pv_inputs.perturb_drafts(toks, 0.7, 1024, 3000, 5)
    rate = np.mean(d != 0)
    assert abs(rate - 0.3 * (1 - 1 / 1024)) < 0.015
