"""Host logic of the asynchronous k-stage drive (Algorithm 1) with fake stages: no GPU.

The fake cache only keeps the length bookkeeping of pv_verify / pv_rollback / pv_cache_readmit and
sleeps for a stage-specific step time, so the interleavings of the real thing (drafter racing
ahead, rejections arriving while a verify is in flight, rollback cascades) all occur."""
import time

import numpy as np
import pytest

from paper_2505_01572_amd import pipeline as pl


class FakeCache:
    def __init__(self, n, step_s, vocab):
        self.n, self.step_s, self.vocab, self.pending = n, step_s, vocab, -1
        self.blk = None
        self.calls = {"verify": 0, "rollback": 0, "readmit": 0}

    def __len__(self):
        return self.n

    def verify(self, prefix_len, draft, stream=None):
        assert prefix_len == self.n, (prefix_len, self.n)
        assert len(draft) >= 1 and all(0 <= t < self.vocab for t in draft)
        time.sleep(self.step_s)
        self.calls["verify"] += 1
        self.blk = (self.n, len(draft))
        n = 1 if (self.pending < 0 or self.pending == draft[0]) else 0     # a random model agrees on nothing else
        self.n += n
        self.pending = self.vocab - 1
        return n, self.pending

    def rollback(self, new_len, stream=None):
        assert 0 <= new_len <= self.n
        self.n, self.pending, self.blk = new_len, -1, None
        self.calls["rollback"] += 1

    def readmit(self, new_len, pending=-1, stream=None):
        assert self.blk is not None and self.n <= new_len <= self.blk[0] + self.blk[1]
        self.n, self.pending = new_len, pending
        self.calls["readmit"] += 1

    def set_pending(self, tok, stream=None):
        self.pending = tok


def _run(levels, step_s, gamma, n_tokens, seed):
    vocab, T0 = 1000, 32
    rng = np.random.default_rng(seed)
    target = rng.integers(0, vocab, n_tokens + 4 * gamma + 16)
    u = rng.random(len(target))
    stages = [pl.Stage(i, FakeCache(T0, step_s[i], vocab), lv, 1 if i == 0 else gamma) for i, lv in enumerate(levels)]
    res = pl.run_pipeline(stages, T0, target, u, vocab, n_tokens, timeout_s=60.0)
    return res, target, stages


@pytest.mark.parametrize("levels,step_s", [((0.7, 1.0), (2e-4, 1e-3)), ((0.6, 0.8, 1.0), (1e-4, 4e-4, 1.5e-3)),
                                           ((0.0, 0.5, 1.0), (1e-4, 2e-4, 5e-4)), ((1.0, 1.0, 1.0), (1e-4, 3e-4, 6e-4))])
def test_output_is_the_last_stages_sequence(levels, step_s):
    res, target, stages = _run(levels, step_s, gamma=8, n_tokens=150, seed=len(levels) * 10 + int(levels[0] * 10))
    assert res["tokens"] >= 150
    assert res["output"] == [int(t) for t in target[: res["tokens"]]]          # lossless, whatever the interleaving
    for s in stages:                                                            # caches never ran past their buffers
        if s.rb is None:                                                        # (a rollback still queued at the stop is fine)
            assert len(s.cache) - 32 == s.m <= len(s.out)
    if 0.0 < levels[-2] < 1.0:
        a = res["stages"][-1]["alpha_measured"]
        assert abs(a - levels[-2]) < 0.15                                       # acceptance rate of the last hop = its level
        assert res["stages"][-1]["rollbacks"] == 0 and res["stages"][0]["rollbacks"] > 0


def test_all_accepted_means_full_blocks_and_no_rollbacks():
    res, _, stages = _run((1.0, 1.0, 1.0), (5e-5, 2e-4, 1e-3), gamma=8, n_tokens=120, seed=5)
    assert all(st["rollbacks"] == 0 for st in res["stages"])
    assert res["stages"][-1]["alpha_measured"] == 1.0
    assert res["stages"][-1]["mean_block"] > 4.0                                # the slow last stage finds full windows waiting


def test_closed_form_helper_matches_eq1_values():
    assert abs(pl.closed_form_tokens_per_step(0.7, 8) - 1.92741) < 1e-4
    assert abs(pl.closed_form_tokens_per_step(0.6, 8) - 1.55656) < 1e-4
    assert pl.closed_form_tokens_per_step(0.5, 1) > 1.0


# ---- synchronous speculative decoding and the autoregressive drive (drivers.py) ----

@pytest.mark.parametrize("level,n_draft", [(0.0, 4), (0.5, 3), (0.8, 7), (1.0, 5)])
def test_sync_speculative_decoding_is_lossless_and_geometric(level, n_draft):
    from paper_2505_01572_amd import drivers as dr
    vocab, T0, n_tokens = 1000, 32, 4000
    rng = np.random.default_rng(17)
    target = rng.integers(0, vocab, n_tokens + 4 * (n_draft + 1) + 16)
    u = rng.random(len(target))
    d = pl.Stage(0, FakeCache(T0, 0.0, vocab), level, 1)
    tc = FakeCache(T0, 0.0, vocab)
    res = dr.speculative_sync(d, tc, T0, target, u, vocab, n_tokens, n_draft)
    assert res["output"] == [int(t) for t in target[:res["tokens"]]]
    assert res["tokens"] >= n_tokens and len(tc) == T0 + res["tokens"]
    assert tc.pending == int(target[res["tokens"]])
    # tokens per round follow the truncated geometric law behind Eq. 5's numerator
    expect = dr.pipespec_closed_form(level, n_draft) if level < 1.0 else n_draft + 1.0
    assert abs(res["tokens_per_round"] - expect) < 0.06 * expect + 0.02
    if 0.0 < level < 1.0:
        assert abs(res["alpha_trials"] - level) < 0.03
    # every round cost n_draft draft steps and one target step
    assert res["draft_steps"] == res["rounds"] * n_draft and tc.calls["verify"] == res["rounds"]


def test_autoregressive_drive_and_closed_forms():
    from paper_2505_01572_amd import drivers as dr

    class Echo(FakeCache):           # next token = (last input + 1) % vocab
        def verify(self, prefix_len, draft, stream=None):
            n, _ = super().verify(prefix_len, draft, stream)
            self.pending = (int(draft[0]) + 1) % self.vocab
            return n, self.pending

    c = Echo(10, 0.0, 50)
    out, secs, steps = dr.autoregressive(c, 10, 7, 20)
    assert out == [(7 + i) % 50 for i in range(21)] and steps == 20 and len(c) == 30
    # Eq. 5 against its parts; Eq. 6 is its numerator; both reduce to 1 token per step at alpha = 0
    assert dr.sd_closed_form(0.0, 5, 4.0) == pytest.approx(1.0 / (5 / 4.0 + 1.0))
    assert dr.sd_closed_form(0.5, 3, 1e12) == pytest.approx(1.875)
    assert dr.pipespec_closed_form(0.5, 3) == pytest.approx(1 + 0.5 + 0.25 + 0.125)
    assert dr.pipespec_closed_form(1.0, 7) == 8.0
    # the product's closed forms agree with the independently written ones the oracle pins to Monte Carlo
    from oracle import ratecheck as rc
    for al, g, cc in ((0.3, 4, 2.0), (0.7, 8, 5.5), (0.9, 7, 12.0)):
        assert dr.sd_closed_form(al, g, cc) == pytest.approx(rc.sd_speedup(al, g, cc))
        assert dr.pipespec_closed_form(al, g) == pytest.approx(rc.pipespec_high_alpha(al, g))
        assert pl.closed_form_tokens_per_step(al, g) == pytest.approx(rc.expected_tokens(al, g))
