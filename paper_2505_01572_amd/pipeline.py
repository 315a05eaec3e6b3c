"""Asynchronous k-stage drive of PipeSpec on one GPU (paper Sec. 3.2, Algorithm 1).

One host thread and one HIP stream per stage.  Stage 0 drafts one token per step; every later
stage verifies whatever its predecessor has produced beyond its own committed position (at
most gamma tokens), appends the matching prefix plus its own next token to its output buffer
O_i, and on a mismatch tells every earlier stage to roll back to the last valid token.  All
arithmetic of a step runs in the library (pv_verify on the stage's cache and stream); this
module only moves token ids between the buffers.

Synthetic acceptance.  The benchmark configuration uses independently drawn random models,
which agree with probability 1/vocab, so the paper's acceptance rates alpha_{i-1,i} cannot arise
from the models themselves.  Each stage therefore still runs its real forward pass over the
real draft block (real time, real K/V), but the token it *emits* at generated index k is taken
from a reference sequence `target[k]` (the last stage's greedy continuation) whenever a shared
uniform draw u[k] falls below the stage's level, and is a stage-specific wrong token
otherwise.  Levels are nested (level_0 < level_1 < ... < level_K = 1), hence stage i accepts a
token of stage i-1 with probability level_{i-1}: alpha_{i-1,i} = level_{i-1}.  The length the
cache keeps after a step is then set with pv_cache_readmit.  The last stage always emits the
target, so the pipeline's output must equal `target` exactly, whatever the interleaving:
that is the losslessness check of the rollback logic.
"""
import threading
import time

import numpy as np


class Stage:
    """One pipeline stage: a cache (anything with verify / rollback / readmit / set_pending),
    its stream, its output buffer O_i and the bookkeeping of Algorithm 1."""

    def __init__(self, index, cache, level, gamma, stream=None):
        self.i, self.cache, self.level, self.gamma, self.stream = index, cache, level, gamma, stream
        self.lock = threading.Lock()
        self.out = []            # O_i: generated tokens, index k = position - prompt_len
        self.m = 0               # tokens of `out` whose K/V are in the cache (inputs consumed)
        self.epoch = 0           # bumped whenever a later stage truncates `out`
        self.rb = None           # smallest index a later stage asked us to roll back to
        self.imposed = -1        # index whose token we last imposed on the earlier stages (not a fresh trial)
        self.steps = self.rows = self.accepted = self.trials = self.rollbacks = 0
        self.busy_s = 0.0


def _settle(cache, want_len, pending, stream):
    """Make the cache hold exactly want_len tokens after a verify whose own (real) acceptance is not
    the one that counts: extend over the block just written, or cut back."""
    if want_len >= len(cache):
        cache.readmit(want_len, pending, stream=stream)
    else:
        cache.rollback(want_len, stream=stream)
        cache.set_pending(pending, stream=stream)


def _wrong_token(target_tok, stage, vocab):
    return int((int(target_tok) + 1 + stage) % vocab)


def run_pipeline(stages, prompt_len, target, u, vocab, n_tokens, max_ahead=None, poll_s=20e-6, timeout_s=120.0):
    """Drive the stages until the last one has committed n_tokens generated tokens.

    stages[i].cache must hold the prompt (prompt_len tokens).  target: reference tokens by generated
    index (len >= n_tokens + gamma + 2), u: uniform draws of the same length.  Returns a dict of
    measurements; out of the last stage is returned under "output".
    """
    K = len(stages) - 1
    max_ahead = max_ahead or 2 * max(s.gamma for s in stages)
    done = threading.Event()
    errors = []
    t_end = time.time() + timeout_s

    def emit(stage, k):          # the token stage `stage` would produce at generated index k
        if stage == K or u[k] < stages[stage].level:
            return int(target[k])
        return _wrong_token(target[k], stage, vocab)

    for s in stages:             # index 0 is every stage's own token after the prompt (free: prefill)
        s.out, s.m, s.rb, s.epoch = [emit(s.i, 0)], 0, None, 0

    def signal_rollback(frm, L, tok):
        """Stage `frm` rejected the draft at index L; its own token there is `tok` (Algorithm 1:
        'signal rejection to earlier stages', 'rollback O_i to match O_j's last token')."""
        for e in range(frm):
            se = stages[e]
            with se.lock:
                if len(se.out) > L and se.out[L] != tok:
                    se.out = se.out[:L] + [tok]
                    se.epoch += 1
                    se.rb = L if se.rb is None else min(se.rb, L)
                    se.rollbacks += 1

    def apply_rollback(s):
        with s.lock:
            L, s.rb = s.rb, None
            if L is None or s.m < L:
                return
            s.m = L
            tok = s.out[s.m]
        s.cache.rollback(prompt_len + s.m, stream=s.stream)
        if s.i > 0:
            s.cache.set_pending(tok, stream=s.stream)

    def drafter(s):
        nxt = stages[1]
        while not done.is_set():
            apply_rollback(s)
            with s.lock:
                if s.rb is not None:
                    continue                                         # a rejection arrived just now: apply it first
                ahead = len(s.out) - nxt.m
                k, tok, epoch = s.m, s.out[s.m] if s.m < len(s.out) else None, s.epoch
            if tok is None or ahead > max_ahead:
                time.sleep(poll_s)
                continue
            t0 = time.perf_counter()
            s.cache.rollback(prompt_len + k, stream=s.stream)        # forget pending: the input token is trusted
            s.cache.verify(prompt_len + k, [tok], stream=s.stream)   # gamma = 1: one greedy decoding step
            s.busy_s += time.perf_counter() - t0
            with s.lock:
                s.steps += 1; s.rows += 1
                if s.epoch != epoch:
                    continue                                         # truncated meanwhile: rollback is pending
                s.m = k + 1
                if len(s.out) == s.m:
                    s.out.append(emit(0, s.m))

    def verifier(s):
        prev = stages[s.i - 1]
        nxt = stages[s.i + 1] if s.i < K else None
        while not done.is_set():
            apply_rollback(s)
            with s.lock:
                if s.rb is not None:
                    continue                                         # a rejection arrived just now: apply it first
                k, first, epoch = s.m, s.out[s.m], s.epoch
                ahead = len(s.out) - (nxt.m if nxt else 0)
            if nxt is not None and ahead > max_ahead:
                time.sleep(poll_s)
                continue
            with prev.lock:
                drafts = list(prev.out[k:k + s.gamma])
            if not drafts:
                time.sleep(poll_s)
                continue
            t0 = time.perf_counter()
            s.cache.verify(prompt_len + k, drafts, stream=s.stream)  # the real forward pass over the block
            n = 0
            while n < len(drafts) and drafts[n] == (first if n == 0 else emit(s.i, k + n)):
                n += 1
            with s.lock:
                s.steps += 1; s.rows += len(drafts)
                stale = s.epoch != epoch
                if not stale:
                    nxt_tok = first if n == 0 else emit(s.i, k + n)
                    s.out = s.out[:k] + drafts[:n] + [nxt_tok]
                    s.m = k + n
                    skip = 1 if (k == s.imposed and n >= 1) else 0      # a re-sent correction always matches
                    s.accepted += n - skip
                    s.trials += n - skip + (1 if n < len(drafts) else 0)
            if stale:
                _settle(s.cache, prompt_len + k, first, s.stream)          # a later stage cut our buffer: keep nothing
            else:
                _settle(s.cache, prompt_len + k + n, nxt_tok, s.stream)
                if n < len(drafts):
                    s.imposed = k + n
                    signal_rollback(s.i, k + n, nxt_tok)
                if s.i == K and s.m >= n_tokens:
                    done.set()
            s.busy_s += time.perf_counter() - t0

    def guard(fn, s):
        try:
            fn(s)
        except Exception as e:          # noqa: BLE001 - reported to the caller below
            errors.append((s.i, e))
            done.set()

    threads = [threading.Thread(target=guard, args=(drafter if s.i == 0 else verifier, s), daemon=True) for s in stages]
    t_start = time.perf_counter()
    for t in threads:
        t.start()
    while not done.is_set() and time.time() < t_end:
        done.wait(0.05)
    timed_out = not done.is_set()
    done.set()
    for t in threads:
        t.join(timeout=30.0)
    elapsed = time.perf_counter() - t_start
    if errors:
        raise RuntimeError(f"stage {errors[0][0]} failed: {errors[0][1]!r}")
    if timed_out:
        raise TimeoutError("pipeline did not reach n_tokens in time")
    last = stages[K]
    res = {"elapsed_s": elapsed, "tokens": last.m, "tokens_per_s": last.m / elapsed, "output": list(last.out[:last.m]),
           "stages": []}
    for s in stages:
        res["stages"].append({
            "steps": s.steps, "rows": s.rows, "accepted": s.accepted, "trials": s.trials, "rollbacks": s.rollbacks,
            "alpha_measured": (s.accepted / s.trials) if s.trials else None,
            "mean_block": (s.rows / s.steps) if s.steps else None,
            "tokens_per_step": (s.m / s.steps) if s.steps else None,
            "steps_per_s": s.steps / elapsed, "busy_frac": s.busy_s / elapsed})
    return res


def closed_form_tokens_per_step(alpha, gamma):
    """Eq. 1 with the steady-state verification probability of Eq. 3 (paper Sec. 3.3)."""
    geo = (1.0 - alpha ** (gamma + 1)) / (1.0 - alpha) if alpha < 1.0 else gamma + 1.0
    rho = alpha / (1.0 - alpha ** (gamma + 1) + alpha)
    return (1.0 - rho) + rho * geo


def load_stage_model(pv, pv_inputs, shp, max_gamma=16):
    """A library model of the given shape with its seeded synthetic weights, generated and
    uploaded chunk by chunk through one pinned host buffer."""
    import torch
    m = pv.Model(shp, max_gamma=max_gamma)
    pinned = torch.empty(m.staging_bytes // 2, dtype=torch.int16, pin_memory=True)
    scratch = pinned.numpy().view(m.np_dtype)
    for kind, layer in pv_inputs.iter_tensors(shp):
        cols = pv_inputs.tensor_shape(shp, kind)[-1]
        q4 = getattr(shp, "weight_bits", 16) == 4 and kind in pv_inputs.Q4_KINDS
        for r0, rows in pv_inputs.iter_row_chunks(shp, kind, layer, m.chunk_rows(cols), scratch=scratch):
            if q4:
                m.load_weights_q4(kind, layer, r0, *pv_inputs.quantize_q4(rows))
            else:
                m.load_weights(kind, layer, r0, rows)
    return m


def main():
    """Config-5 style run: python -m paper_2505_01572_amd.pipeline [--stages 1b,8b,70b_v128k] [--tokens 256]."""
    import argparse
    import json
    import os
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import torch
    import pv_inputs
    import paper_2505_01572_amd as pv

    ap = argparse.ArgumentParser()
    ap.add_argument("--stages", default="1b,8b,70b_v128k")
    ap.add_argument("--levels", default="0.7,0.8")
    ap.add_argument("--gamma", type=int, default=8)
    ap.add_argument("--prefix", type=int, default=1024)
    ap.add_argument("--tokens", type=int, default=256)
    a = ap.parse_args()
    names = a.stages.split(",")
    levels = [float(x) for x in a.levels.split(",")] + [1.0]
    assert len(levels) == len(names)
    shapes = [pv_inputs.CONFIGS[n] for n in names]
    vocab = shapes[-1].vocab
    assert all(s.vocab == vocab for s in shapes), "stages must share a vocabulary"
    prompt = pv_inputs.uniform_tokens(2005, a.prefix, vocab)
    span = a.tokens + 4 * a.gamma + 64
    stages = []
    for i, shp in enumerate(shapes):
        t0 = time.time()
        m = load_stage_model(pv, pv_inputs, shp)
        c = pv.Cache(m, a.prefix + span)
        c.prefill(prompt)
        print(f"[pipeline] stage {i} ({shp.name}) ready in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
        stages.append(Stage(i, c, levels[i], 1 if i == 0 else a.gamma, torch.cuda.Stream()))
    # reference sequence: the last stage's own greedy continuation (gamma = 1 steps), then back to the prompt
    last = stages[-1].cache
    target = [last.pending]
    for k in range(a.tokens + 2 * a.gamma + 8):
        n, nxt = last.verify(a.prefix + k, [target[-1]])
        target.append(nxt)
    last.rollback(a.prefix)
    u = pv_inputs.unit_draws(3005, len(target), stream=7)
    for s in stages:
        s.cache.set_pending(-1)
    res = run_pipeline(stages, a.prefix, np.array(target), u, vocab, a.tokens, timeout_s=600.0)
    assert res["output"] == [int(t) for t in target[:res["tokens"]]], "pipeline output differs from the last stage's greedy decoding"
    fin = res["stages"][-1]
    pred = closed_form_tokens_per_step(fin["alpha_measured"], fin["mean_block"] - 1.0)
    out = {"metric": "pipeline_tokens_per_s", "value": res["tokens_per_s"], "unit": "tok/s", "stages": names, "levels": levels[:-1],
           "gamma": a.gamma, "prefix": a.prefix, "tokens": res["tokens"], "lossless": True,
           "final_stage_tokens_per_step": fin["tokens_per_step"], "closed_form_tokens_per_step": pred,
           "per_stage": res["stages"]}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
