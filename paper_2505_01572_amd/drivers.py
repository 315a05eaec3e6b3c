"""Autoregressive and synchronous speculative-decoding drives on the same verify kernels, next to
the asynchronous pipeline (paper Sec. 2.2, Sec. 3.3 Eq. 5 and Eq. 6, Table 1's sync/async and
single/multi-draft axes).

All arithmetic of a step runs in the library (pv_verify on the stage's cache); this module only
moves token ids.  Acceptance is synthetic exactly as in `pipeline.py`: every model runs its real
forward pass, but the token a draft model *emits* at generated index k is the reference token
target[k] when the shared draw u[k] is below the model's level and a wrong token otherwise, so
that alpha_{d,t} = level_d; the target model always emits the reference, so the output must be
`target` itself (greedy speculative decoding is lossless).
"""
import time

import numpy as np

from .pipeline import Stage, _settle, _wrong_token, run_pipeline, closed_form_tokens_per_step


def autoregressive(cache, prompt_len, first_token, n_tokens, stream=None):
    """Plain greedy decoding: one gamma = 1 step per token.  The cache holds the prompt;
    first_token is the model's own token after the prompt.  Returns (tokens, seconds, steps)."""
    out = [int(first_token)]
    cache.rollback(prompt_len, stream=stream)
    t0 = time.perf_counter()
    for k in range(n_tokens):
        n, nxt = cache.verify(prompt_len + k, [out[-1]], stream=stream)
        if n != 1:
            raise RuntimeError("a trusted single token was not accepted")
        out.append(nxt)
    return out, time.perf_counter() - t0, n_tokens


def speculative_sync(draft, target_cache, prompt_len, target, u, vocab, n_tokens, n_draft, stream=None):
    """Synchronous draft-then-verify speculative decoding with two models (Sec. 2.2; the scheme
    Eq. 5 prices): per round the draft model produces n_draft tokens one after the other, then the
    target model checks [its own last token, the n_draft drafts] in one block and keeps the
    matching prefix plus its own next token; the draft model is rolled back to the kept length.

    draft: a Stage (cache + level) holding the prompt; target_cache holds the prompt too.
    target / u: reference tokens and uniform draws by generated index (len >= n_tokens + n_draft + 2).
    Returns a dict of counts and timings; "output" is the committed sequence.
    """
    def emit_draft(k):
        return int(target[k]) if u[k] < draft.level else _wrong_token(target[k], 0, vocab)

    out = [int(target[0])]       # index 0: the target model's own token after the prompt
    m = 0                        # committed generated tokens whose K/V the target cache holds
    dlen = 0                     # generated tokens whose K/V the draft cache holds
    rounds = rows = drafted = accepted = rejections = draft_steps = 0
    t_draft = t_target = 0.0
    draft.cache.rollback(prompt_len, stream=stream)
    target_cache.rollback(prompt_len, stream=stream)
    target_cache.set_pending(out[0], stream=stream)
    t_start = time.perf_counter()
    while m < n_tokens:
        # draft phase.  First bring the draft cache to the committed sequence: cut what was
        # rejected, then consume what it has not seen yet (the target's correction or bonus token,
        # plus its own last draft when everything was accepted) in one block.
        t0 = time.perf_counter()
        dlen = min(dlen, m)
        feed = out[dlen:m + 1]
        draft.cache.rollback(prompt_len + dlen, stream=stream)              # also forgets pending: the inputs are trusted
        draft.cache.verify(prompt_len + dlen, feed, stream=stream)
        _settle(draft.cache, prompt_len + m + 1, -1, stream)
        dlen = m + 1
        draft_steps += 1
        block = [out[m], emit_draft(m + 1)]
        for i in range(1, n_draft):
            draft.cache.verify(prompt_len + m + i, [block[-1]], stream=stream)
            _settle(draft.cache, prompt_len + m + i + 1, -1, stream)
            dlen += 1
            block.append(emit_draft(m + i + 1))
            draft_steps += 1
        t1 = time.perf_counter()
        # verify phase: one block forward of the target model over [own token, drafts]
        target_cache.verify(prompt_len + m, block, stream=stream)
        n = 1                                                                 # block[0] is the target's own token
        while n < len(block) and block[n] == int(target[m + n]):
            n += 1
        nxt = int(target[m + n])
        _settle(target_cache, prompt_len + m + n, nxt, stream)
        t2 = time.perf_counter()
        out = out[:m] + block[:n] + [nxt]
        rounds += 1; rows += len(block); drafted += n_draft; accepted += n - 1
        rejections += 1 if n < len(block) else 0
        m += n
        t_draft += t1 - t0; t_target += t2 - t1
    elapsed = time.perf_counter() - t_start
    return {"output": out[:m], "tokens": m, "elapsed_s": elapsed, "tokens_per_s": m / elapsed, "rounds": rounds,
            "rows": rows, "tokens_per_round": m / rounds,
            # acceptance rate over the draft positions that were actually compared: a round that keeps
            # j < n_draft drafts compared j + 1 of them
            "alpha_trials": accepted / max(1, accepted + rejections),
            "accepted_drafts": accepted, "rejections": rejections, "drafted": drafted, "draft_steps": draft_steps,
            "draft_s": t_draft, "target_s": t_target}


def sd_closed_form(alpha, n_draft, c):
    """Eq. 5: expected speedup of synchronous speculative decoding over the target model alone;
    c = draft steps per target step (speed ratio), n_draft = drafts per round."""
    geo = (1.0 - alpha ** (n_draft + 1)) / (1.0 - alpha) if alpha < 1.0 else n_draft + 1.0
    return geo / (n_draft / c + 1.0)


def pipespec_closed_form(alpha, n_draft):
    """Eq. 6: high-acceptance approximation of the asynchronous two-stage rate, in tokens per
    target step."""
    return (1.0 - alpha ** (n_draft + 1)) / (1.0 - alpha) if alpha < 1.0 else n_draft + 1.0


def main():
    """python -m paper_2505_01572_amd.drivers [--draft 1b] [--mid 8b] [--target 70b_v128k] [--tokens 128]

    Runs, on one GPU and the same kernels: the target model alone (autoregressive), synchronous
    speculative decoding {draft, target}, the asynchronous two-stage pipeline {draft, target} and
    the asynchronous three-stage pipeline {draft, mid, target}; prints one JSON line with the
    measured rates, speedups over autoregressive decoding and the closed forms at the measured
    acceptance rates and step-time ratio."""
    import argparse
    import json
    import os
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    sys.path.insert(0, root)
    import torch
    import pv_inputs
    import paper_2505_01572_amd as pv
    from .pipeline import load_stage_model

    ap = argparse.ArgumentParser()
    ap.add_argument("--draft", default="1b")
    ap.add_argument("--mid", default="8b")
    ap.add_argument("--target", default="70b_v128k")
    ap.add_argument("--level-draft", type=float, default=0.7)
    ap.add_argument("--level-mid", type=float, default=0.8)
    ap.add_argument("--n-draft", type=int, default=7, help="drafts per round; a block has n_draft + 1 rows")
    ap.add_argument("--prefix", type=int, default=1024)
    ap.add_argument("--tokens", type=int, default=128)
    a = ap.parse_args()
    names = [a.draft, a.mid, a.target]
    shapes = [pv_inputs.CONFIGS[n] for n in names]
    vocab = shapes[-1].vocab
    assert all(s.vocab == vocab for s in shapes), "stages must share a vocabulary"
    prompt = pv_inputs.uniform_tokens(2005, a.prefix, vocab)
    span = a.tokens + 6 * (a.n_draft + 1) + 64
    caches = []
    for shp in shapes:
        t0 = time.time()
        m = load_stage_model(pv, pv_inputs, shp)
        c = pv.Cache(m, a.prefix + span)
        c.prefill(prompt)
        print(f"[drivers] {shp.name} ready in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)
        caches.append(c)
    cd, cm, ct = caches
    gamma = a.n_draft + 1

    # 1. the target alone; its output is the reference sequence
    first = ct.pending
    target, ar_s, _ = autoregressive(ct, a.prefix, first, a.tokens + 4 * gamma + 8)
    ar_rate = (len(target) - 1) / ar_s
    t_target_step = ar_s / (len(target) - 1)
    dfirst = cd.pending
    _, d_s, d_n = autoregressive(cd, a.prefix, dfirst, 64)
    t_draft_step = d_s / d_n
    c_ratio = t_target_step / t_draft_step
    u = pv_inputs.unit_draws(3005, len(target), stream=7)
    target = np.array(target)

    # 2. synchronous speculative decoding {draft, target}
    sd = speculative_sync(Stage(0, cd, a.level_draft, 1), ct, a.prefix, target, u, vocab, a.tokens, a.n_draft)
    assert sd["output"] == [int(t) for t in target[:sd["tokens"]]], "speculative decoding changed the output"

    # 3. asynchronous pipelines
    def run_async(stage_caches, levels):
        stages = []
        for i, (c, lv) in enumerate(zip(stage_caches, levels)):
            c.rollback(a.prefix)
            c.set_pending(-1)
            stages.append(Stage(i, c, lv, 1 if i == 0 else gamma, torch.cuda.Stream()))
        res = run_pipeline(stages, a.prefix, target, u, vocab, a.tokens, timeout_s=600.0)
        assert res["output"] == [int(t) for t in target[:res["tokens"]]], "pipeline output differs from the target's greedy decoding"
        return res

    p2 = run_async([cd, ct], [a.level_draft, 1.0])
    p3 = run_async([cd, cm, ct], [a.level_draft, a.level_mid, 1.0])

    def fin(res):
        f = res["stages"][-1]
        return {"tokens_per_s": res["tokens_per_s"], "speedup_vs_ar": res["tokens_per_s"] / ar_rate,
                "target_steps_per_s": f["steps_per_s"], "tokens_per_target_step": f["tokens_per_step"],
                "alpha_measured": f["alpha_measured"], "mean_block": f["mean_block"],
                "closed_form_tokens_per_step": closed_form_tokens_per_step(f["alpha_measured"], f["mean_block"] - 1.0)}

    out = {"metric": "decoding_drives_tokens_per_s", "unit": "tok/s", "models": names, "prefix": a.prefix, "tokens": a.tokens,
           "n_draft": a.n_draft, "levels": [a.level_draft, a.level_mid],
           "autoregressive": {"tokens_per_s": ar_rate, "target_step_ms": t_target_step * 1e3, "draft_step_ms": t_draft_step * 1e3,
                              "speed_ratio_c": c_ratio},
           "sync_sd": {"tokens_per_s": sd["tokens_per_s"], "speedup_vs_ar": sd["tokens_per_s"] / ar_rate,
                       "tokens_per_round": sd["tokens_per_round"], "alpha_measured": sd["alpha_trials"],
                       "closed_form_speedup_eq5": sd_closed_form(sd["alpha_trials"], a.n_draft, c_ratio),
                       "draft_s": sd["draft_s"], "target_s": sd["target_s"]},
           "async_two_stage": dict(fin(p2), closed_form_eq6=pipespec_closed_form(p2["stages"][-1]["alpha_measured"], a.n_draft)),
           "async_three_stage": fin(p3), "lossless": True}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
