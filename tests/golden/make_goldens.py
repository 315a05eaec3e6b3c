#!/usr/bin/env python3
"""Writes tests/golden/verify_<config>.npz: what the CPU oracle computes for the benchmark
configurations at full depth, for the GPU parity tests to load.

Calls only oracle/ (the plain CPU decoder) and pv_inputs/ (seeded input generators); nothing here
touches the HIP library, and no stored value comes from it.

Per configuration: the seeded prompt is run through every layer, then verify steps
(Algorithm 1, verify branch; Sec. 3.3 after Eq. 1: the correction token) with drafts = the oracle's
own greedy continuation, each position replaced by a uniform token with probability 1 - alpha.
Two drives:
  chain  the model fits in host memory: greedy continuation by single-token decodes, steps follow
         each other (each starts where the last one's accepted prefix ends), like bench.py;
  tree   the model is generated layer by layer (oracle/replay.py) and each pass over the weights
         costs minutes: a few passes find the first greedy tokens, then all steps are verified in one
         pass, each on top of the prompt (as after pv_rollback to the prompt + pv_cache_set_pending).
Stored per step: start position, pending token, draft, per-row argmax, top-2 margin and RMS of the
row's logits, accepted length, correction token, the row's logits at a fixed strided set of ids and at
its 64 largest ids; plus K/V of sampled (layer, position) pairs after the prompt.

    python tests/golden/make_goldens.py 8b            # one of: 1b 7b 8b 70b 70b_v128k 70b_q4  (or a test shape)
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import pv_inputs                      # noqa: E402
from oracle import ref, replay       # noqa: E402

# name -> (drive, prefix, alphas, block sizes of the steps of one chain / of the tree, greedy tokens to find first (tree))
PLANS = {
    "1b": ("chain", 1024, (0.7,), (8, 1, 8, 16, 4, 8), 0),
    "7b": ("chain", 512, (0.5, 0.8), (8, 8, 8, 8), 0),
    "8b": ("chain", 2048, (0.7,), (8, 16, 4, 1, 8, 8), 0),
    "70b": ("tree", 1024, (0.6,), (8, 8, 8, 8, 16, 1), 5),
    "70b_v128k": ("tree", 256, (0.6,), (8, 8, 8, 1), 4),
    "70b_q4": ("tree", 128, (0.6,), (8, 8, 1), 2),            # the 70B shape in 4 bit (Sec. 4.1); prompt cut to 128 (CPU time)
}
TOP = 64


def log(msg):
    print(f"[goldens {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def sample_ids(vocab):
    return np.arange(0, vocab, max(1, vocab // 4096), dtype=np.int32)


class Recorder:
    def __init__(self, shape, gmax):
        self.shape, self.gmax, self.ids = shape, gmax, sample_ids(shape.vocab)
        self.rows = {k: [] for k in ("T", "pending", "gamma", "alpha", "draft", "pred", "accepted", "next_token", "margin", "rms",
                                     "sample_logits", "top_ids", "top_vals")}

    def add(self, T, pending, alpha, draft, logits):
        """Applies the acceptance rule to the block's logits (the same rule ref_verify applies: the rows'
        argmax, ties to the lowest id, longest matching prefix, correction token) and records the step."""
        g, gm = len(draft), self.gmax
        pred = np.argmax(logits, axis=1).astype(np.int32)             # first occurrence of the maximum
        n = 0
        while n < g and draft[n] == ((pending if pending >= 0 else draft[0]) if n == 0 else pred[n - 1]):
            n += 1
        nxt = int(pred[n - 1]) if n >= 1 else int(pending)
        srt = np.sort(logits, axis=1)
        pad = lambda a, fill, dt: np.concatenate([np.asarray(a, dtype=dt), np.full((gm - g,) + np.shape(a)[1:], fill, dtype=dt)])
        top = np.argsort(-logits, axis=1, kind="stable")[:, :TOP].astype(np.int32)
        r = self.rows
        r["T"].append(T); r["pending"].append(pending); r["gamma"].append(g); r["alpha"].append(alpha)
        r["draft"].append(pad(draft, -1, np.int32)); r["pred"].append(pad(pred, -1, np.int32))
        r["accepted"].append(n); r["next_token"].append(nxt)
        r["margin"].append(pad(srt[:, -1] - srt[:, -2], 0.0, np.float64))
        r["rms"].append(pad(np.sqrt((logits ** 2).mean(axis=1)), 0.0, np.float64))
        r["sample_logits"].append(pad(logits[:, self.ids], 0.0, np.float32))
        r["top_ids"].append(pad(top, -1, np.int32))
        r["top_vals"].append(pad(np.take_along_axis(logits, top, axis=1), 0.0, np.float32))
        return n, nxt, pred

    def arrays(self):
        r = self.rows
        out = {f"step_{k}": np.array(r[k]) for k in ("T", "pending", "gamma", "alpha", "accepted", "next_token")}
        out.update({k: np.stack(r[k]) for k in ("draft", "pred", "margin", "rms", "sample_logits", "top_ids", "top_vals")})
        out["sample_ids"] = self.ids
        return out


def kv_sample(shape, export, T):
    """K/V of a few (layer, position) pairs from the oracle's logical export [L][2][len][kv_dim]."""
    L = shape.n_layers
    layers = np.unique(np.array([0, 1, L // 2, L - 1], dtype=np.int32).clip(0, L - 1))
    pos = np.unique(np.array([0, 1, T // 2, T - 2, T - 1], dtype=np.int32).clip(0, T - 1))
    return {"kv_layers": layers, "kv_pos": pos, "kv_sample": export[layers][:, :, pos, :].astype(np.float32)}


def tensor_source(shape, keep):
    """tensors(kind, layer) for the oracle: drawn from the seeded generator, kept in memory if `keep`."""
    held = {}

    def get(kind, layer):
        if (kind, layer) in held:
            return held[(kind, layer)]
        a = pv_inputs.fill_tensor(shape, kind, layer).reshape(pv_inputs.tensor_shape(shape, kind))
        if getattr(shape, "weight_bits", 16) == 4 and kind in pv_inputs.Q4_KINDS:
            # the model's weights ARE the codes and scales; the oracle runs on their float32 values (exact).
            # Rows are independent: the oracle's routine is called on row blocks from a few threads.
            codes, scales = pv_inputs.quantize_q4(a)
            cuts = list(range(0, a.shape[0], 2048)) + [a.shape[0]]
            with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
                parts = list(pool.map(lambda i: ref.dequant_q4(codes[cuts[i]:cuts[i + 1]], scales[cuts[i]:cuts[i + 1]]), range(len(cuts) - 1)))
            a = np.concatenate(parts) if len(parts) > 1 else parts[0]
        if keep:
            held[(kind, layer)] = a
        return a
    return get


def padded_greedy(G, gamma, vocab, seed):
    """The first gamma tokens of the greedy continuation; positions beyond what is known get uniform ids
    (they stand behind a position the draft has to get right first)."""
    blk = pv_inputs.uniform_tokens(seed, gamma, vocab, stream=77)
    k = min(gamma, len(G))
    blk[:k] = G[:k]
    return blk


def make_chain(shape, T, alphas, gammas, out):
    kv_mode = ref.KV_BF16 if shape.dtype == "bf16" else ref.KV_REAL
    gmax, V = max(gammas), shape.vocab
    m = ref.RefModel(shape)
    src = tensor_source(shape, keep=True)
    t0 = time.time()
    for kind, layer in pv_inputs.iter_tensors(shape):
        m.set_tensor(kind, layer, src(kind, layer))
    log(f"{shape.name}: weights drawn in {time.time() - t0:.0f}s")
    prompt = pv_inputs.uniform_tokens(2000 + shape.seed, T, V)
    c = ref.RefCache(m, T + sum(gammas) + gmax + 8, kv_mode)
    t0 = time.time()
    for s in range(0, T, 64):
        last = c.forward_block(prompt[s:s + 64], only_last=True, want_logits=s + 64 >= T)
        if (s // 64) % 4 == 3:
            log(f"{shape.name}: prompt {s + 64}/{T} in {time.time() - t0:.0f}s")
    first = int(np.argmax(last[0]))
    srt = np.sort(last[0])
    extra = kv_sample(shape, c.export(), T)
    rec = Recorder(shape, gmax)
    chains = []
    for ci, alpha in enumerate(alphas):
        c.rollback(T)
        G, Gm = [first], [float(srt[-1] - srt[-2])]      # greedy continuation from position T and the margin each token won by
        Tk, pending, trust, step0 = T, first, False, len(rec.rows["T"])
        for k, g in enumerate(gammas):
            # the greedy tokens this draft is built from: single-token decodes beyond what is known, then back
            have = Tk - T
            while len(G) < have + g:
                for j in range(have, len(G) - 1):
                    c.decode_one(G[j])
                lg = c.decode_one(G[-1])
                s2 = np.sort(lg)
                G.append(int(np.argmax(lg))); Gm.append(float(s2[-1] - s2[-2]))
                c.rollback(Tk)
            blk = np.array(G[have:have + g], dtype=np.int32)
            d = pv_inputs.perturb_drafts(blk, alpha, V, 3000 + shape.seed + 100 * ci, k)
            if trust:
                d[0] = blk[0]
            c.pending = pending
            n_r, t_r, pred_r, lg = c.verify(Tk, d, want_logits=True)
            n, nxt, pred = rec.add(Tk, pending, alpha, d, lg)
            assert (n, nxt) == (n_r, t_r) and np.array_equal(pred, pred_r)          # the recorder's rule is ref_verify's
            assert np.array_equal(d[:n], blk[:n])                                      # only greedy tokens are ever accepted
            if have + n == len(G):                    # the whole known continuation was accepted: the correction token extends it
                mrow = np.sort(lg[n - 1])
                G.append(nxt); Gm.append(float(mrow[-1] - mrow[-2]))
            assert nxt == G[have + n]
            log(f"{shape.name}: alpha {alpha} step {k}: T {Tk} gamma {g} accepted {n} next {nxt}")
            Tk, pending, trust = Tk + n, nxt, n == 0
        chains.append((step0, len(rec.rows["T"]), np.array(G, dtype=np.int32), np.array(Gm)))
    arrs = rec.arrays()
    for i, (a, b, G, Gm) in enumerate(chains):
        arrs[f"chain{i}_steps"] = np.array([a, b], dtype=np.int32)
        arrs[f"chain{i}_greedy"] = G
        arrs[f"chain{i}_greedy_margin"] = Gm
    arrs.update(extra)
    save(out, shape, "chain", T, arrs)


def make_tree(shape, T, alphas, gammas, find, out):
    kv_mode = ref.KV_BF16 if shape.dtype == "bf16" else ref.KV_REAL
    gmax, V = max(gammas), shape.vocab
    run = replay.LayerwiseRun(shape, tensor_source(shape, keep=False), T + gmax + 8, kv_mode,
                              log=lambda msg: log(f"{shape.name}: {msg}"))
    prompt = pv_inputs.uniform_tokens(2000 + shape.seed, T, V)
    t0 = time.time()
    lg = run.run([(0, prompt)], commit=0)[0][-1]
    log(f"{shape.name}: prompt of {T} tokens through {shape.n_layers} layers in {time.time() - t0:.0f}s")
    extra = kv_sample(shape, run.c.export(), T)
    srt = np.sort(lg)
    G, Gm = [int(np.argmax(lg))], [float(srt[-1] - srt[-2])]
    for i in range(find):                                   # one pass over the weights per further greedy token
        lg = run.run([(T, np.array(G, dtype=np.int32))])[0][-1]
        srt = np.sort(lg)
        G.append(int(np.argmax(lg))); Gm.append(float(srt[-1] - srt[-2]))
        log(f"{shape.name}: greedy token {i + 1}/{find} found ({time.time() - t0:.0f}s)")
    alpha = alphas[0]
    drafts = []
    for k, g in enumerate(gammas):
        blk = padded_greedy(G, g, V, 4000 + shape.seed + k)
        d = pv_inputs.perturb_drafts(blk, alpha, V, 3000 + shape.seed, k)
        if k % 2 == 1:
            d[0] = blk[0]                                   # every other step keeps the first position (the steps after a zero-accept step do)
        drafts.append(d)
    logits = run.run([(T, d) for d in drafts])
    rec = Recorder(shape, gmax)
    for d, lg in zip(drafts, logits):
        n, nxt, _ = rec.add(T, G[0], alpha, d, lg)
        assert n == 0 or nxt == G[n] if n < len(G) else True                           # lossless
        log(f"{shape.name}: step gamma {len(d)} accepted {n} next {nxt}")
    arrs = rec.arrays()
    arrs["chain0_steps"] = np.array([0, len(gammas)], dtype=np.int32)
    arrs["chain0_greedy"] = np.array(G, dtype=np.int32)
    arrs["chain0_greedy_margin"] = np.array(Gm)
    arrs.update(extra)
    save(out, shape, "tree", T, arrs)


def save(out, shape, drive, T, arrs):
    meta = {"config": shape.name, "drive": drive, "prefix": T, "n_layers": shape.n_layers, "prompt_seed": 2000 + shape.seed,
            "oracle_real": "f64", "kv_store": "bf16" if shape.dtype == "bf16" else "real", "top": TOP}
    np.savez_compressed(out, meta=np.frombuffer(json.dumps(meta).encode(), dtype=np.uint8), **arrs)
    log(f"wrote {out} ({os.path.getsize(out) / 1e6:.2f} MB)")


def make(name, shape=None, plan=None, out=None):
    shape = shape or pv_inputs.CONFIGS[name]
    drive, T, alphas, gammas, find = plan or PLANS[name]
    out = out or os.path.join(HERE, f"verify_{name}.npz")
    if drive == "chain":
        make_chain(shape, T, alphas, gammas, out)
    else:
        make_tree(shape, T, alphas, gammas, find, out)
    return out


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("config", choices=sorted(PLANS))
    a = ap.parse_args()
    make(a.config)
