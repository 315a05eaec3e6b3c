#!/usr/bin/env python3
"""Benchmark of the verification step (one pass of the whole hot path = one "step").

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b] [--gamma 8] [--prefix T] [--alpha A]

Builds a synthetic LLaMA-shaped verifier (seeded random bf16 weights, uniform-random prompt),
prefills the prompt, obtains the verifier's own greedy continuation with gamma=1 steps, and
then times K verify steps whose drafts are that continuation perturbed at rate 1-alpha.
Weights, KV cache and activations are resident in HBM when the timed region starts; each
step hands over gamma int32 draft ids and reads back two int32 results.

Prints ONE JSON line.  `value` = verified draft positions per second (gamma * steps / s).
`roofline` describes the dominant kernel (the gate/up projection stream), timed with HIP
events on the step's stream in a second, instrumented pass over the same steps.
`cpu_baseline` times the CPU oracle on a bounded slice of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0

# HBM bytes one launch of the dominant kernel moves, from hardware counters: FETCH_SIZE and
# WRITE_SIZE of two separate rocprofv3 --pmc runs of this script, each scaled by what the same
# counter reads for the library's plain copy kernel (--calib-copy) of known size.  Summary and
# commands: profiles/hbm_traffic_pmc_8b_70b.txt.  Keyed by (workload, gamma bucket, kernel).
MEASURED_TRAFFIC = {
    ("8b", "rows<=8", "gateup"): 236364522 + 171176,
    ("70b", "rows<=8", "gateup"): 949250066 + 391260,
}

DEFAULTS = {  # workload -> (prefix, gamma, alpha)
    "tiny": (64, 4, 0.7), "7b": (512, 8, 0.8), "8b": (2048, 8, 0.7), "70b": (1024, 8, 0.6),
    "1b": (1024, 1, 0.7), "70b_v128k": (1024, 8, 0.6), "70b_q4": (1024, 8, 0.6), "8b_q4": (2048, 8, 0.7),
}


def log(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def load_model(pv, pv_inputs, shape, max_gamma, kernel_path=0):
    t0 = time.time()
    m = pv.Model(shape, max_gamma=max_gamma, kernel_path=kernel_path)
    done = 0
    total = shape.n_params()
    # one pinned host buffer, reused for every chunk (no fresh page faults, fast host-to-device copies)
    import torch
    widest = max(pv_inputs.tensor_shape(shape, kind)[-1] for kind, _ in pv_inputs.iter_tensors(shape))
    need = max(m.staging_bytes, 16 * widest * m.np_dtype().itemsize)     # (a model without a staging area still gets 16-row chunks)
    pinned = torch.empty(need // 2, dtype=torch.int16, pin_memory=True)
    scratch = pinned.numpy().view(m.np_dtype)
    last = t0
    for kind, layer in pv_inputs.iter_tensors(shape):
        cols = pv_inputs.tensor_shape(shape, kind)[-1]
        q4 = shape.weight_bits == 4 and kind in pv_inputs.Q4_KINDS
        for r0, rows in pv_inputs.iter_row_chunks(shape, kind, layer, m.chunk_rows(cols), scratch=scratch):
            if q4:
                m.load_weights_q4(kind, layer, r0, *pv_inputs.quantize_q4(rows))
            else:
                m.load_weights(kind, layer, r0, rows)
            done += rows.size
        if time.time() - last > 20:
            last = time.time()
            log(f"weights {done / total * 100:.0f}% ({done * 2 / 1e9:.1f} GB) in {last - t0:.0f}s")
    log(f"weights loaded: {total / 1e9:.2f} G params in {time.time() - t0:.1f}s")
    return m


def cpu_baseline(pv_inputs, shape, gamma, budget_s=20.0):
    """Oracle timed on the host: gamma-row verify steps on 1- and 2-layer slices of the shape
    (prefix 64), repeated until about budget_s seconds of oracle work have been timed, the
    per-step medians extrapolated linearly in the layer count to the full depth."""
    import numpy as np
    from oracle import ref
    from helpers import ref_model
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    times, reps = {}, {}
    for nl in (1, 2):
        s = shape.replace(n_layers=nl)
        rm = ref_model(s)
        c = ref.RefCache(rm, 64 + 4 * gamma, ref.KV_BF16 if s.dtype == "bf16" else ref.KV_REAL)
        c.forward_block(pv_inputs.uniform_tokens(2000, 64, s.vocab), want_logits=False)
        c.pending = -1
        dts, t_used = [], 0.0
        while len(dts) < 3 or (t_used < budget_s / 2 and len(dts) < 400):
            d = pv_inputs.uniform_tokens(2100 + len(dts), gamma, s.vocab)
            t0 = time.time()
            c.verify(len(c), d)
            dt = time.time() - t0
            c.rollback(64)
            dts.append(dt); t_used += dt
        times[nl], reps[nl] = float(np.median(dts)), len(dts)
        del c, rm
    per_layer = max(times[2] - times[1], 1e-9)
    head = max(times[1] - per_layer, 0.0)
    full = head + per_layer * shape.n_layers
    return {"value": gamma / full, "unit": "tok/s", "cores": cores, "kind": "oracle",
            "sample": f"gamma={gamma} verify steps of the fp64 oracle on 1- and 2-layer slices of the {shape.name} shape "
                      f"(prefix 64; {reps[1]} and {reps[2]} steps, about {budget_s:.0f} s of timed work; medians): "
                      f"{per_layer:.3f} s/layer + {head:.3f} s for embedding, final norm and LM head, "
                      f"extrapolated to {shape.n_layers} layers = {full:.2f} s/step"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="8b", choices=sorted(DEFAULTS))
    ap.add_argument("--gamma", type=int, default=None)
    ap.add_argument("--prefix", type=int, default=None)
    ap.add_argument("--alpha", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graphs", action="store_true", help="plain launches instead of HIP-graph replay of the step (comparison runs)")
    ap.add_argument("--prof-kernel", default="gateup")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MiB",
                    help="also launch the library's plain copy kernel on this many MiB three times (the known "
                         "quantity that hardware traffic counters read under rocprofv3 --pmc are scaled by)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import pv_inputs
    import paper_2505_01572_amd as pv

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    shape = pv_inputs.CONFIGS[a.workload]
    T0, gamma, alpha = DEFAULTS[a.workload]
    T0 = a.prefix if a.prefix is not None else T0
    gamma = a.gamma if a.gamma is not None else gamma
    alpha = a.alpha if a.alpha is not None else alpha
    K, W = a.steps, a.warmup
    n_steps = K + W

    model = load_model(pv, pv_inputs, shape, max_gamma=16 if gamma <= 16 else 64)
    max_tokens = T0 + (2 * n_steps + 2) * gamma + 16
    cache = pv.Cache(model, max_tokens)
    if a.no_graphs:
        cache.use_graphs(False)
    prompt = pv_inputs.uniform_tokens(2000 + shape.seed, T0, shape.vocab)
    t0 = time.time()
    cache.prefill(prompt)
    log(f"prefill of {T0} tokens: {time.time() - t0:.2f}s")

    # the verifier's own greedy continuation (gamma=1 steps), then back to the prompt
    first = cache.pending
    need = n_steps * gamma + gamma + 1
    G = np.empty(need, dtype=np.int32)
    G[0] = first
    t0 = time.time()
    for i in range(1, need):
        n, nxt = cache.verify(T0 + i - 1, G[i - 1:i])
        assert n == 1
        G[i] = nxt
    log(f"greedy pre-pass of {need} tokens: {time.time() - t0:.2f}s")
    cache.rollback(T0)
    cache.set_pending(int(first))

    def draft_for(T, step, trust):
        blk = G[T - T0: T - T0 + gamma]
        d = pv_inputs.perturb_drafts(blk, alpha, shape.vocab, 3000 + shape.seed, step)
        if trust:
            d[0] = blk[0]
        return d

    def run_steps(first_step, count, T, trust):
        accepted = 0
        for s in range(first_step, first_step + count):
            n, _ = cache.verify(T, draft_for(T, s, trust))
            T += n
            accepted += n
            trust = n == 0
        return T, trust, accepted

    T, trust, _ = run_steps(0, W, T0, False)
    bytes_first = cache.step_bytes(gamma)
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    T_end, trust_end, accepted = run_steps(W, K, T, trust)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    bytes_last = cache.step_bytes(gamma)
    ms_per_step = elapsed / K * 1e3
    step_bytes = 0.5 * (bytes_first + bytes_last)
    hbm_gbps = step_bytes / (elapsed / K) / 1e9

    # instrumented replay of the same K steps: HIP events around every launch of the dominant kernel
    cache.rollback(T)
    cache.set_pending(int(G[T - T0]))
    cache.profile_select(pv.PROF[a.prof_kernel])
    run_steps(W, K, T, trust)
    ms, launches, kbytes = cache.profile_read()
    cache.profile_select(pv.PROF["none"])
    k_ms = ms / max(launches, 1)
    k_gbps = kbytes / (k_ms * 1e-3) / 1e9 if launches else 0.0

    if a.calib_copy > 0:
        src = torch.full((a.calib_copy << 20,), 1, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            pv.calib_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    traffic = MEASURED_TRAFFIC.get((a.workload, "rows<=8" if gamma <= 8 else "rows<=16", a.prof_kernel))

    out = {
        "metric": "verify_tokens_per_s", "value": gamma * K / elapsed, "unit": "tok/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}-shaped verifier, prefix {T0}, gamma {gamma}, alpha {alpha}, batch 1",
                   "n_layers": shape.n_layers, "d_model": shape.d_model, "vocab": shape.vocab,
                   "page_tokens": shape.page_tokens},
        "steps_per_s": K / elapsed, "committed_tokens_per_s": accepted / elapsed,
        "mean_accepted_len": accepted / K,
        "step_bytes": step_bytes, "step_hbm_gbps": hbm_gbps, "step_hbm_frac": hbm_gbps / HBM_PEAK_GBPS,
        "roofline": {"bound": "hbm", "kernel": f"k_gemm<{a.prof_kernel}>", "achieved": k_gbps, "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": k_gbps / HBM_PEAK_GBPS, "traffic": traffic,
                     "bytes_per_launch": kbytes, "avg_launch_us": k_ms * 1e3, "launches": launches},
    }
    if not a.no_cpu_baseline:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(pv_inputs, shape, gamma)
        log(f"cpu baseline: {time.time() - t0:.1f}s")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
