#!/usr/bin/env python3
"""Benchmark of the verification step (one pass of the whole hot path = one "step").

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 8b] [--gamma 8] [--prefix T] [--alpha A]

Builds a synthetic LLaMA-shaped verifier (seeded random bf16 weights, uniform-random prompt),
prefills the prompt, obtains the verifier's own greedy continuation with gamma=1 steps, and
then times K verify steps whose drafts are that continuation perturbed at rate 1-alpha.
Weights, KV cache and activations are resident in HBM when the timed region starts; each
step hands over gamma int32 draft ids and reads back two int32 results.

Prints ONE JSON line.  The top-level fields describe the headline workload (8B-shaped verifier,
prefix 2048, gamma 8): `value` = verified draft positions per second (gamma * steps / s);
`roofline` = the dominant kernel (the gate/up projection stream), timed with HIP events on the
step's stream in a second, instrumented pass over the same steps; `stream_ceiling` = what a plain
read-only stream of the step's byte count reaches on this device in this run; `prefill_tokens_per_s` =
the prompt's rate when it was fed in (once, 64-row chunks, outside the timed region); `cpu_baseline` =
the CPU oracle timed on a bounded slice of the same workload.  With no --workload / --gamma
given, `also` carries the other points of the metric measured the same way in the same run:
the 8B shape at gamma 1, 4, 16, batched verification of 4 sequences x gamma 8 on the 8B shape, and the
70B-shaped verifier (prefix 1024, gamma 8) with 16-bit and with 4-bit weights.
"""
import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

HBM_PEAK_GBPS = 8000.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")

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


def cpu_baseline(pv_inputs, shape, gamma, prefix, budget_s=20.0):
    """Oracle timed on the host: gamma-row verify steps on 1- and 2-layer slices of the shape at the
    workload's prefix length (the slices' caches are set to that length without running the prompt:
    the keys and values are the zeros they were allocated with, which costs the oracle the same
    arithmetic), repeated until about budget_s seconds of oracle work have been timed, the per-step
    medians extrapolated linearly in the layer count to the full depth."""
    import numpy as np
    from oracle import ref
    from helpers import ref_model
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    times, reps = {}, {}
    for nl in (1, 2):
        s = shape.replace(n_layers=nl)
        rm = ref_model(s)
        c = ref.RefCache(rm, prefix + 4 * gamma, ref.KV_BF16 if s.dtype == "bf16" else ref.KV_REAL)
        c.set_len(prefix)
        dts, t_used = [], 0.0
        while len(dts) < 3 or (t_used < budget_s / 2 and len(dts) < 400):
            d = pv_inputs.uniform_tokens(2100 + len(dts), gamma, s.vocab)
            t0 = time.time()
            c.verify(len(c), d)
            dt = time.time() - t0
            c.rollback(prefix)
            dts.append(dt); t_used += dt
        times[nl], reps[nl] = float(np.median(dts)), len(dts)
        del c, rm
    per_layer = max(times[2] - times[1], 1e-9)
    head = max(times[1] - per_layer, 0.0)
    full = head + per_layer * shape.n_layers
    return {"value": gamma / full, "unit": "tok/s", "cores": cores, "kind": "oracle", "real": "f64",
            "sample": f"gamma={gamma} verify steps of the oracle as the parity tests use it (fp64 build) on 1- and 2-layer slices of "
                      f"the {shape.name} shape at the workload's prefix of {prefix} (cache length set, prompt not run: the prefix's keys and "
                      f"values are zeros; {reps[1]} and {reps[2]} steps, about {budget_s:.0f} s of timed work; medians): "
                      f"{per_layer:.3f} s/layer + {head:.3f} s for embedding, final norm and LM head, "
                      f"extrapolated to {shape.n_layers} layers = {full:.2f} s/step"}


def measured_traffic(workload, gamma, kernel):
    """HBM bytes one launch of `kernel` moves, from the tracked hardware-counter summary (two rocprofv3
    --pmc runs, FETCH_SIZE and WRITE_SIZE, each scaled by the plain copy kernel of known size); None when
    the summary has no entry for this workload and block size.  The summary names the build it was
    taken from: it is evidence about that build, not a reading of this run."""
    try:
        tab = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return None, None
    e = tab.get("entries", {}).get(f"{workload}/rows<={8 if gamma <= 8 else 16}/{kernel}")
    return (e["fetched_bytes"] + e["written_bytes"], tab.get("source")) if e else (None, None)


class Workload:
    """One loaded model with its prompt prefilled and its greedy continuation known."""

    def __init__(self, pv, pv_inputs, name, T0, gammas, n_steps, use_graphs=True):
        import numpy as np
        self.pv, self.pvi, self.name, self.T0 = pv, pv_inputs, name, T0
        self.shape = shape = pv_inputs.CONFIGS[name]
        gmax = max(gammas)
        self.model = load_model(pv, pv_inputs, shape, max_gamma=16 if gmax <= 16 else 64)
        self.cache = pv.Cache(self.model, T0 + (2 * n_steps + 2) * gmax + 16)
        if not use_graphs:
            self.cache.use_graphs(False)
        t0 = time.time()
        self.cache.prefill(pv_inputs.uniform_tokens(2000 + shape.seed, T0, shape.vocab))     # (synchronises)
        self.prefill_s = time.time() - t0
        log(f"{name}: prefill of {T0} tokens: {self.prefill_s:.2f}s")
        # the verifier's own greedy continuation (gamma=1 steps), then back to the prompt
        self.first = self.cache.pending
        need = n_steps * gmax + gmax + 1
        G = np.empty(need, dtype=np.int32)
        G[0] = self.first
        t0 = time.time()
        for i in range(1, need):
            n, nxt = self.cache.verify(T0 + i - 1, G[i - 1:i])
            assert n == 1
            G[i] = nxt
        self.G = G
        log(f"{name}: greedy pre-pass of {need} tokens: {time.time() - t0:.2f}s")

    def _draft(self, T, gamma, alpha, step, trust):
        blk = self.G[T - self.T0: T - self.T0 + gamma]
        d = self.pvi.perturb_drafts(blk, alpha, self.shape.vocab, 3000 + self.shape.seed, step)
        if trust:
            d[0] = blk[0]
        return d

    def _steps(self, first_step, count, T, gamma, alpha, trust):
        accepted = 0
        for s in range(first_step, first_step + count):
            n, _ = self.cache.verify(T, self._draft(T, gamma, alpha, s, trust))
            T += n
            accepted += n
            trust = n == 0
        return T, trust, accepted

    def run(self, gamma, alpha, K, W, prof_kernel=None):
        """W warm-up steps, K timed steps (inputs resident; barrier = device synchronisation on both sides),
        then optionally the same K steps again with HIP events around every launch of one kernel."""
        import torch
        c = self.cache
        c.rollback(self.T0)
        c.set_pending(int(self.first))
        T, trust, _ = self._steps(0, W, self.T0, gamma, alpha, False)
        bytes_first = c.step_bytes(gamma)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        T_end, _, accepted = self._steps(W, K, T, gamma, alpha, trust)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        step_bytes = 0.5 * (bytes_first + c.step_bytes(gamma))
        r = {"gamma": gamma, "prefix": self.T0, "alpha": alpha, "ms_per_step": elapsed / K * 1e3, "steps_per_s": K / elapsed,
             "verified_tokens_per_s": gamma * K / elapsed, "committed_tokens_per_s": accepted / elapsed,
             "mean_accepted_len": accepted / K, "step_bytes": step_bytes,
             "step_hbm_gbps": step_bytes / (elapsed / K) / 1e9, "step_hbm_frac": step_bytes / (elapsed / K) / 1e9 / HBM_PEAK_GBPS,
             "prefill_tokens_per_s": self.T0 / self.prefill_s}     # the prompt, once, in 64-row chunks (untimed region; wall clock with its launch)
        if prof_kernel:
            c.rollback(T)
            c.set_pending(int(self.G[T - self.T0]))
            c.profile_select(self.pv.PROF[prof_kernel])
            self._steps(W, K, T, gamma, alpha, trust)
            ms, launches, kbytes = c.profile_read()
            c.profile_select(self.pv.PROF["none"])
            k_ms = ms / max(launches, 1)
            k_gbps = kbytes / (k_ms * 1e-3) / 1e9 if launches else 0.0
            traffic, source = measured_traffic(self.name, gamma, prof_kernel)
            r["roofline"] = {"bound": "hbm", "kernel": f"k_gemm<{prof_kernel}>", "achieved": k_gbps, "peak": HBM_PEAK_GBPS,
                             "unit": "GB/s", "frac": k_gbps / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": source,
                             "bytes_per_launch": kbytes, "avg_launch_us": k_ms * 1e3, "launches": launches}
        return r

    def run_batch(self, n_seq, gamma, alpha, K, W):
        """Batched verification: n_seq sequences (this one + n_seq - 1 more caches with prompts of their own),
        gamma drafts each, one pass over the weights per step.  Same timing discipline as run()."""
        import numpy as np
        import torch
        pv, pvi, shape, T0 = self.pv, self.pvi, self.shape, self.T0
        n_steps = K + W
        caches, Gs = [self.cache], [self.G]
        need = n_steps * gamma + gamma + 1
        t0 = time.time()
        for i in range(1, n_seq):
            c = pv.Cache(self.model, self.cache.max_tokens)
            c.prefill(pvi.uniform_tokens(2000 + shape.seed + 17 * i, T0, shape.vocab))
            G = np.empty(need, dtype=np.int32)
            G[0] = c.pending
            for k in range(1, need):
                n, nxt = c.verify(T0 + k - 1, G[k - 1:k])
                G[k] = nxt
            caches.append(c); Gs.append(G)
        log(f"{self.name}: {n_seq - 1} more sequences prefilled and pre-passed: {time.time() - t0:.2f}s")
        for c, G in zip(caches, Gs):
            c.rollback(T0); c.set_pending(int(G[0]))
        trust = [False] * n_seq

        def steps(first, count):
            acc = 0
            for st in range(first, first + count):
                drafts = []
                for i, (c, G) in enumerate(zip(caches, Gs)):
                    T = len(c)
                    blk = G[T - T0: T - T0 + gamma]
                    d = pvi.perturb_drafts(blk, alpha, shape.vocab, 3000 + shape.seed + 1000 * i, st)
                    if trust[i]:
                        d[0] = blk[0]
                    drafts.append(d)
                res = pv.verify_batch(caches, drafts)
                for i, (n, _) in enumerate(res):
                    acc += n; trust[i] = n == 0
            return acc
        steps(0, W)
        kv_tok = shape.kv_bytes_per_token()
        weights = self.cache.step_bytes(gamma) - kv_tok * (len(self.cache) + 2 * gamma)
        bytes_first = weights + sum(kv_tok * (len(c) + 2 * gamma) for c in caches)
        torch.cuda.synchronize()
        t_start = time.perf_counter()
        accepted = steps(W, K)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t_start
        step_bytes = 0.5 * (bytes_first + weights + sum(kv_tok * (len(c) + 2 * gamma) for c in caches))
        for c in caches[1:]:
            c.close()
        return {"sequences": n_seq, "gamma": gamma, "rows": n_seq * gamma, "prefix": T0, "alpha": alpha, "ms_per_step": elapsed / K * 1e3,
                "steps_per_s": K / elapsed, "verified_tokens_per_s": n_seq * gamma * K / elapsed, "committed_tokens_per_s": accepted / elapsed,
                "mean_accepted_len": accepted / K / n_seq, "step_bytes": step_bytes,
                "step_hbm_gbps": step_bytes / (elapsed / K) / 1e9, "step_hbm_frac": step_bytes / (elapsed / K) / 1e9 / HBM_PEAK_GBPS}

    def stream_ceiling(self, step_bytes, launch_bytes):
        """Plain read-only streams over the weight arena, timed with events on the stream they run on:
        one of the step's byte count, and launches of one kernel's byte count over successive regions
        (each region is touched once: HBM, not a cache, is what answers)."""
        import torch
        pv, arena = self.pv, self.model.arena
        total = arena.numel()
        sink = torch.zeros(16, dtype=torch.uint8, device=arena.device)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n = min(int(step_bytes), total) // 16 * 16
        best = float("inf")
        for _ in range(3):
            e0.record(); pv.calib_read(arena, n, 0, sink); e1.record(); e1.synchronize()
            best = min(best, e0.elapsed_time(e1))
        out = {"step_bytes_gbps": n / (best * 1e-3) / 1e9, "step_bytes_read": n}
        if launch_bytes:
            lb = int(launch_bytes) // 16 * 16
            reps = max(1, min(32, total // lb))
            e0.record()
            for i in range(reps):
                pv.calib_read(arena, lb, i * lb, sink)
            e1.record(); e1.synchronize()
            out["launch_bytes_gbps"] = lb * reps / (e0.elapsed_time(e1) * 1e-3) / 1e9
            out["launch_bytes"] = lb
        return out

    def close(self):
        import torch
        self.cache.close(); self.model.close()
        self.cache = self.model = None
        gc.collect(); torch.cuda.empty_cache()


def with_ceiling(r, ceil):
    r["stream_ceiling"] = {"gbps": ceil["step_bytes_gbps"], "frac_of_peak": ceil["step_bytes_gbps"] / HBM_PEAK_GBPS,
                           "step_frac_of_ceiling": r["step_hbm_gbps"] / ceil["step_bytes_gbps"],
                           "what": f"plain read-only stream of {ceil['step_bytes_read'] / 1e9:.2f} GB of the weight arena, event-timed, best of 3"}
    if "roofline" in r and "launch_bytes_gbps" in ceil:
        r["roofline"]["stream_ceiling_gbps"] = ceil["launch_bytes_gbps"]
        r["roofline"]["frac_of_ceiling"] = r["roofline"]["achieved"] / ceil["launch_bytes_gbps"]
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default=None, choices=sorted(DEFAULTS))
    ap.add_argument("--gamma", type=int, default=None)
    ap.add_argument("--prefix", type=int, default=None)
    ap.add_argument("--alpha", type=float, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-also", action="store_true", help="headline workload only (no gamma sweep, no 70B-shaped runs)")
    ap.add_argument("--batch", type=int, default=None, metavar="B",
                    help="also time batched verification of B sequences x gamma drafts (default run: 4)")
    ap.add_argument("--no-graphs", action="store_true", help="plain launches instead of HIP-graph replay of the step (comparison runs)")
    ap.add_argument("--prof-kernel", default="gateup")
    ap.add_argument("--calib-copy", type=int, default=0, metavar="MiB",
                    help="also launch the library's plain copy kernel on this many MiB three times (the known "
                         "quantity that hardware traffic counters read under rocprofv3 --pmc are scaled by)")
    a = ap.parse_args()
    if a.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import pv_inputs
    import paper_2505_01572_amd as pv

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    torch.cuda.set_device(0)
    sweep = a.workload is None and a.gamma is None and a.prefix is None and not a.no_also
    name = a.workload or "8b"
    T0, gamma, alpha = DEFAULTS[name]
    T0 = a.prefix if a.prefix is not None else T0
    gamma = a.gamma if a.gamma is not None else gamma
    alpha = a.alpha if a.alpha is not None else alpha
    K, W = a.steps, a.warmup
    gammas = sorted({gamma, 1, 4, 16}) if sweep else [gamma]

    wl = Workload(pv, pv_inputs, name, T0, gammas, K + W, use_graphs=not a.no_graphs)
    shape = wl.shape
    head = wl.run(gamma, alpha, K, W, prof_kernel=a.prof_kernel)
    ceil = wl.stream_ceiling(head["step_bytes"], head["roofline"]["bytes_per_launch"])
    with_ceiling(head, ceil)
    also = {}
    if sweep:
        for g in gammas:
            if g != gamma:
                also[f"{name}_gamma{g}"] = with_ceiling(wl.run(g, alpha, K, W), ceil)
                log(f"{name} gamma {g}: {also[f'{name}_gamma{g}']['ms_per_step']:.3f} ms/step")

    n_batch = a.batch if a.batch is not None else (4 if sweep else 0)
    if n_batch > 1:
        rb = with_ceiling(wl.run_batch(n_batch, gamma, alpha, K, W), ceil)
        also[f"{name}_batch{n_batch}_gamma{gamma}"] = rb
        log(f"{name} batch {n_batch} x gamma {gamma}: {rb['ms_per_step']:.3f} ms/step")

    if a.calib_copy > 0:
        src = torch.full((a.calib_copy << 20,), 1, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            pv.calib_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst
    wl.close()

    if sweep:                                   # the other shape the metric is quoted on, with 16-bit weights and in 4 bit (Sec. 4.1)
        for other in ("70b", "70b_q4"):
            T70, g70, a70 = DEFAULTS[other]
            w70 = Workload(pv, pv_inputs, other, T70, [g70], K + W, use_graphs=not a.no_graphs)
            r70 = w70.run(g70, a70, K, W, prof_kernel=a.prof_kernel)
            with_ceiling(r70, w70.stream_ceiling(r70["step_bytes"], r70["roofline"]["bytes_per_launch"]))
            r70["workload"] = f"{other}-shaped verifier, prefix {T70}, gamma {g70}, alpha {a70}, batch 1"
            also[f"{other}_gamma{g70}"] = r70
            log(f"{other} gamma {g70}: {r70['ms_per_step']:.3f} ms/step")
            w70.close()

    out = {
        "metric": "verify_tokens_per_s", "value": head["verified_tokens_per_s"], "unit": "tok/s",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{shape.name}-shaped verifier, prefix {T0}, gamma {gamma}, alpha {alpha}, batch 1"},
        "steps_per_s": head["steps_per_s"], "committed_tokens_per_s": head["committed_tokens_per_s"],
        "mean_accepted_len": head["mean_accepted_len"],
        "step_bytes": head["step_bytes"], "step_hbm_gbps": head["step_hbm_gbps"], "step_hbm_frac": head["step_hbm_frac"],
        "prefill_tokens_per_s": head["prefill_tokens_per_s"],
        "stream_ceiling": head["stream_ceiling"], "roofline": head["roofline"],
    }
    if also:
        out["also"] = also
    if not a.no_cpu_baseline:
        t0 = time.time()
        out["cpu_baseline"] = cpu_baseline(pv_inputs, shape, gamma, T0)
        log(f"cpu baseline: {time.time() - t0:.1f}s")
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
