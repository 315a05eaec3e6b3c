"""The layer-by-layer oracle drive and the script that writes tests/golden/*.npz, checked on a model
small enough to run both ways (CPU only)."""
import importlib.util
import json
import os

import numpy as np
import pytest

import pv_inputs
from oracle import ref, replay
from helpers import ref_model, greedy_continuation

GQA = pv_inputs.ModelShape("gqa_small", 3, 128, 8, 2, 32, 176, 512, rope_base=500000.0, dtype="bf16", seed=4242)


def _script():
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "make_goldens.py")
    spec = importlib.util.spec_from_file_location("make_goldens", path)
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_layerwise_drive_equals_block_forward_bit_for_bit():
    def tensors(kind, layer):
        return pv_inputs.fill_tensor(GQA, kind, layer, gains="perturbed").reshape(pv_inputs.tensor_shape(GQA, kind))
    prompt = pv_inputs.uniform_tokens(5, 50, GQA.vocab)
    b1, b2 = pv_inputs.uniform_tokens(6, 8, GQA.vocab), pv_inputs.uniform_tokens(7, 5, GQA.vocab)
    run = replay.LayerwiseRun(GQA, tensors, 80, ref.KV_BF16, chunk=16)
    lg = run.run([(0, prompt), (50, b1), (50, b2)], commit=0)
    c = ref.RefCache(ref_model(GQA, gains="perturbed"), 80, ref.KV_BF16)
    last = c.prefill(prompt, chunk=64)                       # another chunking: rows do not depend on it
    assert np.array_equal(lg[0][-1], last)
    a1 = c.forward_block(b1); c.rollback(50)
    a2 = c.forward_block(b2); c.rollback(50)
    assert np.array_equal(lg[1], a1) and np.array_equal(lg[2], a2)
    assert len(run.c) == 50 and np.array_equal(run.c.export(), c.export())
    run.run([(50, b1[:3])], commit=0); c.forward_block(b1[:3])         # commit part of a block, go on from there
    assert np.array_equal(run.run([(53, b2)])[0], c.forward_block(b2))


GQA_Q4 = pv_inputs.ModelShape("gqa_small_q4", 3, 128, 8, 2, 32, 192, 512, rope_base=500000.0, dtype="bf16", seed=4343, weight_bits=4)


@pytest.mark.parametrize("GQA", [GQA, GQA_Q4], ids=["bf16", "q4"])
def test_golden_script_records_what_the_plain_oracle_computes(tmp_path, GQA):
    mg = _script()
    out_c, out_t = str(tmp_path / "chain.npz"), str(tmp_path / "tree.npz")
    mg.make("x", GQA, ("chain", 100, (0.5, 0.8), (8, 16, 1, 4), 0), out_c)
    mg.make("x", GQA, ("tree", 100, (0.6,), (8, 8, 16, 1), 3), out_t)
    rm = ref_model(GQA)                                      # (4-bit shapes: the dequantised codes, by the plain route)
    prompt = pv_inputs.uniform_tokens(2000 + GQA.seed, 100, GQA.vocab)
    for path in (out_c, out_t):
        g = np.load(path)
        meta = json.loads(bytes(g["meta"]).decode())
        assert meta["prefix"] == 100 and meta["n_layers"] == 3
        c = ref.RefCache(rm, 160, ref.KV_BF16)
        c.prefill(prompt)
        assert c.pending == g["chain0_greedy"][0]
        for ci in range(2):                                  # the recorded greedy continuations are the plain single-token ones
            if f"chain{ci}_greedy" in g.files:
                G = g[f"chain{ci}_greedy"]
                assert np.array_equal(G, greedy_continuation(c, len(G)))
                c.rollback(100); c.pending = int(G[0])
        ex = c.export()
        assert np.array_equal(ex[g["kv_layers"]][:, :, g["kv_pos"], :].astype(np.float32), g["kv_sample"])
        seen_accepts = set()
        for k in range(len(g["step_T"])):
            T, gam = int(g["step_T"][k]), int(g["step_gamma"][k])
            # bring the plain cache to the step's start: the greedy tokens of this chain up to T
            ci = [i for i in range(2) if f"chain{i}_steps" in g.files and g[f"chain{i}_steps"][0] <= k < g[f"chain{i}_steps"][1]][0]
            G = g[f"chain{ci}_greedy"]
            c.rollback(100)
            if T > 100:
                c.forward_block(G[:T - 100], want_logits=False)
            c.pending = int(g["step_pending"][k])
            n, nxt, pred, lg = c.verify(T, g["draft"][k, :gam], want_logits=True)
            assert (n, nxt) == (g["step_accepted"][k], g["step_next_token"][k])
            assert np.array_equal(pred, g["pred"][k, :gam])
            assert np.array_equal(lg[:, g["sample_ids"]].astype(np.float32), g["sample_logits"][k, :gam])
            srt = np.sort(lg, axis=1)
            assert np.allclose(srt[:, -1] - srt[:, -2], g["margin"][k, :gam], rtol=0, atol=0)
            assert np.allclose(np.sqrt((lg ** 2).mean(axis=1)), g["rms"][k, :gam], rtol=1e-15)
            assert np.array_equal(np.take_along_axis(lg, g["top_ids"][k, :gam].astype(np.int64), axis=1).astype(np.float32), g["top_vals"][k, :gam])
            assert (g["top_ids"][k, :gam, 0] == pred).all()
            seen_accepts.add(n)
        assert len(seen_accepts) >= 2                        # the drafts do get accepted to different depths
