"""Draft-tree verification (pv_verify_tree; Sec. 2.2 names tree-structured verification as combinable with
the pipeline).  Oracle rule: the step must reach exactly what plain greedy decoding guided by the tree
reaches - walk down from the prefix, at every node take the child that carries the stage's own next
greedy token - and every node's logits must be those of the plain block forward over its
root-to-node chain.  Both follow from the oracle's chain routines alone (ref_forward_block,
ref_decode_one); nothing tree-specific exists on the oracle side.
"""
import numpy as np
import pytest

import pv_inputs
from oracle import ref
from helpers import ref_model, greedy_continuation

pytestmark = pytest.mark.gpu

GQA4 = pv_inputs.ModelShape("tree_gqa", 3, 256, 8, 2, 64, 704, 1024, rope_base=500000.0, dtype="bf16", seed=7301)
MHA = pv_inputs.ModelShape("tree_mha", 2, 256, 4, 4, 64, 512, 1008, dtype="bf16", seed=7302)


@pytest.fixture(scope="module")
def pvlib():
    import torch
    assert torch.cuda.is_available()
    import paper_2505_01572_amd as pv
    return pv


def _chain(parents, i):
    out = []
    while i >= 0:
        out.append(i); i = parents[i]
    return out[::-1]


def _tree(G, n, branching_seed, vocab, keep_depth):
    """n nodes: the greedy tokens G[0..keep_depth) as one root-to-leaf path hidden among random siblings and
    random subtrees (parents always earlier nodes)."""
    rng = np.random.default_rng(branching_seed)
    parents, tokens, on_path = [], [], []
    path_node = -1                      # the node carrying G[d-1]
    d = 0
    while len(parents) < n:
        if d < keep_depth and rng.random() < 0.5:
            # a wrong sibling first now and then, then the right child
            if rng.random() < 0.5 and len(parents) < n - 1:
                parents.append(path_node); tokens.append(int((G[d] + 1 + rng.integers(0, vocab - 1)) % vocab)); on_path.append(False)
            parents.append(path_node); tokens.append(int(G[d])); on_path.append(True)
            path_node = len(parents) - 1; d += 1
        else:
            par = int(rng.integers(-1, len(parents))) if parents else -1
            tok = int(rng.integers(0, vocab))
            # a random node must not accidentally continue the greedy path
            depth = len(_chain(parents, par)) if par >= 0 else 0
            chain_tokens = [tokens[k] for k in _chain(parents, par)] if par >= 0 else []
            if chain_tokens == [int(g) for g in G[:depth]] and tok == int(G[depth]):
                tok = (tok + 1) % vocab
            parents.append(par); tokens.append(tok); on_path.append(False)
    return np.array(tokens, dtype=np.int32), np.array(parents, dtype=np.int32), [i for i, f in enumerate(on_path) if f]


@pytest.mark.parametrize("shape", [GQA4, MHA], ids=lambda s: s.name)
def test_tree_step_equals_greedy_walk_and_chain_forwards(pvlib, shape):
    from gpu_helpers import gpu_model, logit_scale, top2_margin
    gm, rm = gpu_model(shape, gains="perturbed", max_gamma=16), ref_model(shape, gains="perturbed")
    T0 = 150
    prompt = pv_inputs.uniform_tokens(960, T0, shape.vocab)
    gc, rc = pvlib.Cache(gm, 400), ref.RefCache(rm, 400, ref.KV_BF16)
    gc.prefill(prompt); rc.prefill(prompt)
    assert gc.state() == (T0, rc.pending)
    ar = ref.RefCache(rm, 400, ref.KV_BF16); ar.prefill(prompt)
    G = greedy_continuation(ar, 40)                      # the stage's own greedy tokens after the prompt
    T, used = T0, 0
    for step, (n, keep) in enumerate(((20, 5), (64, 9), (7, 0), (33, 12))):
        tokens, parents, want_path = _tree(G[used:], n, 970 + step, shape.vocab, keep)
        n_g, nxt_g, path_g = gc.verify_tree(T, tokens, parents)
        lg_g = gc.debug_logits()
        assert lg_g.shape[0] == n
        # every node's logits = the plain block forward over its chain of ancestors (checked on the path, the leaves of a
        # few other branches and the last node)
        probe = sorted(set(want_path[-1:] + [n - 1, n // 2, 0] + [i for i in range(n) if i not in set(parents)][:4]))
        worst = 0.0
        for i in probe:
            ch = _chain(parents, i)
            lg_r = rc.forward_block(tokens[ch]); rc.rollback(T)
            err = float((np.abs(lg_g[ch] - lg_r) / logit_scale(lg_r)).max())
            worst = max(worst, err)
            assert err < 2e-3, (step, i, err)
        # the walk: the greedy tokens as far as the tree carries them
        m = len(want_path)
        lg_path = rc.forward_block(tokens[want_path]) if m else None
        rc.rollback(T)
        safe = m == 0 or bool((top2_margin(lg_path) > 4 * 2e-3 * logit_scale(lg_path)[:, 0]).all())
        if safe:
            assert (n_g, list(path_g)) == (m, want_path), (step, n_g, path_g, want_path)
            assert nxt_g == G[used + m]
            assert gc.state() == (T + m, int(G[used + m]))
        else:
            m = n_g                                       # a near-tie: follow the library
        # the oracle commits the same path as a chain; the caches must then agree
        if m:
            rc.pending = int(G[used])
            rc.verify(T, tokens[list(path_g)])
        assert len(rc) == len(gc)
        ge, re_ = pv_inputs.bf16_bits_to_f32(gc.export()).astype(np.float64), rc.export()
        assert ge.shape == re_.shape and np.mean(ge != re_) < 0.03 and np.abs(ge - re_).max() <= 2.0 ** -7 * np.abs(re_).max()
        T += m; used += m
        print(f"{shape.name} tree {step}: {n} nodes, accepted {n_g}, worst relative logit error {worst:.2e}")
    # a plain chain step on the cache the tree steps left behind
    d = np.concatenate([[G[used]], pv_inputs.uniform_tokens(990, 5, shape.vocab)]).astype(np.int32)
    rc.pending = int(G[used])
    n_r, t_r, _, lg_r = rc.verify(T, d, want_logits=True)
    assert gc.verify(T, d) == (n_r, t_r)
    assert float((np.abs(gc.debug_logits() - lg_r) / logit_scale(lg_r)).max()) < 2e-3


def test_tree_argument_checks_and_trusted_root(pvlib):
    from gpu_helpers import gpu_model
    gm = gpu_model(GQA4)
    c = pvlib.Cache(gm, 128)
    c.prefill(pv_inputs.uniform_tokens(3, 10, GQA4.vocab))
    st = c.state()
    for bad, code in ((lambda: c.verify_tree(10, [1, 2, 3], [-1, 1, 0]), -1),          # parent not earlier
                      (lambda: c.verify_tree(10, [1, 2, 3], [-1, -2, 0]), -1),
                      (lambda: c.verify_tree(9, [1, 2], [-1, 0]), -2),                  # wrong prefix length
                      (lambda: c.verify_tree(10, [1, GQA4.vocab], [-1, 0]), -3),
                      (lambda: c.verify_tree(10, list(range(65)), [-1] * 65), -3)):
        with pytest.raises(pvlib.PVError) as e:
            bad()
        assert e.value.status == code and c.state() == st
    # pending unknown (after a rollback): the first root is trusted whatever it is
    c.rollback(10)
    n, nxt, path = c.verify_tree(10, [5, 6, 7], [-1, -1, 0])
    assert n >= 1 and path[0] == 0 and c.state() == (10 + n, nxt)
    tiny = gpu_model(pv_inputs.CONFIGS["tiny"])
    t = pvlib.Cache(tiny, 64)
    t.prefill([1, 2, 3])
    with pytest.raises(pvlib.PVError) as e:
        t.verify_tree(3, [4, 5], [-1, 0])                                               # fp32 vector path
    assert e.value.status == -1
