"""Layer-by-layer drive of the CPU oracle for models too deep to hold in host memory.
Test infrastructure only, like everything under oracle/.

The decoder's result for a row depends on the layers in order, but nothing forces a whole step
to finish before the next one starts on layer 0: when every block's input tokens and start
position are known up front, layer l can process the prompt and then every block before layer
l+1 is touched, so that only one layer's weights are alive at a time (a 70B-shaped model has
1.7 GB per layer and 138 GB in all).  Every block starts at or before the end of the prompt's
committed positions + what earlier passes committed, and its rows see the committed positions
and their own block only (the causal rule of the verify step: Algorithm 1, verify branch), so
the keys and values a block writes beyond its start may be overwritten by the next block.

The arithmetic is ref_layer_block's, i.e. exactly what ref_forward_block runs; tests pin this
drive bit for bit against RefCache.prefill / verify on a model small enough for both.
"""
import numpy as np

from . import ref


class LayerwiseRun:
    """One sequence's cache, driven layer-outer.  `tensors(kind, layer)` returns the stored array of a
    tensor (float32, or uint16 bfloat16 bit patterns) and is called once per tensor and pass."""

    def __init__(self, shape, tensors, max_tokens, kv_store, real="f64", chunk=64, log=None):
        self.shape, self.tensors, self.chunk = shape, tensors, chunk
        self.m = ref.RefModel(shape, real=real)
        self.c = ref.RefCache(self.m, max_tokens, kv_store)
        self.log = log or (lambda msg: None)

    def _globals(self, on):
        for kind in ("embed", "final_norm", "lm_head"):
            if on:
                self.m.set_tensor(kind, -1, self.tensors(kind, -1))
            else:
                self.m.drop_tensor(kind, -1)

    def run(self, blocks, commit=None):
        """blocks: list of (start position, token ids).  Every block is run through all layers on top of
        the committed positions [0, start); returns the list of their logits [rows, vocab].  Blocks are
        processed in order within a layer, each writing keys/values at start .. start+rows-1.
        commit: index of the block whose rows stay committed afterwards (the cache length becomes its
        end), or None to leave the length as it is.  A long block (a prompt) is cut into chunks."""
        s = self.shape
        self.m.set_tensor("embed", -1, self.tensors("embed", -1))
        X = [self.m.embed_block(t) for _, t in blocks]
        self.m.drop_tensor("embed", -1)
        end = len(self.c)
        for i, (st, t) in enumerate(blocks):
            assert 0 <= st <= end, "a block must start inside the committed positions"
            if i == commit:
                assert st == end, "the block that stays committed starts at the cache length"
                end = st + len(t)
        per_layer = ("attn_norm", "wq", "wk", "wv", "wo", "ffn_norm", "wg", "wu", "wd")
        for l in range(s.n_layers):
            for kind in per_layer:
                self.m.set_tensor(kind, l, self.tensors(kind, l))
            for (st, _), x in zip(blocks, X):
                for r0 in range(0, x.shape[0], self.chunk):
                    self.c.layer_block(l, st + r0, x[r0:r0 + self.chunk])      # a row slice of a C-contiguous array is contiguous
            for kind in per_layer:
                self.m.drop_tensor(kind, l)
            self.log(f"layer {l + 1}/{s.n_layers}")
        for kind in ("final_norm", "lm_head"):
            self.m.set_tensor(kind, -1, self.tensors(kind, -1))
        out = [self.m.head_block(x) for x in X]
        for kind in ("final_norm", "lm_head"):
            self.m.drop_tensor(kind, -1)
        if commit is not None:
            st, t = blocks[commit]
            self.c.set_len(st + len(t))
        return out
