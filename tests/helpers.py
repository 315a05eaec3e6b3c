"""Shared test plumbing: load synthetic weights into the oracle, drive verify loops."""
import numpy as np

import pv_inputs
from oracle import ref


def ref_model(shape, gains="ones", real="f64", overrides=None):
    """Oracle model filled from the seeded generator. overrides: {(kind, layer): array}."""
    m = ref.RefModel(shape, real=real)
    for kind, layer in pv_inputs.iter_tensors(shape):
        arr = pv_inputs.fill_tensor(shape, kind, layer, gains=gains)
        arr = arr.reshape(pv_inputs.tensor_shape(shape, kind))
        if overrides and (kind, layer) in overrides:
            arr = overrides[(kind, layer)]
        elif getattr(shape, "weight_bits", 16) == 4 and kind in pv_inputs.Q4_KINDS:
            codes, scales = pv_inputs.quantize_q4(arr)          # the model's weights ARE the codes and scales
            arr = ref.dequant_q4(codes, scales)
        m.set_tensor(kind, layer, arr)
    return m


def tensors_f64(shape, gains="ones"):
    """All tensors widened to float64 numpy arrays (for checks written with library routines)."""
    out = {}
    for kind, layer in pv_inputs.iter_tensors(shape):
        a = pv_inputs.fill_tensor(shape, kind, layer, gains=gains)
        if a.dtype == np.uint16:
            a = pv_inputs.bf16_bits_to_f32(a)
        out[(kind, layer)] = a.astype(np.float64).reshape(pv_inputs.tensor_shape(shape, kind))
    return out


def greedy_continuation(cache, n):
    """n greedy tokens after the cached prefix, by one-token decodes. cache.pending must be known."""
    toks = [cache.pending]
    for _ in range(n - 1):
        toks.append(int(np.argmax(cache.decode_one(toks[-1]))))
    return np.array(toks, dtype=np.int32)


def draft_block(G, T0, T, gamma, alpha, vocab, seed, step, trust_first):
    """Synthetic draft for committed length T: the verifier's own greedy tokens G[T-T0 : T-T0+gamma]
    with each position replaced by a uniform token w.p. 1-alpha; position 0 is left intact when
    trust_first (the caller re-sends the verifier's correction token after a zero-accept step)."""
    blk = G[T - T0: T - T0 + gamma]
    d = pv_inputs.perturb_drafts(blk, alpha, vocab, seed, step)
    if trust_first:
        d[0] = blk[0]
    return d
