"""GPU-side test plumbing: build a library model from the seeded generator."""
import numpy as np

import pv_inputs
import paper_2505_01572_amd as pv


def gpu_model(shape, gains="ones", max_gamma=16, kernel_path=pv.PATH_AUTO, overrides=None):
    m = pv.Model(shape, max_gamma=max_gamma, kernel_path=kernel_path)
    for kind, layer in pv_inputs.iter_tensors(shape):
        tshape = pv_inputs.tensor_shape(shape, kind)
        cols = tshape[-1]
        if overrides and (kind, layer) in overrides:
            arr = np.ascontiguousarray(overrides[(kind, layer)]).reshape(-1, cols)
            step = m.chunk_rows(cols)
            for r0 in range(0, arr.shape[0], step):
                m.load_weights(kind, layer, r0, arr[r0:r0 + step])
            continue
        q4 = getattr(shape, "weight_bits", 16) == 4 and kind in pv_inputs.Q4_KINDS
        for r0, rows in pv_inputs.iter_row_chunks(shape, kind, layer, m.chunk_rows(cols), gains=gains):
            if q4:
                m.load_weights_q4(kind, layer, r0, *pv_inputs.quantize_q4(rows))
            else:
                m.load_weights(kind, layer, r0, rows)
    return m


def logit_scale(ref_logits):
    """Per-row RMS of the oracle's logits: the scale bf16 tolerances are relative to."""
    return np.sqrt((np.asarray(ref_logits, dtype=np.float64) ** 2).mean(axis=-1, keepdims=True))


def top2_margin(ref_logits):
    s = np.sort(np.asarray(ref_logits), axis=-1)
    return s[..., -1] - s[..., -2]


def paired_models(shape, max_gamma=16, real="f64"):
    """(library model, oracle model) built from the same generated tensors, each tensor drawn once.
    The oracle borrows the host arrays; the library gets them chunk by chunk."""
    from oracle import ref
    gm = pv.Model(shape, max_gamma=max_gamma)
    rm = ref.RefModel(shape, real=real)
    for kind, layer in pv_inputs.iter_tensors(shape):
        tshape = pv_inputs.tensor_shape(shape, kind)
        arr = pv_inputs.fill_tensor(shape, kind, layer).reshape(tshape)
        a2 = arr.reshape(-1, tshape[-1])
        step = gm.chunk_rows(tshape[-1])
        if getattr(shape, "weight_bits", 16) == 4 and kind in pv_inputs.Q4_KINDS:
            codes, scales = pv_inputs.quantize_q4(a2)           # both sides get the same codes and scales
            rm.set_tensor(kind, layer, ref.dequant_q4(codes, scales))
            for r0 in range(0, a2.shape[0], step):
                gm.load_weights_q4(kind, layer, r0, codes[r0:r0 + step], scales[r0:r0 + step])
            continue
        rm.set_tensor(kind, layer, arr)
        for r0 in range(0, a2.shape[0], step):
            gm.load_weights(kind, layer, r0, a2[r0:r0 + step])
    return gm, rm
