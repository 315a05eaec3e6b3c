"""The C-ABI library loads and exports every symbol include/pipeverify.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "pipeverify.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pv_[a-z0-9_]+)\s*\(", src)))


def test_header_symbols_are_exported():
    from paper_2505_01572_amd import binding
    names = _declared()
    assert "pv_load_weights" in names and "pv_verify" in names and "pv_rollback" in names
    L = ctypes.CDLL(binding._LIB_PATH)
    missing = [n for n in names if not hasattr(L, n)]
    assert not missing, missing
    assert sorted(binding.EXPORTS) == names


def test_strerror_without_gpu():
    from paper_2505_01572_amd import binding
    L = binding.lib()
    assert L.pv_strerror(0) == b"ok"
    assert b"range" in L.pv_strerror(-3)


def test_config_validation_without_gpu():
    """pv_model_bytes is pure host arithmetic: it validates shapes and sizes the arena."""
    from paper_2505_01572_amd import binding
    L = binding.lib()
    cfg = binding.pv_model_config(2, 256, 4, 4, 64, 688, 1024, 1e-5, 10000.0, binding.PV_F32, 16, 16, 0)
    wb, sb = ctypes.c_size_t(), ctypes.c_size_t()
    assert L.pv_model_bytes(ctypes.byref(cfg), ctypes.byref(wb), ctypes.byref(sb)) == 0
    assert wb.value >= 2_106_624 * 4
    cfg.n_kv_heads = 3
    assert L.pv_model_bytes(ctypes.byref(cfg), ctypes.byref(wb), ctypes.byref(sb)) == -1
    cfg.n_kv_heads = 4; cfg.max_gamma = 65
    assert L.pv_model_bytes(ctypes.byref(cfg), ctypes.byref(wb), ctypes.byref(sb)) == -1
    cfg.max_gamma = 16; cfg.page_tokens = 12
    assert L.pv_model_bytes(ctypes.byref(cfg), ctypes.byref(wb), ctypes.byref(sb)) == -1
