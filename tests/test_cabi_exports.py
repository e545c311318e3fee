"""The built C-ABI library loads and exports every symbol include/kvq.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "kvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(kvq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2401_18079_amd import binding
    path = binding.lib_path()
    assert os.path.exists(path), "build the library first: python -m paper_2401_18079_amd.build"
    lib = ctypes.CDLL(path)
    names = declared_symbols()
    assert {"kvq_lut_load", "kvq_quantize_append_k", "kvq_quantize_append_v", "kvq_qk_matvec",
            "kvq_pv_matvec"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTED_SYMBOLS) == names


def test_host_only_helpers():
    import paper_2401_18079_amd as K
    assert K.kvq_codes_bytes(3, 32, 131072) == 131072 * 4096 * 3 // 8
    assert K.kvq_params_bytes(32) % 256 == 0
    assert K.kvq_status_string(3) == "capacity exceeded"
    assert "gfx950" in K.kvq_version()
