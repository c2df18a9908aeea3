"""No GPU needed: the C-ABI library loads and exports every symbol the header declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="aif.h"):
    src = open(os.path.join(ROOT, "include", header)).read()
    return sorted(set(re.findall(r"AIF_API\s+[\w\s\*]+?\b(aif_\w+)\s*\(", src)))


def test_header_declares_the_north_star_entry_points():
    names = _declared()
    for must in ("aif_score_init", "aif_score_request", "aif_score_batch", "aif_topk"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2511_12934_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_12934_amd import build
        build.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(_declared())
    for name in _declared("aif_lsh.h"):
        assert hasattr(lib, name), name
    assert set(binding.LSH_EXPORTS) == set(_declared("aif_lsh.h"))
    for name in _declared("aif_user.h"):
        assert hasattr(lib, name), name
    assert set(binding.USER_EXPORTS) == set(_declared("aif_user.h"))


def test_binding_structs_match_the_c_layout():
    from paper_2511_12934_amd import binding as B
    # x86-64 / LP64 layout of the structs in aif.h
    assert ctypes.sizeof(B.aif_request) == 72
    assert B.aif_request.cand_ids.offset == 40 and B.aif_request.logits_out.offset == 56
    assert ctypes.sizeof(B.aif_config) == 80
    assert B.aif_config.n_items.offset == 8 and B.aif_config.layer_dims.offset == 56
    assert ctypes.sizeof(B.aif_weights) == 32
    # aif_lsh.h
    assert ctypes.sizeof(B.aif_lsh_config) == 40 and B.aif_lsh_config.d_bits.offset == 8
    assert ctypes.sizeof(B.aif_lsh_request) == 56
    assert B.aif_lsh_request.cand_ids.offset == 24 and B.aif_lsh_request.din_out.offset == 40
    # aif_user.h
    assert ctypes.sizeof(B.aif_user_config) == 20 and ctypes.sizeof(B.aif_user_weights) == 32
    assert ctypes.sizeof(B.aif_user_request) == 40 and B.aif_user_request.user_vec_out.offset == 24


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2511_12934_amd import binding as B
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load()


def test_calibration_library_exports_what_the_peaks_driver_calls():
    """The measurement tooling is a library of its own (profiling/libaif_calib.so); profiling/peaks.py calls these."""
    from paper_2511_12934_amd import build
    if not os.path.exists(build.CALIB_LIB):
        build.build()
    lib = ctypes.CDLL(build.CALIB_LIB)
    src = open(os.path.join(ROOT, "paper_2511_12934_amd", "profiling", "peaks.py")).read()
    called = sorted(set(re.findall(r"lib\.(aifcal_\w+)", src)))
    assert {"aifcal_mfma", "aifcal_copy", "aifcal_coissue", "aifcal_attn_loop", "aifcal_valu_costs"} <= set(called)
    for name in called:
        assert hasattr(lib, name), name
