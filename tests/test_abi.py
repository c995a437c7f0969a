"""The C-ABI library loads and exports every symbol that include/rvq.h declares (no compute)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "rvq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rvq_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_entry_points_of_the_boundary():
    names = _declared()
    for must in ("rvq_encode", "rvq_decode", "rvq_ema_update", "rvq_create", "rvq_destroy",
                 "rvq_set_codebooks", "rvq_get_codebooks", "rvq_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2410_15704_amd import binding

    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert set(binding.EXPORTS) == set(_declared())


def test_error_strings_and_config_validation_need_no_gpu():
    from paper_2410_15704_amd import binding as b

    assert b.rvq_strerror(0) == "ok"
    assert "invalid" in b.rvq_strerror(b.RVQ_EINVAL)
    assert b.rvq_version() >= 1000
    # a bad configuration is rejected before any device call
    for bad in (dict(d=100, dhat=32), dict(d=128, dhat=32, K=0), dict(d=128, dhat=32, K=40000),
                dict(d=128, dhat=32, depth=17), dict(d=128, dhat=32, grouping=2),
                dict(d=128, dhat=16, encode_path=b.PATH_SCREEN), dict(d=128, dhat=32, out_dtype=b.BF16)):
        assert b.rvq_create(check=False, **bad) == b.RVQ_EINVAL
    assert b.lib.rvq_destroy(None) == b.RVQ_EINVAL
    assert b.lib.rvq_create(None, None) == b.RVQ_EINVAL
