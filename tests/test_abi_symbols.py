"""The C-ABI library loads (no GPU needed) and exports every entry point include/hivis.h declares."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "hivis.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hivis_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_exported():
    from paper_2509_23928_amd import LIB_PATH, EXPORTED_SYMBOLS
    if not os.path.exists(LIB_PATH):
        from paper_2509_23928_amd.build import build
        build(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), f"{n} declared in hivis.h but not exported"
    assert sorted(EXPORTED_SYMBOLS) == names


def test_binding_refuses_missing_library(tmp_path):
    from paper_2509_23928_amd import binding
    saved = binding._lib
    binding._lib = None
    try:
        with pytest.raises(FileNotFoundError):
            binding.load_library(str(tmp_path / "nope.so"))
    finally:
        binding._lib = saved


def test_create_rejects_bad_config_without_gpu():
    from paper_2509_23928_amd import binding
    lib = binding.load_library()
    cfg = binding.hivis_config(2, 250, 4, 4, 64, 688, 1024, 0, 1, 4, 64, 128, 10000.0, 1e-5, 4)   # d not a multiple of 16
    w = binding.hivis_weights()
    ctx = ctypes.c_void_p()
    rc = lib.hivis_create(ctypes.byref(cfg), ctypes.byref(w), None, ctypes.byref(ctx))
    assert rc == binding.HIVIS_EINVAL and not ctx.value
    assert b"multiple" in lib.hivis_last_error(None)
    assert lib.hivis_destroy(None) == 0


def test_token_clamp_rule_on_the_host():
    """The id a greedy-token kernel stores is forced into [0, vocab): the sentinel of a row without a finite maximum
    (0x7FFFFFFF), negative garbage and vocab itself all land inside the table."""
    from paper_2509_23928_amd import binding
    lib = binding.load_library()
    for V in (16, 1024, 152064):
        assert lib.hivis_clamp_token(0x7FFFFFFF, V) == V - 1
        assert lib.hivis_clamp_token(V, V) == V - 1
        assert lib.hivis_clamp_token(-1, V) == 0 and lib.hivis_clamp_token(-2**31, V) == 0
        for ok in (0, 1, V // 2, V - 1):
            assert lib.hivis_clamp_token(ok, V) == ok
