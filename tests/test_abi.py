"""The C-ABI library loads and exports every symbol include/graphflow.h declares
(CPU only: no compute calls)."""
import ctypes
import os
import re

import pytest

from paper_2605_22566_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "graphflow.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gf_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    syms = _declared_symbols()
    for name in ("gf_resolve_path", "gf_attn_prefill", "gf_attn_decode", "gf_create", "gf_destroy"):
        assert name in syms


@pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libgraphflow.so not built (run __graft_entry__.build())")
def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == _declared_symbols()


@pytest.mark.skipif(not os.path.exists(B.LIB_PATH), reason="libgraphflow.so not built")
def test_strerror_and_null_checks_need_no_gpu():
    lib = B.load_library()
    assert lib.gf_strerror(0) == b"ok"
    assert b"NULL" in lib.gf_strerror(B.GF_ERR_NULL)
    assert lib.gf_destroy(None) == B.GF_ERR_NULL
    assert lib.gf_attn_decode(None, None, None, None, None, None, None, None) == B.GF_ERR_NULL
    assert lib.gf_set_decode_chunk_blocks(None, 2) == B.GF_ERR_NULL


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        B.load_library(str(tmp_path / "nope.so"))
