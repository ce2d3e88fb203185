"""The C-ABI library loads and exports every symbol include/hss_svm.h declares (CPU only: no compute
call is made)."""
import os
import re

import pytest

from paper_2108_04167_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "hss_svm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hss_[a-z0-9_]+|admm_svm_train[a-z_]*|svm_decision)\s*\(", text)))


def test_header_and_binding_agree():
    names = _declared_symbols()
    assert "hss_compress" in names and "admm_svm_train" in names and "hss_ulv_solve" in names
    assert sorted(binding.ABI) == names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("library not built in this tree (run build() first)")
    lib = binding.load()
    for name in _declared_symbols():
        assert hasattr(lib, name), name
    assert lib.hss_strerror(binding.HSS_EINVAL) == b"invalid argument"
    assert lib.hss_strerror(binding.HSS_ESTATE) == b"call out of order"


def test_stats_struct_matches_header_order():
    text = open(os.path.join(ROOT, "include", "hss_svm.h")).read()
    body = text[text.index("typedef struct hss_stats_t {"):text.index("} hss_stats_t;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    body = body[body.index("{") + 1:]
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        m = re.match(r"(int64_t|int32_t|double)\s+(.*)", decl, flags=re.S)
        if m:
            fields += [f.strip() for f in m.group(2).split(",")]
    assert fields == [f for f, _ in binding.HssStats._fields_]
