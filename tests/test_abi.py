"""CPU-side checks of the boundary: the built library loads and exports every symbol the header declares."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sasgd.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sasgd_[A-Za-z_]+)\s*\(", text)))


def test_header_declares_the_protocol_calls():
    syms = declared_symbols()
    for name in ["pullWeights", "getMinibatch", "calcGradient", "pushGradient", "sumGradients", "applyUpdate"]:
        assert "sasgd_" + name in syms


def test_library_exports_every_declared_symbol():
    from paper_1511_05950_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        pytest.skip("libsasgd.so not built (python -m paper_1511_05950_amd.build)")
    lib = binding.load()
    syms = declared_symbols()
    assert sorted(binding.EXPORTS) == syms
    for s in syms:
        assert hasattr(lib, s), s
    assert binding.version().startswith("sasgd-gfx950")


def test_config_struct_layout_matches_header_order():
    from paper_1511_05950_amd import binding
    text = open(HEADER).read()
    body = text[text.index("typedef struct {\n  int32_t lambda;"):text.index("} sasgd_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"(\w+)\s*(?:\)\s*\([^)]*\))?\s*[;,]", body)
    names = [n for n in names if n not in ("user",)]
    fields = [f[0].rstrip("_") for f in binding.SasgdConfig._fields_]
    assert names == fields, (names, fields)
