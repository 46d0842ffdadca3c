"""The C-ABI library loads and exports every symbol that include/slora.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "slora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slora_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_north_star_calls():
    syms = declared_symbols()
    for need in ("slora_pool_init", "slora_adapter_load", "slora_lora_shrink_expand"):
        assert need in syms
    assert len(syms) >= 15


def test_library_exports_every_declared_symbol():
    from paper_2311_03285_amd import slora
    lib = ctypes.CDLL(slora.LIB_PATH)
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} is declared in slora.h but not exported"


def test_binding_has_the_same_names():
    from paper_2311_03285_amd import slora
    for name in declared_symbols():
        assert hasattr(slora, name[len("slora_"):]), name
