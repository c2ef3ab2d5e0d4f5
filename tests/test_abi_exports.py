"""The C-ABI library loads and exports every function include/molret.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "molret.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(?:mol_status_t|size_t|int64_t|const char \*)\s*\*?\s*(\w+)\s*\(", text)
    return sorted(set(names))


def test_header_declares_the_four_path_calls():
    names = declared_functions()
    for required in ("mol_corpus_pack", "hindexer_topk", "mol_score", "mol_topk"):
        assert required in names


def test_library_exports_every_declared_symbol():
    import paper_2306_04039_amd as m
    lib = ctypes.CDLL(m.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in molret.h but not exported"
    from paper_2306_04039_amd.binding import EXPORTS
    assert sorted(EXPORTS) == declared_functions()


def test_host_only_calls_reject_bad_arguments_without_a_gpu():
    import paper_2306_04039_amd as m
    lib = m.load_library()
    assert lib.hindexer_workspace_bytes(None, 4, 10, 0) == 0
    assert lib.mol_workspace_bytes(None, 4, 10, 10) == 0
    assert lib.hindexer_default_lambda(None, 10) == 0
    assert lib.mol_corpus_free(None) == 0
    assert lib.mol_corpus_pack(None, None, None, None, None, None) == -1
    assert b"NULL" in lib.mol_last_error()
