"""The C-ABI library loads and exports every symbol include/grappa.h declares (CPU only:
no compute call is made), and the binding's struct layouts match the header."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "grappa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(grp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    syms = _declared_symbols()
    for s in ("grp_partition", "grp_train_step", "grp_aggregate", "grp_last_error"):
        assert s in syms


def test_library_exports_every_declared_symbol():
    import paper_2602_01872_amd as g
    if not os.path.exists(g.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = g.load()
    for s in _declared_symbols():
        assert hasattr(lib, s), f"{s} declared in grappa.h but not exported"
    assert sorted(g.exported_symbols()) == _declared_symbols()


def test_struct_layouts_match_header():
    import paper_2602_01872_amd as g
    assert C.sizeof(g.ModelDesc) == 4 * (2 + 17 + 2)
    assert C.sizeof(g.StepOpts) == 16 + 8 + 4 * 16 + 16 + 16
    assert g.STATS_BYTES == 40
    assert C.sizeof(g.PartitionView) == 8 * 10
    assert C.sizeof(g.OptimizerDesc) == 24


def test_param_count_and_invalid_model():
    import paper_2602_01872_amd as g
    if not os.path.exists(g.LIB_PATH):
        pytest.skip("library not built")
    assert g.grp_param_count(g.model_desc(g.ARCH_SAGE_MEAN, [100, 256, 256, 47])) == 206895
    assert g.grp_param_count(g.model_desc(g.ARCH_GCN, [64, 64, 8])) == 4680
    assert g.grp_param_count(g.model_desc(g.ARCH_SAGE_MEAN, [64, 128, 16])) == 20624
    assert g.grp_param_count(g.model_desc(g.ARCH_GCN, [64, 0, 8])) == -1
    assert g.grp_param_count(g.model_desc(7, [64, 8])) == -1
