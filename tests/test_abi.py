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
    assert C.sizeof(g.StepOpts) == 16 + 8 + 4 * 16 + 16 + 16 + 8
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


def test_header_is_plain_c_and_its_struct_layouts_are_the_bindings(tmp_path):
    """grappa.h compiles as C99 on its own, and a C program's view of every struct (size and member
    offsets) equals the ctypes declarations the Python binding marshals through."""
    import shutil
    import subprocess
    import paper_2602_01872_amd as g
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "layout.c"
    fields = {
        "grp_partition_view_t": (g.PartitionView, ["n", "nnz", "l2g", "rowptr", "col", "colptr", "row", "d_local_in",
                                                   "d_local_out", "d_global_in"]),
        "grp_partition_weights_t": (g.PartitionWeights, ["csr_w", "csc_w", "w_local_in", "w_global_in"]),
        "grp_model_desc": (g.ModelDesc, ["arch", "n_layers", "dims", "feat_dtype", "gcn_self_loops"]),
        "grp_step_opts": (g.StepOpts, ["estimator", "full_graph", "n_seeds", "seeds", "fanouts", "sampler_seed", "batch_id",
                                       "dropout_rate", "flags", "dropout_seed", "batch_id_dev"]),
        "grp_step_stats": (None, ["loss", "sum_ratio", "R", "S", "nnz_used"]),
        "grp_optimizer_desc": (g.OptimizerDesc, ["kind", "lr", "beta1", "beta2", "eps"]),
    }
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "grappa.h"', 'int main(void) {']
    for name, (_, members) in fields.items():
        lines.append(f'  printf("{name} %zu", sizeof({name}));')
        for m in members:
            lines.append(f'  printf(" %zu", offsetof({name}, {m}));')
        lines.append('  printf("\\n");')
    lines += ['  return 0;', '}']
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(root, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.strip().splitlines()
    seen = {ln.split()[0]: [int(x) for x in ln.split()[1:]] for ln in out}
    for name, (ctype, members) in fields.items():
        size, offs = seen[name][0], seen[name][1:]
        if ctype is None:
            assert size == g.STATS_BYTES and offs == [0, 8, 16, 24, 32]
            continue
        assert size == C.sizeof(ctype), name
        assert offs == [getattr(ctype, m).offset for m in members], name


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_binding_fails_loudly_without_the_built_library(monkeypatch):
    # no fallback path: a missing library is an ImportError at the first call, not a silent CPU route
    from paper_2602_01872_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(os.path.dirname(binding.LIB_PATH), "no_such_library.so"))
    with pytest.raises(ImportError):
        binding.load()


def test_slice_policy_rejects_bad_arguments():
    # host-side setting: needs the built library but no GPU
    import paper_2602_01872_amd as g
    if not os.path.exists(g.LIB_PATH):
        pytest.skip("library not built")
    for bad in ((0, 25), (-5, 25), (1 << 19, -1), (1 << 19, 101)):
        with pytest.raises(g.GrappaError) as ei:
            g.grp_set_slice_policy(*bad)
        assert ei.value.status == g.EINVAL
    g.grp_set_slice_policy()            # the defaults again
