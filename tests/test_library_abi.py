"""CPU-only checks of the boundary: the shared library loads and exports every symbol the
public header declares, and the binding mirrors the header's names.  No compute calls."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "bbmm.h")
LIB = os.path.join(ROOT, "paper_1809_11165_amd", "libbbmm.so")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bbmm_[a-z0-9_]+)\s*\(", text)))


def _ensure_built():
    if not os.path.exists(LIB):
        from paper_1809_11165_amd import build
        build.build()


def test_header_declares_the_documented_entry_points():
    names = _declared_functions()
    for required in ["bbmm_create", "bbmm_destroy", "bbmm_solve_logdet_grad", "bbmm_build_khat",
                     "bbmm_kernel_mm", "bbmm_pivoted_cholesky", "bbmm_precond_solve",
                     "bbmm_make_probes", "bbmm_mbcg", "bbmm_slq_logdet", "bbmm_tridiag_eig_batched",
                     "bbmm_dk_traces"]:
        assert required in names


def test_library_exports_every_declared_symbol():
    _ensure_built()
    lib = ctypes.CDLL(LIB)
    for name in _declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_exactly_the_header_functions():
    from paper_1809_11165_amd import binding
    assert sorted(binding.EXPORTS) == _declared_functions()
    _ensure_built()
    binding.load_library()
    for name in binding.EXPORTS:
        if name in ("bbmm_create", "bbmm_destroy", "bbmm_last_error"):
            continue
        assert hasattr(binding.Context, name), name


def test_struct_layouts_match_the_header_field_order():
    from paper_1809_11165_amd import binding
    text = open(HEADER).read()

    def fields(struct_name):
        clean = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        body = re.search(r"typedef struct \{([^{}]*)\} %s;" % struct_name, clean).group(1)
        out = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            # drop the type words, keep comma separated declarators
            names = re.sub(r"^(const\s+)?(\w+)\s*\**\s*", "", decl)
            for nm in names.split(","):
                out.append(nm.strip().lstrip("*").strip())
        return out

    assert fields("bbmm_problem") == [f[0] for f in binding._Problem._fields_]
    assert fields("bbmm_result") == [f[0] for f in binding._Result._fields_]


def test_context_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_1809_11165_amd import binding
    with pytest.raises(RuntimeError):
        binding.Context()
