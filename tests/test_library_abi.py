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
                     "bbmm_make_probes", "bbmm_mbcg", "bbmm_slq_logdet", "bbmm_slq_from_coeffs",
                     "bbmm_tridiag_eig_batched",
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


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header must compile as C99 on its own, and a C translation unit
    # that takes the address of every declared function must link against the library
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler")
    _ensure_built()
    names = _declared_functions()
    src = tmp_path / "abi.c"
    src.write_text('#include "bbmm.h"\n#include <stdio.h>\ntypedef void (*fn)(void);\nint main(void) {\n'
                   '  fn f[] = {%s};\n  bbmm_problem p; bbmm_result r; (void)p; (void)r;\n'
                   '  printf("%%d\\n", (int)(sizeof f / sizeof f[0]));\n  return bbmm_destroy(0);\n}\n'
                   % ", ".join("(fn)%s" % n for n in names))
    exe = tmp_path / "abi"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.dirname(HEADER), str(src),
                    "-o", str(exe), LIB, "-Wl,-rpath," + os.path.dirname(LIB)], check=True)
    out = subprocess.run([str(exe)], check=True, stdout=subprocess.PIPE, text=True).stdout
    assert int(out) == len(names)


def test_context_refuses_to_run_without_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    from paper_1809_11165_amd import binding
    with pytest.raises(RuntimeError):
        binding.Context()
