"""The C-ABI library loads and exports every symbol include/fusedmm.h declares.
Only host-side calls (no GPU work) are made here."""
import ctypes
import os
import re

import pytest

from paper_2011_06391_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "fusedmm.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fusedmm_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2011_06391_amd import build
        build.build()
    return binding.load()


def test_header_declares_the_documented_entry_points():
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"libfusedmm.so lacks {name}"
        assert isinstance(getattr(lib, name), ctypes._CFuncPtr)


def test_host_only_calls(lib):
    assert binding.fusedmm_version() == 100
    assert binding.fusedmm_status_string(0) == "ok"
    assert "alias" in binding.fusedmm_status_string(binding.FUSEDMM_ERR_ALIAS) or "overlap" in binding.fusedmm_status_string(binding.FUSEDMM_ERR_ALIAS)
    assert binding.fusedmm_status_string(12345) == "unknown status"
    o = binding.fusedmm_ops_preset("tdist")
    assert (o.vop, o.rop, o.sop, o.mop, o.aop) == (binding.VOP["SUB"], binding.ROP["SUMSQ"], binding.SOP["INV_1P"],
                                                   binding.MOP["MUL_T"], 0)
    o = binding.fusedmm_ops_preset("gcn")
    assert (o.vop, o.rop, o.sop, o.mop) == (1, 0, 0, 0)
    with pytest.raises(binding.FusedMMError):
        binding.fusedmm_ops_preset(99)
    # null arguments are reported, not dereferenced
    assert lib.fusedmm_ops_preset(0, None) == binding.FUSEDMM_ERR_INVALID_ARG
    assert lib.fusedmm_plan_create(None, 0, 0, 0, None, None, None, None) == binding.FUSEDMM_ERR_INVALID_ARG
    assert lib.fusedmm_execute(None, None, 32, None, None, 0, None, 0, None, 0, None) == binding.FUSEDMM_ERR_INVALID_ARG
    assert lib.fusedmm_plan_destroy(None) == binding.FUSEDMM_OK


def test_which_kernel_size_a_dimension_runs_on(lib):
    """The dispatch over feature dimensions (host logic, no GPU): every fp32 and fp64 dimension has a size to run on,
    the smallest one that holds it; 2-byte storage takes multiples of 8 up to 1024."""
    sizes = (32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048)
    k = binding.fusedmm_debug_kernel_size
    for d in range(1, binding.FUSEDMM_MAX_D + 1):
        want = d if d in (2, 3, 4, 8, 16) else min(s for s in sizes if s >= d)
        assert k(d, "f32") == want, d
        want64 = min(s for s in sizes if s >= d and s & (s - 1) == 0)
        assert k(d, "f64") == want64, d
        want2 = min(s for s in sizes if s >= d) if d % 8 == 0 and d <= 1024 else 0
        assert k(d, "bf16") == want2, d
    assert k(0, "f32") == 0 and k(binding.FUSEDMM_MAX_D + 1, "f32") == 0 and k(-5, "f64") == 0
    for d, size in ((100, 128), (300, 384), (602, 768), (768, 768), (1433, 1536)):
        assert k(d, "f32") == size


def test_enum_values_match_header():
    text = open(HEADER).read()
    for table, prefix in ((binding.VOP, "FUSEDMM_VOP_"), (binding.ROP, "FUSEDMM_ROP_"), (binding.SOP, "FUSEDMM_SOP_"),
                          (binding.MOP, "FUSEDMM_MOP_")):
        for name, val in table.items():
            m = re.search(prefix + name + r"\s*=\s*(\d+)", text)
            assert m and int(m.group(1)) == val, (prefix + name)
    assert int(re.search(r"#define FUSEDMM_MAX_D (\d+)", text).group(1)) == binding.FUSEDMM_MAX_D


def test_header_is_plain_c_and_the_binding_mirrors_its_structs(tmp_path):
    """include/fusedmm.h compiles as C99 on its own (the boundary has no C++ or torch types), and the
    structures the ctypes binding passes have the header's size and field offsets."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    fields = {"fusedmm_plan_options_t": [f[0] for f in binding.fusedmm_plan_options_t._fields_],
              "fusedmm_ops_t": [f[0] for f in binding.fusedmm_ops_t._fields_]}
    lines = ['#include "fusedmm.h"', "#include <stddef.h>", "#include <stdio.h>", "int main(void) {"]
    for struct, names in fields.items():
        lines.append(f'  printf("{struct} %zu\\n", sizeof({struct}));')
        for name in names:
            lines.append(f'  printf("{struct}.{name} %zu\\n", offsetof({struct}, {name}));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe)], check=True)
    out = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines())
    for struct, names in fields.items():
        cls = getattr(binding, struct)
        assert int(out[struct]) == ctypes.sizeof(cls), struct
        for name in names:
            assert int(out[f"{struct}.{name}"]) == getattr(cls, name).offset, f"{struct}.{name}"
