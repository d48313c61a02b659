"""The C-ABI library loads and exports every entry point the header declares
(no compute calls: runs without a GPU)."""
import ctypes
import os
import re

from paper_2605_16637_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared():
    text = open(os.path.join(ROOT, "include", "hx.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hx_[a-z_]+)\s*\(", text)))


def test_header_and_binding_list_the_same_entry_points():
    assert declared() == sorted(binding.EXPORTS)


def test_library_exports_every_declared_symbol():
    assert os.path.exists(binding.LIB_PATH), "build the library first (__graft_entry__.build())"
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in declared():
        assert hasattr(lib, name), f"{name} is declared in hx.h but not exported"


def test_null_context_is_an_error_not_a_crash():
    lib = binding.load()
    assert lib.hx_stream_status(None, None) == -1
    assert lib.hx_ctx_destroy(None) == -1
    assert lib.hx_last_error(None) == b"NULL context"
    assert lib.hx_ctx_create(None, 0) == -1


def test_struct_layouts_match_the_header(tmp_path):
    """The ctypes structures of the binding against what a C compiler makes of hx.h."""
    import subprocess
    structs = {"hx_model": binding.hx_model, "hx_calls": binding.hx_calls, "hx_prefill_tab": binding.hx_prefill_tab,
               "hx_decode_tab": binding.hx_decode_tab, "hx_links": binding.hx_links, "hx_intervals": binding.hx_intervals,
               "hx_round_args": binding.hx_round_args}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hx.h"', 'int main(void) {']
    for name, cls in structs.items():
        lines.append(f'printf("{name} size %zu\\n", sizeof({name}));')
        for field, _ in cls._fields_:
            lines.append(f'printf("{name} {field} %zu\\n", offsetof({name}, {field}));')
    lines += ['return 0; }']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = subprocess.check_output([str(exe)], text=True).split("\n")
    want = []
    for name, cls in structs.items():
        want.append(f"{name} size {ctypes.sizeof(cls)}")
        for field, _ in cls._fields_:
            want.append(f"{name} {field} {getattr(cls, field).offset}")
    assert [g for g in got if g] == want


def test_every_entry_point_rejects_a_null_context():
    """Each call checks its context before anything else (no GPU needed: nothing is launched)."""
    lib = binding.load()
    for name in binding.EXPORTS:
        if name in ("hx_ctx_create", "hx_last_error"):
            continue
        fn = getattr(lib, name)
        # more NULL/zero arguments than any entry point takes; surplus ones are ignored by the C calling convention
        assert fn(*([None] * 24)) == -1, name
