"""The public header on its own: it compiles as C99 and as C++17 with nothing else included, and every struct
it declares has, field by field, the offsets and the size the Python binding marshals into."""
import ctypes as C
import os
import re
import shutil
import subprocess

import pytest

import paper_2511_14116_amd as fs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
INCLUDE = os.path.join(ROOT, "include")

BOUND = {   # header struct -> the binding's image of it
    "fs_shape": fs.FsShape,
    "fs_kv_view": fs.FsKvView,
    "fs_work_item": fs.ITEM_DTYPE,
    "fs_pair": fs.PAIR_DTYPE,
    "fs_launch_record": fs.RECORD_DTYPE,
    "fs_prefill_entry": fs.PREFILL_ENTRY_DTYPE,
    "fs_prefill_item": fs.PREFILL_ITEM_DTYPE,
    "fs_prefill_pair": fs.PREFILL_PAIR_DTYPE,
}


def _fields(image):
    if isinstance(image, type) and issubclass(image, C.Structure):
        return [(n, getattr(image, n).offset) for n, _ in image._fields_], C.sizeof(image)
    return [(n, image.fields[n][1]) for n in image.names], image.itemsize


def _header_structs():
    with open(os.path.join(INCLUDE, "failsafe.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    return re.findall(r"typedef\s+struct\s*\{[^}]*\}\s*(fs_[a-z_0-9]+)\s*;", text)


def test_every_struct_of_the_header_has_an_image_in_the_binding():
    assert sorted(_header_structs()) == sorted(BOUND)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="no C compiler")
def test_struct_layouts_match_the_binding(tmp_path):
    lines = ["#include <stddef.h>", "#include <stdio.h>", '#include "failsafe.h"', "int main(void) {"]
    for name, image in BOUND.items():
        fields, _ = _fields(image)
        lines.append(f'  printf("{name} size %zu\\n", sizeof({name}));')
        for field, _ in fields:
            lines.append(f'  printf("{name} {field} %zu\\n", offsetof({name}, {field}));')
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines) + "\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", INCLUDE, str(src), "-o", str(exe)],
                   check=True)
    seen = {}
    for line in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.splitlines():
        struct, field, value = line.split()
        seen[(struct, field)] = int(value)
    for name, image in BOUND.items():
        fields, size = _fields(image)
        assert seen[(name, "size")] == size, name
        for field, offset in fields:
            assert seen[(name, field)] == offset, (name, field)
    # no field of the header is missing from the image: the fields tile the struct without a hole
    for name, image in BOUND.items():
        fields, size = _fields(image)
        if isinstance(image, type):
            widths = [C.sizeof(t) for _, t in image._fields_]
        else:
            widths = [image.fields[n][0].itemsize for n in image.names]
        covered = sum(widths)
        assert covered == size or name == "fs_kv_view", name      # the view ends in an int32 and 4 bytes of padding
    assert seen[("fs_kv_view", "size")] == sum(C.sizeof(t) for _, t in fs.FsKvView._fields_) + 4


@pytest.mark.skipif(shutil.which("g++") is None, reason="no C++ compiler")
def test_header_compiles_alone_as_cxx(tmp_path):
    src = tmp_path / "alone.cpp"
    src.write_text('#include "failsafe.h"\nint main() { fs_shape s = {}; return s.n_req + static_cast<int>(sizeof(fs_kv_view)) - 96; }\n')
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-I", INCLUDE, str(src)],
                   check=True)
