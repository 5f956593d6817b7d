"""The C-ABI library loads and exports every symbol the header declares (no GPU needed)."""
import ctypes
import os

import pytest

import paper_2604_24073_amd as fs


def test_library_is_built_in_tree():
    assert os.path.exists(fs.LIB_PATH), "run `python -m paper_2604_24073_amd.build` first"


def test_every_declared_symbol_is_exported():
    lib = fs.load_library()
    names = fs.declared_symbols()
    for required in ("fs_gather_jagged", "fs_unique_ids", "fs_collision_split", "fs_segment_reduce_grads",
                     "fs_rowwise_adagrad_update", "fs_prioritized_step", "fs_ctx_create", "fs_ctx_destroy",
                     "fs_last_error", "fs_check_async"):
        assert required in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/freescale.h but not exported"


def test_version_and_null_context_are_errors_not_crashes():
    lib = fs.load_library()
    assert lib.fs_version() >= 100
    assert lib.fs_gather_jagged(None, None, 0, 64, 0, None, None, 0, 0, None, None) == fs.FS_EINVAL
    assert lib.fs_unique_ids(None, None, 0, 0, None, None, None, None, None, None) == fs.FS_EINVAL
    assert lib.fs_prioritized_step(None, None, None) == fs.FS_EINVAL
    assert lib.fs_ctx_destroy(None) == fs.FS_OK
    assert lib.fs_last_error(None) == b""                                         # no context-free call has failed yet
    # the context-free split rejects what its fixed scratch array cannot hold before it touches the GPU
    too_many = fs.FS_STATIC_SPLIT_MAX_ROWS + 1
    assert lib.fs_collision_split_static(None, None, None, None, too_many, 0, None, None, None, None, None, None,
                                         None, None) == fs.FS_ENOMEM
    assert b"FS_STATIC_SPLIT_MAX_ROWS" in lib.fs_last_error(None)
    assert lib.fs_collision_split_static(None, None, None, None, -1, 0, None, None, None, None, None, None,
                                         None, None) == fs.FS_EINVAL
    assert lib.fs_collision_split_static(None, None, None, None, 10, 0, None, None, None, None, None, None,
                                         ctypes.c_void_p(8), None) == fs.FS_EINVAL   # null lists with cap_t > 0
    assert lib.fs_ctx_create(None, 0, 10, 64) == fs.FS_EINVAL
    h = ctypes.c_void_p()
    assert lib.fs_ctx_create(ctypes.byref(h), 0, 0, 64) == fs.FS_EINVAL          # max_ids < 1
    assert lib.fs_ctx_create(ctypes.byref(h), 0, 10, 4096) == fs.FS_EINVAL       # dim beyond FS_MAX_DIM


def test_step_args_layout_matches_header_order():
    # field order of the ctypes mirror must follow the struct in the header
    text = open(os.path.join(os.path.dirname(fs.LIB_PATH), "..", "include", "freescale.h")).read()
    body = text[text.index("typedef struct fs_step_args {"):text.index("} fs_step_args;")]
    import re
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"[\*\s]([a-z_0-9]+)\s*[;,]", body)
    assert names == [f[0] for f in fs.fs_step_args._fields_]


def test_step_args_size_and_offsets_match_a_c_compiler(tmp_path):
    # the header read by a plain C compiler must lay the record out exactly as the ctypes mirror does
    import subprocess
    root = os.path.join(os.path.dirname(fs.LIB_PATH), "..")
    fields = [f[0] for f in fs.fs_step_args._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "freescale.h"\nint main(void) {\n'
                   '  printf("%zu\\n", sizeof(fs_step_args));\n' +
                   "".join(f'  printf("%zu\\n", offsetof(fs_step_args, {n}));\n' for n in fields) +
                   "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"), str(src),
                    "-o", str(exe)], check=True)
    out = [int(x) for x in subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()]
    assert out[0] == ctypes.sizeof(fs.fs_step_args)
    assert out[1:] == [getattr(fs.fs_step_args, n).offset for n in fields]
