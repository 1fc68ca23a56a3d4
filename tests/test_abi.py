"""Host-side checks of the C ABI: the library loads, exports what the header declares, validates arguments."""
import os
import re

import numpy as np

import paper_2604_02047_amd as g

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "goose.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(goose_[a-z_0-9]+)\s*\(", header))
    assert {"goose_build_mask", "goose_verify_layer", "goose_lm_head_argmax", "goose_accept",
            "goose_compact_kv"} <= declared
    lib = g.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert declared == set(g.EXPORTS)


def test_strerror_and_parent_validation():
    lib = g.load_library()
    assert lib.goose_strerror(0) == b"ok"
    assert b"topological" in lib.goose_strerror(-4)
    assert g.goose_check_parent([-1]) == 0
    assert g.goose_check_parent([-1, 0, 0, 2, 1]) == 0
    assert g.goose_check_parent([-1, 0, 2, 1]) == -4      # child listed before its parent
    assert g.goose_check_parent([-1, 1]) == -4            # self parent
    assert g.goose_check_parent([0, 0]) == -4             # root must be -1
    assert g.goose_check_parent([-1, -1]) == -4           # two roots
    assert g.goose_check_parent(np.full(129, -1)) == -1   # too many nodes
    assert g.goose_check_parent(None) == -1


def test_every_generated_tree_passes_the_host_check():
    import goose_inputs as gi
    for t in [gi.tree_tiny_spine(), gi.tree_spine_7b(0), gi.tree_spine_13b(), gi.tree_spine_33b(),
              gi.tree_spine_stress(), gi.tree_balanced(), gi.tree_random(128, 0)]:
        assert g.goose_check_parent(t.parent) == 0


def test_the_public_header_is_plain_c(tmp_path):
    """include/goose.h is the boundary: it must compile as C99 (no C++ or torch types in the signatures)."""
    import os
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        import pytest
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "h.c"
    src.write_text('#include "goose.h"\nint main(void) { return GOOSE_OK; }\n')
    r = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only",
                        "-I", os.path.join(root, "include"), str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
