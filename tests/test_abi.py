"""The C-ABI library loads (no GPU needed) and exports every entry point include/eoq.h declares;
the Python binding names the same set; argument checks that need no device work return error codes."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "eoq.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(eoq_[a-z0-9_]+)\s*\(", src)))


def load():
    from paper_2105_13890_amd import build
    return ctypes.CDLL(build.build())


def test_every_declared_symbol_is_exported():
    lib = load()
    names = declared_functions()
    assert len(names) >= 20 and "eoq_conv_fwd" in names and "eoq_update_int8" in names
    for n in names:
        assert hasattr(lib, n), f"{n} declared in eoq.h but not exported"


def test_binding_lists_the_same_entry_points():
    import ast
    tree = ast.parse(open(os.path.join(ROOT, "paper_2105_13890_amd", "eoq.py")).read())
    exports = None
    for node in ast.walk(tree):
        if isinstance(node, ast.Assign) and getattr(node.targets[0], "id", "") == "EXPORTS":
            exports = sorted(ast.literal_eval(node.value))
    assert exports == declared_functions()


def test_strerror_and_null_argument_paths():
    lib = load()
    lib.eoq_strerror.restype = ctypes.c_char_p
    assert lib.eoq_strerror(0) == b"ok"
    assert b"workspace" in lib.eoq_strerror(3)
    lib.eoq_workspace_bytes.restype = ctypes.c_size_t
    assert lib.eoq_workspace_bytes(None, 0) == 0
    # null context / descriptor: rejected before any device call
    assert lib.eoq_conv_fwd(None, None, None, None, None, None, None, ctypes.c_size_t(0)) == 1
    assert lib.eoq_quantize(None, None, ctypes.c_size_t(0), 0, 0, None, None) == 1
    assert lib.eoq_destroy(None) == 1
