"""The C-ABI library loads and exports every symbol include/strp.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "strp.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(strp_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_five_entry_points():
    syms = _declared_symbols()
    for name in ("strp_gram", "strp_score_alloc", "strp_mask_topk", "strp_refit", "strp_admm_step"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2510_03246_amd import strp
    if not os.path.exists(strp.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(strp.LIB_PATH)
    for name in _declared_symbols():
        assert hasattr(lib, name), f"{name} declared in strp.h but not exported"
    assert sorted(strp.EXPORTS) == _declared_symbols()


def test_workspace_query_is_a_pure_host_function():
    from paper_2510_03246_amd import strp
    lib = strp.load_library()
    small = strp.ModuleDesc(64, 256, 512, 512, 512, strp.F32, strp.F32, 0)
    big = strp.ModuleDesc(4096, 16384, 262144, 262144, 262144, strp.BF16, strp.BF16, 4915)
    a, b = lib.strp_workspace_bytes(ctypes.byref(small)), lib.strp_workspace_bytes(ctypes.byref(big))
    assert 0 < a < b < 64 << 30
    assert lib.strp_workspace_bytes(None) == 0


def test_binding_fails_loudly_without_library(monkeypatch):
    from paper_2510_03246_amd import strp
    monkeypatch.setattr(strp, "_lib", None)
    monkeypatch.setattr(strp, "LIB_PATH", "/nonexistent/libstrp.so")
    with pytest.raises(FileNotFoundError):
        strp.load_library()


def test_binding_structs_mirror_the_header(tmp_path):
    """Size and last-field offset of every struct the binding marshals, as the C compiler lays the header out."""
    import subprocess
    from paper_2510_03246_amd import strp
    pairs = [("strp_module_desc", "k_max", strp.ModuleDesc), ("strp_score_in", "ldw", strp.ScoreIn),
             ("strp_module_state", "precision", strp.ModuleState), ("strp_params", "stages", strp.Params),
             ("strp_report", "status", strp.Report), ("strp_weight_ref", "ld", strp.WeightRef)]
    src = tmp_path / "layout.c"
    body = "".join(f'  printf("%zu %zu\\n", sizeof({c}), offsetof({c}, {f}));\n' for c, f, _ in pairs)
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "strp.h"\nint main(void) {\n' + body + "  return 0;\n}\n")
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)], check=True, timeout=120)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=30).stdout.split("\n")
    for (cname, field, cls), line in zip(pairs, out):
        size, off = (int(x) for x in line.split())
        assert ctypes.sizeof(cls) == size, cname
        assert getattr(cls, field).offset == off, (cname, field)
