"""CPU-side checks of the boundary: the library builds/loads and exports every entry point that
include/hyb.h declares, and the Python binding names match the C names."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hyb.h")
LIB = os.path.join(ROOT, "paper_2602_21760_amd", "libhyb.so")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(hyb_[a-z0-9_]+)\s*\(", src)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        from paper_2602_21760_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_named_calls():
    names = declared_functions()
    for required in ("hyb_block_forward", "hyb_joint_attention", "hyb_cfg_combine", "hyb_branch_discrepancy",
                     "hyb_euler_step", "hyb_cfg_disc_euler"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), "libhyb.so does not export " + name


def test_binding_covers_every_declared_symbol():
    from paper_2602_21760_amd import binding
    for name in declared_functions():
        assert name in binding.SIGNATURES, "binding has no signature for " + name
    assert set(binding.SIGNATURES) == set(declared_functions())


def test_no_compute_calls_needed_for_queries(lib):
    lib.hyb_version.restype = ctypes.c_int
    assert lib.hyb_version() >= 100
    lib.hyb_last_error_string.restype = ctypes.c_char_p
    assert lib.hyb_last_error_string() is not None
    lib.hyb_discrepancy_workspace_bytes.restype = ctypes.c_size_t
    lib.hyb_discrepancy_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_size_t]
    assert lib.hyb_discrepancy_workspace_bytes(0, 100) == 0
    a = lib.hyb_discrepancy_workspace_bytes(1, 262144)
    b = lib.hyb_discrepancy_workspace_bytes(2, 262144)
    assert a > 0 and a % 256 == 0 and b >= 2 * a - 256


def test_argument_validation_happens_before_any_gpu_work(lib):
    """NULL / shape / dtype errors are reported by the host checks (no device needed)."""
    vp, sz, f, i = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_float, ctypes.c_int
    lib.hyb_cfg_combine.argtypes = [vp, vp, vp, sz, f, i, vp]
    assert lib.hyb_cfg_combine(None, None, None, 0, 1.0, 0, None) == 0          # n == 0: no-op
    assert lib.hyb_cfg_combine(None, None, None, 16, 1.0, 0, None) == 1         # HYB_ERR_NULL
    assert lib.hyb_cfg_combine(None, None, None, 16, 1.0, 7, None) == 3         # HYB_ERR_DTYPE
    assert lib.hyb_cfg_combine(vp(24), vp(32), vp(48), 16, 1.0, 0, None) == 4   # HYB_ERR_ALIGN (not dereferenced)
    lib.hyb_joint_attention.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp]
    assert lib.hyb_joint_attention(vp(16), vp(16), vp(16), vp(16), 1, 1, 8, 8, 32, 0.0, 0, None) == 2   # head_dim
    assert lib.hyb_joint_attention(vp(16), vp(16), vp(16), vp(16), 1, 1, 8, 0, 64, 0.0, 0, None) == 2   # n_kv == 0
    assert lib.hyb_joint_attention(None, None, None, None, 1, 1, 0, 0, 64, 0.0, 0, None) == 0           # n_q == 0
    # workspace form: the query is 0 for fp32 and for shapes that are never split; the cfg 2 shape (24 heads,
    # 4429 rows: 105 query blocks per XCD on 32 CUs) wants scratch, and a short one is an error
    lib.hyb_joint_attention_workspace_bytes.restype = sz
    lib.hyb_joint_attention_workspace_bytes.argtypes = [i, i, i, i]
    assert lib.hyb_joint_attention_workspace_bytes(1, 24, 4429, 0) == 0
    assert lib.hyb_joint_attention_workspace_bytes(1, 3, 4429, 1) == 0          # pairs not a multiple of 8
    need = lib.hyb_joint_attention_workspace_bytes(1, 24, 4429, 1)
    assert need > 0 and need % 256 == 0
    lib.hyb_joint_attention_ws.argtypes = [vp, vp, vp, vp, i, i, i, i, i, f, i, vp, sz, vp]
    assert lib.hyb_joint_attention_ws(vp(16), vp(16), vp(16), vp(16), 1, 24, 4429, 4429, 64, 0.0, 1, vp(256), need - 1, None) == 5
    assert lib.hyb_joint_attention_ws(vp(16), vp(16), vp(16), vp(16), 1, 24, 4429, 4429, 64, 0.0, 1, None, 0, None) == 1
    assert lib.hyb_joint_attention_ws(None, None, None, None, 1, 1, 0, 0, 64, 0.0, 0, None, 0, None) == 0
    lib.hyb_branch_discrepancy.argtypes = [vp, vp, i, sz, i, i, vp, vp, sz, vp]
    assert lib.hyb_branch_discrepancy(vp(16), vp(16), 1, 4096, 2, 0, vp(16), vp(256), 8, None) == 5     # workspace
    assert lib.hyb_branch_discrepancy(vp(16), vp(16), 1, 4096, 3, 0, vp(16), vp(256), 1 << 20, None) == 3
    lib.hyb_last_error_string.restype = ctypes.c_char_p
    assert b"p must be" in lib.hyb_last_error_string()
    # hyb_linear: epilogue values are 0..3 and 5 (HYB_EPI_GEGLU); m == 0 is a no-op for every valid one
    lib.hyb_linear.argtypes = [vp, vp, vp, vp, i, i, i, i, i, i, vp, vp, i, sz, vp]
    for epi, want in ((0, 0), (3, 0), (5, 0), (4, 3), (6, 3), (-1, 3)):
        assert lib.hyb_linear(None, None, None, None, 0, 64, 64, 1, 1, epi, None, None, 1, 0, None) == want, epi
    assert lib.hyb_linear(None, vp(16), None, vp(16), 8, 64, 64, 1, 1, 5, None, None, 1, 0, None) == 1    # NULL a


def test_struct_layouts_match_the_header(tmp_path):
    """The ctypes structures of the binding against sizeof / offsetof of the C declarations (compiled with gcc:
    the header is plain C)."""
    import shutil
    import subprocess
    from paper_2602_21760_amd import binding
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    structs = {"hyb_block_desc": binding.BlockDesc, "hyb_stream_weights": binding.StreamWeights,
               "hyb_block_weights": binding.BlockWeights, "hyb_sdxl_block_desc": binding.SdxlBlockDesc,
               "hyb_sdxl_block_weights": binding.SdxlBlockWeights, "hyb_switch_state": binding.SwitchState}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hyb.h"', 'int main(void) {']
    for cname, ct in structs.items():
        lines.append('printf("%s size %%zu\\n", sizeof(%s));' % (cname, cname))
        for fname, _ in ct._fields_:
            lines.append('printf("%s %s %%zu\\n", offsetof(%s, %s));' % (cname, fname, cname, fname))
    lines.append("return 0; }")
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    got = {tuple(l.split()[:2]): int(l.split()[2]) for l in out if l}
    for cname, ct in structs.items():
        assert got[(cname, "size")] == ctypes.sizeof(ct), cname
        for fname, _ in ct._fields_:
            assert got[(cname, fname)] == getattr(ct, fname).offset, (cname, fname)


def test_missing_library_is_an_error(monkeypatch, tmp_path):
    """No fallback: without libhyb.so the binding raises."""
    from paper_2602_21760_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(Exception):
        binding.lib()
