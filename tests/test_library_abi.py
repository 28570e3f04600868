"""CPU-only checks of the C-ABI library: it loads, exports every function the header declares,
and its host-side argument validation answers before any GPU call."""
import ctypes as C
import os
import re

import pytest

from paper_2310_18313_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fp8lm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fp8lm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert len(names) >= 21
    for name in names:
        assert hasattr(L, name), name
    assert sorted(B.EXPORTS) == names


def test_struct_layouts_match_the_header():
    assert B.lib().fp8lm_sizeof_meta() == C.sizeof(B.Meta) == 112
    assert C.sizeof(B.AdamHparams) == 64 and C.sizeof(B.AutoscaleCfg) == 28 and C.sizeof(B.Tensor) == 16
    assert B.Meta.n_sat.offset == 96 and B.Meta.amax_hist.offset == 16


def _create(tensors):
    arr = (B.Tensor * max(1, len(tensors)))()
    for i, (o, n) in enumerate(tensors):
        arr[i].offset, arr[i].numel = o, n
    h = C.c_void_p()
    st = B.lib().fp8lm_create(C.byref(h), C.cast(arr, C.c_void_p), len(tensors), 0)
    return st, h


def test_create_rejects_bad_tensor_lists_before_touching_the_gpu():
    L = B.lib()
    assert _create([(8, 100)])[0] == -2                    # offset not a multiple of 16
    assert _create([(0, -1)])[0] == -1
    assert _create([(-16, 4)])[0] == -1
    assert _create([(0, 100), (96, 10)])[0] == -3          # overlap
    assert _create([(160, 10), (0, 161)])[0] == -3
    assert L.fp8lm_create(None, None, 0, 0) == -1
    for code, word in ((0, "ok"), (-1, "invalid"), (-2, "misaligned"), (-3, "overlap"), (-4, "HIP"), (-5, "too many")):
        assert word in L.fp8lm_status_string(code).decode()


def test_calls_reject_null_context():
    L = B.lib()
    cfg = B.autoscale_cfg()
    hp = B.adam_hparams(1e-3, 1)
    assert L.fp8lm_amax_scale(None, None, 0, 0, None, C.addressof(cfg), None) == -1
    assert L.fp8lm_cast_fp8(None, None, 0, None, 0, None, C.addressof(cfg), None) == -1
    assert L.fp8lm_adam_step_fp8(None, None, 0, None, None, None, None, None, None, None, None, None,
                                 C.addressof(hp), None) == -1
    assert L.fp8lm_destroy(None) == 0


def test_there_is_no_fallback_when_the_library_is_missing(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libfp8lm.so"))
    with pytest.raises(ImportError):
        B.lib()


def test_c_program_against_the_header_builds_and_fails_loudly_without_a_gpu():
    """tests/c_abi_parity.cpp includes only include/fp8lm.h and links libfp8lm.so: it compiling and linking shows
    the header is plain C-callable; without a GPU its first library call must report the HIP error."""
    import subprocess
    import torch
    import c_abi_build
    import oracle as O
    exe = c_abi_build.build()
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: the run itself is a gpu test")
    r = subprocess.run([exe, O.build()], capture_output=True, text=True, timeout=60)
    assert r.returncode == 2, (r.returncode, r.stdout, r.stderr)
    assert "fp8lm_create" in r.stderr and "HIP runtime error" in r.stderr


def test_header_is_plain_c(tmp_path):
    """include/fp8lm.h compiles as pedantic C99 with every warning on, and its structures have the sizes the
    Python binding assumes."""
    import subprocess
    src = tmp_path / "hdr.c"
    src.write_text(
        '#include "fp8lm.h"\n'
        "#define CHECK(name, cond) typedef char name[(cond) ? 1 : -1]\n"
        f"CHECK(meta_size, sizeof(fp8lm_meta) == {C.sizeof(B.Meta)});\n"
        f"CHECK(cfg_size, sizeof(fp8lm_autoscale_cfg) == {C.sizeof(B.AutoscaleCfg)});\n"
        f"CHECK(hp_size, sizeof(fp8lm_adam_hparams) == {C.sizeof(B.AdamHparams)});\n"
        f"CHECK(tensor_size, sizeof(fp8lm_tensor) == {C.sizeof(B.Tensor)});\n"
        "int main(void) { return 0; }\n")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                        "-fsyntax-only", str(src)], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
