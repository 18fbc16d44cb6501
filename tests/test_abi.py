"""The C-ABI library loads and exports exactly what include/radial.h declares (no GPU needed)."""
import ctypes
import os
import re

from paper_2506_19852_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("radial.h", "radial_diag.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"RADIAL_API\s+[\w\s\*]+?\b(radial_\w+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = _declared()
    assert len(names) == 18 and set(names) == set(binding.EXPORTS)
    lib = ctypes.CDLL(binding.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def test_binding_prototypes_and_error_string():
    lib = binding.load()
    assert binding.radial_last_error() == "" or isinstance(binding.radial_last_error(), str)
    # argument errors are detected before any GPU work
    out = ctypes.c_void_p()
    rc = lib.radial_mask_build(None, None, ctypes.byref(out))
    assert rc == -1 and "NULL" in binding.radial_last_error()
    p = binding.radial_mask_params(4, 16, 100, 1, 0, 1, 1, 0)
    rc = lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out))
    assert rc == -4 and "block" in binding.radial_last_error()
    p = binding.radial_mask_params(0, 16, 64, 1, 0, 1, 1, 0)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -1
    p = binding.radial_mask_params(4, 16, 64, 1, 8, 1, 1, 0)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -1
    assert lib.radial_attn_bwd_workspace(1, 1, 64, 64, None) == 0
    lib.radial_mask_free(None)


def test_header_is_plain_c_and_links(tmp_path):
    """include/radial.h compiles as C99 and a C program links against the library and gets the
    documented error codes back from calls that need no GPU."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        import pytest
        pytest.skip("no C compiler")
    src = os.path.join(ROOT, "tests", "sanitize", "abi_errors.c")
    exe = tmp_path / "abi"
    libdir = os.path.dirname(binding.lib_path())
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", os.path.join(ROOT, "include"),
                           str(src), "-o", str(exe), "-L", libdir, "-lradial", f"-Wl,-rpath,{libdir}"])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", (out.returncode, out.stdout, out.stderr)


def test_size_limits_are_reported_before_any_gpu_work():
    lib = binding.load()
    out = ctypes.c_void_p()
    # N = f*s must stay below 2^31 - block
    p = binding.radial_mask_params(1 << 16, 1 << 15, 128, 1, 0, 1, 1, 0)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -1
    assert "token count" in binding.radial_last_error()
    # more key blocks than the builder's bitmap holds (491 520)
    p = binding.radial_mask_params(1000, 40000, 64, 1, 0, 1, 1, 0)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -4
    assert "key blocks" in binding.radial_last_error()
    # sparsity knob outside its range, negative text-token count
    p = binding.radial_mask_params(4, 64, 64, 1, 0, 40000, 1, 0)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -1
    p = binding.radial_mask_params(4, 64, 64, 1, 0, 1, 1, -3)
    assert lib.radial_mask_build(ctypes.byref(p), None, ctypes.byref(out)) == -1
    assert out.value is None
