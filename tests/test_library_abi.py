"""CPU-side checks of the boundary: the shared library loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2603_08343_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "wht_affine.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(wht_affine_\w+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(binding.library_path())
    names = _declared_functions()
    assert len(names) >= 6
    for name in names:
        assert hasattr(lib, name), f"{name} declared in wht_affine.h but not exported"
    assert set(binding.EXPORTS) == set(names)


def test_version_and_status_strings():
    assert binding.wht_affine_version() >= 100
    seen = {binding.wht_affine_status_string(s) for s in range(0, 7)}
    assert binding.wht_affine_status_string(2).startswith("d must be a power of two")
    assert len(seen) == 7 and "ok" in seen
    assert binding.wht_affine_status_string(99) == "unknown status"


OK, NULLP, DIM, DTYPE, ALIGN, WS = 0, 1, 2, 3, 4, 5
P = 0x1000   # a 16-byte-aligned non-null fake address: validation fails before it is ever used


@pytest.mark.parametrize("args,want", [
    ((0, P, P, P, 4, 256, 0), NULLP),
    ((P, 0, P, P, 4, 256, 0), NULLP),
    ((P, P, 0, P, 4, 256, 0), NULLP),
    ((P, P, P, 0, 4, 256, 0), NULLP),
    ((P, P, P, P, 4, 768, 0), DIM),        # 12 * 2^m widths: bfloat16 only ...
    ((P, P, P, P, 4, 384, 1), DIM),        # ... from 768 ...
    ((P, P, P, P, 4, 24576, 1), DIM),      # ... to 12288
    ((P, P, P, P, 4, 1000, 1), DIM),       # neither 2^n nor 12 * 2^m
    ((P, P, P, P, 4, 1280, 1), DIM),       # 5 * 2^8
    ((P, P, P, P, 0, 768, 1), OK),         # accepted width, N = 0
    ((P, P, P, P, 0, 6144, 1), OK),
    ((P, P, P, P, 0, 12288, 1), OK),
    ((P, P, P, P, 4, 16, 0), DIM),         # below WHT_MIN_D
    ((P, P, P, P, 4, 32768, 1), DIM),      # above WHT_MAX_D
    ((P, P, P, P, 4, 16384, 0), DIM),      # above WHT_MAX_D_F32
    ((P, P, P, P, 4, 0, 0), DIM),
    ((P, P, P, P, 4, -256, 0), DIM),
    ((P, P, P, P, -1, 256, 0), DIM),
    ((P, P, P, P, 4, 256, 2), DTYPE),
    ((P, P, P, P, 4, 256, -1), DTYPE),
    ((P + 8, P, P, P, 4, 256, 0), ALIGN),
    ((P, P + 4, P, P, 4, 256, 0), ALIGN),
    ((P, P, P, P + 2, 4, 256, 1), ALIGN),
    ((P, P, P, P, 0, 256, 1), OK),         # N = 0: nothing to do, nothing enqueued
])
def test_forward_argument_validation(args, want):
    assert binding.wht_affine_forward_raw(*args) == want


def test_forward_residual_argument_validation():
    call = binding.wht_affine_forward_residual_raw
    assert call(P, P, P, 0, P, 4, 256, 1) == NULLP            # resid is required here
    assert call(P, P, P, P + 8, P, 4, 256, 1) == ALIGN
    assert call(P, P, P, P, P, 4, 768, 0) == DIM
    assert call(P, P, P, P, P, 0, 1536, 1) == OK
    assert call(P, P, P, P, P, 4, 256, 3) == DTYPE
    assert call(P, P, P, P, P, 0, 256, 1) == OK


def test_forward_residual_stats_argument_validation():
    call = binding.wht_affine_forward_residual_stats_raw
    assert call(P, P, P, P, P, 0, 4, 256, 1) == NULLP             # the statistic's output is required
    assert call(P, P, P, 0, P, P, 4, 256, 1) == NULLP
    assert call(P, P, P, P, P, P + 2, 4, 256, 1) == ALIGN         # float32: 4-byte aligned
    assert call(P, P, P, P, P, P + 4, 0, 256, 1) == OK
    assert call(P, P, P, P, P, P, 4, 100, 1) == DIM
    assert call(P, P, P, P, P, P, 0, 768, 1) == OK


def test_backward_argument_validation():
    ws = binding.wht_affine_backward_workspace_bytes(100, 1024, 1)
    assert ws > 0 and ws % 16 == 0
    call = binding.wht_affine_backward_raw
    assert call(0, P, P, P, P, P, 100, 1024, 1, P, ws) == NULLP
    assert call(P, P, P, P, 0, P, 100, 1024, 1, P, ws) == NULLP
    assert call(P, P, P, P, P, P, 100, 1000, 1, P, ws) == DIM
    assert call(P, P, P, P, P, P, 100, 1024, 5, P, ws) == DTYPE
    assert call(P, P + 1, P, P, P, P, 100, 1024, 1, P, ws) == ALIGN
    assert call(P, P, P, P, P, P, 100, 1024, 1, 0, ws) == WS
    assert call(P, P, P, P, P, P, 100, 1024, 1, P, ws - 1) == WS
    assert call(P, P, P, P, P, P, 100, 1024, 1, P + 4, ws) == ALIGN
    # optional outputs: dalpha and dbeta come together; something must be asked for
    assert call(P, P, P, P, P, 0, 100, 1024, 1, P, ws) == NULLP
    assert call(P, P, P, 0, 0, 0, 100, 1024, 1, P, ws) == NULLP
    assert call(P, 0, P, P, P, P, 100, 1024, 1, P, ws) == NULLP            # the sums need x
    assert call(P, 0, P, P, 0, 0, 0, 1024, 1, 0, 0) == OK                  # dx only: no x, no workspace
    assert call(P, 0, P, P + 8, 0, 0, 4, 1024, 1, 0, 0) == ALIGN
    assert call(P, P, P, 0, P, P, 100, 1024, 1, 0, 0) == WS                # sums only still need it


def test_workspace_query():
    q = binding.wht_affine_backward_workspace_bytes
    assert q(0, 1024, 1) == 0
    assert q(10, 1000, 1) == 0 and q(10, 1024, 9) == 0
    # one row of 2*d floats per workgroup; never more workgroups than token groups
    assert q(1, 8192, 1) == 2 * 8192 * 4
    assert q(32768, 8192, 1) >= q(64, 8192, 1) > 0
    assert q(32768, 8192, 1) <= 64 << 20
    # rows of 12 * 2^m elements: the partial rows have the row's real length
    assert q(1, 6144, 1) == 2 * 6144 * 4
    assert q(4, 768, 1) == 2 * 768 * 4            # four tokens share a workgroup at d = 768
    assert q(10, 768, 0) == 0 and q(10, 24576, 1) == 0


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libwht_affine.so")
    with pytest.raises(RuntimeError, match="no CPU or eager fallback"):
        binding.library()


def test_product_path_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2603_08343_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "wht_oracle" not in text, f


def test_header_is_plain_c_and_links(tmp_path):
    """include/wht_affine.h must be usable from C (no C++ in the signatures): compile a C99
    translation unit that takes the address of every declared function with the declared
    prototype, link it against the built library, and run it (no GPU call is made)."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text(r'''
#include <stdio.h>
#include "wht_affine.h"
int main(void) {
    int (*fwd)(const void *, const float *, const float *, void *, int64_t, int32_t, int32_t, void *) = wht_affine_forward;
    int (*fwdr)(const void *, const float *, const float *, const void *, void *, int64_t, int32_t, int32_t, void *) = wht_affine_forward_residual;
    int (*fwds)(const void *, const float *, const float *, const void *, void *, float *, int64_t, int32_t, int32_t,
                void *) = wht_affine_forward_residual_stats;
    size_t (*wsq)(int64_t, int32_t, int32_t) = wht_affine_backward_workspace_bytes;
    int (*bwd)(const void *, const void *, const float *, void *, float *, float *, int64_t, int32_t, int32_t,
               void *, size_t, void *) = wht_affine_backward;
    int (*bwds)(const void *, const void *, const float *, void *, float *, float *, int64_t, int32_t, int32_t,
                void *) = wht_affine_backward_static;
    /* argument validation happens before anything touches the GPU */
    if (fwd(NULL, NULL, NULL, NULL, 4, 256, WHT_DTYPE_F32, NULL) != WHT_ERR_NULL_PTR) return 1;
    if (fwdr((void *)16, (float *)16, (float *)16, (void *)16, (void *)16, 4, 100, WHT_DTYPE_BF16, NULL) != WHT_ERR_BAD_DIM) return 2;
    if (wsq(0, 1024, WHT_DTYPE_BF16) != 0) return 3;
    if (fwds((void *)16, (float *)16, (float *)16, (void *)16, (void *)16, NULL, 4, 256, WHT_DTYPE_BF16, NULL)
        != WHT_ERR_NULL_PTR) return 6;
    if (bwd((void *)16, (void *)16, (float *)16, (void *)16, (float *)16, (float *)16, 4, 1024, 7, NULL, 0, NULL)
        != WHT_ERR_BAD_DTYPE) return 4;
    /* the static-scratch variant validates the same way, and refuses what its buffer cannot hold */
    if (bwds(NULL, (void *)16, (float *)16, (void *)16, (float *)16, (float *)16, 4, 1024, WHT_DTYPE_BF16, NULL)
        != WHT_ERR_NULL_PTR) return 7;
    if (bwds((void *)16, (void *)16, (float *)16, (void *)16, (float *)16, (float *)16, 4096, 16384, WHT_DTYPE_BF16, NULL)
        != WHT_ERR_WORKSPACE) return 8;
    if (wsq(4096, 8192, WHT_DTYPE_BF16) > WHT_STATIC_WORKSPACE_BYTES) return 9;
    if (WHT_MIN_D != 32 || WHT_MAX_D != 16384 || WHT_MIN_D_TWELVE != 768 || WHT_MAX_D_TWELVE != 12288) return 5;
    printf("%s|%d\n", wht_affine_status_string(WHT_OK), wht_affine_version());
    return 0;
}
''')
    exe = tmp_path / "use_header"
    libdir = os.path.dirname(binding.library_path())
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic",
                    "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src),
                    "-L", libdir, "-l:libwht_affine.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, (out.returncode, out.stderr)
    assert out.stdout.strip().startswith("ok|")


def test_autograd_wrapper_has_no_cpu_path():
    """The Module builds on the CPU (parameters only) but refuses to run there."""
    import torch
    from paper_2603_08343_amd.autograd import WhtAffine
    layer = WhtAffine(64)
    assert layer.alpha.dtype == torch.float32 and float(layer.alpha.detach().sum()) == 64.0
    assert float(layer.beta.detach().abs().sum()) == 0.0
    if not torch.cuda.is_available():
        with pytest.raises((RuntimeError, ValueError)):
            layer(torch.zeros(2, 64))
