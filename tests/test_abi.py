"""Host-side checks of the C-ABI library: it loads, exports every declared symbol, and its
argument validation and sizing logic behave as the header says.  No kernel is launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2510_04286_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2510_04286_amd import build
        build.build()
    return binding


def test_library_exports_every_declared_symbol(B):
    header = open(os.path.join(ROOT, "include", "slicemoe.h")).read()
    declared = set(re.findall(r"\b(slicemoe_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_layouts_match_the_header(B):
    assert ctypes.sizeof(B.slicemoe_config) == 40
    assert ctypes.sizeof(B.slicemoe_weights) == 9 * ctypes.sizeof(ctypes.c_void_p)
    assert ctypes.sizeof(B.slicemoe_workspace_layout) == 12 * ctypes.sizeof(ctypes.c_size_t)


def test_status_strings(B):
    assert B.slicemoe_status_string(0) == "ok"
    assert "workspace" in B.slicemoe_status_string(B.SLICEMOE_ERR_WORKSPACE)
    assert B.slicemoe_status_string(99) == "unknown status"


def test_config_validation_and_kernel_choice(B):
    ok = B.make_config(16384, 1024, 16, 2, 32, 256)
    assert B.slicemoe_uses_mfma(ok) == 1
    assert B.slicemoe_uses_mfma(B.make_config(512, 256, 4, 2, 8, 256, dtype="f32")) == 0
    assert B.slicemoe_uses_mfma(B.make_config(64, 768, 8, 2, 16, 384)) == 1  # ds = 96, the paper's own shape
    assert B.slicemoe_uses_mfma(B.make_config(64, 768, 16, 2, 16, 192)) == 1  # ds = 48: zero-padded K-steps and tiles
    assert B.slicemoe_uses_mfma(B.make_config(64, 768, 2, 2, 16, 1536)) == 1  # ds = 384: first router layer read from memory
    assert B.slicemoe_uses_mfma(B.make_config(64, 640, 16, 2, 16, 160)) == 0  # ds = 40: generic kernels
    assert B.slicemoe_uses_mfma(B.make_config(64, 1024, 16, 2, 32, 256, flags=B.SLICEMOE_FLAG_FORCE_GENERIC)) == 0
    for bad in [B.make_config(8, 100, 3, 2, 4, 16),      # d % S != 0
                B.make_config(8, 64, 4, 5, 4, 16),       # k > E
                B.make_config(-1, 64, 4, 2, 4, 16),
                B.make_config(8, 64, 4, 0, 4, 16),
                B.make_config(8, 64, 4, 2, 65, 16),      # E > 64
                B.make_config(8, 64, 4, 9, 16, 16),      # k > 8
                B.make_config(8, 640, 16, 2, 16, 160, flags=B.SLICEMOE_FLAG_REQUIRE_MFMA)]:
        assert B.slicemoe_uses_mfma(bad) == -1
        assert B.slicemoe_workspace_bytes(bad) == 0 and B.slicemoe_packed_bytes(bad) == 0
    L = B.lib()
    bad = B.make_config(8, 100, 3, 2, 4, 16)
    assert L.slicemoe_forward(ctypes.byref(bad), None, None, None, None, 0, None) == B.SLICEMOE_ERR_INVALID_ARG
    big = B.make_config(8, 64, 4, 2, 65, 16)
    assert L.slicemoe_dispatch(ctypes.byref(big), None, None, None, None, None, None, None, 0, None) == B.SLICEMOE_ERR_UNSUPPORTED
    # null pointers and short workspaces are reported before anything touches the GPU
    assert L.slicemoe_forward(ctypes.byref(ok), None, None, None, None, 0, None) == B.SLICEMOE_ERR_INVALID_ARG
    assert L.slicemoe_combine(ctypes.byref(ok), None, None, None, None) == B.SLICEMOE_ERR_INVALID_ARG
    w = B.slicemoe_weights()
    one = ctypes.c_void_p(256)  # never dereferenced: the workspace check comes first
    assert L.slicemoe_forward(ctypes.byref(ok), one, ctypes.byref(w), one, one, 1024, None) == B.SLICEMOE_ERR_WORKSPACE
    assert L.slicemoe_dispatch(ctypes.byref(ok), one, one, one, one, one, one, one, 16, None) == B.SLICEMOE_ERR_WORKSPACE


def test_train_router_parameter_checks(B):
    """Out-of-range parameters and missing tables of draws are INVALID_ARG before anything touches the GPU."""
    L = B.lib()
    ok = B.make_config(64, 1024, 16, 2, 32, 256)
    w = B.slicemoe_weights()
    one = ctypes.c_void_p(256)   # never dereferenced
    odd = ctypes.c_void_p(260)   # not 16-byte aligned

    def route(tp, noise, drop_u):
        return L.slicemoe_route_train(ctypes.byref(ok), one, ctypes.byref(w), tp, noise, drop_u, one, one, None, 0, None)

    def forward(tp, noise, drop_u):
        return L.slicemoe_forward_train(ctypes.byref(ok), one, ctypes.byref(w), tp, noise, drop_u, one, one, 0, None)

    P = B.slicemoe_route_train_params
    for call in (route, forward):
        assert call(None, None, None) == B.SLICEMOE_ERR_INVALID_ARG
        for bad in (P(0.0, 0.0, 0.0), P(-1.0, 0.0, 0.0), P(float("nan"), 0.0, 0.0), P(float("inf"), 0.0, 0.0),
                    P(1.0, -0.1, 0.0), P(1.0, float("nan"), 0.0), P(1.0, 0.0, 1.0), P(1.0, 0.0, -0.1),
                    P(1.0, 0.0, float("nan")), P(1.0, 0.0, 0.0, float("nan")), P(1.0, 0.0, 0.0, float("inf"))):
            assert call(ctypes.byref(bad), one, one) == B.SLICEMOE_ERR_INVALID_ARG
        assert call(ctypes.byref(P(1.0, 0.5, 0.0)), None, None) == B.SLICEMOE_ERR_INVALID_ARG   # noise table missing
        assert call(ctypes.byref(P(1.0, 0.5, 0.0)), odd, None) == B.SLICEMOE_ERR_INVALID_ARG    # misaligned
        assert call(ctypes.byref(P(1.0, 0.0, 0.2)), None, None) == B.SLICEMOE_ERR_INVALID_ARG   # drop_u missing
    # valid parameters get as far as the workspace check of the whole-layer call
    assert forward(ctypes.byref(P(0.7, 0.5, 0.2)), one, one) == B.SLICEMOE_ERR_WORKSPACE
    assert forward(ctypes.byref(P(0.7, 0.5, 0.2, -0.1)), one, one) == B.SLICEMOE_ERR_WORKSPACE   # any finite weight
    assert ctypes.sizeof(P) == 16
    bad_cfg = B.make_config(8, 100, 3, 2, 4, 16)
    assert L.slicemoe_route_train(ctypes.byref(bad_cfg), one, ctypes.byref(w), ctypes.byref(P(1.0, 0.0, 0.0)), None, None,
                                  one, one, None, 0, None) == B.SLICEMOE_ERR_INVALID_ARG


def test_capacity_and_sizes(B):
    from paper_2510_04286_amd import workload as wl
    for name, c in wl.CONFIGS.items():
        cfg = B.config_of(c)
        assert B.slicemoe_capacity(cfg) == c.capacity()
        L = B.slicemoe_get_workspace_layout(cfg)
        assert L.total == B.slicemoe_workspace_bytes(cfg) > 0
        offs = [L.topk_idx, L.topk_p, L.counts_raw, L.counts, L.offsets, L.perm, L.inv, L.y, L.stats, L.scratch, L.packed]
        assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
        assert L.perm - L.offsets >= (c.E + 1) * 4 and L.stats - L.y >= c.Na * c.ds * (2 if c.dtype == 'bf16' else 4)
        assert B.slicemoe_dispatch_workspace_bytes(cfg) >= -(-c.Na // 1024) * c.E * 4
        assert (B.slicemoe_packed_bytes(cfg) > 0) == (c.dtype == "bf16")
    assert B.slicemoe_capacity(B.make_config(100, 64, 4, 2, 8, 16, capacity_factor=1.1)) == 111  # ceil(1.1f*800/8)


C_CALLER = r"""
#include <stdio.h>
#include "slicemoe.h"
int main(void)
{
    slicemoe_config c;
    c.T = 16384; c.d = 1024; c.S = 16; c.k = 2; c.E = 32; c.Hr = 256; c.He = 256;
    c.capacity_factor = 0.0f; c.dtype = SLICEMOE_BF16; c.flags = 0;
    printf("%zu %zu %s\n", slicemoe_workspace_bytes(&c), slicemoe_backward_workspace_bytes(&c),
           slicemoe_status_string(SLICEMOE_ERR_WORKSPACE));
    c.S = 3;   /* d %% S != 0 */
    printf("%zu %d\n", slicemoe_workspace_bytes(&c), (int)slicemoe_route(&c, 0, 0, 0, 0, 0, 0, 0));
    return 0;
}
"""


def test_header_is_plain_c_and_the_library_links_from_c(B, tmp_path):
    """The boundary is a C ABI: the header compiles as pedantic C99 without any HIP include, and a C program linked
    against the shared library gets the same sizes as the Python binding (size queries and argument checks only)."""
    import subprocess
    from paper_2510_04286_amd import workload as wl
    src = tmp_path / "caller.c"
    src.write_text(C_CALLER.replace("%%", "%"))
    exe = tmp_path / "caller"
    libdir = os.path.dirname(B.LIB_PATH)
    libname = os.path.basename(B.LIB_PATH)
    assert libname.startswith("lib") and libname.endswith(".so")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-l" + libname[3:-3], "-Wl,-rpath," + libdir,
                    "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    cfg = B.config_of(wl.CONFIGS["headline"])
    first = out[0].split(" ", 2)
    assert int(first[0]) == B.slicemoe_workspace_bytes(cfg)
    assert int(first[1]) == B.slicemoe_backward_workspace_bytes(cfg)
    assert first[2] == B.lib().slicemoe_status_string(B.SLICEMOE_ERR_WORKSPACE).decode()
    assert out[1].split() == ["0", str(B.SLICEMOE_ERR_INVALID_ARG)]
