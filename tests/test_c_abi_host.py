"""Host-side checks of the C ABI that need no GPU: the shared library loads, exports every
symbol that include/la.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "la.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2006_16236_amd import build
    if not os.path.exists(build.LIB):
        build.build_library(force=True)
    from paper_2006_16236_amd import binding
    return binding.raw()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(la_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2006_16236_amd import binding
    names = declared_functions()
    assert {"la_causal_fwd", "la_causal_bwd", "la_global_fwd", "la_recurrent_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in la.h but not exported"
    assert set(binding.EXPORTS) == set(names)


def test_version_and_status_strings(lib):
    from paper_2006_16236_amd import binding
    assert binding.la_version() >= 100
    seen = set()
    for st in range(0, -9, -1):
        s = binding.status_string(st)
        assert s and s != "unknown status" and s not in seen
        seen.add(s)
    assert binding.status_string(-99) == "unknown status"
    assert binding.la_kernel_name(2) == "causal_pass_fwd" and binding.la_kernel_name(99) == "unknown"


def test_workspace_queries(lib):
    from paper_2006_16236_amd import binding as b
    assert b.la_causal_fwd_workspace(256, 8, 512, 64, 64) == 0          # 2048 sequences: one segment each
    long = b.la_causal_fwd_workspace(2, 8, 65536, 64, 64)
    assert long == 16 * 128 * (64 * 64 + 64) * 4                        # 128 segments of 512 tokens
    assert b.la_causal_bwd_workspace(2, 8, 65536, 64, 64) > 2 * long
    assert b.la_global_fwd_workspace(1, 1, 1, 32, 32) >= (32 * 32 + 32) * 4
    assert b.la_global_bwd_workspace(1, 1, 1, 32, 32) >= 2 * (32 * 32 + 32) * 4 + 8
    assert b.la_causal_fwd_workspace(1, 1, 100, 48, 64) == 0            # invalid D: query returns 0
    assert b.la_causal_fwd_workspace(0, 1, 100, 64, 64) == 0


def test_argument_errors_are_reported_before_any_launch(lib):
    """Fake (never dereferenced) device addresses: every call must fail in validation."""
    from paper_2006_16236_amd import binding as b
    p = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10004)
    null = ctypes.c_void_p(None)
    f = ctypes.c_float
    fwd = lib.la_causal_fwd
    assert fwd(null, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fwd(p, p, p, null, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fwd(p, p, p, p, null, 0, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_SHAPE
    assert fwd(p, p, p, p, null, 1, 1, 0, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_SHAPE
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(-1.0), 0, null, 0, null) == b.LA_ERR_SHAPE
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(float("nan")), 0, null, 0, null) == b.LA_ERR_SHAPE
    assert fwd(p, p, p, p, null, 1 << 20, 1 << 10, 1 << 20, 64, 64, f(0), 0, null, 0, null) == b.LA_ERR_SHAPE
    assert fwd(p, p, p, p, null, 1, 1, 16, 48, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 128, f(1e-6), 0, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 7, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, odd, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_ALIGN
    # the token-major entry points validate the same way
    fwd_t, bwd_t = lib.la_causal_fwd_bnhd, lib.la_causal_bwd_bnhd
    assert fwd_t(null, p, p, p, null, 1, 4, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fwd_t(p, p, p, p, null, 1, 4, 16, 48, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd_t(p, p, odd, p, null, 1, 4, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_ALIGN
    assert bwd_t(p, p, p, null, p, null, null, p, p, p, 1, 4, 16, 64, 64, f(1e-6), 0, p, 1 << 30,
                 null) == b.LA_ERR_NULL
    assert bwd_t(p, p, p, null, p, null, p, p, p, p, 1, 4, 16, 64, 64, f(1e-6), 0, null, 0,
                 null) == b.LA_ERR_WORKSPACE
    # a long sequence needs a workspace
    assert fwd(p, p, p, p, null, 1, 1, 4096, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE
    assert fwd(p, p, p, p, null, 1, 1, 4096, 64, 64, f(1e-6), 0, p, 1024, null) == b.LA_ERR_WORKSPACE

    # the forward without a workspace argument: same validation; sizes beyond its built-in
    # scratch array are refused before any GPU call
    fna = lib.la_causal_fwd_noalloc
    assert fna(null, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null) == b.LA_ERR_NULL
    assert fna(p, p, p, p, null, 1, 1, 16, 48, 64, f(1e-6), 0, null) == b.LA_ERR_UNSUPPORTED
    assert fna(p, odd, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null) == b.LA_ERR_ALIGN
    # (1000 sequences cut in three: 3000 states of 16.6 KB)
    assert b.la_causal_fwd_workspace(125, 8, 4096, 64, 64) > b.LA_NOALLOC_SCRATCH_BYTES
    assert fna(p, p, p, p, null, 125, 8, 4096, 64, 64, f(1e-6), 0, null) == b.LA_ERR_SCRATCH
    assert b.la_causal_fwd_workspace(2, 8, 1 << 16, 64, 64) <= b.LA_NOALLOC_SCRATCH_BYTES

    fws = lib.la_causal_fwd_state
    assert fws(p, p, p, p, null, p, null, null, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fws(p, p, p, null, null, p, null, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fws(p, p, p, null, null, null, null, null, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_NULL
    assert fws(p, p, p, odd, p, p, null, null, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_ALIGN
    assert fws(p, p, p, null, null, p, null, null, null, 1, 1, 4096, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE

    bwd = lib.la_causal_bwd
    assert bwd(p, p, p, p, p, null, null, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_NULL
    assert bwd(p, p, p, p, p, null, p, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE
    assert bwd(p, p, p, p, p, null, p, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 8, null) == b.LA_ERR_WORKSPACE
    assert bwd(p, p, p, p, p, null, p, p, p, odd, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_ALIGN
    assert bwd(p, p, p, p, p, odd, p, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_ALIGN

    bws = lib.la_causal_bwd_state
    # Q K V S0 z0 O den fwd_ws dO dS1 dz1 dQ dK dV dS0 dz0
    ok16 = [p, p, p, null, null, p, p, null, p, null, null, p, p, p, null, null]
    tail = (1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null)
    for pos in (3, 9, 14):                      # one half of a state pair without the other
        args = list(ok16)
        args[pos] = p
        assert bws(*args, *tail) == b.LA_ERR_NULL
    args = list(ok16)
    args[8] = null
    assert bws(*args, *tail) == b.LA_ERR_NULL
    args = list(ok16)
    args[14], args[15] = p, odd
    assert bws(*args, *tail) == b.LA_ERR_ALIGN
    assert bws(*ok16, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE

    # element type codes: 0..4 are known (fp32, bf16, the same with Q, K as feature values, fp32 poly2)
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 5, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), -1, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 4096, 64, 64, f(1e-6), 3, null, 0, null) == b.LA_ERR_WORKSPACE
    assert b.la_causal_bwd_workspace(2, 8, 4096, 64, 64, b.LA_BF16_FEATURES) == \
        b.la_causal_bwd_workspace(2, 8, 4096, 64, 64, b.LA_BF16)

    # the degree-2 polynomial map: 8 raw values per token, nothing else
    assert fwd(p, p, p, p, null, 1, 1, 16, 64, 64, f(0.5), b.LA_F32_POLY2, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 16, 4, 64, f(0.5), b.LA_F32_POLY2, null, 0, null) == b.LA_ERR_UNSUPPORTED
    assert fwd(p, p, p, p, null, 1, 1, 4096, 8, 64, f(0.5), b.LA_F32_POLY2, null, 0, null) == b.LA_ERR_WORKSPACE
    assert b.la_causal_fwd_workspace(1, 1, 4096, 8, 64, b.LA_F32_POLY2) == b.la_causal_fwd_workspace(1, 1, 4096, 64, 64)
    assert b.la_causal_fwd_workspace(1, 1, 4096, 8, 64) == 0            # D = 8 without the map: unsupported

    glob = lib.la_global_fwd
    assert glob(p, p, p, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE
    assert glob(p, p, null, p, null, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 20, null) == b.LA_ERR_NULL
    assert glob(p, p, p, p, odd, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 20, null) == b.LA_ERR_ALIGN

    gbwd = lib.la_global_bwd
    assert gbwd(p, p, p, p, p, null, null, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_NULL
    assert gbwd(p, p, p, p, p, null, p, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, null, 0, null) == b.LA_ERR_WORKSPACE
    assert gbwd(p, p, p, p, p, null, p, p, p, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 8, null) == b.LA_ERR_WORKSPACE
    assert gbwd(p, p, p, p, p, null, p, p, odd, p, 1, 1, 16, 64, 64, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_ALIGN
    assert gbwd(p, p, p, p, p, null, p, p, p, p, 1, 1, 16, 64, 40, f(1e-6), 0, p, 1 << 30, null) == b.LA_ERR_UNSUPPORTED

    step = lib.la_recurrent_step
    assert step(p, p, p, null, p, p, 1, 1, 64, 64, f(1e-6), 0, null) == b.LA_ERR_NULL
    assert step(p, p, p, p, p, p, 1, 1, 16, 64, f(1e-6), 0, null) == b.LA_ERR_UNSUPPORTED
    assert step(p, p, p, p, p, p, 1, -1, 64, 64, f(1e-6), 0, null) == b.LA_ERR_SHAPE
    steps = lib.la_recurrent_steps
    assert steps(p, p, p, p, p, null, 4, 1, 1, 64, 64, f(1e-6), 0, null) == b.LA_ERR_NULL
    assert steps(p, p, p, p, p, p, 0, 1, 1, 64, 64, f(1e-6), 0, null) == b.LA_ERR_SHAPE
    assert steps(p, p, p, p, p, p, 4, 1, 1, 64, 48, f(1e-6), 0, null) == b.LA_ERR_UNSUPPORTED


def test_aliasing_is_refused(lib):
    """Overlap of a written buffer with any other buffer, found from pointers and sizes alone
    (fake addresses, nothing is launched)."""
    from paper_2006_16236_amd import binding as b
    f, vp, null = ctypes.c_float, ctypes.c_void_p, ctypes.c_void_p(None)
    B, H, N, D, M = 1, 2, 16, 64, 64                          # one chunk: no forward workspace
    tensor = B * H * N * D * 4
    base = 0x100000
    at = lambda i: vp(base + i * 2 * tensor)                  # disjoint, 16-byte aligned
    Q, K, V, O, dO, dQ, dK, dV, den, ws = (at(i) for i in range(10))
    dims = (B, H, N, D, M, f(1e-6), 0)
    fwd, bwd = lib.la_causal_fwd, lib.la_causal_bwd
    assert fwd(Q, K, V, V, null, *dims, null, 0, null) == b.LA_ERR_ALIAS               # O is V
    assert fwd(Q, K, V, vp(Q.value + tensor - 16), null, *dims, null, 0, null) == b.LA_ERR_ALIAS  # O starts inside Q
    big = 1 << 30
    assert bwd(Q, K, V, null, den, null, dO, dQ, dQ, dV, *dims, ws, big, null) == b.LA_ERR_ALIAS  # dK is dQ
    assert bwd(Q, K, V, null, den, null, dO, dQ, dK, dO, *dims, ws, big, null) == b.LA_ERR_ALIAS  # dV is dO
    assert bwd(Q, K, V, null, den, null, dO, dQ, dK, dV, *dims, dV, big, null) == b.LA_ERR_ALIAS  # ws is dV
    step = lib.la_recurrent_step
    q, k, v, S, z, out = (at(i) for i in range(6))
    assert step(q, k, v, S, z, S, B, H, D, M, f(1e-6), 0, null) == b.LA_ERR_ALIAS      # out is the state


def test_schedule_knobs_change_the_workspace(lib, monkeypatch):
    from paper_2006_16236_amd import binding as b
    try:
        monkeypatch.setenv("LA_TARGET_WAVES", "1")
        b.la_tuning_reload()
        assert b.la_causal_fwd_workspace(1, 1, 4096, 64, 64) == 0
        monkeypatch.setenv("LA_TARGET_WAVES", str(1 << 20))
        monkeypatch.setenv("LA_MIN_SEG_CHUNKS", "1")
        # the environment is read once: without a reload the query still answers for the old values
        assert b.la_causal_fwd_workspace(1, 1, 4096, 64, 64) == 0
        b.la_tuning_reload()
        assert b.la_causal_fwd_workspace(1, 1, 4096, 64, 64) == 256 * (64 * 64 + 64) * 4
    finally:
        monkeypatch.undo()
        b.la_tuning_reload()


def test_binding_refuses_host_tensors(lib):
    import torch
    from paper_2006_16236_amd import binding as b
    x = torch.zeros(1, 1, 16, 64)
    with pytest.raises(ValueError):
        b.la_causal_fwd(x, x, x, x)
    with pytest.raises(TypeError):
        b.la_causal_fwd(x.double(), x, x, x)


def test_binding_checks_every_tensor_against_the_sizes(lib):
    """The C ABI cannot see tensor sizes, so the binding must: a tensor of the wrong shape,
    element type or device is refused before any call (host tensors suffice to show it: the
    shape and dtype checks come first)."""
    import torch
    from paper_2006_16236_amd import binding as b
    B, H, N, D, M = 2, 3, 20, 64, 32
    Q, K = torch.zeros(B, H, N, D), torch.zeros(B, H, N, D)
    V, O, dO = torch.zeros(B, H, N, M), torch.zeros(B, H, N, M), torch.zeros(B, H, N, M)
    den = torch.zeros(B, H, N)
    dQ, dK, dV = torch.zeros_like(Q), torch.zeros_like(K), torch.zeros_like(V)

    def refused(fn, *args, match, **kw):
        with pytest.raises(ValueError, match=match):
            fn(*args, **kw)

    refused(b.la_causal_fwd, Q, K[:, :, :-1].contiguous(), V, O, match="K: shape")          # shorter K
    refused(b.la_causal_fwd, Q, K, V[..., :16].contiguous(), O, match="O: shape")           # V, O disagree
    refused(b.la_causal_fwd, Q, K, V, O[:, :1].contiguous(), match="O: shape")
    refused(b.la_causal_fwd, Q, K.bfloat16(), V, O, match="K: dtype")                       # fp32 Q, bf16 K
    refused(b.la_causal_fwd, Q, K, V, O, den.double(), match="den: dtype")                  # fp64 den
    refused(b.la_causal_fwd, Q, K, V, O, den[:, :, :-1].contiguous(), match="den: shape")
    refused(b.la_causal_fwd, Q, K, V.transpose(1, 2).contiguous().transpose(1, 2), O, match="V must be contiguous")
    refused(b.la_causal_fwd_noalloc, Q, K, V[:, :, 1:].contiguous(), O, match="V: shape")
    refused(b.la_global_fwd, Q, K, V, O, den=den.half(), match="den: dtype")
    refused(b.la_causal_bwd, Q, K, V, None, den, dO.bfloat16(), dQ, dK, dV, match="dO: dtype")   # autocast dO
    refused(b.la_causal_bwd, Q, K, V, None, den, dO, dQ, dK[:, :, :4].contiguous(), dV, match="dK: shape")
    refused(b.la_causal_bwd, Q, K, V, None, den, dO, dQ, dK, dQ, match="dV: shape")
    refused(b.la_global_bwd, Q, K, V, O[..., :8].contiguous(), den, dO, dQ, dK, dV, match="O: shape")
    refused(b.la_causal_bwd, Q, K, V, None, den, dO, dQ, dK, dV, fwd_ws=[1, 2], match="fwd_ws")
    # token-major: Q is [B, N, H, D]; den stays [B, H, N]
    Qt, Vt = Q.transpose(1, 2).contiguous(), V.transpose(1, 2).contiguous()
    refused(b.la_causal_fwd_bnhd, Qt, Qt, Vt, Vt.clone(), torch.zeros(B, N, H), match="den: shape")
    refused(b.la_global_fwd_bnhd, Qt, K, Vt, Vt.clone(), match="K: shape")
    # state tensors are fp32 [B,H,D,M] / [B,H,D]
    S, z = torch.zeros(B, H, D, M), torch.zeros(B, H, D)
    refused(b.la_causal_fwd_state, Q, K, V, O, den, S.double(), z, match="S0: dtype")
    refused(b.la_causal_fwd_state, Q, K, V, O, den, S, z, S, z[:, :, :-1].contiguous(), match="z1: shape")
    refused(b.la_causal_bwd_state, Q, K, V, None, den, dO, dQ, dK, dV, dS1=S.transpose(2, 3).contiguous(),
            dz1=z, match="dS1: shape")
    q, k, v, out = torch.zeros(B, H, D), torch.zeros(B, H, D), torch.zeros(B, H, M), torch.zeros(B, H, M)
    refused(b.la_recurrent_step, q, k, v, S.half(), z, out, match="S: dtype")
    refused(b.la_recurrent_step, q, k[:, :-1].contiguous(), v, S, z, out, match="k: shape")
    refused(b.la_recurrent_steps, q[None], k[None], v[None], S, z, out, match="out: shape")
    # everything consistent: the only objection left is that these are host tensors
    refused(b.la_causal_bwd, Q, K, V, None, den, dO, dQ, dK, dV, match="device tensors")
    refused(b.la_recurrent_step, q, k, v, S, z, out, match="device tensors")


def test_header_is_plain_c_and_links_against_the_library(lib, tmp_path):
    """include/la.h compiles as C99 and as C++11 with pedantic warnings as errors, and a plain C
    program that calls the host-only entry points links against the shared library and runs."""
    import subprocess
    from paper_2006_16236_amd import binding as b
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    src = tmp_path / "client.c"
    src.write_text(
        '#include <stdio.h>\n#include "la.h"\n'
        'int main(void) {\n'
        '    size_t ws = la_causal_bwd_workspace(2, 8, 4096, 64, 64, LA_F32);\n'
        '    printf("%d %s %lu\\n", la_version(), la_status_string(LA_ERR_ALIAS), (unsigned long)ws);\n'
        '    return la_causal_fwd(0, 0, 0, 0, 0, 1, 1, 16, 64, 64, 1e-6f, LA_F32, 0, 0, 0) == LA_ERR_NULL ? 0 : 1;\n'
        '}\n')
    for cc, std, lang in (("gcc", "-std=c99", "c"), ("g++", "-std=c++11", "c++")):
        subprocess.run([cc, std, "-Wall", "-Wextra", "-pedantic", "-Werror", "-I", inc, "-fsyntax-only",
                        "-x", lang, str(src)], check=True)
    exe = tmp_path / "client"
    libdir = os.path.dirname(b.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-I", inc, str(src), "-o", str(exe), "-L", libdir, "-l:libla_hip.so",
                    f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(" ", 1)
    assert int(out[0]) == b.la_version() and "overlaps" in out[1]
    assert out[1].rstrip().endswith(str(b.la_causal_bwd_workspace(2, 8, 4096, 64, 64)))
