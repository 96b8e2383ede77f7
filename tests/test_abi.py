"""Host-side checks that need no GPU: the shared library loads, exports every
function the header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2403_07816_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2403_07816_amd.build import build
        build(verbose=False)
    return B.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "btx_moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(btx_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = declared_functions()
    for required in ("btx_moe_route", "btx_moe_ff_forward", "btx_moe_ff_backward", "btx_merge_average"):
        assert required in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} is declared in btx_moe.h but not exported"
    assert lib.btx_version() >= 1
    assert lib.btx_status_string(0) == b"ok"


def test_binding_covers_every_declared_symbol():
    assert sorted(B._SIGNATURES) == declared_functions()


def test_route_rejects_bad_arguments(lib):
    p = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    null = None

    def route(T=8, d=64, E=4, k=2, mode=0, lb=0, U=null, x=p, ws_bytes=1 << 20, dtype=0, tau=1.0, cf=0.0):
        return lib.btx_moe_route(x, dtype, p, null, U, T, d, E, k, mode, lb, 0.0, tau, cf, p, p, p, p, p, p, p, p, p, p, p,
                                 ws_bytes, null)

    assert route(k=5) == 1                 # k > E
    assert route(k=0) == 1
    assert route(E=65, k=1) == 1           # more experts than a wavefront has lanes
    assert route(d=60) == 1                # d not a multiple of 8
    assert route(mode=4) == 1
    assert route(mode=3, k=1) == 1         # Gumbel sampling needs its noise
    assert route(mode=3, k=1, U=p, tau=0.0) == 1   # and a positive temperature
    assert route(mode=1, k=2) == 1         # Switch needs k = 1
    assert route(mode=2, k=1) == 1         # sampling needs U
    assert route(mode=0, U=p) == 1         # U only with sampling
    assert route(lb=2) == 1
    assert route(cf=-0.5) == 1             # capacity factor: 0 (none) or positive
    assert route(dtype=7) == 1
    assert route(x=null) == 1
    assert route(x=ctypes.c_void_p(264)) == 1      # rows move as 16-byte pieces: 16-byte aligned tensors
    assert route(ws_bytes=16) == 3         # workspace too small
    assert route(T=0) == 0                 # empty batch: nothing to do
    assert route(T=-1) == 1


def test_forward_backward_and_merge_reject_bad_arguments(lib):
    p = ctypes.c_void_p(256)
    null = None

    def fwd(T=8, d=64, f=64, E=4, k=2, s13=64 * 64, s2=64 * 64, h1=p, h3=p, ws=1 << 30, out=p, x=p, W2=p):
        return lib.btx_moe_ff_forward(x, p, p, W2, 0, s13, s2, T, d, f, E, k, p, p, p, p, null, out, h1, h3, p, ws, null)

    assert fwd(f=12) == 1
    assert fwd(s13=10) == 1                # expert stride smaller than one expert
    assert fwd(s13=64 * 64 + 4) == 1       # ... or one that puts an expert off the 16-byte grid
    assert fwd(s2=64 * 64 + 8, ws=0) == 3  # a padded stride on the grid is fine (the call gets as far as the workspace)
    assert fwd(x=ctypes.c_void_p(264)) == 1 and fwd(W2=ctypes.c_void_p(258)) == 1 and fwd(out=ctypes.c_void_p(8)) == 1
    assert fwd(h3=null) == 1               # h1/h3 come as a pair
    assert fwd(out=null) == 1
    assert fwd(ws=0) == 3
    assert fwd(T=0) == 0

    def bwd(T=8, k=2, mode=0, lb=0, flags=0, dW=(p, p, p), dwt=0, dt=0, ws=1 << 30, noise=null, tau=1.0):
        return lib.btx_moe_ff_backward(p, p, p, p, p, p, dt, 64 * 64, 64 * 64, T, 64, 64, 4, k, mode, lb, 0.0, 0.0,
                                       flags, noise, tau, p, p, p, p, p, p, p, p, p, p, p, p, p, null, dW[0], dW[1],
                                       dW[2], dwt,
                                       p, ws, null)

    assert bwd(dW=(p, null, p)) == 1       # weight gradients: all three or none
    assert bwd(dW=(p, p, ctypes.c_void_p(264))) == 1   # misaligned
    assert bwd(flags=1, lb=0) == 1         # gradient through u only in gate-mean mode
    assert bwd(flags=8) == 1
    assert bwd(dt=0, dwt=1) == 1           # fp32 layer cannot return bf16 weight gradients
    assert bwd(mode=1, k=2) == 1
    assert bwd(mode=3, k=1) == 1           # Gumbel backward needs the noise again
    assert bwd(mode=0, noise=p) == 1       # and no other mode takes it
    assert bwd(mode=3, k=1, noise=p, tau=-1.0) == 1
    assert bwd(ws=0) == 3
    assert bwd(T=0) == 0

    arr = (ctypes.c_void_p * 2)(256, 512)
    assert lib.btx_merge_average(arr, 0, p, 16, 0, null) == 1
    assert lib.btx_merge_average(arr, 17, p, 16, 0, null) == 1
    assert lib.btx_merge_average(arr, 2, ctypes.c_void_p(257), 16, 0, null) == 1   # misaligned
    assert lib.btx_merge_average(arr, 2, p, 0, 0, null) == 0
    assert lib.btx_merge_average(arr, 2, p, -1, 0, null) == 1

    wts = (ctypes.c_float * 2)(0.5, 0.5)
    assert lib.btx_merge_weighted(arr, wts, 0, p, 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, wts, 17, p, 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, None, 2, p, 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, (ctypes.c_float * 2)(0.5, float("nan")), 2, p, 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, (ctypes.c_float * 2)(0.5, float("inf")), 2, p, 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, wts, 2, ctypes.c_void_p(257), 16, 0, null) == 1
    assert lib.btx_merge_weighted(arr, wts, 2, p, 0, 0, null) == 0
    assert lib.btx_merge_weighted(arr, wts, 2, p, -1, 0, null) == 1


def test_norm_route_and_norm_backward_reject_bad_arguments(lib):
    p, null = ctypes.c_void_p(256), ctypes.c_void_p(0)
    q = ctypes.c_void_p(512)

    def nr(h=p, gain=p, eps=1e-5, xn=q, rstd=p, T=4, d=64, E=4, k=2, ws=1 << 20):
        return lib.btx_moe_norm_route(h, 0, gain, eps, xn, rstd, p, null, null, T, d, E, k, 0, 0, 0.0, 1.0, 0.0,
                                      p, p, p, p, p, p, p, p, p, p, p, ws, null)
    assert nr(gain=null) == 1
    assert nr(xn=null) == 1
    assert nr(rstd=null) == 1
    assert nr(xn=p) == 1                    # xn must not alias h
    assert nr(eps=-1.0) == 1
    assert nr(d=60) == 1
    assert nr(k=5) == 1
    assert nr(ws=0) == 3
    assert nr(T=0) == 0

    def nb(dxn=p, h=p, gain=p, rstd=p, dres=null, dt=0, T=4, d=64, dH=q, dgain=p, ws=1 << 20):
        return lib.btx_rmsnorm_backward(dxn, h, gain, rstd, dres, dt, T, d, dH, dgain, p, ws, null)
    assert nb(dxn=null) == 1
    assert nb(gain=null) == 1
    assert nb(rstd=null) == 1
    assert nb(dH=null) == 1
    assert nb(dgain=null) == 1
    assert nb(dt=7) == 1
    assert nb(d=60) == 1
    assert nb(d=16392) == 1
    assert nb(ws=0) == 3
    assert nb(T=0) == 0
    assert lib.btx_rmsnorm_backward_workspace_bytes(16384, 4096) == 1024 * 4096 * 4
    assert lib.btx_rmsnorm_backward_workspace_bytes(0, 4096) == 0


def test_mix_experts_rejects_bad_arguments(lib):
    bad = 1
    a, b, c, x, y, z = (ctypes.c_void_p(0x1000 * i) for i in range(1, 7))
    ok_tail = (x, y, z, None)
    assert lib.btx_mix_experts(a, b, c, 1, 4, 64, 96, 0, 5, *ok_tail) == bad      # 96 % 5 != 0
    assert lib.btx_mix_experts(a, b, c, 1, 4, 64, 96, 2, 3, *ok_tail) == bad      # unknown mode
    assert lib.btx_mix_experts(a, b, c, 1, 5, 64, 96, 1, 0, *ok_tail) == bad      # blend: 96 % 5 != 0
    assert lib.btx_mix_experts(a, b, c, 1, 4, 64, 96, 0, 32, *ok_tail) == bad     # 128 experts
    assert lib.btx_mix_experts(a, b, c, 1, 4, 64, 96, 0, 3, a, y, z, None) == bad  # output aliases input
    assert lib.btx_mix_experts(None, b, c, 1, 4, 64, 96, 0, 3, *ok_tail) == bad
    assert lib.btx_mix_experts(a, b, c, 7, 4, 64, 96, 0, 3, *ok_tail) == bad      # dtype


def test_adamw_rejects_bad_arguments(lib):
    bad = 1
    a, b, c, g = (ctypes.c_void_p(0x1000 * i) for i in range(1, 5))

    def step(master=a, grad=g, n=64, t=1, b1=0.9, b2=0.95, eps=1e-8, gdt=1, lowp=None):
        return lib.btx_adamw_step(master, b, c, grad, gdt, lowp, n, t, 1e-4, b1, b2, eps, 0.1, None)

    assert step(t=0) == bad
    assert step(b1=1.0) == bad
    assert step(b2=-0.1) == bad
    assert step(eps=-1.0) == bad
    assert step(master=None) == bad
    assert step(grad=ctypes.c_void_p(0x4008)) == bad      # misaligned
    assert step(lowp=ctypes.c_void_p(0x5004)) == bad
    assert step(gdt=5) == bad
    assert step(n=-1) == bad
    assert step(n=0) == 0


def test_shapes_beyond_the_kernels_limits_are_refused_before_any_launch(lib):
    p, null = ctypes.c_void_p(256), None

    def fwd(T, d, f, E, k, dt):
        return lib.btx_moe_ff_forward(p, p, p, p, dt, d * f, d * f, T, d, f, E, k, p, p, p, p, null, p, p, p, p,
                                      1 << 62, null)
    unsupported = 2
    assert fwd(8_400_000, 64, 64, 4, 1, 1) == unsupported     # bf16 MFMA path: padded rows * 512 bytes overflow 32 bits
    assert fwd(4_200_000, 64, 64, 4, 1, 0) == unsupported     # plain path: more row tiles than the grid's y dimension
    assert fwd(4_200_000, 64, 72, 4, 1, 1) == unsupported     # bf16 with an f the MFMA kernels do not take


def test_missing_library_raises(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libbtx_moe.so")
    with pytest.raises(RuntimeError):
        B.load_library()
