"""The entry point for callers that cannot allocate: btx_moe_route_noalloc, called through the raw
C ABI, against btx_moe_route on the same inputs.  Two calls in a row, the second with a smaller
input: the fixed workspace still holds the first call's contents then."""
import ctypes

import pytest
import torch

from paper_2403_07816_amd import binding as B
from paper_2403_07816_amd import synth

pytestmark = pytest.mark.gpu

NAMES = ("topk_idx", "gates", "probs", "counts", "offsets", "perm", "inv_pos", "gate_sum", "prob_sum", "lb_loss")


def ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def route_both(lib, x, Wr, b, U, k, mode, alpha, tau, cf, check_free=False):
    T, d = x.shape
    E = Wr.shape[1]
    dt = B.BTX_BF16 if x.dtype == torch.bfloat16 else B.BTX_F32
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ws_bytes = lib.btx_moe_route_workspace_bytes(T, d, E, k)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    want, got = B.alloc_routing(T, E, k, "cuda"), B.alloc_routing(T, E, k, "cuda")
    for r in (want, got):                       # an output the call fails to write must show
        for n in NAMES:
            getattr(r, n).fill_(-7)
    outs = lambda r: [ptr(getattr(r, n)) for n in NAMES]
    st = lib.btx_moe_route(ptr(x), dt, ptr(Wr), ptr(b), ptr(U), T, d, E, k, mode, B.BTX_LB_TOKEN_FRAC, alpha, tau, cf,
                           *outs(want), ptr(ws), ws_bytes, stream)
    assert st == 0
    torch.cuda.synchronize()
    before, free_before = torch.cuda.memory_allocated(), torch.cuda.mem_get_info()[0]
    st = lib.btx_moe_route_noalloc(ptr(x), dt, ptr(Wr), ptr(b), ptr(U), T, d, E, k, mode, B.BTX_LB_TOKEN_FRAC, alpha, tau,
                                   cf, *outs(got), stream)
    assert st == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    if check_free:       # from the second call on nothing is loaded lazily any more: the device's free memory stays put
        assert torch.cuda.mem_get_info()[0] == free_before
    for n in NAMES:
        assert torch.equal(getattr(got, n), getattr(want, n)), n


def test_route_noalloc_matches_route_on_two_calls_in_a_row():
    lib = B.load_library()
    assert lib.btx_moe_route_noalloc_max_workspace_bytes() == 4 << 20
    big = synth.make_layer(3000, 512, 64, 1, dtype=torch.bfloat16, unit_rms=True, router_E=32)
    x, Wr = big["x"].cuda(), big["W_router"].cuda()
    route_both(lib, x, Wr, None, None, 8, B.BTX_ROUTE_TOPK_RENORM, 0.01, 1.0, 0.0)
    # second call, smaller in every dimension, other routing mode, with a capacity limit and a bias
    small = synth.make_layer(333, 128, 64, 1, dtype=torch.float32, router_E=5, router_bias=[2.0, 0, 0, 0, -1.0],
                             with_U=True)
    route_both(lib, small["x"].cuda(), small["W_router"].cuda(), small["b_router"].cuda(), small["U"].cuda(), 1,
               B.BTX_ROUTE_SAMPLE_TOP1, 0.01, 1.0, 1.25, check_free=True)
    # and the first problem once more
    route_both(lib, x, Wr, None, None, 8, B.BTX_ROUTE_TOPK_RENORM, 0.01, 1.0, 0.0, check_free=True)


def test_route_noalloc_refuses_what_does_not_fit():
    lib = B.load_library()
    p = ctypes.c_void_p(256)
    T, d, E, k = 1 << 20, 4096, 64, 2
    assert lib.btx_moe_route_workspace_bytes(T, d, E, k) > lib.btx_moe_route_noalloc_max_workspace_bytes()
    st = lib.btx_moe_route_noalloc(p, B.BTX_BF16, p, None, None, T, d, E, k, 0, 0, 0.0, 1.0, 0.0, p, p, p, p, p, p, p, p,
                                   p, p, None)
    assert st == 3     # BTX_ERR_WORKSPACE, nothing launched
    # the same argument checks as btx_moe_route for what does fit
    assert lib.btx_moe_route_noalloc(p, B.BTX_BF16, p, None, None, 64, 64, 4, 5, 0, 0, 0.0, 1.0, 0.0, p, p, p, p, p, p,
                                     p, p, p, p, None) == 1
    assert lib.btx_moe_route_noalloc(p, B.BTX_BF16, p, None, None, 0, 64, 4, 2, 0, 0, 0.0, 1.0, 0.0, p, p, p, p, p, p,
                                     p, p, p, p, None) == 0
