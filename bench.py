#!/usr/bin/env python3
"""Benchmark of the MoE feed-forward layer (route -> forward -> backward) on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already
resident in HBM: btx_moe_route, btx_moe_ff_forward (saving h1/h3) and
btx_moe_ff_backward (dX, dW_router, db_router, dW1/dW3/dW2, load-balancing gradient).
Prints ONE JSON line: layer tokens/s, the MFMA roofline of the dominant expert-GEMM
kernel (timed live with HIP events recorded inside the library around every stage), and
the CPU oracle timed on a bounded sample of the same batch.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2403_07816_amd import binding as B  # noqa: E402
from paper_2403_07816_amd import synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, vendor figure
WORKLOAD = dict(name="llama2-7b-shaped MoE-FF layer, fwd+bwd, T=16384 (4 seq x 4096), d=4096, f=11008, E=4, top-2, "
                     "bf16, load-balancing loss alpha=0.01",
                T=16384, d=4096, f=11008, E=4, k=2, alpha=0.01)
# FETCH_SIZE / WRITE_SIZE read this fraction of the known traffic of a plain streaming kernel (combine_kernel;
# see profiles/layer_fwd_bwd_c2_pmc_counters.txt): 128-byte reads are counted as 64 bytes on this chip
FETCH_FACTOR, WRITE_FACTOR = 0.5028, 1.000
# routing variants that can be timed; top2 is the benchmark configuration
VARIANTS = {
    "top2": dict(name="top-2", k=2, mode=0, bias=None, tau=1.0, cf=0.0),
    "switch-cf1.5": dict(name="Switch top-1, router bias +2 on expert 0, capacity factor 1.5", k=1, mode=1,
                         bias=[2.0, 0.0, 0.0, 0.0], tau=1.0, cf=1.5),
    "gumbel": dict(name="Gumbel-softmax sample top-1, tau 0.5", k=1, mode=3, bias=None, tau=0.5, cf=0.0),
    # the sublayer inside its block: out = h + FF_MoE(rmsnorm(h)); normalisation folded into the router kernel,
    # residual added in combine, the normalisation's backward (with the residual gradient) as a last stage
    "norm-block": dict(name="top-2 inside its block (RMSNorm in front, residual add)", k=2, mode=0, bias=None, tau=1.0,
                       cf=0.0, block=True),
    # 4 FFs split into 8 chunks each (Sec. 3.3 "Splitting Experts"): 32 experts of width 1376, top-8
    "split8-top8": dict(name="32 split experts of width 1376, top-8", k=8, mode=0, bias=None, tau=1.0, cf=0.0, E=32,
                        f=1376),
    # soft routing (Sec. 3.3): every expert active, gates = softmax; the same path with k = E
    "soft": dict(name="soft routing (top-4 of 4)", k=4, mode=0, bias=None, tau=1.0, cf=0.0),
    # inference: router and forward only, nothing kept for a backward pass
    "forward": dict(name="top-2, forward only", k=2, mode=0, bias=None, tau=1.0, cf=0.0, forward_only=True),
}
GEMM_STAGES = {"up_swiglu": 4, "down": 2, "bwd_act": 2, "bwd_dx": 4, "dw13": 4, "dw2": 2}   # x d*f*R flops


class HipEvents:
    """Raw hipEvent_t handles (the library records them on the stream it launches on)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.ev = (ctypes.c_void_p * n)()
        for i in range(n):
            e = ctypes.c_void_p()
            assert self.hip.hipEventCreate(ctypes.byref(e)) == 0
            self.ev[i] = e.value

    def slice(self, start, count):
        return ctypes.cast(ctypes.byref(self.ev, start * ctypes.sizeof(ctypes.c_void_p)),
                           ctypes.POINTER(ctypes.c_void_p)), count

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), ctypes.c_void_p(self.ev[a]), ctypes.c_void_p(self.ev[b]))
        if rc != 0:                          # a stage that launched nothing never records its events
            self.hip.hipGetLastError()       # do not leave the failed query behind as a sticky error
            return 0.0
        return ms.value


def profiled_traffic(stage):
    """HBM bytes per launch of the GEMM kernel of `stage`, from the committed rocprofv3 PMC
    summary (FETCH_SIZE + WRITE_SIZE in KiB, scaled by the copy-kernel calibration stated
    in that file); None when the summary is missing."""
    path = os.path.join(ROOT, "profiles", "layer_fwd_bwd_c2_pmc_counters.txt")
    if not os.path.exists(path):
        return None
    fetch = write = None
    inside = False
    for line in open(path):
        if not line.startswith(" "):
            inside = line.startswith("mfma_gemm_kernel<") and line.strip().endswith(" " + stage)
        elif inside and "FETCH_SIZE" in line:
            fetch = float(line.split()[1])
        elif inside and "WRITE_SIZE" in line:
            write = float(line.split()[1])
    if fetch is None or write is None:
        return None
    return (fetch / FETCH_FACTOR + write / WRITE_FACTOR) * 1024.0


def sustained_mfma_tflops(data, ms_target=40.0):
    """Register-fed bf16 MFMA rate on `data` (TFLOP/s): what the matrix cores sustain on this
    chip, at the clock it settles to under that load, with operands like the layer's."""
    B.btx_probe_mfma(data, 256, 2000)                      # warm-up, also settles the clock
    torch.cuda.synchronize()
    iters = 4000
    for _ in range(2):                                     # second pass: ~ms_target long
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        flops = B.btx_probe_mfma(data, 256, iters)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        iters = max(1000, int(iters * ms_target / ms))
    return flops / (ms * 1e-3) / 1e12


def hbm_stages(stage_ms, T, d, E, k, s=2, block=False):
    """The streaming stages against the 8 TB/s HBM peak: algorithmic bytes per token (bf16 rows of d*s bytes) and
    the rate they were moved at.  route: x read once + indices, gates, probabilities written; combine: k rows read,
    one written; gather_x_bwd: x and dY each read once per routed slot and written once per slot, transposed;
    router_bwd: x read (dW_router), k rows of dxs read and one row of dX written."""
    per_token = {"route": d * s + k * 8 + E * 4, "combine": d * s * (k + 1), "gather_x_bwd": 2 * d * s * 2 * k,
                 "router_bwd": d * s * (k + 2)}
    if block:   # route also writes the normalised rows; combine also reads the residual; norm_bwd: dXn, h, dY in, dH out
        per_token.update({"route": 2 * d * s + k * 8 + E * 4 + 4, "combine": d * s * (k + 2), "norm_bwd": 4 * d * s})
    return {n: {"bytes_per_token": b, "ms": stage_ms[n], "tb_per_s": b * T / (stage_ms[n] * 1e-3) / 1e12,
                "frac_of_hbm_peak": b * T / (stage_ms[n] * 1e-3) / 8e12}
            for n, b in per_token.items() if stage_ms.get(n, 0) > 0}


def cpu_baseline(L, W, sample_tokens):
    """The oracle, as it stands, on the first `sample_tokens` tokens of the batch."""
    from oracle import btx_oracle as O
    f64 = lambda t: None if t is None else t.detach().float().cpu().numpy().astype(np.float64)
    x, dY = f64(L["x"][:sample_tokens]), f64(L["dY"][:sample_tokens])
    Wr = f64(L["W_router"])
    W1 = [f64(L["W1"][e]) for e in range(W["E"])]
    W3 = [f64(L["W3"][e]) for e in range(W["E"])]
    W2 = [f64(L["W2"][e]) for e in range(W["E"])]
    t0 = time.perf_counter()
    fwd = O.moe_forward(x, Wr, None, W1, W3, W2, W["k"], O.ROUTE_TOPK_RENORM, None, W["alpha"], O.LB_TOKEN_FRAC)
    O.moe_backward(x, Wr, None, W1, W3, W2, W["k"], O.ROUTE_TOPK_RENORM, dY, fwd, W["alpha"], O.LB_TOKEN_FRAC, 1.0)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {sample_tokens} tokens of the same batch, fwd+bwd in fp64 numpy, {dt:.1f} s"}


def library_gemm_context(L, R, d, f, reps=10):
    """Context only: the vendor library's plain GEMMs (torch.matmul) on the shapes of the six expert
    products, all R rows against one expert's weights, no grouping and no fused epilogue.  Not part
    of the measured path and never compared as a target: it shows what a tuned dense GEMM reaches on
    the same box, data and clock."""
    dev = L["x"].device
    xs = L["x"].repeat((R + L["x"].shape[0] - 1) // L["x"].shape[0], 1)[:R].contiguous()
    dys = L["dY"].repeat((R + L["dY"].shape[0] - 1) // L["dY"].shape[0], 1)[:R].contiguous()
    W1, W3, W2 = L["W1"][0], L["W3"][0], L["W2"][0]
    a = torch.randn((R, f), device=dev, dtype=torch.float32).bfloat16()
    cases = {
        "up_swiglu": (4, lambda: (xs @ W1, xs @ W3)),
        "down": (2, lambda: a @ W2),
        "bwd_act": (2, lambda: dys @ W2.t()),
        "bwd_dx": (4, lambda: (a @ W1.t(), a @ W3.t())),
        "dw13": (4, lambda: (xs.t() @ a, xs.t() @ a)),
        "dw2": (2, lambda: a.t() @ dys),
    }
    out = {}
    for name, (c, fn) in cases.items():
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = {"ms": ms, "tflops": c * d * f * R / (ms * 1e-3) / 1e12}
    total = sum(v["ms"] for v in out.values())
    return {"kind": "torch.matmul, dense, one expert's weights, no fused epilogue (context, not a target)",
            "ms": total, "tflops": 18.0 * d * f * R / (total * 1e-3) / 1e12, "per_kernel": out}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tokens", type=int, default=WORKLOAD["T"], help="override T (parity/dev runs only)")
    ap.add_argument("--cpu-sample", type=int, default=8192, help="tokens the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--variant", default="top2", choices=sorted(VARIANTS),
                    help="routing variant; only top2 is the benchmark of record, the others are extra measurements")
    ap.add_argument("--library-gemm", action="store_true",
                    help="also time the vendor library's plain GEMMs on the same shapes (context only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    W = dict(WORKLOAD)
    W["T"] = args.tokens
    V = VARIANTS[args.variant]
    W["k"] = V["k"]
    W["E"], W["f"] = V.get("E", W["E"]), V.get("f", W["f"])
    T, d, f, E, k, alpha = W["T"], W["d"], W["f"], W["E"], W["k"], W["alpha"]
    dev = "cuda:0"
    torch.cuda.set_device(0)
    L = synth.make_layer(T, d, f, E, dtype=torch.bfloat16, device=dev, unit_rms=True, with_dY=True,
                         router_bias=V["bias"], with_gumbel=V["mode"] == B.BTX_ROUTE_GUMBEL_TOP1)
    noise = L["U"] if V["mode"] == B.BTX_ROUTE_GUMBEL_TOP1 else None
    lib = B.load_library()

    # everything a step writes is allocated once, outside the timed region
    routing = B.alloc_routing(T, E, k, dev)
    out = torch.empty_like(L["x"])
    saved = (torch.empty((T * k, f), dtype=torch.bfloat16, device=dev),
             torch.empty((T * k, f), dtype=torch.bfloat16, device=dev))
    grads = B.Grads(torch.empty_like(L["x"]), torch.empty((d, E), dtype=torch.float32, device=dev),
                    torch.empty(E, dtype=torch.float32, device=dev), torch.empty_like(L["W1"]),
                    torch.empty_like(L["W3"]), torch.empty_like(L["W2"]))
    ws_bytes = max(lib.btx_moe_route_workspace_bytes(T, d, E, k),
                   lib.btx_moe_ff_forward_workspace_bytes(T, d, f, E, k, B.BTX_BF16),
                   lib.btx_moe_ff_backward_workspace_bytes(T, d, f, E, k, B.BTX_BF16))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    block = V.get("block", False)
    if block:   # raw rows of varying length, a gain near one; xn, rstd and dH are allocated here, outside the timing
        gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 77)
        h_raw = (L["x"].float() * torch.exp(0.5 * torch.randn((T, 1), generator=gen, device=dev))).to(torch.bfloat16)
        gain = 1.0 + 0.1 * torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
        xn, rstd, dH = torch.empty_like(h_raw), torch.empty(T, dtype=torch.float32, device=dev), torch.empty_like(h_raw)
        dgain = torch.empty(d, dtype=torch.float32, device=dev)
        ws_bytes = max(ws_bytes, lib.btx_rmsnorm_backward_workspace_bytes(T, d))
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def step():
        if block:
            B.btx_moe_norm_route(h_raw, gain, 1e-5, L["W_router"], L["b_router"], noise, k, V["mode"],
                                 B.BTX_LB_TOKEN_FRAC, alpha, out=routing, workspace=ws, xn=xn, rstd=rstd)
            B.btx_moe_ff_forward(xn, L["W1"], L["W3"], L["W2"], routing, save=True, out=out, saved=saved, workspace=ws,
                                 residual=h_raw)
            B.btx_moe_ff_backward(L["dY"], xn, L["W_router"], L["W1"], L["W3"], L["W2"], routing, saved[0], saved[1],
                                  V["mode"], B.BTX_LB_TOKEN_FRAC, alpha, 1.0, 0, out=grads, workspace=ws)
            B.btx_rmsnorm_backward(grads.dX, h_raw, gain, rstd, dres=L["dY"], dH=dH, workspace=ws, dgain=dgain)
            return
        B.btx_moe_route(L["x"], L["W_router"], L["b_router"], noise, k, V["mode"], B.BTX_LB_TOKEN_FRAC, alpha,
                        out=routing, workspace=ws, tau=V["tau"], capacity_factor=V["cf"])
        if V.get("forward_only"):
            B.btx_moe_ff_forward(L["x"], L["W1"], L["W3"], L["W2"], routing, save=False, out=out, workspace=ws)
            return
        B.btx_moe_ff_forward(L["x"], L["W1"], L["W3"], L["W2"], routing, save=True, out=out, saved=saved, workspace=ws)
        B.btx_moe_ff_backward(L["dY"], L["x"], L["W_router"], L["W1"], L["W3"], L["W2"], routing, saved[0], saved[1],
                              V["mode"], B.BTX_LB_TOKEN_FRAC, alpha, 1.0, 0, out=grads, workspace=ws, noise=noise,
                              tau=V["tau"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    n_stage = len(B.STAGE_NAMES)
    events = HipEvents(2 * n_stage * args.steps)
    step_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for s in range(args.steps):
        ptr, n = events.slice(2 * n_stage * s, n_stage)
        lib.btx_profile_stages(ptr, n)
        step_ev[s][0].record()
        step()
        step_ev[s][1].record()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    lib.btx_profile_stages(None, 0)
    step_ms = sorted(a.elapsed_time(b) for a, b in step_ev)

    stage_ms = {}
    for i, name in enumerate(B.STAGE_NAMES):
        v = [events.elapsed_ms(2 * n_stage * s + 2 * i, 2 * n_stage * s + 2 * i + 1) for s in range(args.steps)]
        stage_ms[name] = float(np.mean(v))
    R = int(routing.offsets[-1].item())     # grouped rows the expert GEMMs worked on (T*k unless pairs were dropped)
    gemm = {n: {"ms": stage_ms[n], "tflops": c * d * f * R / (stage_ms[n] * 1e-3) / 1e12}
            for n, c in GEMM_STAGES.items() if stage_ms[n] > 0}
    gemm_coef = float(sum(GEMM_STAGES[n] for n in gemm))    # 18 for forward + backward
    dominant = max(gemm, key=lambda n: gemm[n]["ms"])
    gemm_ms = sum(v["ms"] for v in gemm.values())
    gemm_tflops = gemm_coef * d * f * R / (gemm_ms * 1e-3) / 1e12

    ms_per_step = elapsed / args.steps * 1e3
    sustained = sustained_mfma_tflops(L["x"])
    result = {
        "metric": "MoE-FF layer tokens/s fwd+bwd (d4096,f11008,E4,top2)" if not V.get("forward_only")
                  else "MoE-FF layer tokens/s forward only (d4096,f11008,E4,top2)",
        "value": T * args.steps / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": (W["name"] if args.variant == "top2" else
                                W["name"].replace("top-2", V["name"]).replace("f=11008, E=4, ", "" if "E" in V else "f=11008, E=4, ")
                                .replace("fwd+bwd, " if V.get("forward_only") else "\0", ""))
                   if T == WORKLOAD["T"] else f"dev run, T={T}, {V['name']}", "tokens": T, "routed_rows": R, "d_model": d,
                   "d_ff": f, "experts": E, "top_k": k},
        "roofline": {"bound": "mfma", "kernel": f"mfma_gemm_kernel ({dominant})", "achieved": gemm[dominant]["tflops"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": gemm[dominant]["tflops"] / PEAK_BF16_TFLOPS,
                     "traffic": profiled_traffic(dominant) if T == WORKLOAD["T"] and args.variant == "top2" else None,
                     "algorithmic_flops": GEMM_STAGES[dominant] * d * f * R,
                     # register-fed MFMA loop on the same x: the ceiling at the clock the chip sustains
                     "sustained_mfma_peak": sustained, "frac_of_sustained": gemm[dominant]["tflops"] / sustained},
        "expert_gemms": {"ms": gemm_ms, "tflops": gemm_tflops, "frac_of_peak": gemm_tflops / PEAK_BF16_TFLOPS,
                         "frac_of_sustained": gemm_tflops / sustained,
                         "layer_frac_of_peak": gemm_coef * d * f * R / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                         "per_kernel": gemm},
        "stage_ms": stage_ms,
        "step_ms": {"median": step_ms[len(step_ms) // 2], "min": step_ms[0], "max": step_ms[-1]},
        "hbm_stages": hbm_stages(stage_ms, T, d, E, k, block=block),
    }
    if args.cpu_sample > 0 and args.variant == "top2":   # the oracle is timed on the benchmark configuration only
        result["cpu_baseline"] = cpu_baseline(L, W, min(args.cpu_sample, T))
    if args.library_gemm:
        result["library_gemm"] = library_gemm_context(L, R, d, f)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
