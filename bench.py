#!/usr/bin/env python3
"""Benchmark of the MoE feed-forward layer (route -> forward -> backward) on one MI355X.

A step is one pass of the whole hot path over one synthetic batch that is already
resident in HBM: btx_moe_route, btx_moe_ff_forward (saving h1/h3) and
btx_moe_ff_backward (dX, dW_router, db_router, dW1/dW3/dW2, load-balancing gradient).
Prints ONE JSON line: layer tokens/s of the benchmark configuration (T=16384, d=4096,
f=11008, E=4, top-2, bf16), the MFMA roofline of the dominant expert-GEMM kernel (timed
live with HIP events recorded inside the library around every stage), and the CPU oracle
timed on a bounded sample of the same batch.  Before anything is timed, the step's
outputs are compared with the oracle on a few tokens and two runs are compared byte for
byte.  Under "configs" the same measurements for the other named configurations
(forward at T=4096; Switch and sample top-1 with an overloaded expert; 32 split experts,
top-8) and the parameter averaging at the 7B non-FF parameter set.
"""
from __future__ import annotations

import argparse
import ctypes
import hashlib
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
PEAK_HBM_TBS = 8.0          # MI355X HBM3E, vendor figure
D_MODEL, D_FF = 4096, 11008
ALPHA = 0.01
# the named configurations; "top2" is the benchmark of record, the others are reported under "configs"
VARIANTS = {
    "top2": dict(name="top-2", T=16384, E=4, f=D_FF, k=2, mode=B.BTX_ROUTE_TOPK_RENORM),
    "c1-forward": dict(name="top-2, forward only, one 4096-token sequence", T=4096, E=4, f=D_FF, k=2,
                       mode=B.BTX_ROUTE_TOPK_RENORM, forward_only=True),
    "c3a-switch": dict(name="Switch top-1 (dropless), router bias +2 on expert 0", T=16384, E=4, f=D_FF, k=1,
                       mode=B.BTX_ROUTE_SWITCH_TOP1, bias=[2.0, 0.0, 0.0, 0.0]),
    "c3b-sample": dict(name="sample top-1 by inverse CDF of a supplied uniform, router bias +2 on expert 0", T=16384,
                       E=4, f=D_FF, k=1, mode=B.BTX_ROUTE_SAMPLE_TOP1, bias=[2.0, 0.0, 0.0, 0.0]),
    # 4 FFs split into 8 chunks each (Sec. 3.3 "Splitting Experts"): 32 experts of width 1376, top-8
    "c4-split8-top8": dict(name="32 split experts of width 1376, top-8", T=16384, E=32, f=1376, k=8,
                           mode=B.BTX_ROUTE_TOPK_RENORM, split=8),
    # further measurements, only on request (--variant)
    "switch-cf1.5": dict(name="Switch top-1, router bias +2 on expert 0, capacity factor 1.5", T=16384, E=4, f=D_FF,
                         k=1, mode=B.BTX_ROUTE_SWITCH_TOP1, bias=[2.0, 0.0, 0.0, 0.0], cf=1.5),
    "gumbel": dict(name="Gumbel-softmax sample top-1, tau 0.5", T=16384, E=4, f=D_FF, k=1,
                   mode=B.BTX_ROUTE_GUMBEL_TOP1, tau=0.5),
    "soft": dict(name="soft routing (top-4 of 4)", T=16384, E=4, f=D_FF, k=4, mode=B.BTX_ROUTE_TOPK_RENORM),
    "forward": dict(name="top-2, forward only", T=16384, E=4, f=D_FF, k=2, mode=B.BTX_ROUTE_TOPK_RENORM,
                    forward_only=True),
    # the sublayer inside its block: out = h + FF_MoE(rmsnorm(h)); normalisation folded into the router kernel,
    # residual added in combine, the normalisation's backward (with the residual gradient) as a last stage
    "norm-block": dict(name="top-2 inside its block (RMSNorm in front, residual add)", T=16384, E=4, f=D_FF, k=2,
                       mode=B.BTX_ROUTE_TOPK_RENORM, block=True),
}
REPORTED = ["c1-forward", "c3a-switch", "c3b-sample", "c4-split8-top8"]
GEMM_STAGES = {"up_swiglu": 4, "down": 2, "bwd_act": 2, "bwd_dx": 4, "dw13": 4, "dw2": 2}   # x d*f*R flops
PMC_PROFILE = os.path.join(ROOT, "profiles", "layer_fwd_bwd_c2_pmc_counters.txt")
GEMM_SOURCE = os.path.join(ROOT, "paper_2403_07816_amd", "csrc", "gemm_mfma.hip")


def describe(V, T):
    passes = "forward only" if V.get("forward_only") else "fwd+bwd"
    return (f"llama2-7b-shaped MoE-FF layer, {passes}, T={T}, d={D_MODEL}, f={V['f']}, E={V['E']}, {V['name']}, bf16, "
            f"load-balancing loss alpha={ALPHA}")


def metric_name(V):
    passes = "forward only" if V.get("forward_only") else "fwd+bwd"
    return f"MoE-FF layer tokens/s {passes} (d{D_MODEL},f{V['f']},E{V['E']},top{V['k']})"


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

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(ctypes.c_void_p(e))


def source_digest():
    return hashlib.sha256(open(GEMM_SOURCE, "rb").read()).hexdigest()[:16]


def profiled_traffic(stage):
    """HBM bytes per launch of the GEMM kernel of `stage`, taken from the committed rocprofv3 counter
    summary (two --pmc runs: FETCH_SIZE, then WRITE_SIZE, KiB per dispatch, each divided by what the same
    counter reads per KiB moved by a plain streaming kernel of known size in the same run; the factors are
    stated in that file).  It is a profile of an earlier run of this same kernel, not of this run: the
    summary names the digest of the kernel source it was taken with, and when that no longer matches the
    source in the tree the figure is withheld (None)."""
    if not os.path.exists(PMC_PROFILE):
        return None, "no committed counter summary"
    fetch = write = digest = None
    factors = {}
    inside = False
    for line in open(PMC_PROFILE):
        if line.startswith("# gemm_mfma.hip sha256/16:"):
            digest = line.split(":")[1].strip()
        elif line.startswith("# calibration:"):
            for tok in line.split():
                if "=" in tok:
                    kname, v = tok.split("=")
                    factors[kname] = float(v)
        elif not line.startswith(" "):
            inside = line.startswith("mfma_gemm_kernel<") and line.strip().endswith(" " + stage)
        elif inside and "FETCH_SIZE" in line:
            fetch = float(line.split()[1])
        elif inside and "WRITE_SIZE" in line:
            write = float(line.split()[1])
    src = os.path.relpath(PMC_PROFILE, ROOT)
    if digest != source_digest():
        return None, f"{src} was taken with another version of the kernel source"
    if fetch is None or write is None or "FETCH_SIZE" not in factors or "WRITE_SIZE" not in factors:
        return None, f"{src} has no counters for {stage}"
    return (fetch / factors["FETCH_SIZE"] + write / factors["WRITE_SIZE"]) * 1024.0, src


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
                "frac_of_hbm_peak": b * T / (stage_ms[n] * 1e-3) / (PEAK_HBM_TBS * 1e12)}
            for n, b in per_token.items() if stage_ms.get(n, 0) > 0}


def host_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def f64(t):
    return None if t is None else t.detach().float().cpu().numpy().astype(np.float64)


_W64 = {}


def experts_f64(W):
    """Per-expert float64 host copies of a stacked weight tensor, made once per tensor."""
    key = (W.data_ptr(), tuple(W.shape))
    if key not in _W64:
        _W64[key] = [f64(W[e]) for e in range(W.shape[0])]
    return _W64[key]


def cpu_baseline(L, V, sample_tokens):
    """The oracle, as it stands, on the first `sample_tokens` tokens of the batch."""
    from oracle import btx_oracle as O
    x, dY = f64(L["x"][:sample_tokens]), f64(L["dY"][:sample_tokens])
    Wr = f64(L["W_router"])
    W1, W3, W2 = experts_f64(L["W1"]), experts_f64(L["W3"]), experts_f64(L["W2"])
    t0 = time.perf_counter()
    fwd = O.moe_forward(x, Wr, None, W1, W3, W2, V["k"], O.ROUTE_TOPK_RENORM, None, ALPHA, O.LB_TOKEN_FRAC)
    O.moe_backward(x, Wr, None, W1, W3, W2, V["k"], O.ROUTE_TOPK_RENORM, dY, fwd, ALPHA, O.LB_TOKEN_FRAC, 1.0)
    dt = time.perf_counter() - t0
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": host_threads(), "kind": "oracle",
            "sample": f"first {sample_tokens} tokens of the same batch, fwd+bwd in fp64 numpy, {dt:.1f} s"}


class Layer:
    """One configuration: its tensors, everything a step writes (allocated once, outside any timed
    region) and the step itself."""

    def __init__(self, V, T, dev, shared=None):
        self.V, self.T, self.dev = V, T, dev
        d, f, E, k = D_MODEL, V["f"], V["E"], V["k"]
        self.d, self.f, self.E, self.k = d, f, E, k
        split = V.get("split", 1)
        if shared is not None and shared.T >= T and shared.V.get("split", 1) == 1 and shared.V["E"] == E // split and \
                shared.V["f"] == f * split:
            # the same seed-shaped experts, rows and gradient as the benchmark configuration
            src = shared.L
            L = {n: src[n] for n in ("W1", "W3", "W2")}
            L["x"], L["dY"] = src["x"][:T].contiguous(), src["dY"][:T].contiguous()
            extra = synth.make_layer(T, d, 8, 1, device=dev, router_E=E, router_bias=V.get("bias"),
                                     with_U=V["mode"] == B.BTX_ROUTE_SAMPLE_TOP1,
                                     with_gumbel=V["mode"] == B.BTX_ROUTE_GUMBEL_TOP1)
            L["W_router"], L["b_router"], L["U"] = extra["W_router"], extra["b_router"], extra["U"]
        else:
            L = synth.make_layer(T, d, f * split, E // split, dtype=torch.bfloat16, device=dev, unit_rms=True,
                                 with_dY=True, router_E=E, router_bias=V.get("bias"),
                                 with_U=V["mode"] == B.BTX_ROUTE_SAMPLE_TOP1,
                                 with_gumbel=V["mode"] == B.BTX_ROUTE_GUMBEL_TOP1)
        if split > 1:
            L = dict(L)
            L["W1"], L["W3"], L["W2"] = B.split_experts(L["W1"], L["W3"], L["W2"], split)
        self.L = L
        self.noise = L["U"] if V["mode"] == B.BTX_ROUTE_GUMBEL_TOP1 else None
        lib = B.load_library()
        self.routing = B.alloc_routing(T, E, k, dev)
        self.out = torch.empty_like(L["x"])
        self.fwd_only = bool(V.get("forward_only"))
        self.block = bool(V.get("block"))
        ws_bytes = max(lib.btx_moe_route_workspace_bytes(T, d, E, k),
                       lib.btx_moe_ff_forward_workspace_bytes(T, d, f, E, k, B.BTX_BF16),
                       lib.btx_moe_ff_backward_workspace_bytes(T, d, f, E, k, B.BTX_BF16),
                       lib.btx_rmsnorm_backward_workspace_bytes(T, d) if self.block else 0)
        self.ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
        self.saved = self.grads = None
        if not self.fwd_only:
            self.saved = (torch.empty((T * k, f), dtype=torch.bfloat16, device=dev),
                          torch.empty((T * k, f), dtype=torch.bfloat16, device=dev))
            self.grads = B.Grads(torch.empty_like(L["x"]), torch.empty((d, E), dtype=torch.float32, device=dev),
                                 torch.empty(E, dtype=torch.float32, device=dev), torch.empty_like(L["W1"]),
                                 torch.empty_like(L["W3"]), torch.empty_like(L["W2"]))
        if self.block:   # raw rows of varying length, a gain near one
            gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 77)
            self.h_raw = (L["x"].float() * torch.exp(0.5 * torch.randn((T, 1), generator=gen, device=dev))).to(torch.bfloat16)
            self.gain = 1.0 + 0.1 * torch.randn(d, generator=gen, device=dev, dtype=torch.float32)
            self.xn, self.rstd = torch.empty_like(self.h_raw), torch.empty(T, dtype=torch.float32, device=dev)
            self.dH, self.dgain = torch.empty_like(self.h_raw), torch.empty(d, dtype=torch.float32, device=dev)

    def step(self):
        L, V, k = self.L, self.V, self.k
        tau, cf = V.get("tau", 1.0), V.get("cf", 0.0)
        if self.block:
            B.btx_moe_norm_route(self.h_raw, self.gain, 1e-5, L["W_router"], L["b_router"], self.noise, k, V["mode"],
                                 B.BTX_LB_TOKEN_FRAC, ALPHA, out=self.routing, workspace=self.ws, xn=self.xn, rstd=self.rstd)
            B.btx_moe_ff_forward(self.xn, L["W1"], L["W3"], L["W2"], self.routing, save=True, out=self.out,
                                 saved=self.saved, workspace=self.ws, residual=self.h_raw)
            B.btx_moe_ff_backward(L["dY"], self.xn, L["W_router"], L["W1"], L["W3"], L["W2"], self.routing, self.saved[0],
                                  self.saved[1], V["mode"], B.BTX_LB_TOKEN_FRAC, ALPHA, 1.0, 0, out=self.grads,
                                  workspace=self.ws)
            B.btx_rmsnorm_backward(self.grads.dX, self.h_raw, self.gain, self.rstd, dres=L["dY"], dH=self.dH,
                                   workspace=self.ws, dgain=self.dgain)
            return
        U = L["U"] if V["mode"] in (B.BTX_ROUTE_SAMPLE_TOP1, B.BTX_ROUTE_GUMBEL_TOP1) else None
        B.btx_moe_route(L["x"], L["W_router"], L["b_router"], U, k, V["mode"], B.BTX_LB_TOKEN_FRAC, ALPHA,
                        out=self.routing, workspace=self.ws, tau=tau, capacity_factor=cf)
        if self.fwd_only:
            B.btx_moe_ff_forward(L["x"], L["W1"], L["W3"], L["W2"], self.routing, save=False, out=self.out, workspace=self.ws)
            return
        B.btx_moe_ff_forward(L["x"], L["W1"], L["W3"], L["W2"], self.routing, save=True, out=self.out, saved=self.saved,
                             workspace=self.ws)
        B.btx_moe_ff_backward(L["dY"], L["x"], L["W_router"], L["W1"], L["W3"], L["W2"], self.routing, self.saved[0],
                              self.saved[1], V["mode"], B.BTX_LB_TOKEN_FRAC, ALPHA, 1.0, 0, out=self.grads,
                              workspace=self.ws, noise=self.noise, tau=tau)

    def outputs(self):
        """Everything a step returns."""
        r = self.routing
        res = [self.out, r.topk_idx, r.gates, r.probs, r.counts, r.offsets, r.perm, r.inv_pos, r.gate_sum, r.prob_sum,
               r.lb_loss]
        if self.grads is not None:
            g = self.grads
            res += [g.dX, g.dW_router, g.db_router, g.dW1, g.dW3, g.dW2]
        return res

    def deterministic(self):
        """Two steps, every returned tensor compared byte for byte (no kernel uses atomics)."""
        self.step()
        first = [t.clone() for t in self.outputs()]
        for t in self.outputs():
            t.zero_()
        self.step()
        torch.cuda.synchronize()
        return all(torch.equal(a, b) for a, b in zip(first, self.outputs()))

    def parity(self, n_tokens=12, tol=2e-2):
        """The step's out and dX rows of a few tokens against the oracle (which is forced onto the
        step's routing of those tokens and given the whole batch's load-balancing statistics)."""
        from oracle import btx_oracle as O
        V, k, T = self.V, self.k, self.T
        if self.block:
            return None
        self.step()
        torch.cuda.synchronize()
        L, r = self.L, self.routing
        rng = np.random.default_rng(7)
        toks = np.unique(np.concatenate([[0, T - 1], rng.integers(0, T, n_tokens)]))
        tt = torch.from_numpy(toks).to(self.dev)
        W1, W3, W2 = experts_f64(L["W1"]), experts_f64(L["W3"]), experts_f64(L["W2"])
        U = None if L["U"] is None else f64(L["U"][tt])
        idx = r.topk_idx[tt].cpu().numpy().astype(np.int64)
        dropped = (r.inv_pos[tt] < 0).cpu().numpy()
        sub = O.moe_forward(f64(L["x"][tt]), f64(L["W_router"]), f64(L["b_router"]), W1, W3, W2, k, V["mode"], U,
                            forced_idx=idx, tau=V.get("tau", 1.0), forced_dropped=dropped)

        def rel(a, b):
            return float(np.linalg.norm(a - b) / np.linalg.norm(b))
        errs = {"out": rel(f64(self.out[tt]), sub["out"])}
        if not self.fwd_only:
            counts = r.counts.cpu().numpy().astype(np.float64)
            stats = {"u": counts / (T * k), "pbar": f64(r.prob_sum) / T, "T": T}
            ref = O.moe_backward(f64(L["x"][tt]), f64(L["W_router"]), f64(L["b_router"]), W1, W3, W2, k, V["mode"],
                                 f64(L["dY"][tt]), sub, ALPHA, O.LB_TOKEN_FRAC, 1.0, batch_stats=stats, want_dW=False,
                                 tau=V.get("tau", 1.0))
            errs["dX"] = rel(f64(self.grads.dX[tt]), ref["dX"])
        return {"tokens": int(toks.size), "rel_err": errs, "tol": tol, "ok": all(e <= tol for e in errs.values())}

    def timed(self, steps, warmup):
        lib = B.load_library()
        T, d, f, E, k = self.T, self.d, self.f, self.E, self.k
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        n_stage = len(B.STAGE_NAMES)
        events = HipEvents(2 * n_stage * steps)
        step_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for s in range(steps):
            ptr, n = events.slice(2 * n_stage * s, n_stage)
            lib.btx_profile_stages(ptr, n)
            step_ev[s][0].record()
            self.step()
            step_ev[s][1].record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        lib.btx_profile_stages(None, 0)
        step_ms = sorted(a.elapsed_time(b) for a, b in step_ev)
        stage_ms = {}
        for i, name in enumerate(B.STAGE_NAMES):
            v = [events.elapsed_ms(2 * n_stage * s + 2 * i, 2 * n_stage * s + 2 * i + 1) for s in range(steps)]
            stage_ms[name] = float(np.mean(v))
        events.destroy()
        R = int(self.routing.offsets[-1].item())   # grouped rows the expert GEMMs worked on (T*k unless pairs were dropped)
        gemm = {n: {"ms": stage_ms[n], "tflops": c * d * f * R / (stage_ms[n] * 1e-3) / 1e12,
                    "frac_of_peak": c * d * f * R / (stage_ms[n] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
                for n, c in GEMM_STAGES.items() if stage_ms[n] > 0}
        gemm_coef = float(sum(GEMM_STAGES[n] for n in gemm))    # 18 for forward + backward, 6 for forward
        gemm_ms = sum(v["ms"] for v in gemm.values())
        gemm_tflops = gemm_coef * d * f * R / (gemm_ms * 1e-3) / 1e12
        ms_per_step = elapsed / steps * 1e3
        return {"elapsed": elapsed, "ms_per_step": ms_per_step, "tokens_per_s": T * steps / elapsed, "routed_rows": R,
                "step_ms": {"median": step_ms[len(step_ms) // 2], "min": step_ms[0], "max": step_ms[-1]},
                "stage_ms": stage_ms, "gemm": gemm,
                "expert_gemms": {"ms": gemm_ms, "tflops": gemm_tflops, "frac_of_peak": gemm_tflops / PEAK_BF16_TFLOPS,
                                 "layer_frac_of_peak": gemm_coef * d * f * R / (ms_per_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                                 "per_kernel": gemm},
                "hbm_stages": hbm_stages(stage_ms, T, d, E, k, block=self.block)}


def merge_bench(dev, steps=10, warmup=2, cpu_elems=1 << 26):
    """btx_merge_average over 4 perturbed copies of the 7B non-FF parameter set (32 layers x 4 attention
    matrices [4096,4096] plus the embeddings [32000,4096], bf16), each copy one flat buffer: HBM-bound,
    (N+1) * 2 bytes per element.  The oracle's merge_average is timed on the first `cpu_elems` elements."""
    from oracle import btx_oracle as O
    N, numel = 4, 128 * 4096 * 4096 + 32000 * 4096
    gen = torch.Generator(device=dev).manual_seed(synth.BASE_SEED + 8)
    base = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32) / 64.0
    copies = []
    for _ in range(N):
        pert = torch.randn(numel, generator=gen, device=dev, dtype=torch.float32) * (0.1 / 64.0)
        copies.append((base + pert).to(torch.bfloat16))
        del pert
    del base
    out = torch.empty_like(copies[0])
    for _ in range(warmup):
        B.btx_merge_average(copies, out=out)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    for a, b in ev:
        a.record()
        B.btx_merge_average(copies, out=out)
        b.record()
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in ev)
    mean_ms = float(np.mean(ms))
    nbytes = (N + 1) * 2 * numel
    # parity on the timed output: the first and last elements against the oracle, bit for bit
    pos = torch.cat([torch.arange(0, 1 << 16, device=dev), torch.arange(numel - (1 << 16), numel, device=dev)])
    want = O.round_to_bf16(O.merge_average([c[pos].float().cpu().numpy() for c in copies]))
    ok = bool(np.array_equal(out[pos].float().cpu().numpy(), want))
    host = [c[:cpu_elems].float().cpu().numpy() for c in copies]
    t0 = time.perf_counter()
    O.round_to_bf16(O.merge_average(host))
    dt = time.perf_counter() - t0
    return {"workload": f"mean of {N} bf16 copies of {numel} elements (128 x [4096,4096] + [32000,4096])",
            "algorithmic_bytes": nbytes, "ms": mean_ms, "ms_min": ms[0],
            "roofline": {"bound": "hbm", "kernel": "merge_bf16_kernel", "achieved": nbytes / (mean_ms * 1e-3) / 1e9,
                         "peak": PEAK_HBM_TBS * 1e3, "unit": "GB/s", "frac": nbytes / (mean_ms * 1e-3) / (PEAK_HBM_TBS * 1e12)},
            "parity_checked": ok,
            "cpu_baseline": {"value": (N + 1) * 2 * cpu_elems / dt / 1e9, "unit": "GB/s (same (N+1)*2 bytes per element)",
                             "cores": host_threads(), "kind": "oracle",
                             "sample": f"first {cpu_elems} elements of every copy, float64 numpy, {dt:.1f} s"}}


def config_report(V, T, r, parity, det):
    return {"metric": metric_name(V), "workload": describe(V, T), "value": r["tokens_per_s"], "unit": "tokens/s",
            "ms_per_step": r["ms_per_step"], "routed_rows": r["routed_rows"], "step_ms": r["step_ms"],
            "expert_gemms": r["expert_gemms"], "stage_ms": r["stage_ms"], "hbm_stages": r["hbm_stages"],
            "parity_checked": parity, "deterministic": det}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--tokens", type=int, default=0, help="override T (dev runs only)")
    ap.add_argument("--cpu-sample", type=int, default=8192, help="tokens the CPU oracle is timed on (0 = skip)")
    ap.add_argument("--variant", default="top2", choices=sorted(VARIANTS),
                    help="configuration to time as the headline; only top2 is the benchmark of record")
    ap.add_argument("--no-configs", action="store_true", help="skip the other named configurations and the merge")
    ap.add_argument("--merge-only", action="store_true", help="only the parameter averaging (profiling runs)")
    ap.add_argument("--no-selfcheck", action="store_true", help="skip the parity and determinism checks (profiling runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    dev = "cuda:0"
    torch.cuda.set_device(0)
    B.btx_init()
    if args.merge_only:
        print(json.dumps(merge_bench(dev)))
        return
    V = VARIANTS[args.variant]
    T = args.tokens or V["T"]
    main_layer = Layer(V, T, dev)
    parity = det = None
    if not args.no_selfcheck:
        parity = main_layer.parity()
        det = main_layer.deterministic()
    r = main_layer.timed(args.steps, args.warmup)
    gemm = r["gemm"]
    dominant = max(gemm, key=lambda n: gemm[n]["ms"])
    record = args.variant == "top2" and T == V["T"]
    traffic, traffic_src = profiled_traffic(dominant) if record else (None, "only kept for the benchmark configuration")
    result = {
        "metric": metric_name(V), "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": describe(V, T) if T == V["T"] else "dev run, " + describe(V, T), "tokens": T,
                   "routed_rows": r["routed_rows"], "d_model": D_MODEL, "d_ff": V["f"], "experts": V["E"], "top_k": V["k"]},
        "roofline": {"bound": "mfma", "kernel": f"mfma_gemm_kernel ({dominant})", "achieved": gemm[dominant]["tflops"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": gemm[dominant]["tflops"] / PEAK_BF16_TFLOPS,
                     "traffic": traffic, "traffic_source": traffic_src,
                     "algorithmic_flops": GEMM_STAGES[dominant] * D_MODEL * V["f"] * r["routed_rows"]},
        "expert_gemms": r["expert_gemms"], "stage_ms": r["stage_ms"], "step_ms": r["step_ms"],
        "hbm_stages": r["hbm_stages"],
        "parity_checked": None if parity is None else parity["ok"], "parity": parity, "deterministic": det,
    }
    if args.cpu_sample > 0 and args.variant == "top2":   # the oracle is timed on the benchmark configuration only
        result["cpu_baseline"] = cpu_baseline(main_layer.L, V, min(args.cpu_sample, T))
    if record and not args.no_configs:
        configs = {}
        for name in REPORTED:
            Vc = VARIANTS[name]
            layer = Layer(Vc, Vc["T"], dev, shared=main_layer)
            p = None if args.no_selfcheck else layer.parity()
            dt = None if args.no_selfcheck else layer.deterministic()
            configs[name] = config_report(Vc, Vc["T"], layer.timed(10, 3), p, dt)
            if Vc.get("split", 1) > 1:
                _W64.clear()             # the split copies are not needed again
            del layer
            torch.cuda.empty_cache()
        _W64.clear()
        del main_layer
        torch.cuda.empty_cache()
        configs["c4-merge-average"] = merge_bench(dev)
        result["configs"] = configs
    print(json.dumps(result))


if __name__ == "__main__":
    main()
