"""Plain CPU oracle for the token-routed Mixture-of-Experts feed-forward layer
of Branch-Train-MiX (arXiv 2403.07816) and for its parameter averaging.

THIS IS TEST INFRASTRUCTURE.  It is slow on purpose, it shares no code with
the HIP library, and the library never calls it.  Only the tests, the smoke
check and the bench's cpu_baseline leg import it.

Everything is numpy float64.  A matmul serves as a step where the definition
has a matrix product; there is no tiling, grouping, permutation or fusion.

What each function follows:
  route            Sec. 3.2 (router W_l x, Top-k: softmax over the kept k
                   logits); Sec. 3.3 "Routing method" (Switch = top-1 with the
                   softmax probability as gate; sample-top-1 in the reading
                   described below)
  lb_statistics    Sec. 3.3 "Load balancing" (u_i, p_i, L_LB)
  expert_ff        the feed-forward sublayer of the seed model (Sec. 4.1:
                   Llama-2 7B, i.e. the gated 3-matrix SwiGLU form; Table 4's
                   active-parameter column confirms three d x d_ff matrices)
  moe_forward      the layer equation of Sec. 3.2: sum_i g_i(W_l x) FF_i(x)
  moe_backward     chain rule on the above with the discrete selection held
                   fixed (the paper writes no backward; it only finetunes the
                   layer by gradient descent)
  split_experts    Sec. 3.3 "Splitting Experts"
  rmsnorm          the pre-normalisation in front of the sublayer (seed model, Sec. 4.1)
  merge_average    Sec. 3.2: non-FF parameters are averaged elementwise
  merge_weighted   the same merge with caller-chosen coefficients
  grouping         the token->expert grouping implied by skipping zero gates

Readings where the paper is silent (also listed in the design notes):
  * ties in top-k / argmax go to the lower expert index; the k chosen experts
    are listed by descending logit;
  * an optional router bias is added to the logits;
  * sample-top-1 takes one uniform number U[t] per token and picks the first
    expert whose cumulative softmax probability exceeds it; gate = that
    expert's softmax probability (parity unpinned: the paper's Gumbel-softmax
    form needs E noises per token and a temperature);
  * u_i in the load-balancing loss: LB_TOKEN_FRAC uses the fraction of routed
    (token, slot) pairs counts_i/(T*k); LB_GATE_MEAN is the printed formula,
    the batch mean of the gate value.  Which one the authors ran is parity
    unpinned; both satisfy sum_i u_i = 1 for top-k.  u is a constant for the
    gradient unless grad_through_u is set (LB_GATE_MEAN only).
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

ROUTE_TOPK_RENORM = 0
ROUTE_SWITCH_TOP1 = 1
ROUTE_SAMPLE_TOP1 = 2
ROUTE_GUMBEL_TOP1 = 3

LB_TOKEN_FRAC = 0
LB_GATE_MEAN = 1

F64 = np.float64


# --------------------------------------------------------------------------
# small pieces
# --------------------------------------------------------------------------
def softmax(s: np.ndarray) -> np.ndarray:
    """Row-wise softmax with the row maximum subtracted first."""
    s = np.asarray(s, dtype=F64)
    z = np.exp(s - s.max(axis=-1, keepdims=True))
    return z / z.sum(axis=-1, keepdims=True)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def silu_grad(z: np.ndarray) -> np.ndarray:
    sig = 1.0 / (1.0 + np.exp(-z))
    return sig * (1.0 + z * (1.0 - sig))


def expert_ff(x: np.ndarray, W1: np.ndarray, W3: np.ndarray, W2: np.ndarray) -> np.ndarray:
    """FF(x) = (silu(x W1) * (x W3)) W2, no biases."""
    x = np.asarray(x, dtype=F64)
    return (silu(x @ np.asarray(W1, F64)) * (x @ np.asarray(W3, F64))) @ np.asarray(W2, F64)


# --------------------------------------------------------------------------
# routing
# --------------------------------------------------------------------------
def router_logits(x, W_router, b_router=None) -> np.ndarray:
    s = np.asarray(x, F64) @ np.asarray(W_router, F64)
    if b_router is not None:
        s = s + np.asarray(b_router, F64)[None, :]
    return s


def capacity(T: int, k: int, E: int, capacity_factor: float) -> int:
    """Rows an expert may take: ceil(capacity_factor * T*k / E) (Sec. 4.3: "a hard limit
    after which routed tokens will be dropped"); 0 = no limit."""
    if capacity_factor <= 0:
        return 0
    return int(math.ceil(float(capacity_factor) * T * k / E))


def dropped_pairs(idx: np.ndarray, E: int, cap: int) -> np.ndarray:
    """dropped[t,j]: the pair (t,j) is beyond its expert's capacity.  Pairs are served in
    (t, j) order, so the first `cap` pairs of every expert are kept."""
    T, k = idx.shape
    dropped = np.zeros((T, k), dtype=bool)
    if cap <= 0:
        return dropped
    taken = np.zeros(E, dtype=np.int64)
    for t in range(T):
        for j in range(k):
            e = idx[t, j]
            if taken[e] >= cap:
                dropped[t, j] = True
            else:
                taken[e] += 1
    return dropped


def route(x, W_router, b_router, k: int, mode: int, U=None, forced_idx=None, tau: float = 1.0,
          capacity_factor: float = 0.0, forced_dropped=None) -> Dict[str, np.ndarray]:
    """Logits, full softmax, chosen experts idx[T,k] and their gates[T,k].

    forced_idx[T,k] (entries < 0 = not forced) overrides the selection of
    individual tokens; the gate formulas are then applied to the forced set.
    forced_dropped[T,k] replaces the capacity decision (for evaluating a sample of
    a batch whose drops were decided on the whole batch).

    ROUTE_GUMBEL_TOP1 (Sec. 3.3 "Sample Top-1", training time): U is the Gumbel
    noise G[T,E] drawn by the caller and tau the temperature; the soft sample is
    y = softmax((logits + G) / tau), all of it but its largest entry is zeroed,
    so the gate is that largest entry and only its expert is computed.  "probs"
    stays the plain softmax of the logits, which is what the load-balancing loss
    uses; the soft sample is returned as "gate_probs".
    """
    s = router_logits(x, W_router, b_router)
    T, E = s.shape
    assert 1 <= k <= E
    p = softmax(s)
    gate_probs = None
    if mode == ROUTE_TOPK_RENORM:
        # descending logit, ties -> lower index (stable sort of the negated logits)
        idx = np.argsort(-s, axis=1, kind="stable")[:, :k]
    elif mode == ROUTE_SWITCH_TOP1:
        assert k == 1
        idx = np.argsort(-s, axis=1, kind="stable")[:, :1]
    elif mode == ROUTE_SAMPLE_TOP1:
        assert k == 1 and U is not None
        U = np.asarray(U, F64)
        idx = np.empty((T, 1), dtype=np.int64)
        for t in range(T):
            c = 0.0
            chosen = E - 1
            for e in range(E):
                c += p[t, e]
                if c > U[t]:
                    chosen = e
                    break
            idx[t, 0] = chosen
    elif mode == ROUTE_GUMBEL_TOP1:
        assert k == 1 and U is not None and tau > 0
        noisy = s + np.asarray(U, F64)
        gate_probs = softmax(noisy / tau)
        idx = np.argsort(-noisy, axis=1, kind="stable")[:, :1]
    else:
        raise ValueError("unknown route mode")
    idx = idx.astype(np.int64)
    if forced_idx is not None:
        forced_idx = np.asarray(forced_idx)
        rows = forced_idx[:, 0] >= 0
        idx[rows] = forced_idx[rows]
    if mode == ROUTE_TOPK_RENORM:
        gates = softmax(np.take_along_axis(s, idx, axis=1))
    elif mode == ROUTE_GUMBEL_TOP1:
        gates = np.take_along_axis(gate_probs, idx, axis=1)
    else:
        gates = np.take_along_axis(p, idx, axis=1)
    res = {"logits": s, "probs": p, "idx": idx, "gates": gates,
           "dropped": (np.asarray(forced_dropped, dtype=bool) if forced_dropped is not None
                       else dropped_pairs(idx, E, capacity(T, k, E, capacity_factor)))}
    if gate_probs is not None:
        res["gate_probs"] = gate_probs
    return res


def dense_gates(idx: np.ndarray, gates: np.ndarray, E: int) -> np.ndarray:
    """The routing function's output as the paper writes it: a length-E vector
    per token that is zero outside the chosen experts."""
    T, k = idx.shape
    g = np.zeros((T, E), dtype=F64)
    for t in range(T):
        for j in range(k):
            g[t, idx[t, j]] = gates[t, j]
    return g


def lb_statistics(idx, gates, probs, alpha: float, lb_mode: int) -> Dict[str, np.ndarray]:
    """counts_i, sum_t g_i, sum_t softmax_i, u_i, p_i and L_LB = alpha*N*sum u_i p_i."""
    T, E = probs.shape
    k = idx.shape[1]
    g = dense_gates(idx, gates, E)
    counts = np.zeros(E, dtype=np.int64)
    for t in range(T):
        for j in range(k):
            counts[idx[t, j]] += 1
    gate_sum = g.sum(axis=0)
    prob_sum = np.asarray(probs, F64).sum(axis=0)
    pbar = prob_sum / T
    if lb_mode == LB_TOKEN_FRAC:
        u = counts.astype(F64) / (T * k)
    elif lb_mode == LB_GATE_MEAN:
        u = gate_sum / T
    else:
        raise ValueError("unknown lb mode")
    loss = alpha * E * float(np.sum(u * pbar))
    return {"counts": counts, "gate_sum": gate_sum, "prob_sum": prob_sum, "u": u, "pbar": pbar,
            "lb_loss": loss}


def grouping(idx: np.ndarray, E: int, dropped: Optional[np.ndarray] = None) -> Dict[str, np.ndarray]:
    """Group the kept (token, slot) pairs by expert, keeping (t, j) order inside
    a group.  perm[r] = t*k+j of the pair at grouped row r; inv_pos[t,j] = r, or -1
    for a dropped pair; offsets[e] = first grouped row of expert e."""
    T, k = idx.shape
    flat = idx.reshape(-1)
    keep = np.ones(T * k, dtype=bool) if dropped is None else ~np.asarray(dropped).reshape(-1)
    order = np.argsort(flat, kind="stable").astype(np.int64)
    perm = order[keep[order]]
    inv = -np.ones(T * k, dtype=np.int64)
    inv[perm] = np.arange(perm.size)
    counts = np.bincount(flat[keep], minlength=E)
    offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    return {"offsets": offsets, "perm": perm, "inv_pos": inv.reshape(T, k)}


# --------------------------------------------------------------------------
# the layer
# --------------------------------------------------------------------------
def moe_forward(x, W_router, b_router, W1, W3, W2, k: int, mode: int = ROUTE_TOPK_RENORM, U=None,
                alpha: float = 0.0, lb_mode: int = LB_TOKEN_FRAC, forced_idx=None,
                keep_y: bool = False, tau: float = 1.0, capacity_factor: float = 0.0,
                forced_dropped=None) -> Dict[str, np.ndarray]:
    """out_t = sum_i g_i(W_l x_t) FF_i(x_t), evaluating FF_i only where the
    gate is non-zero (the paper's own remark that zero-gate experts are
    skipped); W1/W3/W2 are sequences of per-expert matrices.  With a capacity
    factor the pairs beyond an expert's capacity contribute nothing."""
    x = np.asarray(x, F64)
    T, d = x.shape
    E = len(W1)
    r = route(x, W_router, b_router, k, mode, U, forced_idx, tau, capacity_factor, forced_dropped)
    idx, gates = r["idx"], r["gates"]
    kept = ~r["dropped"]
    out = np.zeros((T, d), dtype=F64)
    y = np.zeros((T, k, d), dtype=F64) if keep_y else None
    for e in range(E):
        tt, jj = np.nonzero((idx == e) & kept)
        if tt.size == 0:
            continue
        ye = expert_ff(x[tt], W1[e], W3[e], W2[e])
        out[tt] += gates[tt, jj][:, None] * ye
        if keep_y:
            y[tt, jj] = ye
    res = dict(r)
    res.update(lb_statistics(idx, gates, r["probs"], alpha, lb_mode))
    res["out"] = out
    if keep_y:
        res["y"] = y
    return res


def moe_forward_all_experts(x, W_router, b_router, W1, W3, W2, k: int, mode: int = ROUTE_TOPK_RENORM,
                            U=None, tau: float = 1.0) -> np.ndarray:
    """The layer equation taken literally: every expert on every token, times
    the dense (mostly zero) gate vector.  Used to pin moe_forward."""
    x = np.asarray(x, F64)
    E = len(W1)
    r = route(x, W_router, b_router, k, mode, U, None, tau)
    g = dense_gates(r["idx"], r["gates"], E)
    out = np.zeros_like(x)
    for e in range(E):
        out += g[:, e:e + 1] * expert_ff(x, W1[e], W3[e], W2[e])
    return out


def lb_grad_logits(probs, u, alpha: float, T_batch: int) -> np.ndarray:
    """d L_LB / d logits with u held constant:
    (alpha*N/T) * p_tj * (u_j - sum_e u_e p_te)."""
    probs = np.asarray(probs, F64)
    E = probs.shape[1]
    return (alpha * E / T_batch) * probs * (u[None, :] - (probs * u[None, :]).sum(axis=1, keepdims=True))


def moe_backward(x, W_router, b_router, W1, W3, W2, k: int, mode: int, dY, fwd: Dict[str, np.ndarray],
                 alpha: float = 0.0, lb_mode: int = LB_TOKEN_FRAC, lb_grad_scale: float = 0.0,
                 grad_through_u: bool = False, batch_stats: Optional[Dict] = None,
                 want_dW: bool = True, tau: float = 1.0) -> Dict[str, np.ndarray]:
    """Gradients of  <dY, out> + lb_grad_scale * L_LB  with idx held fixed.

    fwd is moe_forward's result for the same inputs (idx, gates, probs are
    read from it).  batch_stats={"u","pbar","T"} substitutes the whole batch's
    load-balancing statistics when x is only a sample of that batch.
    """
    x = np.asarray(x, F64)
    dY = np.asarray(dY, F64)
    T, d = x.shape
    E = len(W1)
    idx, gates, probs = fwd["idx"], fwd["gates"], fwd["probs"]
    kept = ~fwd["dropped"] if "dropped" in fwd else np.ones(idx.shape, dtype=bool)
    Wr = np.asarray(W_router, F64)
    if batch_stats is None:
        st = lb_statistics(idx, gates, probs, alpha, lb_mode)
        u, pbar, T_batch = st["u"], st["pbar"], T
    else:
        u, pbar, T_batch = batch_stats["u"], batch_stats["pbar"], batch_stats["T"]

    dX = np.zeros((T, d), dtype=F64)
    dg = np.zeros((T, k), dtype=F64)
    dW1: List[Optional[np.ndarray]] = [None] * E
    dW3: List[Optional[np.ndarray]] = [None] * E
    dW2: List[Optional[np.ndarray]] = [None] * E
    for e in range(E):
        W1e, W3e, W2e = np.asarray(W1[e], F64), np.asarray(W3[e], F64), np.asarray(W2[e], F64)
        tt, jj = np.nonzero((idx == e) & kept)   # a dropped pair has no output, hence dg = 0
        xe = x[tt]
        h1 = xe @ W1e
        h3 = xe @ W3e
        a = silu(h1) * h3
        ye = a @ W2e
        dg[tt, jj] = np.sum(dY[tt] * ye, axis=1)
        dy = gates[tt, jj][:, None] * dY[tt]
        da = dy @ W2e.T
        dh1 = da * h3 * silu_grad(h1)
        dh3 = da * silu(h1)
        dX[tt] += dh1 @ W1e.T + dh3 @ W3e.T
        if want_dW:
            dW2[e] = a.T @ dy
            dW1[e] = xe.T @ dh1
            dW3[e] = xe.T @ dh3

    dg_ff = dg                                   # <dY_t, FF_e(x_t)> alone, reported beside the total
    if grad_through_u:
        # u_i = mean_t g_ti, so L_LB also depends on every gate: dL/dg_ti = alpha*N*p_i/T
        assert lb_mode == LB_GATE_MEAN
        dg = dg + lb_grad_scale * (alpha * E / T_batch) * pbar[idx]

    ds = np.zeros((T, E), dtype=F64)
    if mode == ROUTE_TOPK_RENORM:
        inner = np.sum(gates * dg, axis=1, keepdims=True)
        ds_sel = gates * (dg - inner)
        for t in range(T):
            for j in range(k):
                ds[t, idx[t, j]] += ds_sel[t, j]
    elif mode == ROUTE_GUMBEL_TOP1:
        # gate = y_e with y = softmax((s + G)/tau): d gate / d s_j = y_e (delta_ej - y_j) / tau
        yv = fwd["gate_probs"]
        for t in range(T):
            e = idx[t, 0]
            row = -yv[t, e] * yv[t]
            row[e] += yv[t, e]
            ds[t] = dg[t, 0] * row / tau
    else:
        for t in range(T):
            e = idx[t, 0]
            pe = probs[t, e]
            row = -pe * probs[t]
            row[e] += pe
            ds[t] = dg[t, 0] * row
    if lb_grad_scale != 0.0:
        ds += lb_grad_scale * lb_grad_logits(probs, u, alpha, T_batch)

    dX += ds @ Wr.T
    return {"dX": dX, "dW_router": x.T @ ds, "db_router": ds.sum(axis=0), "ds": ds, "dg": dg, "dg_ff": dg_ff,
            "dW1": dW1, "dW3": dW3, "dW2": dW2}


def dW_columns(x, W1e, W3e, W2e, tokens, token_gates, dY, cols) -> Dict[str, np.ndarray]:
    """For one expert, whose routed tokens are `tokens` with gates
    `token_gates`: columns `cols` of dW1 and dW3 and rows `cols` of dW2.
    The same definitions as moe_backward, restricted to those d_ff indices, so
    that a few columns of a full-size gradient can be checked one by one."""
    xe = np.asarray(x, F64)[tokens]
    dy = np.asarray(token_gates, F64)[:, None] * np.asarray(dY, F64)[tokens]
    cols = np.asarray(cols)
    h1 = xe @ np.asarray(W1e[:, cols], F64)
    h3 = xe @ np.asarray(W3e[:, cols], F64)
    a = silu(h1) * h3
    da = dy @ np.asarray(W2e[cols, :], F64).T
    dh1 = da * h3 * silu_grad(h1)
    dh3 = da * silu(h1)
    return {"dW1": xe.T @ dh1, "dW3": xe.T @ dh3, "dW2": a.T @ dy}


# --------------------------------------------------------------------------
# MiX construction pieces
# --------------------------------------------------------------------------
def split_experts(W1: Sequence[np.ndarray], W3: Sequence[np.ndarray], W2: Sequence[np.ndarray], C: int):
    """Split every FF along d_ff into C chunks: expert i*C+c takes columns
    [c*f/C, (c+1)*f/C) of W1_i and W3_i and the same rows of W2_i."""
    o1, o3, o2 = [], [], []
    for i in range(len(W1)):
        f = W1[i].shape[1]
        assert f % C == 0
        fc = f // C
        for c in range(C):
            o1.append(np.asarray(W1[i])[:, c * fc:(c + 1) * fc])
            o3.append(np.asarray(W3[i])[:, c * fc:(c + 1) * fc])
            o2.append(np.asarray(W2[i])[c * fc:(c + 1) * fc, :])
    return o1, o3, o2


def blend_experts(W1: Sequence[np.ndarray], W3: Sequence[np.ndarray], W2: Sequence[np.ndarray]):
    """Sec. 3.3 "Blending Experts": every FF is cut along d_ff into N chunks (N = number of
    FFs) and MoE expert n is built from the n-th chunk of every domain FF, domain after
    domain.  Width stays d_ff; the hidden units are only dealt out differently."""
    N = len(W1)
    f = np.asarray(W1[0]).shape[1]
    assert f % N == 0
    fc = f // N
    o1, o3, o2 = [], [], []
    for n in range(N):
        o1.append(np.concatenate([np.asarray(W1[i])[:, n * fc:(n + 1) * fc] for i in range(N)], axis=1))
        o3.append(np.concatenate([np.asarray(W3[i])[:, n * fc:(n + 1) * fc] for i in range(N)], axis=1))
        o2.append(np.concatenate([np.asarray(W2[i])[n * fc:(n + 1) * fc, :] for i in range(N)], axis=0))
    return o1, o3, o2


def merge_average(tensors: Sequence[np.ndarray]) -> np.ndarray:
    """Elementwise mean of N same-shape tensors, in float64."""
    acc = np.zeros_like(np.asarray(tensors[0], F64))
    for t in tensors:
        acc = acc + np.asarray(t, F64)
    return acc / len(tensors)


def rmsnorm(h: np.ndarray, gain: np.ndarray, eps: float):
    """Root-mean-square normalisation of every token row, the pre-normalisation in front of
    the feed-forward sublayer of the seed model's blocks (Sec. 4.1: Llama-2 7B):
        xn[t,c] = h[t,c] * rstd[t] * gain[c],   rstd[t] = 1 / sqrt(mean_c h[t,c]^2 + eps).
    Returns (xn [T,d], rstd [T]) in float64.  The block then computes
    out = h + FF_MoE(xn): the layer of Sec. 3.2 takes xn where that section writes x."""
    h = np.asarray(h, F64)
    gain = np.asarray(gain, F64)
    rstd = 1.0 / np.sqrt(np.mean(h * h, axis=1) + eps)
    return h * rstd[:, None] * gain[None, :], rstd


def rmsnorm_backward(dxn: np.ndarray, h: np.ndarray, gain: np.ndarray, eps: float):
    """Chain rule through rmsnorm: with xhat = h * rstd and q = gain * dxn,
        dh[t]    = rstd[t] * (q[t] - xhat[t] * mean_c(q[t,c] * xhat[t,c])),
        dgain[c] = sum_t dxn[t,c] * xhat[t,c].
    Returns (dh [T,d], dgain [d]) in float64."""
    dxn, h, gain = np.asarray(dxn, F64), np.asarray(h, F64), np.asarray(gain, F64)
    rstd = 1.0 / np.sqrt(np.mean(h * h, axis=1) + eps)
    xhat = h * rstd[:, None]
    q = dxn * gain[None, :]
    dh = rstd[:, None] * (q - xhat * np.mean(q * xhat, axis=1, keepdims=True))
    return dh, np.sum(dxn * xhat, axis=0)


def merge_weighted(tensors: Sequence[np.ndarray], weights: Sequence[float]) -> np.ndarray:
    """Elementwise weighted sum  sum_n w_n * tensors[n]  in float64, terms added in input
    order.  Generalises the uniform mean of Sec. 3.2 (w_n = 1/N) to caller-chosen
    coefficients; the paper itself only averages, so whether the authors ever weighted a
    merge is parity unpinned.  The weights are taken as given (not normalised)."""
    assert len(tensors) == len(weights) and len(tensors) >= 1
    acc = np.zeros_like(np.asarray(tensors[0], F64))
    for t, w in zip(tensors, weights):
        acc = acc + np.float64(w) * np.asarray(t, F64)
    return acc


def adamw_step(p, g, m, v, step: int, lr: float, beta1: float, beta2: float, eps: float, weight_decay: float):
    """One AdamW update (Sec. 4.1 names the optimizer and its weight decay, 0.1; the moment
    decay rates and eps are inputs): decoupled weight decay, bias-corrected moments,
        m <- b1 m + (1-b1) g,  v <- b2 v + (1-b2) g^2,
        p <- p - lr * ( (m/(1-b1^t)) / (sqrt(v/(1-b2^t)) + eps) + wd * p ),   t = step >= 1.
    Returns the new (p, m, v) in float64."""
    p, g, m, v = (np.asarray(a, F64) for a in (p, g, m, v))
    assert step >= 1
    m = beta1 * m + (1.0 - beta1) * g
    v = beta2 * v + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v


def round_to_bf16(v: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (ties to even), returned as
    float32.  One rounding, straight from float64.  Values are assumed finite
    and inside bfloat16's normal range."""
    v = np.ascontiguousarray(v, dtype=F64)
    bits = v.view(np.uint64)
    drop = np.uint64(52 - 7)                      # float64 mantissa bits that bf16 cannot hold
    lsb = (bits >> drop) & np.uint64(1)
    rounded = (bits + ((np.uint64(1) << (drop - np.uint64(1))) - np.uint64(1)) + lsb) >> drop << drop
    return rounded.view(F64).astype(np.float32)


def ff_active_params(d: int, f: int, k: int, n_layers: int) -> int:
    """Feed-forward parameters touched per token: k experts x three d x f
    matrices x layers (used to check the 3-matrix reading against Table 4)."""
    return n_layers * k * 3 * d * f
