"""Pins for the CPU oracle: every check compares it with something other than
itself (a textbook routine, brute force, a closed form, a finite difference,
or a number the paper prints)."""
import itertools
import os

import numpy as np
import pytest
import scipy.special

from oracle import btx_oracle as O

RNG = np.random.default_rng(7)


def tiny_layer(T=6, d=8, f=12, E=4, scale=1.0, rng=None):
    rng = RNG if rng is None else rng
    x = rng.normal(size=(T, d))
    Wr = rng.normal(size=(d, E)) * scale
    W1 = [rng.normal(size=(d, f)) / np.sqrt(d) for _ in range(E)]
    W3 = [rng.normal(size=(d, f)) / np.sqrt(d) for _ in range(E)]
    W2 = [rng.normal(size=(f, d)) / np.sqrt(f) for _ in range(E)]
    return x, Wr, W1, W3, W2


# ---------------------------------------------------------------- routing --
def test_softmax_matches_scipy():
    s = RNG.normal(size=(50, 7)) * 5
    np.testing.assert_allclose(O.softmax(s), scipy.special.softmax(s, axis=1), rtol=1e-13)


@pytest.mark.parametrize("E,k", [(4, 1), (4, 2), (5, 3), (6, 6)])
def test_topk_is_max_sum_subset_bruteforce(E, k):
    """Top-k = the size-k subset with the largest logit sum; gates = softmax
    over exactly those logits (Sec. 3.2)."""
    x, Wr, *_ = tiny_layer(T=40, d=5, E=E)
    r = O.route(x, Wr, None, k, O.ROUTE_TOPK_RENORM)
    s = x @ Wr
    for t in range(x.shape[0]):
        best = max(itertools.combinations(range(E), k), key=lambda c: sum(s[t, i] for i in c))
        assert set(r["idx"][t]) == set(best)
        # listed by descending logit
        assert all(s[t, r["idx"][t, j]] >= s[t, r["idx"][t, j + 1]] for j in range(k - 1))
        z = np.exp(s[t, r["idx"][t]])
        np.testing.assert_allclose(r["gates"][t], z / z.sum(), rtol=1e-12)


def test_topk_tie_goes_to_lower_index():
    x = np.ones((1, 2))
    Wr = np.array([[0.5, 1.0, 1.0, 0.5], [0.5, 1.0, 1.0, 0.5]])
    r = O.route(x, Wr, None, 3, O.ROUTE_TOPK_RENORM)
    assert list(r["idx"][0]) == [1, 2, 0]
    r1 = O.route(x, Wr, None, 1, O.ROUTE_SWITCH_TOP1)
    assert list(r1["idx"][0]) == [1]


def test_gates_sum_to_one_and_equal_renormalised_softmax():
    x, Wr, *_ = tiny_layer(T=64, d=8, E=6)
    r = O.route(x, Wr, None, 2, O.ROUTE_TOPK_RENORM)
    np.testing.assert_allclose(r["gates"].sum(axis=1), 1.0, rtol=1e-13)
    p = scipy.special.softmax(x @ Wr, axis=1)
    sel = np.take_along_axis(p, r["idx"], axis=1)
    np.testing.assert_allclose(r["gates"], sel / sel.sum(axis=1, keepdims=True), rtol=1e-12)


def test_soft_routing_is_topk_with_k_equal_E():
    x, Wr, *_ = tiny_layer(T=20, d=8, E=5)
    r = O.route(x, Wr, None, 5, O.ROUTE_TOPK_RENORM)
    g = O.dense_gates(r["idx"], r["gates"], 5)
    np.testing.assert_allclose(g, scipy.special.softmax(x @ Wr, axis=1), rtol=1e-12)


def test_switch_gate_is_softmax_prob_of_argmax_and_bias_is_added():
    x, Wr, *_ = tiny_layer(T=50, d=8, E=4)
    b = np.array([2.0, 0.0, 0.0, 0.0])
    r = O.route(x, Wr, b, 1, O.ROUTE_SWITCH_TOP1)
    s = x @ Wr + b
    p = scipy.special.softmax(s, axis=1)
    assert np.array_equal(r["idx"][:, 0], np.argmax(s, axis=1))
    np.testing.assert_allclose(r["gates"][:, 0], p.max(axis=1), rtol=1e-12)


def test_sample_top1_is_inverse_cdf_and_follows_the_softmax():
    T, E = 20000, 4
    x = np.zeros((T, 3))
    Wr = np.zeros((3, E))
    b = np.log(np.array([0.1, 0.2, 0.3, 0.4]))
    U = np.random.default_rng(3).random(T)
    r = O.route(x, Wr, b, 1, O.ROUTE_SAMPLE_TOP1, U=U)
    cdf = np.cumsum([0.1, 0.2, 0.3, 0.4])
    expected = np.minimum(np.searchsorted(cdf, U, side="right"), E - 1)
    far = np.min(np.abs(U[:, None] - cdf[None, :]), axis=1) > 1e-12
    assert np.array_equal(r["idx"][far, 0], expected[far])
    freq = np.bincount(r["idx"][:, 0], minlength=E) / T
    np.testing.assert_allclose(freq, [0.1, 0.2, 0.3, 0.4], atol=0.012)
    np.testing.assert_allclose(r["gates"][:, 0], np.array([0.1, 0.2, 0.3, 0.4])[r["idx"][:, 0]], rtol=1e-12)
    # U beyond the accumulated sum falls to the last expert
    r2 = O.route(x[:1], Wr, b, 1, O.ROUTE_SAMPLE_TOP1, U=np.array([1.0]))
    assert r2["idx"][0, 0] == E - 1


def test_gumbel_top1_special_cases():
    """Pins of the Gumbel soft sample (Sec. 3.3): without noise at tau = 1 it is Switch
    routing; with two experts its gate is a logistic function of the noisy logit gap; a
    constant added to every noise value changes nothing; a high temperature flattens the gate
    to 1/E without moving the arg-max; and the chosen expert follows the softmax (Gumbel-max)."""
    rng = np.random.default_rng(5)
    x, Wr, W1, W3, W2 = tiny_layer(T=9, d=6, f=5, E=4, rng=rng)
    b = rng.normal(size=4) * 0.2
    zero = np.zeros((9, 4))
    sw = O.route(x, Wr, b, 1, O.ROUTE_SWITCH_TOP1)
    gz = O.route(x, Wr, b, 1, O.ROUTE_GUMBEL_TOP1, zero, tau=1.0)
    np.testing.assert_array_equal(gz["idx"], sw["idx"])
    np.testing.assert_allclose(gz["gates"], sw["gates"], rtol=1e-13)
    np.testing.assert_allclose(gz["probs"], sw["probs"], rtol=1e-13)
    G = -np.log(-np.log(rng.random((9, 4))))
    a = O.route(x, Wr, b, 1, O.ROUTE_GUMBEL_TOP1, G, tau=0.7)
    c = O.route(x, Wr, b, 1, O.ROUTE_GUMBEL_TOP1, G + 3.25, tau=0.7)
    np.testing.assert_array_equal(a["idx"], c["idx"])
    np.testing.assert_allclose(a["gates"], c["gates"], rtol=1e-12)
    np.testing.assert_allclose(a["probs"], sw["probs"], rtol=1e-13)       # LB probabilities ignore noise and tau
    np.testing.assert_array_equal(a["idx"][:, 0], np.argmax(a["logits"] + G, axis=1))
    hot = O.route(x, Wr, b, 1, O.ROUTE_GUMBEL_TOP1, G, tau=1e9)
    np.testing.assert_array_equal(hot["idx"], a["idx"])
    np.testing.assert_allclose(hot["gates"], 0.25, rtol=1e-6)
    # two experts: gate = 1 / (1 + exp(-|gap| / tau))
    x2, Wr2, *_ = tiny_layer(T=9, d=6, f=5, E=2, rng=rng)
    G2 = -np.log(-np.log(rng.random((9, 2))))
    r2 = O.route(x2, Wr2, None, 1, O.ROUTE_GUMBEL_TOP1, G2, tau=0.5)
    gap = np.abs((r2["logits"] + G2)[:, 0] - (r2["logits"] + G2)[:, 1])
    np.testing.assert_allclose(r2["gates"][:, 0], 1.0 / (1.0 + np.exp(-gap / 0.5)), rtol=1e-12)
    # Gumbel-max: arg-max of logits + Gumbel noise is a draw from softmax(logits)
    s = np.array([[0.3, -1.0, 1.2, 0.1]])
    n = 40000
    Gn = -np.log(-np.log(rng.random((n, 4))))
    picks = np.argmax(s + Gn, axis=1)
    freq = np.bincount(picks, minlength=4) / n
    np.testing.assert_allclose(freq, O.softmax(s)[0], atol=0.01)


def test_grouping_bruteforce():
    idx = RNG.integers(0, 5, size=(37, 3))
    g = O.grouping(idx, 5)
    rows = []
    for e in range(5):
        assert g["offsets"][e] == len(rows)
        for t in range(37):
            for j in range(3):
                if idx[t, j] == e:
                    rows.append(t * 3 + j)
    assert g["offsets"][5] == len(rows) == 37 * 3
    assert list(g["perm"]) == rows
    for r, tj in enumerate(rows):
        assert g["inv_pos"][tj // 3, tj % 3] == r


# ---------------------------------------------------------------- forward --
def test_expert_ff_matches_loops():
    x, _, W1, W3, W2 = tiny_layer(T=3, d=4, f=5)
    got = O.expert_ff(x, W1[0], W3[0], W2[0])
    for t in range(3):
        a = np.zeros(5)
        for j in range(5):
            h1 = sum(x[t, c] * W1[0][c, j] for c in range(4))
            h3 = sum(x[t, c] * W3[0][c, j] for c in range(4))
            a[j] = h1 / (1 + np.exp(-h1)) * h3
        for c in range(4):
            np.testing.assert_allclose(got[t, c], sum(a[j] * W2[0][j, c] for j in range(5)), rtol=1e-12)


@pytest.mark.parametrize("mode,k", [(O.ROUTE_TOPK_RENORM, 2), (O.ROUTE_SWITCH_TOP1, 1), (O.ROUTE_TOPK_RENORM, 4)])
def test_skipping_zero_gate_experts_changes_nothing(mode, k):
    x, Wr, W1, W3, W2 = tiny_layer(T=17)
    a = O.moe_forward(x, Wr, None, W1, W3, W2, k, mode)["out"]
    b = O.moe_forward_all_experts(x, Wr, None, W1, W3, W2, k, mode)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_forward_bruteforce_over_all_subsets():
    """For tiny T: evaluate sum_{i in S} softmax_S(s)_i FF_i(x) for every
    subset S of size k and check the layer picked the max-logit-sum one."""
    x, Wr, W1, W3, W2 = tiny_layer(T=5)
    out = O.moe_forward(x, Wr, None, W1, W3, W2, 2)["out"]
    s = x @ Wr
    for t in range(5):
        best, best_sum = None, -np.inf
        for S in itertools.combinations(range(4), 2):
            if s[t, list(S)].sum() > best_sum:
                best, best_sum = S, s[t, list(S)].sum()
        z = np.exp(s[t, list(best)])
        g = z / z.sum()
        ref = sum(g[n] * O.expert_ff(x[t:t + 1], W1[i], W3[i], W2[i])[0] for n, i in enumerate(best))
        np.testing.assert_allclose(out[t], ref, rtol=1e-11)


@pytest.mark.parametrize("k", [1, 2, 3])
def test_identical_experts_reduce_to_the_dense_seed_ff(k):
    """Sparse-upcycling special case (Sec. 4.1.2): E copies of one FF with
    renormalised top-k gates equal that FF for any router."""
    x, Wr, W1, W3, W2 = tiny_layer(T=30)
    W1 = [W1[0]] * 4
    W3 = [W3[0]] * 4
    W2 = [W2[0]] * 4
    out = O.moe_forward(x, Wr, None, W1, W3, W2, k)["out"]
    h1 = x @ W1[0]
    dense = ((h1 * scipy.special.expit(h1)) * (x @ W3[0])) @ W2[0]
    np.testing.assert_allclose(out, dense, rtol=1e-11, atol=1e-13)


def test_identical_experts_backward_corollaries():
    x, Wr, W1, W3, W2 = tiny_layer(T=30)
    W1 = [W1[0]] * 4
    W3 = [W3[0]] * 4
    W2 = [W2[0]] * 4
    dY = RNG.normal(size=x.shape)
    fwd = O.moe_forward(x, Wr, None, W1, W3, W2, 2)
    g = O.moe_backward(x, Wr, None, W1, W3, W2, 2, O.ROUTE_TOPK_RENORM, dY, fwd)
    # dense SwiGLU backward written out directly
    h1, h3 = x @ W1[0], x @ W3[0]
    sig = scipy.special.expit(h1)
    a = h1 * sig * h3
    da = dY @ W2[0].T
    dh1 = da * h3 * (sig + h1 * sig * (1 - sig))
    dh3 = da * h1 * sig
    np.testing.assert_allclose(g["dX"], dh1 @ W1[0].T + dh3 @ W3[0].T, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(sum(g["dW2"]), a.T @ dY, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(sum(g["dW1"]), x.T @ dh1, rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(sum(g["dW3"]), x.T @ dh3, rtol=1e-10, atol=1e-12)
    assert np.abs(g["dW_router"]).max() < 1e-12


# ----------------------------------------------------------- load balance --
@pytest.mark.parametrize("lb_mode", [O.LB_TOKEN_FRAC, O.LB_GATE_MEAN])
def test_lb_closed_forms(lb_mode):
    x, Wr, *_ = tiny_layer(T=64, d=8, E=4)
    r = O.route(x, Wr, None, 2, O.ROUTE_TOPK_RENORM)
    st = O.lb_statistics(r["idx"], r["gates"], r["probs"], 0.01, lb_mode)
    np.testing.assert_allclose(st["pbar"].sum(), 1.0, rtol=1e-13)
    np.testing.assert_allclose(st["u"].sum(), 1.0, rtol=1e-13)
    assert st["counts"].sum() == 64 * 2
    # the loss written as in Sec. 3.3, from scratch
    g = O.dense_gates(r["idx"], r["gates"], 4)
    u = g.mean(axis=0) if lb_mode == O.LB_GATE_MEAN else (g > 0).sum(axis=0) / (64 * 2)
    p = scipy.special.softmax(x @ Wr, axis=1).mean(axis=0)
    np.testing.assert_allclose(st["lb_loss"], 0.01 * 4 * np.sum(u * p), rtol=1e-12)


@pytest.mark.parametrize("lb_mode", [O.LB_TOKEN_FRAC, O.LB_GATE_MEAN])
def test_lb_uniform_routing_gives_alpha(lb_mode):
    """Zero router => uniform softmax; tokens spread evenly => L_LB = alpha."""
    E, T = 4, 8
    probs = np.full((T, E), 1.0 / E)
    idx = np.array([[t % E, (t + 1) % E] for t in range(T)])
    gates = np.full((T, 2), 0.5)
    st = O.lb_statistics(idx, gates, probs, 0.01, lb_mode)
    np.testing.assert_allclose(st["lb_loss"], 0.01, rtol=1e-13)


# --------------------------------------------------------------- backward --
def _loss(x, Wr, b, W1, W3, W2, k, mode, U, dY, forced, alpha, lam, u_frozen, lb_mode, tau=1.0, cf=0.0):
    f = O.moe_forward(x, Wr, b, W1, W3, W2, k, mode, U, alpha, lb_mode, forced_idx=forced, tau=tau,
                      capacity_factor=cf)
    L = np.sum(dY * f["out"])
    if lam != 0.0:
        if u_frozen is None:
            L += lam * f["lb_loss"]
        else:
            L += lam * alpha * len(W1) * np.sum(u_frozen * f["probs"].mean(axis=0))
    return L


@pytest.mark.parametrize("mode,k,lb_mode,through_u", [
    (O.ROUTE_TOPK_RENORM, 2, O.LB_TOKEN_FRAC, False),
    (O.ROUTE_TOPK_RENORM, 2, O.LB_GATE_MEAN, False),
    (O.ROUTE_TOPK_RENORM, 3, O.LB_GATE_MEAN, True),
    (O.ROUTE_SWITCH_TOP1, 1, O.LB_TOKEN_FRAC, False),
    (O.ROUTE_SWITCH_TOP1, 1, O.LB_GATE_MEAN, True),
    (O.ROUTE_SAMPLE_TOP1, 1, O.LB_TOKEN_FRAC, False),
    (O.ROUTE_GUMBEL_TOP1, 1, O.LB_TOKEN_FRAC, False),
    (O.ROUTE_GUMBEL_TOP1, 1, O.LB_GATE_MEAN, True),
])
def test_backward_matches_finite_differences(mode, k, lb_mode, through_u):
    rng = np.random.default_rng(11)
    T, d, f, E = 5, 6, 7, 4
    x, Wr, W1, W3, W2 = tiny_layer(T, d, f, E, rng=rng)
    b = rng.normal(size=E) * 0.3
    U = rng.random(T)
    tau = 1.0
    if mode == O.ROUTE_GUMBEL_TOP1:
        U, tau = -np.log(-np.log(rng.random((T, E)))), 0.6
    dY = rng.normal(size=(T, d))
    alpha, lam = 0.7, 1.3   # large on purpose so that the LB terms are visible
    fwd = O.moe_forward(x, Wr, b, W1, W3, W2, k, mode, U, alpha, lb_mode, tau=tau)
    forced = fwd["idx"].copy()
    u_frozen = None if (through_u or lb_mode == O.LB_TOKEN_FRAC) else fwd["u"].copy()
    g = O.moe_backward(x, Wr, b, W1, W3, W2, k, mode, dY, fwd, alpha, lb_mode, lam, through_u, tau=tau)

    def fd(arr, which, setter):
        num = np.zeros_like(arr)
        eps = 1e-6
        for i in np.ndindex(arr.shape):
            old = arr[i]
            arr[i] = old + eps
            lp = _loss(x, Wr, b, W1, W3, W2, k, mode, U, dY, forced, alpha, lam, u_frozen, lb_mode, tau)
            arr[i] = old - eps
            lm = _loss(x, Wr, b, W1, W3, W2, k, mode, U, dY, forced, alpha, lam, u_frozen, lb_mode, tau)
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        return num

    np.testing.assert_allclose(g["dX"], fd(x, "x", None), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(g["dW_router"], fd(Wr, "Wr", None), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(g["db_router"], fd(b, "b", None), rtol=2e-6, atol=2e-8)
    for e in range(E):
        if np.any(fwd["idx"] == e):
            np.testing.assert_allclose(g["dW1"][e], fd(W1[e], "W1", None), rtol=2e-6, atol=2e-8)
            np.testing.assert_allclose(g["dW3"][e], fd(W3[e], "W3", None), rtol=2e-6, atol=2e-8)
            np.testing.assert_allclose(g["dW2"][e], fd(W2[e], "W2", None), rtol=2e-6, atol=2e-8)


def test_capacity_keeps_the_first_pairs_of_every_expert():
    """Sec. 4.3: a hard limit after which routed tokens are dropped.  Pins: the limit itself,
    service in (token, slot) order, a dropped pair adds nothing to the output, and a limit
    nobody reaches changes nothing."""
    assert O.capacity(10, 1, 4, 1.5) == 4 and O.capacity(16, 2, 4, 1.0) == 8 and O.capacity(7, 1, 4, 0.0) == 0
    rng = np.random.default_rng(3)
    x, Wr, W1, W3, W2 = tiny_layer(T=10, d=6, f=5, E=4, rng=rng)
    b = np.array([9.0, 0.0, 0.0, 0.0])          # everybody wants expert 0
    r = O.route(x, Wr, b, 1, O.ROUTE_SWITCH_TOP1, capacity_factor=1.5)
    assert np.all(r["idx"] == 0)
    np.testing.assert_array_equal(r["dropped"][:, 0], np.arange(10) >= 4)
    f = O.moe_forward(x, Wr, b, W1, W3, W2, 1, O.ROUTE_SWITCH_TOP1, capacity_factor=1.5)
    assert not f["out"][4:].any()
    np.testing.assert_allclose(f["out"][:4], f["gates"][:4] * O.expert_ff(x[:4], W1[0], W3[0], W2[0]), rtol=1e-12)
    np.testing.assert_array_equal(f["counts"], [10, 0, 0, 0])        # statistics see the routing, not the drops
    g = O.grouping(r["idx"], 4, r["dropped"])
    np.testing.assert_array_equal(g["offsets"], [0, 4, 4, 4, 4])
    np.testing.assert_array_equal(g["perm"], [0, 1, 2, 3])
    np.testing.assert_array_equal(g["inv_pos"][:, 0], [0, 1, 2, 3] + [-1] * 6)
    # top-2 in (t, j) order, brute force against the dense layer equation with dropped gates zeroed
    x, Wr, W1, W3, W2 = tiny_layer(T=9, d=6, f=5, E=3, rng=rng)
    r = O.route(x, Wr, None, 2, O.ROUTE_TOPK_RENORM, capacity_factor=0.5)
    cap = O.capacity(9, 2, 3, 0.5)
    assert cap == 3
    seen = np.zeros(3, dtype=int)
    for t in range(9):
        for j in range(2):
            e = r["idx"][t, j]
            assert r["dropped"][t, j] == (seen[e] >= cap)
            seen[e] += not r["dropped"][t, j]
    f = O.moe_forward(x, Wr, None, W1, W3, W2, 2, capacity_factor=0.5)
    dense = O.dense_gates(r["idx"], np.where(r["dropped"], 0.0, r["gates"]), 3)
    want = sum(dense[:, e:e + 1] * O.expert_ff(x, W1[e], W3[e], W2[e]) for e in range(3))
    np.testing.assert_allclose(f["out"], want, rtol=1e-12, atol=1e-14)
    # a sample of the batch evaluated with the whole batch's drop decisions gives the same rows
    sel = np.array([1, 4, 8])
    sub = O.moe_forward(x[sel], Wr, None, W1, W3, W2, 2, forced_idx=r["idx"][sel], forced_dropped=r["dropped"][sel])
    np.testing.assert_allclose(sub["out"], f["out"][sel], rtol=1e-12, atol=1e-14)
    # a limit nobody reaches
    a = O.moe_forward(x, Wr, None, W1, W3, W2, 2, capacity_factor=3.0)
    z = O.moe_forward(x, Wr, None, W1, W3, W2, 2)
    assert not a["dropped"].any()
    np.testing.assert_array_equal(a["out"], z["out"])


@pytest.mark.parametrize("mode,k,cf", [(O.ROUTE_SWITCH_TOP1, 1, 0.75), (O.ROUTE_TOPK_RENORM, 2, 0.5)])
def test_backward_with_dropped_pairs_matches_finite_differences(mode, k, cf):
    rng = np.random.default_rng(17)
    T, d, f, E = 8, 5, 6, 3
    x, Wr, W1, W3, W2 = tiny_layer(T, d, f, E, rng=rng)
    b = rng.normal(size=E) * 0.3
    dY = rng.normal(size=(T, d))
    alpha, lam = 0.7, 1.3
    fwd = O.moe_forward(x, Wr, b, W1, W3, W2, k, mode, None, alpha, O.LB_TOKEN_FRAC, capacity_factor=cf)
    assert fwd["dropped"].any() and not fwd["dropped"].all()
    forced = fwd["idx"].copy()
    g = O.moe_backward(x, Wr, b, W1, W3, W2, k, mode, dY, fwd, alpha, O.LB_TOKEN_FRAC, lam)

    def fd(arr):
        num = np.zeros_like(arr)
        eps = 1e-6
        for i in np.ndindex(arr.shape):
            old = arr[i]
            arr[i] = old + eps
            lp = _loss(x, Wr, b, W1, W3, W2, k, mode, None, dY, forced, alpha, lam, None, O.LB_TOKEN_FRAC, cf=cf)
            arr[i] = old - eps
            lm = _loss(x, Wr, b, W1, W3, W2, k, mode, None, dY, forced, alpha, lam, None, O.LB_TOKEN_FRAC, cf=cf)
            arr[i] = old
            num[i] = (lp - lm) / (2 * eps)
        return num

    np.testing.assert_allclose(g["dX"], fd(x), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(g["dW_router"], fd(Wr), rtol=2e-6, atol=2e-8)
    np.testing.assert_allclose(g["db_router"], fd(b), rtol=2e-6, atol=2e-8)
    for e in range(E):
        np.testing.assert_allclose(g["dW1"][e], fd(W1[e]), rtol=2e-6, atol=2e-8)
        np.testing.assert_allclose(g["dW3"][e], fd(W3[e]), rtol=2e-6, atol=2e-8)
        np.testing.assert_allclose(g["dW2"][e], fd(W2[e]), rtol=2e-6, atol=2e-8)


def test_dW_columns_agrees_with_full_backward_definition_by_loops():
    """dW_columns is pinned by writing the sums out token by token."""
    rng = np.random.default_rng(5)
    x, Wr, W1, W3, W2 = tiny_layer(T=9, d=4, f=6, rng=rng)
    dY = rng.normal(size=x.shape)
    r = O.route(x, Wr, None, 2, O.ROUTE_TOPK_RENORM)
    e = 1
    tt, jj = np.nonzero(r["idx"] == e)
    cols = [0, 4]
    got = O.dW_columns(x, W1[e], W3[e], W2[e], tt, r["gates"][tt, jj], dY, cols)
    dW1 = np.zeros((4, 2)); dW3 = np.zeros((4, 2)); dW2 = np.zeros((2, 4))
    for t, j in zip(tt, jj):
        g = r["gates"][t, j]
        for n, c in enumerate(cols):
            h1 = x[t] @ W1[e][:, c]
            h3 = x[t] @ W3[e][:, c]
            sig = 1 / (1 + np.exp(-h1))
            da = g * (dY[t] @ W2[e][c, :])
            dW2[n] += h1 * sig * h3 * g * dY[t]
            dW1[:, n] += x[t] * da * h3 * (sig * (1 + h1 * (1 - sig)))
            dW3[:, n] += x[t] * da * h1 * sig
    np.testing.assert_allclose(got["dW1"], dW1, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(got["dW3"], dW3, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(got["dW2"], dW2, rtol=1e-11, atol=1e-13)


def test_sampled_backward_with_batch_stats_equals_full_backward_rows():
    rng = np.random.default_rng(9)
    x, Wr, W1, W3, W2 = tiny_layer(T=12, rng=rng)
    dY = rng.normal(size=x.shape)
    fwd = O.moe_forward(x, Wr, None, W1, W3, W2, 2, alpha=0.5)
    full = O.moe_backward(x, Wr, None, W1, W3, W2, 2, 0, dY, fwd, alpha=0.5, lb_grad_scale=1.0)
    sel = np.array([1, 5, 10])
    sub_fwd = O.moe_forward(x[sel], Wr, None, W1, W3, W2, 2, alpha=0.5)
    sub = O.moe_backward(x[sel], Wr, None, W1, W3, W2, 2, 0, dY[sel], sub_fwd, alpha=0.5, lb_grad_scale=1.0,
                         batch_stats={"u": fwd["u"], "pbar": fwd["pbar"], "T": 12}, want_dW=False)
    np.testing.assert_allclose(sub["dX"], full["dX"][sel], rtol=1e-11, atol=1e-13)


# ------------------------------------------------------------ split/merge --
def test_split_chunks_sum_to_the_unsplit_ff():
    x, _, W1, W3, W2 = tiny_layer(T=7, d=8, f=12, E=2)
    s1, s3, s2 = O.split_experts(W1, W3, W2, 3)
    assert len(s1) == 6 and s1[0].shape == (8, 4) and s2[0].shape == (4, 8)
    for i in range(2):
        total = sum(O.expert_ff(x, s1[i * 3 + c], s3[i * 3 + c], s2[i * 3 + c]) for c in range(3))
        np.testing.assert_allclose(total, O.expert_ff(x, W1[i], W3[i], W2[i]), rtol=1e-11, atol=1e-13)
    # zero router, k = E = C on one FF's chunks: uniform gates 1/C => FF(x)/C
    out = O.moe_forward(x, np.zeros((8, 3)), None, s1[:3], s3[:3], s2[:3], 3)["out"]
    np.testing.assert_allclose(out, O.expert_ff(x, W1[0], W3[0], W2[0]) / 3, rtol=1e-11, atol=1e-13)


def test_blend_deals_hidden_units_out_without_changing_their_sum():
    x, _, W1, W3, W2 = tiny_layer(T=5, d=8, f=12, E=3)
    b1, b3, b2 = O.blend_experts(W1, W3, W2)
    assert len(b1) == 3 and b1[0].shape == (8, 12) and b2[0].shape == (12, 8)
    # every hidden unit still exists exactly once: the sum over experts of FF(x) is unchanged
    total = sum(O.expert_ff(x, W1[i], W3[i], W2[i]) for i in range(3))
    blended = sum(O.expert_ff(x, b1[n], b3[n], b2[n]) for n in range(3))
    np.testing.assert_allclose(blended, total, rtol=1e-11, atol=1e-13)
    # expert n holds chunk n of every domain, domain after domain (f/N = 4 columns each)
    np.testing.assert_array_equal(b1[1][:, 8:12], np.asarray(W1[2])[:, 4:8])
    np.testing.assert_array_equal(b2[2][0:4, :], np.asarray(W2[0])[8:12, :])
    # dealing out twice puts every chunk back
    c1, c3, c2 = O.blend_experts(b1, b3, b2)
    for i in range(3):
        np.testing.assert_array_equal(c1[i], W1[i])
        np.testing.assert_array_equal(c3[i], W3[i])
        np.testing.assert_array_equal(c2[i], W2[i])
    # blended expert = what splitting into N chunks and regrouping by chunk index gives
    s1, s3, s2 = O.split_experts(W1, W3, W2, 3)
    for n in range(3):
        np.testing.assert_array_equal(b1[n], np.concatenate([s1[i * 3 + n] for i in range(3)], axis=1))
        np.testing.assert_array_equal(b2[n], np.concatenate([s2[i * 3 + n] for i in range(3)], axis=0))


def test_adamw_step_closed_forms_and_library_routine():
    """Pins of the AdamW update: the first step moves every weight by lr*(sign(g) + wd*p) when
    eps is negligible; a zero gradient leaves pure decay; and a sequence of steps follows
    torch.optim.AdamW (decoupled decay, bias correction) in float64."""
    rng = np.random.default_rng(9)
    p = rng.normal(size=(5, 7))
    g = rng.normal(size=(5, 7))
    z = np.zeros_like(p)
    p1, m1, v1 = O.adamw_step(p, g, z, z, 1, 1e-2, 0.9, 0.95, 1e-30, 0.1)
    np.testing.assert_allclose(p1, p - 1e-2 * (np.sign(g) + 0.1 * p), rtol=1e-12)
    np.testing.assert_allclose(m1, 0.1 * g, rtol=1e-13)
    np.testing.assert_allclose(v1, 0.05 * g * g, rtol=1e-13)
    p0, m0, v0 = O.adamw_step(p, z, z, z, 1, 1e-2, 0.9, 0.95, 1e-8, 0.1)
    np.testing.assert_allclose(p0, p * (1 - 1e-3), rtol=1e-13)
    assert not m0.any() and not v0.any()
    import torch
    tp = torch.tensor(p, dtype=torch.float64, requires_grad=True)
    opt = torch.optim.AdamW([tp], lr=3e-3, betas=(0.9, 0.95), eps=1e-8, weight_decay=0.1)
    po, mo, vo = p, z, z
    for step in range(1, 6):
        gs = rng.normal(size=p.shape)
        tp.grad = torch.tensor(gs, dtype=torch.float64)
        opt.step()
        po, mo, vo = O.adamw_step(po, gs, mo, vo, step, 3e-3, 0.9, 0.95, 1e-8, 0.1)
        np.testing.assert_allclose(po, tp.detach().numpy(), rtol=1e-12, atol=1e-15)


def test_merge_average():
    a = RNG.normal(size=(5, 7)).astype(np.float32)
    for n in (1, 2, 3, 4, 7):
        assert np.array_equal(O.merge_average([a] * n).astype(np.float32), a)
    ints = [np.array([1.0, 2.0, -8.0]), np.array([3.0, 2.0, 4.0]), np.array([5.0, 2.0, 1.0])]
    assert np.array_equal(O.merge_average(ints), np.array([3.0, 2.0, -1.0]))


# ------------------------------------------------------------------ rmsnorm --
def test_rmsnorm_against_the_library_routine_and_its_invariants():
    import torch
    h = RNG.normal(size=(7, 24)) * np.exp(RNG.normal(size=(7, 1)))
    gain = 1.0 + 0.1 * RNG.normal(size=24)
    xn, rstd = O.rmsnorm(h, gain, 1e-5)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(h), (24,), torch.from_numpy(gain), 1e-5).numpy()
    np.testing.assert_allclose(xn, ref, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt((h * h).mean(axis=1) + 1e-5), rtol=1e-14)
    # unit gain, no eps: every row has mean square 1, and scaling a row changes nothing
    x1, _ = O.rmsnorm(h, np.ones(24), 0.0)
    np.testing.assert_allclose((x1 * x1).mean(axis=1), 1.0, rtol=1e-13)
    x2, _ = O.rmsnorm(h * np.array([[3.0], [0.5], [7.0], [1.0], [2.0], [11.0], [0.25]]), np.ones(24), 0.0)
    np.testing.assert_allclose(x2, x1, rtol=1e-13, atol=1e-15)


def test_rmsnorm_backward_against_autograd_finite_differences_and_loops():
    import torch
    T, d, eps = 5, 12, 1e-5
    h = RNG.normal(size=(T, d))
    gain = 1.0 + 0.2 * RNG.normal(size=d)
    dxn = RNG.normal(size=(T, d))
    dh, dgain = O.rmsnorm_backward(dxn, h, gain, eps)
    # library autodiff of the library routine
    th = torch.from_numpy(h).requires_grad_(True)
    tg = torch.from_numpy(gain).requires_grad_(True)
    (torch.nn.functional.rms_norm(th, (d,), tg, eps) * torch.from_numpy(dxn)).sum().backward()
    np.testing.assert_allclose(dh, th.grad.numpy(), rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(dgain, tg.grad.numpy(), rtol=1e-11, atol=1e-13)
    # central differences on L = sum(dxn * xn)
    loss = lambda hh, gg: float((O.rmsnorm(hh, gg, eps)[0] * dxn).sum())
    for (t, c) in [(0, 0), (2, 5), (4, 11)]:
        e = np.zeros_like(h); e[t, c] = 1e-6
        assert abs((loss(h + e, gain) - loss(h - e, gain)) / 2e-6 - dh[t, c]) < 1e-7
    for c in (0, 7):
        e = np.zeros_like(gain); e[c] = 1e-6
        assert abs((loss(h, gain + e) - loss(h, gain - e)) / 2e-6 - dgain[c]) < 1e-7
    # dgain by loops
    rstd = 1.0 / np.sqrt((h * h).mean(axis=1) + eps)
    for c in (1, 9):
        assert abs(sum(dxn[t, c] * h[t, c] * rstd[t] for t in range(T)) - dgain[c]) < 1e-12
    # with unit gain and no eps the output does not depend on the length of h: dh is orthogonal to h
    dh0, _ = O.rmsnorm_backward(dxn, h, np.ones(d), 0.0)
    np.testing.assert_allclose((dh0 * h).sum(axis=1), 0.0, atol=1e-13)


def test_merge_weighted():
    """Pins: a one-hot weight selects that model; uniform weights 1/N (exact in binary) give the
    mean; small integers come out exactly; np.average (a library routine) agrees when the
    weights sum to one; the result is linear in the weights."""
    ts = [RNG.normal(size=(6, 5)) for _ in range(4)]
    assert np.array_equal(O.merge_weighted(ts, [0, 0, 1, 0]), ts[2])
    assert np.array_equal(O.merge_weighted(ts, [0.25] * 4), O.merge_average(ts))
    ints = [np.array([1.0, 2.0, -8.0]), np.array([3.0, 2.0, 4.0])]
    assert np.array_equal(O.merge_weighted(ints, [2.0, -1.0]), np.array([-1.0, 2.0, -20.0]))
    w = [0.5, 0.25, 0.125, 0.125]
    np.testing.assert_allclose(O.merge_weighted(ts, w), np.average(np.stack(ts), axis=0, weights=w), rtol=1e-14)
    w2 = [0.1, -0.3, 0.7, 0.2]
    np.testing.assert_allclose(O.merge_weighted(ts, [a + 2 * b for a, b in zip(w, w2)]),
                               O.merge_weighted(ts, w) + 2 * O.merge_weighted(ts, w2), rtol=1e-13, atol=1e-15)


def test_round_to_bf16_matches_torch_and_rounds_once():
    import torch
    v = RNG.normal(size=10000) * np.exp(RNG.normal(size=10000) * 5)
    v32 = v.astype(np.float32).astype(np.float64)     # exactly representable in fp32 => torch rounds once too
    ref = torch.from_numpy(v32.astype(np.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(O.round_to_bf16(v32), ref)
    # a value just above a bf16 tie must round up although fp32 would first hide the excess
    tie = 1.0 + 2.0 ** -8
    assert O.round_to_bf16(np.array([tie]))[0] == 1.0                      # tie -> even
    assert O.round_to_bf16(np.array([tie + 2.0 ** -40]))[0] == np.float32(1.0 + 2.0 ** -7)
    assert O.round_to_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == np.float32(1.0 + 2.0 ** -6)


def test_three_matrix_ff_matches_table4_active_params():
    """Table 4 prints 6.7 / 11.1 / 19.7 B active parameters for 1 / 2 / 4
    active experts; the differences fix the FF as three 4096 x 11008 matrices
    per expert in each of 32 layers."""
    path = os.path.join(os.path.dirname(__file__), "golden", "table4_active_params.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    printed = {int(k): float(v) for k, v in rows}
    base = printed[1] * 1e9 - O.ff_active_params(4096, 11008, 1, 32)
    for k, v in printed.items():
        total = base + O.ff_active_params(4096, 11008, k, 32)
        # both printed numbers are rounded to 0.1, so allow 0.05 + 0.05; a 2-matrix FF would miss by 1.4
        assert abs(total / 1e9 - v) <= 0.1001, (k, total)


def test_capacity_is_taken_on_the_number_that_is_passed():
    """ceil(cf * T*k / E) is sensitive to the last bit of cf when the product is an integer: 0.8 gives
    208 rows at T*k/E = 260, the float32 nearest to 0.8 (what a C float argument carries) 209."""
    assert O.capacity(1040, 1, 4, 0.8) == 208
    assert O.capacity(1040, 1, 4, float(np.float32(0.8))) == 209
    assert O.capacity(1040, 1, 4, 1.25) == 325 and O.capacity(1041, 1, 4, 1.25) == 326
    assert O.capacity(16384, 1, 4, 1.5) == 6144 and O.capacity(900, 1, 4, 1.5) == 338
