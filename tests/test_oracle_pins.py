"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle itself.

Every test here runs on the CPU only.  Citations name the passage of the paper that fixes the
property being checked.
"""
import json
import math
import os

import numpy as np
import pytest

from oracle import wersa_oracle as wo

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(seed, B=2, H=2, n=64, d=4, m=16, L=3, q_mean=0.7):
    r = np.random.default_rng(seed)
    p = dict(
        Q=r.standard_normal((B, H, n, d)) + q_mean,
        K=r.standard_normal((B, H, n, d)),
        V=r.standard_normal((B, H, n, d)),
        Omega=r.standard_normal((d, m)),
        sigma=1.3,
        Wg=r.standard_normal((H, L + 1, d)),
        bg=0.1 * r.standard_normal((H, L + 1)),
        omega=1.0 + 0.1 * r.standard_normal(L + 1),
        L=L,
    )
    p["dO"] = r.standard_normal((B, H, n, d))
    return p


# ---------------------------------------------------------------- Haar transform
def test_haar_hand_example():
    """Appendix A analysis equations worked by hand on an 8-sample signal."""
    with open(os.path.join(GOLDEN, "haar_hand_example.json")) as f:
        g = json.load(f)
    x = np.array(g["x"], float)[:, None]
    coeffs, n = wo.haar_dwt(x, g["L"])
    s2 = math.sqrt(2.0)
    assert n == 8
    np.testing.assert_allclose(coeffs[0][:, 0] * s2, g["d1_times_sqrt2"], atol=1e-14)
    np.testing.assert_allclose(coeffs[1][:, 0], g["d2"], atol=1e-14)
    np.testing.assert_allclose(coeffs[2][:, 0] * s2, g["d3_times_sqrt2"], atol=1e-14)
    np.testing.assert_allclose(coeffs[3][:, 0] * s2, g["a3_times_sqrt2"], atol=1e-14)
    assert abs(sum(float(np.sum(c * c)) for c in coeffs) - g["energy"]) < 1e-12
    low = wo.haar_filter(x, np.array([0.0, 0.0, 0.0, 1.0]), 3)
    np.testing.assert_allclose(low[:, 0], g["lowpass_only_reconstruction"], atol=1e-14)


@pytest.mark.parametrize("n,L", [(64, 3), (256, 6), (128, 1), (48, 3), (100, 2), (8, 3)])
def test_perfect_reconstruction_and_energy(n, L):
    """Appendix A inverse equations undo the analysis; the transform is orthonormal."""
    x = np.random.default_rng(n + L).standard_normal((n, 5))
    coeffs, n0 = wo.haar_dwt(x, L)
    assert n0 == n and len(coeffs) == L + 1
    # band sizes: d_l has npad / 2^l rows (Algorithm 2 return order d_1..d_L, a_L)
    npad = coeffs[0].shape[0] * 2
    for l in range(1, L + 1):
        assert coeffs[l - 1].shape[0] == npad >> l
    assert coeffs[L].shape[0] == npad >> L
    np.testing.assert_allclose(wo.haar_idwt(coeffs, n), x, atol=1e-13)
    np.testing.assert_allclose(wo.haar_filter(x, np.ones(L + 1), L), x, atol=1e-13)
    e_x = np.sum(x * x)
    e_c = sum(np.sum(c * c) for c in coeffs)
    assert abs(e_x - e_c) < 1e-10 * e_x


def _block_mean(x, size):
    """Replace every aligned block of `size` rows by its mean (zero padding the tail)."""
    n = x.shape[0]
    npad = -(-n // size) * size
    xp = np.zeros((npad,) + x.shape[1:])
    xp[:n] = x
    mean = xp.reshape(npad // size, size, -1).mean(axis=1, keepdims=True)
    return np.broadcast_to(mean, (npad // size, size, xp.shape[1])).reshape(npad, -1)[:n]


@pytest.mark.parametrize("n,L", [(64, 3), (256, 6), (48, 3), (100, 2), (192, 5), (300, 7), (1000, 9), (700, 12)])
def test_block_mean_closed_form(n, L):
    """Gated Haar filter == F_0 x + sum_l (F_l - F_{l-1}) * (mean over aligned 2^l blocks).

    Follows from the Haar scaling function being an indicator (Appendix A): the level-l
    approximation is 2^{l/2} times the block mean.  Fixes the band order of F and shows the
    result does not depend on how far beyond a multiple of 2^L the signal is zero padded.
    """
    r = np.random.default_rng(7 * n + L)
    x = r.standard_normal((n, 3))
    F = r.uniform(0.1, 1.5, L + 1)
    ref = F[0] * x
    for l in range(1, L + 1):
        ref = ref + (F[l] - F[l - 1]) * _block_mean(x, 1 << l)
    np.testing.assert_allclose(wo.haar_filter(x, F, L), ref, atol=1e-13)


def test_filter_special_cases_and_symmetry():
    r = np.random.default_rng(3)
    n, L = 128, 4
    x, y = r.standard_normal((n, 6)), r.standard_normal((n, 6))
    np.testing.assert_allclose(wo.haar_filter(x, np.full(L + 1, 0.37), L), 0.37 * x, atol=1e-13)
    only_a = np.zeros(L + 1)
    only_a[L] = 1.0
    np.testing.assert_allclose(wo.haar_filter(x, only_a, L), _block_mean(x, 1 << L), atol=1e-13)
    only_d1 = np.zeros(L + 1)
    only_d1[0] = 1.0
    np.testing.assert_allclose(wo.haar_filter(x, only_d1, L), x - _block_mean(x, 2), atol=1e-13)
    F = r.uniform(0, 1, L + 1)
    lhs = np.sum(wo.haar_filter(x, F, L) * y)
    rhs = np.sum(x * wo.haar_filter(y, F, L))
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)


# ---------------------------------------------------------------- gate
def test_gate_formula():
    """F_i = sigmoid(g(Q_avg)_i) * omega_i with a linear g (Section 3.1 step 4)."""
    r = np.random.default_rng(5)
    qbar, W, b, om = r.standard_normal(6), r.standard_normal((4, 6)), r.standard_normal(4), r.uniform(0.5, 2, 4)
    logits, s, F = wo.gate(qbar, W, b, om)
    for i in range(4):
        zi = sum(W[i, j] * qbar[j] for j in range(6)) + b[i]
        assert abs(logits[i] - zi) < 1e-14
        assert abs(s[i] - math.exp(zi) / (1 + math.exp(zi))) < 1e-14
        assert abs(F[i] - om[i] * s[i]) < 1e-14
    # zero logits give sigmoid 1/2
    _, s0, F0 = wo.gate(qbar, 0 * W, 0 * b, om)
    np.testing.assert_allclose(s0, 0.5)
    np.testing.assert_allclose(F0, 0.5 * om)


# ---------------------------------------------------------------- linear attention
@pytest.mark.parametrize("n", [32, 200])
def test_linear_attention_equals_explicit_kernel_matrix(n):
    """Appendix A linear attention identity and the Section 3.1 attention equation:
    phi(Q)(phi(K)^T V) / (phi(Q) phi(K)^T 1 + eps) equals the explicit n x n product."""
    L = 3
    p = _rand_problem(11, B=1, H=1, n=n, d=8, m=32, L=L)
    eps = 1e-3
    f = wo.forward_slice(p["Q"][0, 0], p["K"][0, 0], p["V"][0, 0], p["Omega"], p["sigma"],
                         p["Wg"][0], p["bg"][0], p["omega"], L, eps, 1e-6)
    # independent recomputation: explicit attention matrix, entry by entry feature products
    m = p["Omega"].shape[1]
    QF = wo.haar_filter(p["Q"][0, 0], f["F"], L)
    KF = wo.haar_filter(p["K"][0, 0], f["F"], L)
    pq = np.maximum(QF @ p["Omega"] / p["sigma"], 0) / math.sqrt(m)
    pk = np.maximum(KF @ p["Omega"] / p["sigma"], 0) / math.sqrt(m)
    A = np.zeros((n, n))
    for i in range(n):
        for j in range(n):
            A[i, j] = float(np.dot(pq[i], pk[j]))
    O_ref = (A @ p["V"][0, 0]) / (A.sum(axis=1) + eps)[:, None]
    np.testing.assert_allclose(f["O"], O_ref, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(f["D"], A.sum(axis=1) + eps, rtol=1e-12)


def test_convexity_and_unit_values():
    """phi >= 0, so with eps = 0 each output row is a convex combination of rows of V."""
    p = _rand_problem(13, B=1, H=1, n=96, d=8, m=64, L=2)
    args = (p["Q"][0, 0], p["K"][0, 0])
    tail = (p["Omega"], p["sigma"], p["Wg"][0], p["bg"][0], p["omega"], 2)
    f = wo.forward_slice(*args, p["V"][0, 0], *tail, 0.0, 1e-6)
    V = p["V"][0, 0]
    assert np.all(f["O"] <= V.max(axis=0)[None, :] + 1e-12)
    assert np.all(f["O"] >= V.min(axis=0)[None, :] - 1e-12)
    eps = 0.05
    f1 = wo.forward_slice(*args, np.ones_like(V), *tail, eps, 1e-6)
    np.testing.assert_allclose(f1["O"], ((f1["D"] - eps) / f1["D"])[:, None] * np.ones_like(V), rtol=1e-12)


# ---------------------------------------------------------------- random features
def _arccos_kernel(q, k, sigma):
    """E_w[relu(q.w/sigma) relu(k.w/sigma)], w ~ N(0, I): degree-1 arc-cosine kernel (textbook)."""
    nq, nk = np.linalg.norm(q), np.linalg.norm(k)
    th = math.acos(max(-1.0, min(1.0, float(q @ k) / (nq * nk))))
    return nq * nk * (math.sin(th) + (math.pi - th) * math.cos(th)) / (2 * math.pi * sigma ** 2)


def test_random_feature_kernel_converges_at_rate_inv_sqrt_m():
    """Appendix B, random-features bullet: E|phi(q)^T phi(k) - kappa| <= C / sqrt(m).

    phi(q)^T phi(k) with the 1/sqrt(m) scaling and the bandwidth is a Monte-Carlo estimate of
    the ReLU-feature expectation; its RMS error must fall like m^-1/2.
    """
    r = np.random.default_rng(17)
    d, sigma = 8, 1.7
    q, k = r.standard_normal(d), r.standard_normal(d)
    target = _arccos_kernel(q, k, sigma)
    ms = [64, 256, 1024, 4096, 16384]
    rms = []
    for m in ms:
        errs = []
        for s in range(24):
            Om = np.random.default_rng(1000 * m + s).standard_normal((d, m))
            _, pq = wo.feature_map(q[None, :], Om, sigma, 1e-6)
            _, pk = wo.feature_map(k[None, :], Om, sigma, 1e-6)
            errs.append(float(pq[0] @ pk[0]) - target)
        rms.append(math.sqrt(np.mean(np.square(errs))))
    slope = np.polyfit(np.log(ms), np.log(rms), 1)[0]
    assert -0.65 < slope < -0.35, (slope, rms)
    assert rms[-1] < 0.03 * abs(target), (rms, target)


def test_bandwidth_floor():
    """Algorithm 1 bandwidth line: bw = max(beta, floor)."""
    x = np.random.default_rng(2).standard_normal((5, 4))
    Om = np.random.default_rng(3).standard_normal((4, 8))
    U1, _ = wo.feature_map(x, Om, 1e-9, 0.5)
    U2, _ = wo.feature_map(x, Om, 0.5, 1e-6)
    np.testing.assert_allclose(U1, U2)


# ---------------------------------------------------------------- homogeneity in sigma
def test_sigma_homogeneity_and_closed_form_dsigma():
    """ReLU is positively homogeneous: with eps = 0 the output does not depend on sigma, and
    with eps > 0 d loss / d sigma = (2 eps / sigma) * sum_t dD_t."""
    p = _rand_problem(19)
    common = dict(Omega=p["Omega"], Wg=p["Wg"], bg=p["bg"], omega=p["omega"], L=p["L"])
    o1 = wo.forward(p["Q"], p["K"], p["V"], sigma=0.8, eps=0.0, **common)["O"]
    o2 = wo.forward(p["Q"], p["K"], p["V"], sigma=2.9, eps=0.0, **common)["O"]
    np.testing.assert_allclose(o1, o2, rtol=1e-10, atol=1e-12)
    eps = 1e-2
    g = wo.backward(p["Q"], p["K"], p["V"], sigma=p["sigma"], dO=p["dO"], eps=eps, **common)
    closed = 2.0 * eps / p["sigma"] * g["dD_sum"]
    assert abs(g["dsigma"] - closed) < 1e-9 * max(1.0, abs(closed))
    # a common rescaling of all F_i acts like 1/sigma: sum_i omega_i * domega_i == -sigma * dsigma
    # holds only without the pooled path, i.e. d/d(log c) of F -> cF equals -d/d(log sigma)
    assert abs(float(np.sum(p["omega"] * g["domega"])) + p["sigma"] * g["dsigma"]) < 1e-9


# ---------------------------------------------------------------- finite differences
def _loss(p, eps, **over):
    q = dict(p)
    q.update(over)
    O = wo.forward(q["Q"], q["K"], q["V"], q["Omega"], q["sigma"], q["Wg"], q["bg"], q["omega"],
                   q["L"], eps=eps)["O"]
    return float(np.sum(O * p["dO"]))


@pytest.mark.parametrize("n,L", [(64, 3), (40, 2)])
def test_backward_matches_central_finite_differences(n, L):
    """The backward is the derivative of the forward: central differences in float64 on a tiny
    problem with a shifted Q (so the pooled-query path matters), two batches and two heads (so
    the cross-slice sums of the parameter gradients are exercised), and n = 40 (zero padding)."""
    eps = 1e-2
    p = _rand_problem(23 + n, n=n, L=L)
    g = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"],
                    L, p["dO"], eps=eps)
    h = 1e-6
    r = np.random.default_rng(99)

    def check(name, gname, count):
        arr = p[name]
        flat_idx = r.choice(arr.size, size=min(count, arr.size), replace=False)
        for fi in flat_idx:
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            fd = (_loss(p, eps, **{name: ap}) - _loss(p, eps, **{name: am})) / (2 * h)
            an = g[gname][idx]
            assert abs(fd - an) < 2e-6 * max(1.0, abs(an)), (name, idx, fd, an)

    check("Q", "dQ", 12)
    check("K", "dK", 12)
    check("V", "dV", 8)
    check("Wg", "dWg", 10)
    check("bg", "dbg", 8)
    check("omega", "domega", L + 1)
    fd = (_loss(p, eps, sigma=p["sigma"] + h) - _loss(p, eps, sigma=p["sigma"] - h)) / (2 * h)
    assert abs(fd - g["dsigma"]) < 2e-6 * max(1.0, abs(fd))


# ---------------------------------------------------------------- ablation special cases
def test_ablation_special_cases():
    """Appendix E switches as special cases: all filters 1 is plain ReLU-feature linear attention
    on the unfiltered Q, K; zero gate weights make F independent of Q."""
    p = _rand_problem(29, B=1, H=1, n=64, d=4, m=16, L=3)
    Q, K, V = p["Q"][0, 0], p["K"][0, 0], p["V"][0, 0]
    # F == 1: huge bias saturates the sigmoid, omega = 1
    big = np.full(4, 50.0)
    f = wo.forward_slice(Q, K, V, p["Omega"], 1.0, 0 * p["Wg"][0], big, np.ones(4), 3, 1e-6, 1e-6)
    m = 16
    pq = np.maximum(Q @ p["Omega"], 0) / math.sqrt(m)
    pk = np.maximum(K @ p["Omega"], 0) / math.sqrt(m)
    ref = (pq @ (pk.T @ V)) / ((pq @ pk.sum(axis=0)) + 1e-6)[:, None]
    np.testing.assert_allclose(f["O"], ref, rtol=1e-9)
    # Wg == 0: gradient through the pooled query vanishes, dWg is still dlogits x qbar
    g0 = wo.backward_slice(Q, K, V, p["Omega"], 1.0, 0 * p["Wg"][0], p["bg"][0], p["omega"], 3,
                           1e-6, 1e-6, p["dO"][0, 0])
    QF = wo.haar_filter(Q, g0["dF"] * 0 + wo.gate(Q.mean(0), 0 * p["Wg"][0], p["bg"][0], p["omega"])[2], 3)
    # with Wg = 0, dQ is exactly the filter applied to dQ_F (self-adjoint operator)
    F = wo.gate(Q.mean(0), 0 * p["Wg"][0], p["bg"][0], p["omega"])[2]
    np.testing.assert_allclose(g0["dQ"], wo.haar_filter(g0["dQF"], F, 3), atol=1e-12)
    assert QF.shape == Q.shape


# ---------------------------------------------------------------- attention block
def _rand_block(seed, B=2, H=2, n=16, d=3, m=8, L=2):
    r = np.random.default_rng(seed)
    hidden = H * d
    p = _rand_problem(seed + 1, B=B, H=H, n=n, d=d, m=m, L=L)
    p.update(X=r.standard_normal((B, n, hidden)) + 0.3,
             WQ=r.standard_normal((hidden, hidden)) / math.sqrt(hidden),
             WK=r.standard_normal((hidden, hidden)) / math.sqrt(hidden),
             WV=r.standard_normal((hidden, hidden)) / math.sqrt(hidden),
             WO=r.standard_normal((hidden, hidden)) / math.sqrt(hidden),
             dY=r.standard_normal((B, n, hidden)), H=H)
    return p


def _block_args(p, **over):
    q = dict(p, **over)
    return (q["X"], q["WQ"], q["WK"], q["WV"], q["WO"], q["H"], q["Omega"], q["sigma"], q["Wg"],
            q["bg"], q["omega"], q["L"])


def test_block_head_layout_and_identity_weights():
    """Section 3.1 step 2: head h owns columns [h d, (h+1) d).  With identity projections the
    block is the core applied to the head-split input, so it is pinned to the pinned core; a
    column permutation folded into W^out must permute the output columns the same way."""
    p = _rand_block(41)
    hidden = p["X"].shape[2]
    eye = np.eye(hidden)
    H, d = p["H"], hidden // p["H"]
    f = wo.block_forward(*_block_args(p, WQ=eye, WK=eye, WV=eye, WO=eye), eps=1e-3)
    for b in range(p["X"].shape[0]):
        for h in range(H):
            xs = p["X"][b][:, h * d:(h + 1) * d]
            s = wo.forward_slice(xs, xs, xs, p["Omega"], p["sigma"], p["Wg"][h], p["bg"][h],
                                 p["omega"], p["L"], 1e-3, 1e-6)
            np.testing.assert_allclose(f["Y"][b][:, h * d:(h + 1) * d], s["O"], rtol=1e-12, atol=1e-14)
    perm = np.random.default_rng(5).permutation(hidden)
    fp = wo.block_forward(*_block_args(p, WQ=eye, WK=eye, WV=eye, WO=eye[:, perm]), eps=1e-3)
    np.testing.assert_allclose(fp["Y"], f["Y"][:, :, perm], rtol=1e-12, atol=1e-14)
    # split and merge are inverse to each other
    T = np.random.default_rng(6).standard_normal((2, 5, hidden))
    np.testing.assert_array_equal(wo.merge_heads(wo.split_heads(T, H)), T)


def test_block_is_linear_in_value_and_output_weights():
    """Y is linear in W^V and in W^out (the normaliser does not depend on V)."""
    p = _rand_block(43)
    y1 = wo.block_forward(*_block_args(p), eps=1e-3)["Y"]
    y2 = wo.block_forward(*_block_args(p, WV=2.5 * p["WV"]), eps=1e-3)["Y"]
    y3 = wo.block_forward(*_block_args(p, WO=-0.5 * p["WO"]), eps=1e-3)["Y"]
    np.testing.assert_allclose(y2, 2.5 * y1, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(y3, -0.5 * y1, rtol=1e-11, atol=1e-13)


def test_block_backward_matches_central_finite_differences():
    """Every gradient of the block against central differences of its forward (float64)."""
    eps = 1e-2
    p = _rand_block(47)
    g = wo.block_backward(*_block_args(p), p["dY"], eps=eps)
    h = 1e-6
    r = np.random.default_rng(3)

    def loss(**over):
        return float(np.sum(wo.block_forward(*_block_args(p, **over), eps=eps)["Y"] * p["dY"]))

    for name, gname, count in (("X", "dX", 12), ("WQ", "dWQ", 8), ("WK", "dWK", 8), ("WV", "dWV", 8),
                               ("WO", "dWO", 8), ("Wg", "dWg", 6), ("bg", "dbg", 4),
                               ("omega", "domega", 3)):
        arr = p[name]
        for fi in r.choice(arr.size, size=min(count, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h)
            an = g[gname][idx]
            assert abs(fd - an) < 3e-6 * max(1.0, abs(an)), (name, idx, fd, an)
    fd = (loss(sigma=p["sigma"] + h) - loss(sigma=p["sigma"] - h)) / (2 * h)
    assert abs(fd - g["dsigma"]) < 3e-6 * max(1.0, abs(fd))


# ---------------------------------------------------------------- the pins bite
def test_projection_rounding_hook_changes_only_what_it_says():
    """`proj_dtype` of the feature map (used by the GPU tests so that both sides take the ReLU
    decision of Section 3.1 step 7 on the same numbers): None and float64 are the same function
    bit for bit; float16 equals rounding X_F by hand before the unchanged map, moves U by at most
    2^-11 |X_F| |Omega| / sigma entry by entry, and touches nothing upstream of the projection."""
    r = np.random.default_rng(71)
    XF = r.standard_normal((40, 6)) * 3.0
    Om = r.standard_normal((6, 24))
    U0, P0 = wo.feature_map(XF, Om, 1.3, 1e-6)
    U64, P64 = wo.feature_map(XF, Om, 1.3, 1e-6, np.float64)
    assert np.array_equal(U0, U64) and np.array_equal(P0, P64)
    U16, P16 = wo.feature_map(XF, Om, 1.3, 1e-6, np.float16)
    Uh, Ph = wo.feature_map(XF.astype(np.float16).astype(np.float64), Om, 1.3, 1e-6)
    assert np.array_equal(U16, Uh) and np.array_equal(P16, Ph)
    bound = 2.0 ** -11 * (np.abs(XF) @ np.abs(Om)) / 1.3
    assert np.all(np.abs(U16 - U0) <= bound * (1 + 1e-12))
    assert np.any(U16 != U0)                       # it does round
    # through the whole forward: everything up to X_F is untouched, float64 is the identity
    p = _rand_problem(73, B=1, H=1, n=48, d=6, m=24, L=3)
    args = (p["Q"][0, 0], p["K"][0, 0], p["V"][0, 0], p["Omega"], p["sigma"], p["Wg"][0], p["bg"][0], p["omega"],
            p["L"], 1e-4, 1e-6)
    f0, f64, f16 = (wo.forward_slice(*args, proj_dtype=t) for t in (None, np.float64, np.float16))
    for name in f0:
        assert np.array_equal(f0[name], f64[name]), name
    for name in ("qbar", "logits", "s", "F", "QF", "KF"):
        assert np.array_equal(f0[name], f16[name]), name
    np.testing.assert_array_equal(f16["UQ"], wo.feature_map(f0["QF"].astype(np.float16).astype(np.float64),
                                                            p["Omega"], p["sigma"], 1e-6)[0])
    assert 0 < np.max(np.abs(f16["O"] - f0["O"])) < 1e-2
    # and through the backward: float64 is the identity there too
    g0 = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], p["L"], p["dO"])
    g64 = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], p["L"], p["dO"],
                      proj_dtype=np.float64)
    for name in ("O", "dQ", "dK", "dV", "dWg", "dbg", "domega"):
        assert np.array_equal(g0[name], g64[name]), name


def test_block_store_hook_is_applied_where_it_says_and_nowhere_else():
    """`store` of the block functions (a GPU test rounds the stored intermediates to bf16 with it):
    the identity hook equals no hook bit for bit; a marking hook is called on exactly Q', K', V', A
    (forward) and additionally dA, dQ', dK', dV' (backward), in that order, each with the value the
    unhooked run holds at that point when the hook returns its argument unchanged."""
    p = _rand_block(75)
    f0 = wo.block_forward(*_block_args(p))
    fi = wo.block_forward(*_block_args(p), store=lambda a: a)
    for name in f0:
        assert np.array_equal(f0[name], fi[name]), name
    seen = []

    def mark(a):
        seen.append(np.array(a, copy=True))
        return a
    wo.block_forward(*_block_args(p), store=mark)
    assert len(seen) == 4
    for got, name in zip(seen, ("Qp", "Kp", "Vp", "A")):
        assert np.array_equal(got, f0[name]), name
    g0 = wo.block_backward(*_block_args(p), p["dY"])
    seen.clear()
    gi = wo.block_backward(*_block_args(p), p["dY"], store=mark)
    for name in g0:
        assert np.array_equal(np.asarray(g0[name]), np.asarray(gi[name])), name
    assert len(seen) == 8
    for got, name in zip(seen, ("Qp", "Kp", "Vp", "A", "dA", "dQp", "dKp", "dVp")):
        assert np.array_equal(got, g0[name]), name
    # a hook that does change its argument changes the result (it is really in the data path)
    rb = lambda a: a.astype(np.float16).astype(np.float64)
    gr = wo.block_backward(*_block_args(p), p["dY"], store=rb)
    assert np.array_equal(gr["Qp"], rb(g0["Qp"]))
    assert 0 < np.max(np.abs(gr["dX"] - g0["dX"])) < 5e-2 * np.max(np.abs(g0["dX"]))


def test_planted_mistakes_are_caught(monkeypatch):
    """Each plausible mistake, planted in the oracle (on the CPU), must fail at least one pin:
    a swapped Haar pair sign, a dropped 1/sqrt(2), a transposed operand in S, a dropped epsilon,
    a missing 1/sqrt(m), a wrong band order of the filter."""
    import oracle.wersa_oracle as mod

    def expect_failure(pins):
        failed = 0
        for pin in pins:
            try:
                pin()
            except AssertionError:
                failed += 1
        assert failed >= 1, "no pin noticed the planted mistake"

    haar_pins = [test_haar_hand_example, lambda: test_perfect_reconstruction_and_energy(64, 3),
                 lambda: test_block_mean_closed_form(64, 3)]
    attn_pins = [lambda: test_linear_attention_equals_explicit_kernel_matrix(16),
                 test_random_feature_kernel_converges_at_rate_inv_sqrt_m, test_convexity_and_unit_values]

    # 1. detail = (odd - even)/sqrt(2) instead of (even - odd)/sqrt(2)
    real_dwt = mod.haar_dwt

    def dwt_wrong_sign(X, L):
        coeffs, n = real_dwt(X, L)
        return [-c for c in coeffs[:-1]] + [coeffs[-1]], n
    monkeypatch.setattr(mod, "haar_dwt", dwt_wrong_sign)
    expect_failure(haar_pins)
    monkeypatch.setattr(mod, "haar_dwt", real_dwt)

    # 2. analysis without the 1/sqrt(2) normalisation
    def dwt_unnormalised(X, L):
        coeffs, n = real_dwt(X, L)
        return [c * mod.SQRT2 for c in coeffs], n
    monkeypatch.setattr(mod, "haar_dwt", dwt_unnormalised)
    expect_failure(haar_pins)
    monkeypatch.setattr(mod, "haar_dwt", real_dwt)

    # 3. filter applied with the band order reversed
    real_fidwt = mod.filtered_idwt
    monkeypatch.setattr(mod, "filtered_idwt", lambda coeffs, F, n: real_fidwt(coeffs, F[::-1], n))
    expect_failure([lambda: test_block_mean_closed_form(64, 3), test_filter_special_cases_and_symmetry])
    monkeypatch.setattr(mod, "filtered_idwt", real_fidwt)

    # 4. feature map without the 1/sqrt(m) factor, and with the bandwidth multiplied instead of divided
    real_fm = mod.feature_map

    def fm_no_sqrt_m(XF, Omega, sigma, bw_floor, proj_dtype=None):
        U, Phi = real_fm(XF, Omega, sigma, bw_floor, proj_dtype)
        return U, Phi * math.sqrt(Omega.shape[1])
    monkeypatch.setattr(mod, "feature_map", fm_no_sqrt_m)
    expect_failure(attn_pins)

    def fm_bandwidth_inverted(XF, Omega, sigma, bw_floor, proj_dtype=None):
        return real_fm(XF, Omega, 1.0 / max(sigma, bw_floor), bw_floor, proj_dtype)
    monkeypatch.setattr(mod, "feature_map", fm_bandwidth_inverted)
    expect_failure([test_bandwidth_floor, test_sigma_homogeneity_and_closed_form_dsigma] + attn_pins)
    monkeypatch.setattr(mod, "feature_map", real_fm)

    # 5. a backward with one term dropped (the pooled-query path) fails the finite differences
    real_bwd = mod.backward_slice

    def bwd_no_pooled_path(*args, **kw):
        r = real_bwd(*args, **kw)
        Q, L = args[0], args[8]
        r = dict(r)
        r["dQ"] = mod.haar_filter(r["dQF"], mod.gate(Q.mean(0), args[5], args[6], args[7])[2], L)
        return r
    monkeypatch.setattr(mod, "backward_slice", bwd_no_pooled_path)
    expect_failure([lambda: test_backward_matches_central_finite_differences(64, 3)])
    monkeypatch.setattr(mod, "backward_slice", real_bwd)

    # 6. head split that interleaves heads instead of giving each a contiguous column block
    real_split = mod.split_heads

    def split_interleaved(T, H):
        B, n, hidden = T.shape
        return T.reshape(B, n, hidden // H, H).transpose(0, 3, 1, 2)
    monkeypatch.setattr(mod, "split_heads", split_interleaved)
    expect_failure([test_block_head_layout_and_identity_weights])
    monkeypatch.setattr(mod, "split_heads", real_split)

    # 7. a transposed operand in the KV reduction: S = phi(K) V in place of phi(K)^T V (the shapes
    #    still agree when n == m), everything after it computed from that S
    real_fwd = mod.forward_slice

    def fwd_transposed_S(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, *a, **kw):
        f = dict(real_fwd(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, *a, **kw))
        assert f["PhiK"].shape[0] == f["PhiK"].shape[1], "the planted mistake needs n == m"
        f["S"] = f["PhiK"] @ np.asarray(V, np.float64)
        f["N"] = f["PhiQ"] @ f["S"]
        f["O"] = f["N"] / f["D"][:, None]
        return f
    monkeypatch.setattr(mod, "forward_slice", fwd_transposed_S)
    expect_failure([lambda: test_linear_attention_equals_explicit_kernel_matrix(32)])

    # 8. the normaliser without its epsilon: D = phi(Q) z
    def fwd_no_eps(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, *a, **kw):
        f = dict(real_fwd(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, *a, **kw))
        f["D"] = f["D"] - eps
        f["O"] = f["N"] / f["D"][:, None]
        return f
    monkeypatch.setattr(mod, "forward_slice", fwd_no_eps)
    expect_failure([lambda: test_linear_attention_equals_explicit_kernel_matrix(32), test_convexity_and_unit_values])
    monkeypatch.setattr(mod, "forward_slice", real_fwd)


# ---------------------------------------------------------------- Algorithm 1 variant: separate random matrices
def test_separate_key_matrix_explicit_kernel_and_gradients():
    """Algorithm 1 draws separate projection matrices for Q and K.  Pins: passing the shared
    matrix as Omega_K changes nothing; with a different Omega_K the output equals the explicit
    n x n attention built from phi_Q = ReLU(Q_F Omega_Q), phi_K = ReLU(K_F Omega_K); all
    gradients match central differences."""
    L, n, eps = 2, 48, 1e-2
    p = _rand_problem(61, B=1, H=1, n=n, d=4, m=16, L=L)
    OmK = np.random.default_rng(62).standard_normal(p["Omega"].shape)
    args = (p["Q"][0, 0], p["K"][0, 0], p["V"][0, 0], p["Omega"], p["sigma"], p["Wg"][0], p["bg"][0],
            p["omega"], L, eps, 1e-6)
    f_shared = wo.forward_slice(*args)
    f_same = wo.forward_slice(*args, Omega_K=p["Omega"])
    np.testing.assert_array_equal(f_shared["O"], f_same["O"])
    f = wo.forward_slice(*args, Omega_K=OmK)
    m = OmK.shape[1]
    pq = np.maximum(f["QF"] @ p["Omega"] / p["sigma"], 0) / math.sqrt(m)
    pk = np.maximum(f["KF"] @ OmK / p["sigma"], 0) / math.sqrt(m)
    A = pq @ pk.T
    np.testing.assert_allclose(f["O"], (A @ p["V"][0, 0]) / (A.sum(axis=1) + eps)[:, None], rtol=1e-11)
    assert np.abs(f["O"] - f_shared["O"]).max() > 1e-3   # the second matrix is really used
    g = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, p["dO"],
                    eps=eps, Omega_K=OmK)
    h = 1e-6
    r = np.random.default_rng(5)

    def loss(**over):
        q = dict(p, **over)
        O = wo.forward(q["Q"], q["K"], q["V"], q["Omega"], q["sigma"], q["Wg"], q["bg"], q["omega"], L, eps=eps,
                       Omega_K=OmK)["O"]
        return float(np.sum(O * p["dO"]))

    for name, gname in (("Q", "dQ"), ("K", "dK"), ("V", "dV"), ("Wg", "dWg"), ("omega", "domega")):
        arr = p[name]
        for fi in r.choice(arr.size, size=min(6, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h)
            assert abs(fd - g[gname][idx]) < 3e-6 * max(1.0, abs(fd)), (name, idx, fd, g[gname][idx])


# ---------------------------------------------------------------- Algorithm 1 variant: gate pooled over heads
def test_pooled_gate_definition_special_cases_and_gradients():
    """Algorithm 1's gate: one linear map on the concatenated pooled queries, one filter per batch
    element.  Pins: the logits equal W_filter . concat(qbar_h) written out by hand; with a single
    head it is the per-head gate; every head of a batch element gets the same F; all gradients
    match central differences (the cross-head sum of dF included)."""
    L, eps = 2, 1e-2
    p = _rand_problem(71, B=2, H=3, n=32, d=4, m=16, L=L)
    qbars, lg, sg, Fg = wo.pooled_gate(p["Q"][1], p["Wg"], p["bg"], p["omega"])
    Wfilter = np.concatenate([p["Wg"][h] for h in range(3)], axis=1)          # (L+1, H*d)
    qcat = np.concatenate([p["Q"][1, h].mean(axis=0) for h in range(3)])      # (H*d,)
    np.testing.assert_allclose(lg, Wfilter @ qcat + p["bg"].sum(axis=0), rtol=1e-12)
    np.testing.assert_allclose(Fg, p["omega"] / (1.0 + np.exp(-lg)), rtol=1e-12)
    # one head: identical to the per-head gate
    p1 = _rand_problem(72, B=2, H=1, n=32, d=4, m=16, L=L)
    a = wo.forward(p1["Q"], p1["K"], p1["V"], p1["Omega"], p1["sigma"], p1["Wg"], p1["bg"], p1["omega"], L, eps=eps)
    b = wo.forward(p1["Q"], p1["K"], p1["V"], p1["Omega"], p1["sigma"], p1["Wg"], p1["bg"], p1["omega"], L, eps=eps,
                   pooled=True)
    np.testing.assert_allclose(a["O"], b["O"], rtol=1e-12)
    f = wo.forward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, eps=eps,
                   pooled=True, keep=("O", "F"))
    for bb in range(2):
        for h in range(1, 3):
            np.testing.assert_array_equal(f["F"][bb, h], f["F"][bb, 0])
    g = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, p["dO"],
                    eps=eps, pooled=True)
    np.testing.assert_allclose(g["O"], f["O"], rtol=1e-12)
    h_ = 1e-6
    r = np.random.default_rng(7)

    def loss(**over):
        q = dict(p, **over)
        O = wo.forward(q["Q"], q["K"], q["V"], q["Omega"], q["sigma"], q["Wg"], q["bg"], q["omega"], L, eps=eps,
                       pooled=True)["O"]
        return float(np.sum(O * p["dO"]))

    for name, gname, count in (("Q", "dQ", 10), ("K", "dK", 6), ("V", "dV", 4), ("Wg", "dWg", 10), ("bg", "dbg", 6),
                               ("omega", "domega", 3)):
        arr = p[name]
        for fi in r.choice(arr.size, size=min(count, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h_
            am[idx] -= h_
            fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h_)
            assert abs(fd - g[gname][idx]) < 3e-6 * max(1.0, abs(fd)), (name, idx, fd, g[gname][idx])


# ---------------------------------------------------------------- Algorithm 1 variant: LayerNorm output stage
def test_layernorm_output_stage_properties_and_gradients():
    """Algorithm 1 normalises the linear-attention output with LayerNorm.  Pins: each output row
    has zero mean and variance var / (var + eps); the output does not change when V gets a
    common scale (up to the eps term) nor when a constant is added to every column of the
    numerator; the written-out formula on the explicit n x n numerator; all gradients match
    central differences; d sigma equals its closed form -(2 / sigma) sum_t <dO_t, O_t> eps rstd_t^2."""
    L, eps = 2, 1e-3
    p = _rand_problem(81, B=1, H=2, n=40, d=6, m=16, L=L)
    kw = dict(eps=eps, layernorm=True)
    f = wo.forward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L,
                   keep=("O", "N", "D", "PhiQ", "PhiK"), **kw)
    O, N, rstd = f["O"], f["N"], f["D"]
    np.testing.assert_allclose(O.mean(axis=-1), 0.0, atol=1e-12)
    var = N.var(axis=-1)
    np.testing.assert_allclose(O.var(axis=-1), var / (var + eps), rtol=1e-10)
    np.testing.assert_allclose(rstd, 1.0 / np.sqrt(var + eps), rtol=1e-12)
    A = f["PhiQ"][0, 1] @ f["PhiK"][0, 1].T                      # explicit n x n kernel matrix, head 1
    Nref = A @ p["V"][0, 1]
    np.testing.assert_allclose(O[0, 1], (Nref - Nref.mean(1, keepdims=True)) / np.sqrt(Nref.var(1, keepdims=True) + eps),
                               rtol=1e-10, atol=1e-12)
    # scale invariance in V up to eps (tiny eps -> invariant)
    a = wo.forward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, eps=1e-14,
                   layernorm=True)["O"]
    b = wo.forward(p["Q"], p["K"], 3.0 * p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, eps=1e-14,
                   layernorm=True)["O"]
    np.testing.assert_allclose(a, b, rtol=1e-7, atol=1e-9)
    g = wo.backward(p["Q"], p["K"], p["V"], p["Omega"], p["sigma"], p["Wg"], p["bg"], p["omega"], L, p["dO"], **kw)
    h = 1e-6
    r = np.random.default_rng(9)

    def loss(**over):
        q = dict(p, **over)
        return float(np.sum(wo.forward(q["Q"], q["K"], q["V"], q["Omega"], q["sigma"], q["Wg"], q["bg"], q["omega"],
                                       L, **kw)["O"] * p["dO"]))

    for name, gname, count in (("Q", "dQ", 10), ("K", "dK", 8), ("V", "dV", 8), ("Wg", "dWg", 6), ("bg", "dbg", 4),
                               ("omega", "domega", 3)):
        arr = p[name]
        for fi in r.choice(arr.size, size=min(count, arr.size), replace=False):
            idx = np.unravel_index(fi, arr.shape)
            ap, am = arr.copy(), arr.copy()
            ap[idx] += h
            am[idx] -= h
            fd = (loss(**{name: ap}) - loss(**{name: am})) / (2 * h)
            assert abs(fd - g[gname][idx]) < 5e-6 * max(1.0, abs(fd)), (name, idx, fd, g[gname][idx])
    fd = (loss(sigma=p["sigma"] + h) - loss(sigma=p["sigma"] - h)) / (2 * h)
    assert abs(fd - g["dsigma"]) < 5e-6 * max(1.0, abs(fd))
    closed = -(2.0 / p["sigma"]) * np.sum(np.sum(p["dO"] * O, axis=-1) * eps * rstd ** 2)
    np.testing.assert_allclose(g["dsigma"], closed, rtol=1e-7)


def test_planted_mistakes_in_the_variants_are_caught(monkeypatch):
    """The pins of the Algorithm 1 variants notice plausible mistakes planted into the oracle (on
    the CPU): a LayerNorm backward without its projection terms, a LayerNorm with the unbiased
    variance, a pooled gate that averages the heads' logits instead of summing them, and a key
    side that silently keeps the query-side random matrix."""
    mod = wo

    def expect_failure(pins):
        failed = 0
        for pin in pins:
            try:
                pin()
            except AssertionError:
                failed += 1
        assert failed >= 1, "no pin noticed the planted mistake"

    # 1. LayerNorm backward as a plain row scaling (mean and projection terms dropped)
    real_bwd = mod.backward_slice

    def bwd_ln_scaling_only(*args, **kw):
        if not kw.get("layernorm"):
            return real_bwd(*args, **kw)
        dO = args[11]
        return real_bwd(*args[:11], dO - 0.0 * dO, **dict(kw, layernorm=False))   # the plain path's gradients
    monkeypatch.setattr(mod, "backward_slice", bwd_ln_scaling_only)
    expect_failure([test_layernorm_output_stage_properties_and_gradients])
    monkeypatch.setattr(mod, "backward_slice", real_bwd)

    # 2. LayerNorm with the unbiased variance (divide by d - 1)
    real_fwd = mod.forward_slice

    def fwd_ln_unbiased(*args, **kw):
        f = real_fwd(*args, **kw)
        if kw.get("layernorm") or (len(args) > 14 and args[14]):
            f = dict(f)
            N, eps = f["N"], args[9]
            d = N.shape[1]
            var = N.var(axis=1, ddof=1)
            f["D"] = 1.0 / np.sqrt(var + eps)
            f["O"] = (N - N.mean(axis=1, keepdims=True)) * f["D"][:, None]
        return f
    monkeypatch.setattr(mod, "forward_slice", fwd_ln_unbiased)
    expect_failure([test_layernorm_output_stage_properties_and_gradients])
    monkeypatch.setattr(mod, "forward_slice", real_fwd)

    # 3. pooled gate that averages the heads' logits instead of summing them
    real_pg = mod.pooled_gate

    def pooled_gate_mean(Qb, Wg, bg, omega):
        qbars, lg, s, F = real_pg(Qb, Wg, bg, omega)
        lg = lg / Qb.shape[0]
        s = 1.0 / (1.0 + np.exp(-lg))
        return qbars, lg, s, s * omega
    monkeypatch.setattr(mod, "pooled_gate", pooled_gate_mean)
    expect_failure([test_pooled_gate_definition_special_cases_and_gradients])
    monkeypatch.setattr(mod, "pooled_gate", real_pg)

    # 4. key side keeps the query-side random matrix
    def fwd_ignores_key_matrix(*args, **kw):
        kw = dict(kw)
        kw["Omega_K"] = None
        args = list(args)
        if len(args) > 12:
            args[12] = None
        return real_fwd(*args, **kw)
    monkeypatch.setattr(mod, "forward_slice", fwd_ignores_key_matrix)
    expect_failure([test_separate_key_matrix_explicit_kernel_and_gradients])
    monkeypatch.setattr(mod, "forward_slice", real_fwd)
