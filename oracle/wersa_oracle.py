"""fp64 CPU oracle for WERSA attention (forward and backward).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
HIP kernels are checked against.  It shares no code with the GPU path and the
product never calls it: only tests, the smoke check and the CPU-baseline leg
of the benchmark import it.

Everything is written per (batch, head) slice with NumPy in float64, in the
order the paper states the method (Section 3.1 steps 3-8; Appendix D,
Algorithms 1 and 2).  Library primitives used as steps: ``@`` (matmul),
``mean``, ``maximum``.  No blocking, fusion or reordering.

Readings of the paper taken here (each one is a choice where the text is
silent or disagrees with itself):

* Normalisation follows the Section 3.1 attention equation (divide by
  phi(Q_F) phi(K_F)^T 1 + eps); the LayerNorm of Algorithm 1 is available as
  an option (layernorm).
* One shared random matrix Omega (Section 3.1 step 7) and the 1/sqrt(m) factor
  of Algorithm 1's random projection lines.  Algorithm 1's separate matrices for
  Q and K are available as an option (Omega_K).
* The gate g is a single linear map per head (Algorithm 1's W_filter), applied
  to that head's own pooled query (Section 3.1 step 4), plus a bias; the
  per-scale weights omega are shared by all heads.  Algorithm 1's form (one
  map on the pooled queries of all heads, one filter per batch element) is
  available as an option (pooled).
* The same filter F (computed from Q) multiplies the coefficients of both Q
  and K (Section 3.1 step 6).
* Band order of F: index 0 is the finest detail band d_1, index L-1 is d_L,
  index L is the approximation a_L (return order of Algorithm 2's DWT).
* Haar pair convention (Appendix A, Appendix C, Algorithm 2): pair
  (x[2k], x[2k+1]), approximation = (even+odd)/sqrt(2), detail =
  (even-odd)/sqrt(2).
* Zero padding to the next power of two before the transform, trim after the
  inverse (Algorithm 2); the pooled query uses the original n rows.
* sigma_eff = max(sigma, bw_floor) (Algorithm 1's bandwidth line); one scalar
  for the whole call.
* Sub-gradient of ReLU at exactly 0 is 0.

Decision precision (optional, default off): the ReLU derivative 1[U > 0] is a binary decision
taken by floating point.  When a kernel is checked whose projection consumes X_F in a reduced
precision, `proj_dtype` (for example numpy.float16) rounds X_F once to that type before the
projection, so that both sides take the decision on the same numbers; everything else stays
float64.  With proj_dtype=None the oracle is the plain float64 definition.

Pins (tests/test_oracle_pins.py): hand-derived Haar coefficients, perfect
reconstruction, energy preservation, block-mean closed form, explicit n x n
kernel-matrix attention, arc-cosine kernel limit and m^-1/2 rate, convexity,
sigma homogeneity, central finite differences for every gradient, ablation
special cases; for the attention block: identity projections reduce it to the
pinned core per head, column permutation of W^out, linearity in W^V and W^out,
central finite differences for every block gradient; the two optional hooks
(`proj_dtype`, `store`) are pinned as the identity when inactive and as exactly
the stated rounding when active.  Absolute output values on real data: parity
unpinned (the paper prints no worked numeric example).
"""
import math

import numpy as np

SQRT2 = math.sqrt(2.0)


# ----------------------------------------------------------------------------
# Haar transform along the sequence axis (Appendix A equations; Algorithm 2)
# ----------------------------------------------------------------------------
def next_pow2(n):
    return 1 << max(0, math.ceil(math.log2(n))) if n > 1 else 1


def haar_dwt(X, L):
    """L-level Haar analysis of X (n, d) along axis 0.

    Returns ([d_1, ..., d_L, a_L], n): details finest first, then the last
    approximation (Algorithm 2, VectorizedDWT).  X is zero-padded to the next
    power of two first.
    """
    n = X.shape[0]
    npad = next_pow2(n)
    if npad < (1 << L):
        npad = 1 << L
    approx = np.zeros((npad,) + X.shape[1:], dtype=np.float64)
    approx[:n] = X
    details = []
    for _ in range(L):
        even = approx[0::2]
        odd = approx[1::2]
        details.append((even - odd) / SQRT2)
        approx = (even + odd) / SQRT2
    return details + [approx], n


def haar_idwt(coeffs, n):
    """Inverse of haar_dwt; trims to the original n rows (VectorizedIDWT)."""
    approx = coeffs[-1]
    for detail in reversed(coeffs[:-1]):
        even = (approx + detail) / SQRT2
        odd = (approx - detail) / SQRT2
        nxt = np.empty((2 * approx.shape[0],) + approx.shape[1:], dtype=np.float64)
        nxt[0::2] = even
        nxt[1::2] = odd
        approx = nxt
    return approx[:n]


def filtered_idwt(coeffs, F, n):
    """Multiply band i by F[i], then inverse transform (FilteredIDWT)."""
    return haar_idwt([c * F[i] for i, c in enumerate(coeffs)], n)


def haar_filter(X, F, L):
    """X_F = W^-1 (F (.) W X)  (Section 3.1 step 6)."""
    coeffs, n = haar_dwt(X, L)
    return filtered_idwt(coeffs, F, n)


# ----------------------------------------------------------------------------
# Gate (Section 3.1 step 4, equations for Q'_avg, F and F_i)
# ----------------------------------------------------------------------------
def gate(qbar, Wg_h, bg_h, omega):
    """qbar (d,), Wg_h (L+1, d), bg_h (L+1,), omega (L+1,) -> logits, s, F."""
    logits = Wg_h @ qbar + bg_h
    s = 1.0 / (1.0 + np.exp(-logits))
    return logits, s, s * omega


# ----------------------------------------------------------------------------
# Random feature map (Section 3.1 step 7; Algorithm 1 projection lines)
# ----------------------------------------------------------------------------
def feature_map(XF, Omega, sigma, bw_floor, proj_dtype=None):
    m = Omega.shape[1]
    sigma_eff = max(float(sigma), float(bw_floor))
    if proj_dtype is not None:
        XF = XF.astype(proj_dtype).astype(np.float64)
    U = (XF @ Omega) / sigma_eff
    Phi = np.maximum(U, 0.0) / math.sqrt(m)
    return U, Phi


# ----------------------------------------------------------------------------
# Forward, one (b, h) slice
# ----------------------------------------------------------------------------
def forward_slice(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, proj_dtype=None,
                  Omega_K=None, gate_given=None, layernorm=False):
    """Q, K, V (n, d) -> dict of every stage tensor, 'O' is the output.

    Omega_K: a second random matrix for the key side (Algorithm 1 draws separate projection
    matrices for Q and K); None = the one shared matrix of Section 3.1 step 7.
    gate_given: (logits, s, F) computed outside (the gate pooled over heads), else this head's own.
    layernorm: Algorithm 1's output stage, O = LayerNorm(phi(Q_F) (phi(K_F)^T V)) over the d
    columns of each row (no affine parameters, biased variance, eps inside the root), in place
    of Section 3.1's division by the normaliser; D then holds 1 / sqrt(var + eps)."""
    OmK = Omega if Omega_K is None else np.asarray(Omega_K, np.float64)
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    qbar = Q.mean(axis=0)
    logits, s, F = gate(qbar, Wg_h, bg_h, omega) if gate_given is None else gate_given
    QF = haar_filter(Q, F, L)
    KF = haar_filter(K, F, L)
    UQ, PhiQ = feature_map(QF, Omega, sigma, bw_floor, proj_dtype)
    UK, PhiK = feature_map(KF, OmK, sigma, bw_floor, proj_dtype)
    S = PhiK.T @ V                       # (m, d)  phi(K_F)^T V
    z = PhiK.T @ np.ones(K.shape[0])     # (m,)    phi(K_F)^T 1
    N = PhiQ @ S
    if layernorm:
        mu = N.mean(axis=1)
        var = ((N - mu[:, None]) ** 2).mean(axis=1)
        D = 1.0 / np.sqrt(var + eps)          # rstd
        O = (N - mu[:, None]) * D[:, None]
    else:
        D = PhiQ @ z + eps
        O = N / D[:, None]
    return dict(qbar=qbar, logits=logits, s=s, F=F, QF=QF, KF=KF, UQ=UQ, UK=UK,
                PhiQ=PhiQ, PhiK=PhiK, S=S, z=z, N=N, D=D, O=O)


# ----------------------------------------------------------------------------
# Backward, one (b, h) slice: chain rule through forward_slice, step by step
# in reverse.  The paper states no backward; this is the derivative of the
# forward above (checked by finite differences in the pins).
# ----------------------------------------------------------------------------
def _haar_filter_vjp(X, F, L, dXF):
    """Given dL/dX_F, return dL/dX and dL/dF for X_F = W^-1 (F (.) W X).

    The padded Haar transform matrix W is orthonormal, so the transpose of the
    inverse transform is the forward transform and vice versa; the transpose of
    'trim to n rows' is 'zero-pad back', which haar_dwt does on entry.
    """
    cx, n = haar_dwt(X, L)           # coefficients of the input
    cg, _ = haar_dwt(dXF, L)         # (W^-1)^T applied to the padded cotangent
    dF = np.array([np.sum(cx[i] * cg[i]) for i in range(L + 1)])
    dX = haar_idwt([cg[i] * F[i] for i in range(L + 1)], n)   # W^T (F (.) .)
    return dX, dF


def backward_slice(Q, K, V, Omega, sigma, Wg_h, bg_h, omega, L, eps, bw_floor, dO,
                   fwd=None, proj_dtype=None, Omega_K=None, gate_outside=False, layernorm=False):
    """Returns dict dQ, dK, dV (n, d), dWg_h (L+1, d), dbg_h, domega (L+1,),
    dsigma (scalar, term-by-term chain rule form), plus intermediates."""
    Q = np.asarray(Q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    dO = np.asarray(dO, np.float64)
    f = fwd if fwd is not None else forward_slice(Q, K, V, Omega, sigma, Wg_h, bg_h,
                                                  omega, L, eps, bw_floor, proj_dtype, Omega_K,
                                                  layernorm=layernorm)
    OmK = Omega if Omega_K is None else np.asarray(Omega_K, np.float64)
    n, d = Q.shape
    m = Omega.shape[1]
    sigma_eff = max(float(sigma), float(bw_floor))
    D, O, S, z = f["D"], f["O"], f["S"], f["z"]
    PhiQ, PhiK, UQ, UK = f["PhiQ"], f["PhiK"], f["UQ"], f["UK"]

    if layernorm:
        # O = (N - mean) * rstd, per row: the standard LayerNorm derivative (D holds rstd)
        dN = D[:, None] * (dO - dO.mean(axis=1, keepdims=True) - O * (dO * O).mean(axis=1, keepdims=True))
        dD = np.zeros(n)
        dPhiQ = dN @ S.T
        dS = PhiQ.T @ dN
        dz = np.zeros(m)
    else:
        # O = N / D
        dN = dO / D[:, None]
        dD = -np.sum(dO * O, axis=1) / D
        # N = PhiQ S ; D = PhiQ z + eps
        dPhiQ = dN @ S.T + np.outer(dD, z)
        dS = PhiQ.T @ dN
        dz = PhiQ.T @ dD
    # S = PhiK^T V ; z = PhiK^T 1
    dPhiK = V @ dS.T + np.outer(np.ones(n), dz)
    dV = PhiK @ dS
    # Phi = max(U, 0)/sqrt(m)
    dUQ = dPhiQ * (UQ > 0.0) / math.sqrt(m)
    dUK = dPhiK * (UK > 0.0) / math.sqrt(m)
    # U = X_F Omega / sigma_eff
    dQF = (dUQ @ Omega.T) / sigma_eff
    dKF = (dUK @ OmK.T) / sigma_eff
    if float(sigma) > float(bw_floor):
        dsigma = -(np.sum(dUQ * UQ) + np.sum(dUK * UK)) / sigma_eff
    else:
        dsigma = 0.0
    # X_F = W^-1 (F (.) W X), for Q and K with the same F
    dQ, dF_q = _haar_filter_vjp(Q, f["F"], L, dQF)
    dK, dF_k = _haar_filter_vjp(K, f["F"], L, dKF)
    dF = dF_q + dF_k
    if gate_outside:   # the caller owns the gate (pooled over heads): hand back dF, no pooled-query term yet
        return dict(dQ=dQ, dK=dK, dV=dV, dsigma=dsigma, dS=dS, dz=dz, dD=dD, dF=dF, dQF=dQF, dKF=dKF)
    # F = s * omega ; s = sigmoid(logits) ; logits = Wg qbar + bg ; qbar = mean(Q)
    s = f["s"]
    domega = dF * s
    ds = dF * omega
    dlogits = ds * s * (1.0 - s)
    dWg_h = np.outer(dlogits, f["qbar"])
    dbg_h = dlogits
    dqbar = Wg_h.T @ dlogits
    dQ = dQ + dqbar[None, :] / n
    return dict(dQ=dQ, dK=dK, dV=dV, dWg_h=dWg_h, dbg_h=dbg_h, domega=domega,
                dsigma=dsigma, dS=dS, dz=dz, dD=dD, dF=dF, dQF=dQF, dKF=dKF)


# ----------------------------------------------------------------------------
# Whole call over (B, H, n, d)
# ----------------------------------------------------------------------------
def pooled_gate(Qb, Wg, bg, omega):
    """Algorithm 1's gate: the per-head pooled queries of one batch element, concatenated over the
    heads, go through ONE linear map to L+1 logits; every head of that batch element shares the
    filter.  With the per-head parameter layout Wg (H, L+1, d), bg (H, L+1) the map is
    logits_i = sum_h (Wg[h, i] . qbar_h + bg[h, i]).  Qb is (H, n, d)."""
    qbars = np.asarray(Qb, np.float64).mean(axis=1)                  # (H, d)
    logits = np.einsum("hid,hd->i", np.asarray(Wg, np.float64), qbars) + np.asarray(bg, np.float64).sum(axis=0)
    s = 1.0 / (1.0 + np.exp(-logits))
    return qbars, logits, s, s * np.asarray(omega, np.float64)


def forward(Q, K, V, Omega, sigma, Wg, bg, omega, L, eps=1e-6, bw_floor=1e-6,
            slices=None, keep=("O",), proj_dtype=None, Omega_K=None, pooled=False, layernorm=False):
    """Q, K, V (B, H, n, d); Omega (d, m); Wg (H, L+1, d); bg (H, L+1); omega (L+1,).

    Returns dict of stacked stage tensors named in `keep`, each (B, H, ...).
    `slices` optionally restricts the work to a list of (b, h) pairs; other
    slices are left as zeros.
    """
    B, H = Q.shape[:2]
    Omega = np.asarray(Omega, np.float64)
    out = {}
    todo = slices if slices is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in todo:
        given = None
        if pooled:
            _, lg, sg, Fg = pooled_gate(Q[b], Wg, bg, omega)
            given = (lg, sg, Fg)
        f = forward_slice(Q[b, h], K[b, h], V[b, h], Omega, sigma,
                          np.asarray(Wg[h], np.float64), np.asarray(bg[h], np.float64),
                          np.asarray(omega, np.float64), L, eps, bw_floor, proj_dtype, Omega_K, given,
                          layernorm)
        for name in keep:
            if name not in out:
                out[name] = np.zeros((B, H) + np.shape(f[name]), np.float64)
            out[name][b, h] = f[name]
    return out


def backward_pooled(Q, K, V, Omega, sigma, Wg, bg, omega, L, dO, eps=1e-6, bw_floor=1e-6,
                    proj_dtype=None, Omega_K=None, layernorm=False):
    """Backward with the gate pooled over heads (pooled_gate): dF of the heads of a batch element
    add up before the sigmoid's derivative; the pooled-query term then goes back to each head."""
    B, H, n, d = Q.shape
    Omega = np.asarray(Omega, np.float64)
    omega = np.asarray(omega, np.float64)
    Wg = np.asarray(Wg, np.float64)
    g = dict(dQ=np.zeros((B, H, n, d)), dK=np.zeros((B, H, n, d)), dV=np.zeros((B, H, n, d)),
             dWg=np.zeros((H, L + 1, d)), dbg=np.zeros((H, L + 1)), domega=np.zeros(L + 1),
             dsigma=0.0, O=np.zeros((B, H, n, d)), dD_sum=0.0)
    for b in range(B):
        qbars, lg, sg, Fg = pooled_gate(Q[b], Wg, bg, omega)
        dF = np.zeros(L + 1)
        for h in range(H):
            args = (Q[b, h], K[b, h], V[b, h], Omega, sigma, Wg[h], np.asarray(bg[h], np.float64), omega, L,
                    eps, bw_floor)
            f = forward_slice(*args, proj_dtype, Omega_K, (lg, sg, Fg), layernorm)
            r = backward_slice(*args, dO[b, h], fwd=f, Omega_K=Omega_K, gate_outside=True, layernorm=layernorm)
            g["O"][b, h] = f["O"]
            g["dQ"][b, h], g["dK"][b, h], g["dV"][b, h] = r["dQ"], r["dK"], r["dV"]
            g["dsigma"] += r["dsigma"]
            g["dD_sum"] += float(np.sum(r["dD"]))
            dF += r["dF"]
        g["domega"] += dF * sg
        dlogits = dF * omega * sg * (1.0 - sg)
        for h in range(H):
            g["dWg"][h] += np.outer(dlogits, qbars[h])
            g["dbg"][h] += dlogits
            g["dQ"][b, h] += (Wg[h].T @ dlogits)[None, :] / n
    return g


def backward(Q, K, V, Omega, sigma, Wg, bg, omega, L, dO, eps=1e-6, bw_floor=1e-6,
             slices=None, proj_dtype=None, Omega_K=None, pooled=False, layernorm=False):
    """Gradients of sum(O * dO) w.r.t. Q, K, V, Wg, bg, omega, sigma.

    Parameter gradients are summed over every slice processed (all of them
    unless `slices` restricts the work).
    """
    if pooled:
        assert slices is None, "the pooled gate couples the heads of a batch element"
        return backward_pooled(Q, K, V, Omega, sigma, Wg, bg, omega, L, dO, eps, bw_floor, proj_dtype, Omega_K,
                               layernorm)
    B, H, n, d = Q.shape
    Omega = np.asarray(Omega, np.float64)
    omega = np.asarray(omega, np.float64)
    g = dict(dQ=np.zeros((B, H, n, d)), dK=np.zeros((B, H, n, d)), dV=np.zeros((B, H, n, d)),
             dWg=np.zeros((H, L + 1, d)), dbg=np.zeros((H, L + 1)), domega=np.zeros(L + 1),
             dsigma=0.0, O=np.zeros((B, H, n, d)), dD_sum=0.0)
    todo = slices if slices is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in todo:
        Wg_h = np.asarray(Wg[h], np.float64)
        bg_h = np.asarray(bg[h], np.float64)
        f = forward_slice(Q[b, h], K[b, h], V[b, h], Omega, sigma, Wg_h, bg_h, omega, L,
                          eps, bw_floor, proj_dtype, Omega_K, layernorm=layernorm)
        r = backward_slice(Q[b, h], K[b, h], V[b, h], Omega, sigma, Wg_h, bg_h, omega, L,
                           eps, bw_floor, dO[b, h], fwd=f, Omega_K=Omega_K, layernorm=layernorm)
        g["O"][b, h] = f["O"]
        g["dQ"][b, h] = r["dQ"]
        g["dK"][b, h] = r["dK"]
        g["dV"][b, h] = r["dV"]
        g["dWg"][h] += r["dWg_h"]
        g["dbg"][h] += r["dbg_h"]
        g["domega"] += r["domega"]
        g["dsigma"] += r["dsigma"]
        g["dD_sum"] += float(np.sum(r["dD"]))
    return g


# ----------------------------------------------------------------------------
# Attention block: input/output projections around the core (Section 3.1 steps 1-2 and the
# closing lines of Algorithm 1: linear projections, head splitting, merged heads times W_out)
# ----------------------------------------------------------------------------
def split_heads(T, H):
    """(B, n, H*d) -> (B, H, n, d): head h owns columns [h*d, (h+1)*d) (Section 3.1 step 2)."""
    B, n, hidden = T.shape
    return T.reshape(B, n, H, hidden // H).transpose(0, 2, 1, 3)


def merge_heads(T):
    """(B, H, n, d) -> (B, n, H*d), the inverse of split_heads (Algorithm 1, merge line)."""
    B, H, n, d = T.shape
    return T.transpose(0, 2, 1, 3).reshape(B, n, H * d)


def block_forward(X, WQ, WK, WV, WO, H, Omega, sigma, Wg, bg, omega, L, eps=1e-6, bw_floor=1e-6,
                  proj_dtype=None, store=None):
    """Self-attention block on X (B, n, hidden): Q' = X W^Q, K' = X W^K, V' = X W^V, heads split,
    WERSA core per head, heads merged, Y = A W^out.  Weights are (hidden_in, hidden_out).

    `store`, when given, is applied to Q', K', V' and A right after each is formed (a test uses
    it to round the intermediates to the storage type of the kernel under test); None keeps
    everything in float64.
    """
    X = np.asarray(X, np.float64)
    keepf = (lambda a: a) if store is None else store
    Qp = keepf(X @ np.asarray(WQ, np.float64))
    Kp = keepf(X @ np.asarray(WK, np.float64))
    Vp = keepf(X @ np.asarray(WV, np.float64))
    core = forward(split_heads(Qp, H), split_heads(Kp, H), split_heads(Vp, H), Omega, sigma, Wg, bg,
                   omega, L, eps, bw_floor, proj_dtype=proj_dtype)
    A = keepf(merge_heads(core["O"]))
    Y = A @ np.asarray(WO, np.float64)
    return dict(Y=Y, A=A, Qp=Qp, Kp=Kp, Vp=Vp)


def block_backward(X, WQ, WK, WV, WO, H, Omega, sigma, Wg, bg, omega, L, dY, eps=1e-6,
                   bw_floor=1e-6, proj_dtype=None, store=None):
    """Gradients of sum(Y * dY) w.r.t. X, the four weight matrices and the core's parameters
    (chain rule through block_forward; the core's part is `backward`)."""
    X = np.asarray(X, np.float64)
    dY = np.asarray(dY, np.float64)
    WQ, WK, WV, WO = (np.asarray(w, np.float64) for w in (WQ, WK, WV, WO))
    keepf = (lambda a: a) if store is None else store
    f = block_forward(X, WQ, WK, WV, WO, H, Omega, sigma, Wg, bg, omega, L, eps, bw_floor,
                      proj_dtype=proj_dtype, store=store)
    B, n, hidden = X.shape
    X2, dY2, A2 = X.reshape(B * n, hidden), dY.reshape(B * n, hidden), f["A"].reshape(B * n, hidden)
    dWO = A2.T @ dY2
    dA = keepf(dY @ WO.T)
    g = backward(split_heads(f["Qp"], H), split_heads(f["Kp"], H), split_heads(f["Vp"], H), Omega,
                 sigma, Wg, bg, omega, L, split_heads(dA, H), eps, bw_floor, proj_dtype=proj_dtype)
    dQp, dKp, dVp = (keepf(merge_heads(g[k])) for k in ("dQ", "dK", "dV"))
    dX = dQp @ WQ.T + dKp @ WK.T + dVp @ WV.T
    dWQ = X2.T @ dQp.reshape(B * n, hidden)
    dWK = X2.T @ dKp.reshape(B * n, hidden)
    dWV = X2.T @ dVp.reshape(B * n, hidden)
    return dict(Y=f["Y"], A=f["A"], Qp=f["Qp"], Kp=f["Kp"], Vp=f["Vp"], dA=dA, dQp=dQp, dKp=dKp,
                dVp=dVp, dX=dX, dWQ=dWQ, dWK=dWK, dWV=dWV, dWO=dWO, dWg=g["dWg"], dbg=g["dbg"],
                domega=g["domega"], dsigma=g["dsigma"])
