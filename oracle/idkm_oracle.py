"""CPU oracle for implicit differentiable soft k-means (IDKM).  TEST INFRASTRUCTURE ONLY.

Plain numpy float64, written from the paper, slow on purpose.  Nothing here is
shared with, imported by, or imports the HIP path; only tests, the smoke check
and the benchmark's CPU-baseline leg may call it.

Shapes (row-major): W[m,d] weight vectors, C[k,d] codebook, A[m,k] attention,
Wq[m,d] = A C soft-quantised weights, G[m,d] = dL/dWq upstream gradient.

Two energies are supported, selected by `dist`:
  0  e_ij = ||w_i - c_j||     the paper's distance matrix (Sec. 3.2, Alg. 1 step "distance matrix")
  1  e_ij = ||w_i - c_j||^2   the squared variant

Every function cites the passage of the paper it writes out.  Parity status:
every function below is pinned by tests/test_oracle_*.py against closed forms,
invariants, brute force (hard Lloyd), central finite differences, a dense
linear solve and an independent autodiff of the matrix form; the code packing
against Python big-integer arithmetic and a hand-worked stream; none is unpinned.
"""
from __future__ import annotations

import numpy as np

DIST_L2 = 0
DIST_SQL2 = 1


def _f64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


# --------------------------------------------------------------------------- forward

def energy(W, C, dist):
    """Distance matrix D[m,k], d_ij = ||w_i - c_j|| (Alg. 1, distance-matrix step), or its square."""
    W, C = _f64(W), _f64(C)
    m, d = W.shape
    k = C.shape[0]
    sq = np.zeros((m, k))
    for r in range(d):
        diff = W[:, r][:, None] - C[:, r][None, :]
        sq += diff * diff
    return sq if dist == DIST_SQL2 else np.sqrt(sq)


def attention(W, C, tau, dist):
    """A = rowsoftmax_tau(-D)  (Eq. "aterms", Eq. "arow").

    softmax_tau(x)_j = exp(x_j/tau) / sum_l exp(x_l/tau).  The row minimum of D is
    subtracted before exponentiating; this leaves the quotient unchanged.
    """
    E = energy(W, C, dist)
    E -= E.min(axis=1, keepdims=True)
    P = np.exp(-E / tau)
    return P / P.sum(axis=1, keepdims=True)


def mstep(A, W, C_prev):
    """C+ = diag(A^T 1)^-1 A^T W  (Eq. "centers"); returns (C+, n) with n = A^T 1.

    A cluster whose mass n_j is exactly zero keeps its previous centre (the paper
    is silent; in exact arithmetic the mass is positive).
    """
    W = _f64(W)
    n = A.sum(axis=0)
    S = A.T @ W
    Cp = np.array(C_prev, dtype=np.float64, copy=True)
    ok = n > 0
    Cp[ok] = S[ok] / n[ok][:, None]
    return Cp, n


def F(C, W, tau, dist):
    """The fixed-point map F(C, W) (Eq. "deepeqc"): one E-step followed by one M-step."""
    A = attention(W, C, tau, dist)
    return mstep(A, W, C)[0]


def soft_kmeans(W, C0, tau, tol, max_iter, dist):
    """Algorithm 1: repeat C+ = F(C, W) until ||C+ - C||_F < tol (or max_iter evaluations of F).

    Returns dict(C, iters, converged, residual); C is the last C+, iters counts
    evaluations of F, residual is the last ||C+ - C||_F.
    """
    W = _f64(W)
    C = _f64(C0).copy()
    res = np.inf
    it = 0
    for it in range(1, max_iter + 1):
        Cp = F(C, W, tau, dist)
        res = float(np.linalg.norm(Cp - C))
        C = Cp
        if res < tol:
            break
    return dict(C=C, iters=it, converged=bool(res < tol), residual=res)


def soft_quantize(W, C, tau, dist):
    """r_tau(W, C) = A(W, C) C  (Eq. "softquant", Eq. "softquantmatrix" in row-major shapes)."""
    return attention(W, C, tau, dist) @ _f64(C)


def hard_assign_f32(W32, C32):
    """Index of the closest codeword q(w_i, C) (Sec. 3, product-quantisation set-up), decided in float32.

    The key is evaluated in float32 with every operation rounded separately:
    d == 1: |w - c|;  d > 1: sum_r (w_r - c_r)^2 accumulated in index order.
    Ties go to the lowest index.  Deciding in the kernel's precision makes the
    integer result comparable bit for bit.
    """
    W32 = np.asarray(W32, dtype=np.float32)
    C32 = np.asarray(C32, dtype=np.float32)
    m, d = W32.shape
    k = C32.shape[0]
    if d == 1:
        key = np.abs(W32[:, 0][:, None] - C32[:, 0][None, :])
    else:
        key = np.zeros((m, k), dtype=np.float32)
        for r in range(d):
            diff = (W32[:, r][:, None] - C32[:, r][None, :]).astype(np.float32)
            key = (key + (diff * diff).astype(np.float32)).astype(np.float32)
    return np.argmin(key, axis=1).astype(np.int32)


def hard_quantize(W32, C32):
    """q(W, C): every w_i replaced by its closest codeword (Sec. 3, the map written with a bold q), float32 rows of C."""
    C32 = np.asarray(C32, dtype=np.float32)
    return C32[hard_assign_f32(W32, C32)]


def cluster_objective(W, C, assign):
    """Sum_i ||w_i - c_assign(i)||^2 (Eq. "clusterobj"), float64."""
    W, C = _f64(W), _f64(C)
    diff = W - C[np.asarray(assign)]
    return float(np.sum(diff * diff))


def code_bits(k):
    """Bits per code for a codebook of k codewords: the b with 2^b >= k (k = 2^b in the paper), at least 1."""
    b = 1
    while (1 << b) < k:
        b += 1
    return b


def pack_codes(assign, k):
    """The stored form of a quantised layer (Sec. 3: one of k = 2^b codewords per sub-vector, b bits each).

    Code i occupies bits [i b, (i+1) b) of one little-endian bit stream (bit t of the stream is bit t mod 32 of
    32-bit word t div 32); the last word is padded with zero bits.  Returns uint32[ceil(m b / 32)].
    """
    a = np.asarray(assign, dtype=np.int64)
    b = code_bits(k)
    assert a.min(initial=0) >= 0 and a.max(initial=0) < k
    m = a.shape[0]
    nwords = (m * b + 31) // 32
    bits = np.zeros(nwords * 32, dtype=np.uint8)
    for t in range(b):
        bits[t:m * b:b] = (a >> t) & 1
    by = np.packbits(bits, bitorder="little")
    return by.view("<u4").astype(np.uint32)


def unpack_codes(words, m, k):
    """Inverse of pack_codes: int32[m]."""
    b = code_bits(k)
    by = np.asarray(words, dtype="<u4").view(np.uint8)
    bits = np.unpackbits(by, bitorder="little")[:m * b].reshape(m, b).astype(np.int64)
    return (bits << np.arange(b)[None, :]).sum(axis=1).astype(np.int32)


# --------------------------------------------------------------------------- derivatives of F

def _delta(W, C, E, dist, r):
    """delta_ij,r = d e_ij / d w_i,r  (and d e_ij / d c_j,r = -delta_ij,r); zero where w_i == c_j."""
    diff = W[:, r][:, None] - C[:, r][None, :]
    if dist == DIST_SQL2:
        return 2.0 * diff
    out = np.zeros_like(diff)
    np.divide(diff, E, out=out, where=E > 0)
    return out


def vjp_F(C, W, tau, dist, g):
    """Vector-Jacobian products of F at (C, W) with a cotangent g[k,d].

    Returns ((dF/dC)^T g  [k,d],  (dF/dW)^T g  [m,d]).  These are the two
    Jacobians of Eq. "grad", obtained by differentiating F_j = s_j / n_j,
    s_j = sum_i a_ij w_i, n_j = sum_i a_ij through the softmax of Eq. "aterms":
        d a_il / d e_ij = -(1/tau) a_il (1[l=j] - a_ij).
    With h_j = g_j / n_j, beta_ij = h_j . (w_i - F_j), gamma_ij = a_ij (beta_ij - sum_l a_il beta_il):
        ((dF/dC)^T g)_j = (1/tau) sum_i gamma_ij delta_ij
        ((dF/dW)^T g)_i = sum_j a_ij h_j - (1/tau) sum_j gamma_ij delta_ij
    """
    W, C, g = _f64(W), _f64(C), _f64(g)
    m, d = W.shape
    E = energy(W, C, dist)
    Es = E - E.min(axis=1, keepdims=True)
    P = np.exp(-Es / tau)
    A = P / P.sum(axis=1, keepdims=True)
    Fv, n = mstep(A, W, C)
    h = np.zeros_like(g)
    ok = n > 0
    h[ok] = g[ok] / n[ok][:, None]
    beta = W @ h.T - (h * Fv).sum(axis=1)[None, :]
    bbar = (A * beta).sum(axis=1, keepdims=True)
    gamma = A * (beta - bbar)
    JCg = np.zeros_like(C)
    JWg = A @ h
    for r in range(d):
        dl = _delta(W, C, E, dist, r)
        gd = gamma * dl
        JCg[:, r] = gd.sum(axis=0) / tau
        JWg[:, r] -= gd.sum(axis=1) / tau
    return JCg, JWg


def jacobian_C(C, W, tau, dist):
    """Dense dF/dC as a (k d) x (k d) matrix J[(j,r),(l,s)] = d F_jr / d c_ls, from k d unit cotangents."""
    C = _f64(C)
    k, d = C.shape
    J = np.zeros((k * d, k * d))
    for idx in range(k * d):
        g = np.zeros(k * d)
        g[idx] = 1.0
        J[idx, :] = vjp_F(C, W, tau, dist, g.reshape(k, d))[0].reshape(-1)
    return J


def loss_cotangents(W, C, tau, dist, G):
    """Cotangents of the loss through Wq = A(W, C) C at fixed upstream G = dL/dWq.

    Returns (v[k,d], direct[m,d]):  v = dL/dC with W held fixed (both factors of
    A C depend on C), direct = dL/dW with C held fixed (through A only).
    Algorithm 2 evaluates the loss on r_tau(W, C*) with autodiff on, so both
    dependences are part of the gradient.
    With p_ij = G_i . c_j and rho_ij = a_ij (p_ij - sum_l a_il p_il):
        v_j = sum_i a_ij G_i + (1/tau) sum_i rho_ij delta_ij
        direct_i = -(1/tau) sum_j rho_ij delta_ij
    """
    W, C, G = _f64(W), _f64(C), _f64(G)
    m, d = W.shape
    E = energy(W, C, dist)
    Es = E - E.min(axis=1, keepdims=True)
    P = np.exp(-Es / tau)
    A = P / P.sum(axis=1, keepdims=True)
    p = G @ C.T
    pbar = (A * p).sum(axis=1, keepdims=True)
    rho = A * (p - pbar)
    v = A.T @ G
    direct = np.zeros_like(W)
    for r in range(d):
        dl = _delta(W, C, E, dist, r)
        rd = rho * dl
        v[:, r] += rd.sum(axis=0) / tau
        direct[:, r] = -rd.sum(axis=1) / tau
    return v, direct


# --------------------------------------------------------------------------- backward

def solve_dense(C, W, tau, dist, v):
    """g = (I - dF/dC)^-T v by Gaussian elimination: the inverse of Eq. "inv" applied as a VJP."""
    C = _f64(C)
    k, d = C.shape
    J = jacobian_C(C, W, tau, dist)
    g = np.linalg.solve(np.eye(k * d) - J.T, _f64(v).reshape(-1))
    return g.reshape(k, d)


def solve_iterative(C, W, tau, dist, v, tol, max_iter, alpha=1.0):
    """Vector form of the averaged fixed-point iteration of Sec. 4.2 (Eq. "backiter", averaging step):
        g <- alpha (v + (dF/dC)^T g) + (1 - alpha) g,   g_0 = v,
    stopped when ||g_new - g||_F <= tol ||v||_F or after max_iter passes.  If the
    step norm is non-finite or grows on 5 consecutive passes the iteration is
    declared divergent and restarted from g = v with alpha halved (at most 6
    halvings), as the paper prescribes for its alpha = 0.25.
    Returns dict(g, iters (all passes, all attempts), converged, residual, alpha).
    """
    v = _f64(v)
    vnorm = float(np.linalg.norm(v))
    passes = 0
    halvings = 0
    while True:
        g = v.copy()
        prev = np.inf
        grow = 0
        diverged = False
        converged = False
        dn = np.inf
        for _ in range(max_iter):
            u = vjp_F(C, W, tau, dist, g)[0]
            passes += 1
            gn = alpha * (v + u) + (1.0 - alpha) * g
            dn = float(np.linalg.norm(gn - g))
            g = gn
            if not np.isfinite(dn):
                diverged = True
                break
            if dn <= tol * vnorm:
                converged = True
                break
            grow = grow + 1 if dn > prev else 0
            if grow >= 5:
                diverged = True
                break
            prev = dn
        if diverged and halvings < 6:
            alpha *= 0.5
            halvings += 1
            continue
        return dict(g=g, iters=passes, converged=converged, residual=dn, alpha=alpha)


def backward(W, C, tau, dist, G, mode, tol=1e-6, max_iter=1000, alpha=1.0):
    """dL/dW for L(A(W, C*(W)) C*(W)) at the solution C (Alg. 2, per-layer backward steps).

    mode "implicit": g solves (I - dF/dC)^T g = v by the iteration of Sec. 4.2.
    mode "dense":    same system by Gaussian elimination (the definition, Eq. "grad"/"inv").
    mode "jfb":      g = v, the zeroth-order Neumann truncation M* = I (Sec. 4.3, Eq. "jfbgrad").
    dL/dW = direct + (dF/dW)^T g.  Returns dict(dW, g, v, iters, converged, residual, alpha).
    """
    v, direct = loss_cotangents(W, C, tau, dist, G)
    info = dict(iters=0, converged=True, residual=0.0, alpha=alpha)
    if mode == "jfb":
        g = v
    elif mode == "dense":
        g = solve_dense(C, W, tau, dist, v)
    elif mode == "implicit":
        s = solve_iterative(C, W, tau, dist, v, tol, max_iter, alpha)
        g = s["g"]
        info = dict(iters=s["iters"], converged=s["converged"], residual=s["residual"], alpha=s["alpha"])
    else:
        raise ValueError(mode)
    dW = direct + vjp_F(C, W, tau, dist, g)[1]
    return dict(dW=dW, g=g, v=v, **info)


def inverse_matrix_iteration(J, alpha=0.25, tol=1e-12, max_iter=100000):
    """The paper's own matrix iteration for M* = (I - dF/dC)^-1 (Eq. "backiter2" with averaging):
        M(t+1) = alpha (J M(t) + I) + (1 - alpha) M(t),  M(0) = I.
    Kept to show that the vector form above solves the same system."""
    n = J.shape[0]
    M = np.eye(n)
    for t in range(1, max_iter + 1):
        Mn = alpha * (J @ M + np.eye(n)) + (1 - alpha) * M
        dn = np.linalg.norm(Mn - M)
        M = Mn
        if dn <= tol:
            break
    return M, t
