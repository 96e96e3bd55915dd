"""fp64 attention forward and backward from the plain definitions (test infrastructure only).

Everything here is the textbook form the paper starts from (Sec. 2.2): the full
N x N score matrix is materialised, nothing is tiled, fused or reordered.  One
(batch, head) problem is an N x d triple Q, K, V; the 4-D wrappers loop over heads.

Conventions (the paper is silent on both; the choices are stated, not derived):
  * causal masking: query row r attends to key columns c <= r; when the numbers of queries and
    keys differ (N_q x d queries against N_k x d keys / values) the mask is aligned at the bottom
    right, c <= r + (N_k - N_q): the last query sees every key.  A query that sees no key at
    all (only possible when N_q > N_k) has P = 0, O = 0, L = -inf and takes no part in any
    gradient;
  * the softmax scale alpha multiplies the scores S = alpha Q K^T, and therefore
    appears once more in dQ and dK (Eq. 2 / Appendix E.2: dS = alpha P o (dP - delta)).
"""
import numpy as np


def scores(Q, K, alpha, causal):
    """S = alpha Q K^T (Sec. 2.2); masked entries are -inf."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    S = alpha * (Q @ K.T)
    if causal:
        n_q, n_k = S.shape
        r = np.arange(n_q)[:, None]
        c = np.arange(n_k)[None, :]
        S = np.where(c > r + (n_k - n_q), -np.inf, S)
    return S


def softmax_rows(S):
    """Row softmax and row logsumexp of S, via the safe form exp(S - rowmax S) (Sec. 3.3.2)."""
    m = np.max(S, axis=1, keepdims=True)
    empty = np.isneginf(m)                      # rows with every entry masked
    E = np.exp(S - np.where(empty, 0.0, m))
    ell = np.sum(E, axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        P = np.where(empty, 0.0, E / ell)
        L = np.where(empty, -np.inf, m + np.log(ell))[:, 0]
    return P, L


def forward(Q, K, V, alpha, causal):
    """One head.  Returns O = softmax(alpha Q K^T) V  [N,d]  and  L = logsumexp rows  [N]."""
    S = scores(Q, K, alpha, causal)
    P, L = softmax_rows(S)
    O = P @ np.asarray(V, dtype=np.float64)
    return O, L


def backward(Q, K, V, dO, alpha, causal, delta=None):
    """One head.  Gradients of a loss whose derivative w.r.t. O is dO (Alg. 2 without tiling).

        P     = softmax(alpha Q K^T)
        dV    = P^T dO
        dP    = dO V^T
        delta = rowsum(dO o O)                      (Alg. 2; Claim 1)
        dS    = P o (dP - delta)                    (Alg. 2; Eq. 2)
        dQ    = alpha dS K ,  dK = alpha dS^T Q     (Eq. 2, Appendix E.2)

    `delta` may be supplied to study the effect of a perturbed delta (Eq. 2);
    by default it is computed from the fp64 O.
    Returns dQ, dK, dV, delta.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    S = scores(Q, K, alpha, causal)
    P, _ = softmax_rows(S)
    O = P @ V
    dV = P.T @ dO
    dP = dO @ V.T
    if delta is None:
        delta = np.sum(dO * O, axis=1)
    dS = P * (dP - np.asarray(delta, dtype=np.float64)[:, None])
    dQ = alpha * (dS @ K)
    dK = alpha * (dS.T @ Q)
    return dQ, dK, dV, delta


def forward_backward(Q, K, V, dO, alpha, causal, row_block=None):
    """One head, everything at once: O, L, dQ, dK, dV, delta.

    Query rows are independent of one another in S, P, O, L, delta, dP, dS and dQ, and dK, dV are
    sums over query rows; `row_block` only bounds memory by visiting the rows in slabs
    (row_block=None: one slab, i.e. the full N x N matrices).  The arithmetic per entry is the
    same as in forward() / backward().
    """
    Q = np.asarray(Q, dtype=np.float64); K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64); dO = np.asarray(dO, dtype=np.float64)
    N, d = Q.shape
    Nk = K.shape[0]
    rb = N if row_block is None else int(row_block)
    O = np.empty((N, d)); L = np.empty(N); delta = np.empty(N)
    dQ = np.empty((N, d)); dK = np.zeros((Nk, d)); dV = np.zeros((Nk, d))
    for r0 in range(0, N, rb):
        r1 = min(N, r0 + rb)
        S = alpha * (Q[r0:r1] @ K.T)
        if causal:
            r = np.arange(r0, r1)[:, None]
            c = np.arange(Nk)[None, :]
            S = np.where(c > r + (Nk - N), -np.inf, S)
        P, L[r0:r1] = softmax_rows(S)
        O[r0:r1] = P @ V
        delta[r0:r1] = np.sum(dO[r0:r1] * O[r0:r1], axis=1)
        dV += P.T @ dO[r0:r1]
        dP = dO[r0:r1] @ V.T
        dS = P * (dP - delta[r0:r1, None])
        dQ[r0:r1] = alpha * (dS @ K)
        dK += alpha * (dS.T @ Q[r0:r1])
    return O, L, dQ, dK, dV, delta


def forward_backward_bh(Q, K, V, dO, alpha, causal, heads=None, row_block=None):
    """[B,H,N,d] wrapper.  `heads` = optional list of (b,h) pairs to compute (others skipped).

    Returns a dict of arrays shaped like the inputs ([B,H,N] for L and delta); entries of
    heads that were not requested are NaN.
    """
    Q = np.asarray(Q); B, H, N, d = Q.shape
    out = {k: np.full((B, H, N, d), np.nan) for k in ("O", "dQ", "dK", "dV")}
    out["L"] = np.full((B, H, N), np.nan)
    out["delta"] = np.full((B, H, N), np.nan)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in todo:
        O, L, dQ, dK, dV, delta = forward_backward(Q[b, h], K[b, h], V[b, h], dO[b, h], alpha, causal,
                                                     row_block)
        out["O"][b, h] = O; out["L"][b, h] = L
        out["dQ"][b, h] = dQ; out["dK"][b, h] = dK; out["dV"][b, h] = dV
        out["delta"][b, h] = delta
    return out
