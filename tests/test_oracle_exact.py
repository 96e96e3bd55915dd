"""Pins for oracle.exact (CPU only): brute force, finite differences, closed forms and the
identities the paper states (Sec. 2.2, Sec. 3.2, Eq. 2)."""
import math

import numpy as np
import pytest

from oracle import exact


def _rand(seed, N, d, scale=1.0):
    rng = np.random.default_rng(seed)
    return [scale * rng.standard_normal((N, d)) for _ in range(4)]


def _brute_forward(Q, K, V, alpha, causal):
    """Literal per-element loops over the definition of softmax attention."""
    N, d = Q.shape
    O = np.zeros((N, d)); L = np.zeros(N)
    for r in range(N):
        cols = [c for c in range(K.shape[0]) if (not causal or c <= r)]
        s = [alpha * sum(Q[r, k] * K[c, k] for k in range(d)) for c in cols]
        mx = max(s)
        w = [math.exp(v - mx) for v in s]
        tot = sum(w)
        for i in range(d):
            O[r, i] = sum(w[j] * V[cols[j], i] for j in range(len(cols))) / tot
        L[r] = mx + math.log(tot)
    return O, L


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,d", [(1, 1), (5, 3), (8, 4)])
def test_forward_matches_brute_force(N, d, causal):
    Q, K, V, _ = _rand(N * 10 + d, N, d)
    O, L = exact.forward(Q, K, V, 0.7, causal)
    Ob, Lb = _brute_forward(Q, K, V, 0.7, causal)
    assert np.allclose(O, Ob, rtol=0, atol=1e-14)
    assert np.allclose(L, Lb, rtol=0, atol=1e-14)


def _loss(Q, K, V, dO, alpha, causal):
    O, _ = exact.forward(Q, K, V, alpha, causal)
    return float(np.sum(O * dO))


@pytest.mark.parametrize("causal", [False, True])
def test_backward_matches_central_finite_differences(causal):
    """loss = sum(O o dO) has dloss/dO = dO, so its numerical gradient is (dQ, dK, dV)."""
    N, d, alpha = 12, 5, 0.45
    Q, K, V, dO = _rand(3, N, d)
    dQ, dK, dV, _ = exact.backward(Q, K, V, dO, alpha, causal)
    h = 1e-5
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        num = np.zeros_like(X)
        for i in range(N):
            for j in range(d):
                old = X[i, j]
                X[i, j] = old + h; fp = _loss(Q, K, V, dO, alpha, causal)
                X[i, j] = old - h; fm = _loss(Q, K, V, dO, alpha, causal)
                X[i, j] = old
                num[i, j] = (fp - fm) / (2 * h)
        err = np.max(np.abs(num - G)) / np.max(np.abs(G))
        assert err < 1e-7, (name, err)


def test_backward_finite_differences_directional_on_tiny_workload():
    """Same check at the size of the smallest benchmark configuration (N=128, d=64), along
    random directions instead of per element."""
    from paper_2510_04212_amd import synth
    w = synth.WORKLOADS["tiny"]
    x = synth.head_f64(w, 0, 0)
    Q, K, V, dO = x["Q"], x["K"], x["V"], x["dO"]
    dQ, dK, dV, _ = exact.backward(Q, K, V, dO, w.alpha, w.causal)
    rng = np.random.default_rng(5)
    h = 1e-5
    for name, X, G in (("Q", Q, dQ), ("K", K, dK), ("V", V, dV)):
        for _ in range(4):
            D = rng.standard_normal(X.shape)
            args = {"Q": Q, "K": K, "V": V}
            args[name] = X + h * D; fp = _loss(args["Q"], args["K"], args["V"], dO, w.alpha, w.causal)
            args[name] = X - h * D; fm = _loss(args["Q"], args["K"], args["V"], dO, w.alpha, w.causal)
            num = (fp - fm) / (2 * h)
            ana = float(np.sum(G * D))
            assert abs(num - ana) <= 1e-7 * max(1.0, abs(ana)), (name, num, ana)


@pytest.mark.parametrize("causal", [False, True])
def test_rows_of_P_sum_to_one_and_L_is_logsumexp(causal):
    Q, K, V, _ = _rand(9, 33, 8, 2.0)
    S = exact.scores(Q, K, 0.3, causal)
    P, L = exact.softmax_rows(S)
    assert np.max(np.abs(P.sum(1) - 1)) < 1e-14
    with np.errstate(divide="ignore"):
        ref = np.log(np.sum(np.exp(S), axis=1))
    assert np.allclose(L, ref, atol=1e-12)
    if causal:
        assert np.all(P[np.triu_indices(33, 1)] == 0)


def test_closed_forms():
    N, d, alpha = 17, 6, 0.5
    Q, K, V, dO = _rand(21, N, d)
    # causal row 0 sees only key 0
    O, L = exact.forward(Q, K, V, alpha, True)
    assert np.allclose(O[0], V[0], atol=1e-15)
    assert abs(L[0] - alpha * Q[0] @ K[0]) < 1e-14
    # Q = 0: uniform attention over the visible keys
    O, L = exact.forward(np.zeros_like(Q), K, V, alpha, True)
    for r in range(N):
        assert np.allclose(O[r], V[:r + 1].mean(0), atol=1e-14)
        assert abs(L[r] - math.log(r + 1)) < 1e-14
    # all keys equal: same
    O, L = exact.forward(Q, np.tile(K[:1], (N, 1)), V, alpha, False)
    assert np.allclose(O, np.tile(V.mean(0), (N, 1)), atol=1e-13)
    # V constant per column: O equals it
    Vc = np.tile(V[:1], (N, 1))
    O, _ = exact.forward(Q, K, Vc, alpha, False)
    assert np.allclose(O, Vc, atol=1e-14)
    # dO = 0: no gradient; and dV for Q = 0 non-causal is the column mean of dO in every row
    dQ, dK, dV, delta = exact.backward(Q, K, V, np.zeros_like(dO), alpha, True)
    assert not dQ.any() and not dK.any() and not dV.any() and not delta.any()
    dQ, dK, dV, _ = exact.backward(np.zeros_like(Q), K, V, dO, alpha, False)
    assert np.allclose(dV, np.tile(dO.sum(0) / N, (N, 1)), atol=1e-14)
    assert np.allclose(dK, 0, atol=1e-15)          # dK = alpha dS^T Q with Q = 0


@pytest.mark.parametrize("causal", [False, True])
def test_delta_identity_and_dS_rows_sum_to_zero(causal):
    """Sec. 3.2: rowsum(dO o O) = rowsum(dP o P); hence the rows of dS sum to zero."""
    Q, K, V, dO = _rand(31, 40, 8)
    alpha = 0.35
    S = exact.scores(Q, K, alpha, causal)
    P, _ = exact.softmax_rows(S)
    O = P @ V
    dP = dO @ V.T
    d1 = np.sum(dO * O, axis=1)
    d2 = np.sum(dP * P, axis=1)
    assert np.allclose(d1, d2, atol=1e-13)
    dS = P * (dP - d1[:, None])
    assert np.max(np.abs(dS.sum(1))) < 1e-13
    _, _, _, delta = exact.backward(Q, K, V, dO, alpha, causal)
    assert np.allclose(delta, d1, atol=1e-15)


@pytest.mark.parametrize("causal", [False, True])
def test_delta_perturbation_closed_form(causal):
    """Eq. 2: replacing delta by delta + v changes dQ by  -alpha diag(v) (P K)  exactly
    (dQ_hp - dQ_lp = alpha diag(delta_lp - delta_hp) P K), and leaves dV unchanged."""
    Q, K, V, dO = _rand(41, 24, 7)
    alpha = 0.6
    dQ, dK, dV, delta = exact.backward(Q, K, V, dO, alpha, causal)
    v = np.random.default_rng(1).standard_normal(24) * 1e-2
    dQ2, dK2, dV2, _ = exact.backward(Q, K, V, dO, alpha, causal, delta=delta + v)
    P, _ = exact.softmax_rows(exact.scores(Q, K, alpha, causal))
    assert np.allclose(dQ - dQ2, alpha * np.diag(v) @ (P @ K), atol=1e-14)
    assert np.allclose(dK - dK2, alpha * (P * v[:, None]).T @ Q, atol=1e-14)
    assert np.array_equal(dV, dV2)


def test_bh_wrapper_selects_heads():
    rng = np.random.default_rng(2)
    Q, K, V, dO = [rng.standard_normal((2, 3, 9, 4)) for _ in range(4)]
    out = exact.forward_backward_bh(Q, K, V, dO, 0.5, True, heads=[(1, 2)])
    O, L, dQ, dK, dV, delta = exact.forward_backward(Q[1, 2], K[1, 2], V[1, 2], dO[1, 2], 0.5, True)
    assert np.array_equal(out["O"][1, 2], O) and np.array_equal(out["dK"][1, 2], dK)
    assert np.isnan(out["O"][0, 0]).all()


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("row_block", [None, 1, 7, 16])
def test_forward_backward_slabs_equal_separate_functions(causal, row_block):
    """forward_backward() (optionally visiting query rows in slabs) must reproduce forward() and
    backward(), which the tests above pin."""
    Q, K, V, dO = _rand(51, 37, 5)
    O, L = exact.forward(Q, K, V, 0.4, causal)
    dQ, dK, dV, delta = exact.backward(Q, K, V, dO, 0.4, causal)
    got = exact.forward_backward(Q, K, V, dO, 0.4, causal, row_block=row_block)
    for a, b in zip(got, (O, L, dQ, dK, dV, delta)):
        assert np.max(np.abs(a - b)) < 1e-13
