"""Pins for the oracle with different numbers of queries and keys (N_q x N_k scores, causal
mask aligned at the bottom right): reductions to the square problem, which is pinned on its own
(tests/test_oracle_exact.py), finite differences, and agreement of the tiled algorithms in
binary64 with the plain definition."""
import numpy as np
import pytest

from oracle import exact, flash


def _rand(rng, nq, nk, d):
    return (rng.standard_normal((nq, d)), rng.standard_normal((nk, d)), rng.standard_normal((nk, d)),
            rng.standard_normal((nq, d)))


def test_fewer_queries_than_keys_is_the_tail_of_the_square_problem():
    """N_q < N_k, causal: the N_q queries are the LAST N_q rows of the square N_k problem (the
    decoding-with-a-prefix case); gradients of K, V equal the square problem's with dO = 0 on the
    other rows."""
    rng = np.random.default_rng(11)
    nq, nk, d = 5, 13, 4
    Qf, K, V, dOf = _rand(rng, nk, nk, d)
    dOf[: nk - nq] = 0.0
    O_sq, L_sq, dQ_sq, dK_sq, dV_sq, _ = exact.forward_backward(Qf, K, V, dOf, 0.7, True)
    O, L, dQ, dK, dV, _ = exact.forward_backward(Qf[nk - nq:], K, V, dOf[nk - nq:], 0.7, True)
    assert np.allclose(O, O_sq[nk - nq:], rtol=0, atol=1e-14) and np.allclose(L, L_sq[nk - nq:], atol=1e-14)
    assert np.allclose(dQ, dQ_sq[nk - nq:], atol=1e-14)
    assert np.allclose(dK, dK_sq, atol=1e-14) and np.allclose(dV, dV_sq, atol=1e-14)
    # the same through forward() / backward()
    O2, L2 = exact.forward(Qf[nk - nq:], K, V, 0.7, True)
    g = exact.backward(Qf[nk - nq:], K, V, dOf[nk - nq:], 0.7, True)
    assert np.array_equal(O2, O) and np.allclose(g[0], dQ, atol=1e-14) and np.allclose(g[1], dK, atol=1e-14)


def test_more_queries_than_keys_leading_rows_see_nothing():
    """N_q > N_k, causal: the first N_q - N_k queries see no key (O = 0, L = -inf, no gradient);
    the rest is the square N_k problem."""
    rng = np.random.default_rng(12)
    nq, nk, d = 11, 4, 3
    Q, K, V, dO = _rand(rng, nq, nk, d)
    O, L, dQ, dK, dV, delta = exact.forward_backward(Q, K, V, dO, 1.3, True)
    e = nq - nk
    assert (O[:e] == 0).all() and np.isneginf(L[:e]).all() and (dQ[:e] == 0).all() and (delta[:e] == 0).all()
    ref = exact.forward_backward(Q[e:], K, V, dO[e:], 1.3, True)
    for got, want in zip((O[e:], L[e:], dQ[e:], dK, dV), ref[:5]):
        assert np.allclose(got, want, atol=1e-14)


@pytest.mark.parametrize("nq,nk,causal", [(6, 9, True), (9, 6, True), (5, 8, False)])
def test_rectangular_gradients_by_finite_differences(nq, nk, causal):
    rng = np.random.default_rng(nq * 100 + nk)
    d, alpha = 3, 0.9
    Q, K, V, G = _rand(rng, nq, nk, d)
    loss = lambda q, k, v: float(np.sum(exact.forward(q, k, v, alpha, causal)[0] * G))
    dQ, dK, dV, _ = exact.backward(Q, K, V, G, alpha, causal)
    h = 1e-6
    for X, dX, idx in ((Q, dQ, 0), (K, dK, 1), (V, dV, 2)):
        num = np.zeros_like(X)
        for i in range(X.shape[0]):
            for j in range(X.shape[1]):
                args = [Q.copy(), K.copy(), V.copy()]
                args[idx][i, j] += h; up = loss(*args)
                args[idx][i, j] -= 2 * h; dn = loss(*args)
                num[i, j] = (up - dn) / (2 * h)
        assert np.allclose(num, dX, rtol=1e-6, atol=1e-8)


@pytest.mark.parametrize("nq,nk", [(20, 52), (52, 20), (33, 33), (1, 70), (70, 1)])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("variant", [flash.STANDARD, flash.MITIGATED])
def test_tiled_algorithms_in_binary64_equal_the_definition(nq, nk, causal, variant):
    """Alg. 1 / Alg. 3 and Alg. 2 over key tiles of 8 (ragged last tile, tiles that some rows do not
    see at all) against the untiled fp64 definition."""
    rng = np.random.default_rng(nq + 7 * nk)
    Q, K, V, dO = _rand(rng, nq, nk, 4)
    ref = exact.forward_backward(Q, K, V, dO, 0.6, causal)
    f = flash.forward(Q, K, V, 0.6, causal, variant, Bc=8, prec=flash.FP64)
    assert np.allclose(f["O"], ref[0], atol=1e-12)
    seen = ~np.isneginf(ref[1])
    assert np.array_equal(np.isneginf(f["L"]), ~seen) and np.allclose(f["L"][seen], ref[1][seen], atol=1e-12)
    dQ, dK, dV, delta = flash.backward(Q, K, V, f["O"], dO, f["L"], 0.6, causal, Bc=8, Br=16, prec=flash.FP64)
    for got, want in zip((dQ, dK, dV), ref[2:5]):
        assert np.isfinite(got).all() and np.allclose(got, want, atol=1e-12)
    dr = flash.delta_recomputed(Q, K, V, dO, f["L"], 0.6, causal, Bc=8, prec=flash.FP64)
    assert np.allclose(dr, ref[5], atol=1e-12)


def test_bf16_dataflow_on_rows_that_see_nothing():
    """The low-precision emulation keeps O = 0 / L = -inf on unseen rows and finite values
    elsewhere, for both normalisers."""
    rng = np.random.default_rng(3)
    from oracle.bf16 import round_to_bf16
    Q, K, V, dO = [round_to_bf16(x.astype(np.float32)) for x in _rand(rng, 40, 24, 8)]
    for variant in (flash.STANDARD, flash.MITIGATED):
        f = flash.forward(Q, K, V, 0.35, True, variant, Bc=8)
        assert (f["O"][:16] == 0).all() and np.isneginf(f["L"][:16]).all()
        assert np.isfinite(f["O"]).all() and np.isfinite(f["L"][16:]).all()
        g = flash.backward(Q, K, V, f["O"], dO, f["L"], 0.35, True, Bc=8, Br=8)
        assert all(np.isfinite(x).all() for x in g[:3]) and (g[0][:16] == 0).all()
