"""Multi-step training harness around ONE attention head, on the CPU (test infrastructure only).

The paper follows, over training steps, how the low-precision delta_lp = rowsum(dO o O_lp)
differs from delta_hp = rowsum(dO o O_hp) and how the sum over tokens of that difference keeps
one sign, so that the error it puts into the query projection's gradient,

    dW^Q_hp - dW^Q_lp = alpha * sum_T (delta_lp - delta_hp)[T] * (P K)[T]^T X[T]        (Sec. 3.3.1)

accumulates over steps instead of cancelling (Claim 2, the cumulative curve of Sec. 3.3.1).
The paper's curve comes from GPT-2 training on OpenWebText; this harness reproduces the
mechanism on synthetic data: an attention layer whose input features X are fixed, whose key,
value and upstream-gradient tensors are fixed, and whose query projection W^Q (initialised to
the identity) is trained by plain gradient descent on the linear loss <O, G>:

    Q   = bf16( X bf16(W^Q) )            products exact, sums in binary64, one rounding via binary32
    O   = attention forward (oracle.flash.forward: Alg. 1 or Alg. 3, bf16 dataflow)
    dO  = G
    delta_lp, delta_hp as above; the step records  sum_T (delta_lp - delta_hp)[T]
    dQ  = Alg. 2 with the chosen delta
    dW^Q = X^T dQ (binary64 sums, stored binary32);   W^Q <- W^Q - lr dW^Q

Everything a step computes outside the attention calls is written out here with numpy.
"""
import numpy as np

from . import flash
from .bf16 import round_to_bf16


def project(X, W):
    """Q = bf16(X bf16(W)): X bf16-valued [N,D], W binary32 [D,d]."""
    Wb = round_to_bf16(np.asarray(W, dtype=np.float32)).astype(np.float64)
    Q64 = np.asarray(X, dtype=np.float64) @ Wb
    return round_to_bf16(Q64.astype(np.float32))


def grad_diff_closed_form(P, K, X, delta_lp, delta_hp, alpha):
    """Right-hand side of the identity of Sec. 3.3.1:
    alpha * sum_T (delta_lp - delta_hp)[T] (P K)[T]^T X[T], as a [d, D] matrix."""
    PK = np.asarray(P, dtype=np.float64) @ np.asarray(K, dtype=np.float64)
    c = np.asarray(delta_lp, dtype=np.float64) - np.asarray(delta_hp, dtype=np.float64)
    return alpha * (PK * c[:, None]).T @ np.asarray(X, dtype=np.float64)


def run(X, K, V, G, alpha, causal, steps, lr, variant=flash.STANDARD, delta_mode="lp", beta=2.0,
        eps=1e-3, Bc=64):
    """One head.  X, K, V, G: bf16-valued [N,d] arrays.  delta_mode: which delta the backward
    pass uses, "lp" (from the bf16 O) or "hp" (from the unrounded O, Sec. 3.2).
    Returns per-step arrays: sum_delta_diff, loss, rows_tied (rows with at least two unit
    probabilities), update_err (Frobenius norm of dW^Q_lp - dW^Q_hp of the step),
    cum_update_err (Frobenius norm of that difference summed over the steps so far: it grows
    like the step count when the per-step errors share a direction, like its square root
    when they do not), and the final W^Q (binary32 [d,d])."""
    X = np.asarray(X, dtype=np.float32)
    G32 = np.asarray(G, dtype=np.float32)
    d = X.shape[1]
    W = np.eye(d, dtype=np.float32)
    rec = {"sum_delta_diff": [], "loss": [], "rows_tied": [], "update_err": [], "cum_update_err": []}
    cumD = np.zeros((d, d), dtype=np.float64)
    for _ in range(steps):
        Q = project(X, W)
        f = flash.forward(Q, K, V, alpha, causal, variant, beta, eps, Bc)
        delta_lp = np.sum(G32 * f["O"], axis=1, dtype=np.float32)
        delta_hp = np.sum(G32 * f["Ohp"], axis=1, dtype=np.float32)
        dQ_lp, _, _, _ = flash.backward(Q, K, V, f["O"], G32, f["L"], alpha, causal, Bc, Bc)
        dQ_hp, _, _, _ = flash.backward(Q, K, V, f["Ohp"], G32, f["L"], alpha, causal, Bc, Bc)
        dW_lp = X.astype(np.float64).T @ dQ_lp.astype(np.float64)
        dW_hp = X.astype(np.float64).T @ dQ_hp.astype(np.float64)
        cumD += dW_lp - dW_hp
        rec["update_err"].append(float(np.linalg.norm(dW_lp - dW_hp)))
        rec["cum_update_err"].append(float(np.linalg.norm(cumD)))
        dW = (dW_lp if delta_mode == "lp" else dW_hp).astype(np.float32)
        W = (W - np.float32(lr) * dW).astype(np.float32)
        rec["sum_delta_diff"].append(float(np.sum(delta_lp.astype(np.float64) - delta_hp.astype(np.float64))))
        rec["loss"].append(float(np.sum(f["O"].astype(np.float64) * G32.astype(np.float64))))
        rec["rows_tied"].append(int(np.sum(f["ones"] >= 2)))
    out = {k: np.asarray(v) for k, v in rec.items()}
    out["W"] = W
    return out
