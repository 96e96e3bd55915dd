"""The paper's tiled attention (online softmax over key tiles) in a chosen working precision
(test infrastructure only).

forward()   the flash-attention forward (Alg. 1): per key tile, a running normaliser m, the
            unnormalised probabilities P-bar = exp(S - m), their running row sum l and the
            running unnormalised output, all rescaled when m grows; O = O-bar / l and
            L = m + log l at the end (Sec. 2.2).  With variant = MITIGATED the normaliser of a
            tile row follows Sec. 4 (Alg. 3): beta r_m or 0 instead of the tile row maximum r_m
            when r_m is attained, within eps, more than once.
backward()  the flash-attention backward (Alg. 2): P = exp(S - L) recomputed per tile pair,
            delta = rowsum(dO o O), dS = P o (dP - delta), and the three gradient sums.

A `Precision` fixes the arithmetic:
  FP64  every step in binary64, no rounding points.  In this mode the functions must agree
        with oracle.exact to rounding error for every tile size and both variants (online
        softmax is exact; Alg. 3 only changes the softmax shift, Sec. 4).
  BF16  the low-precision dataflow the paper analyses (Sec. 3.3.2): operands are bf16 values,
        every product/sum is carried in binary32, and results are rounded to bf16 at stated
        points.  The rounding points and the reasons for them:
          (r1) P-bar is rounded to bf16 before it is used (it is a bf16 tensor in the paper's
               low-precision flow: the inputs of the P-bar V product are results of earlier
               bf16 operations, Sec. 3.3.2);
          (r2) the row sum l is taken over the ROUNDED P-bar, in binary32, so numerator and
               denominator use the same numbers (the paper uses one tensor P-bar for both);
          (r3) the unnormalised output O-bar = P-bar V is accumulated in binary32 over ALL key
               tiles and rounded to bf16 once, BEFORE the division by l (the paper's
               "(.)_lp": dot product in FP32, final result rounded to BF16; its analysed
               setting is tile = N, Sec. 3.2);
          (r4) O = O-bar / l is rounded to bf16 again when stored;
          (r5) m, l and L stay in binary32;
          (r6) backward: delta = rowsum(dO o O) uses the bf16 O of (r4) (this is delta_lp,
               Claim 1); P = exp(S - L) in binary32 is rounded to bf16 only as the operand of
               P^T dO; dS = P o (dP - delta) uses the binary32 P and is rounded to bf16 as the
               operand of dS K and dS^T Q; accumulators are binary32; alpha multiplies the
               binary32 dQ, dK accumulators once at the end; dQ, dK, dV are stored as bf16.
        Scores S stay in binary32 and alpha is applied to the binary32 Q K^T (never by
        pre-scaling Q in bf16).
          (r7) the exponential returns 0 where its result would be a subnormal binary32 number
               (below 2^-126): Sec. 4 warns that a larger beta risks underflow without fixing
               where underflow sets in; whether a row loses all of its probabilities (l = 0,
               0/0) is decided in the arithmetic of the kernels, whose exponential instruction
               produces no subnormal results.  Sums and products keep subnormals.

Rows of the score matrix are independent in the forward pass, so the query block size B_r has
no numerical effect there and all rows are processed together; B_c (the key tile) matters for
Alg. 3 because its test looks at one tile row at a time.
"""
from dataclasses import dataclass
from typing import Callable

import numpy as np

from .bf16 import round_to_bf16
from .fp8 import round_to_e4m3

STANDARD = 0    # Alg. 1
MITIGATED = 1   # Alg. 3


@dataclass(frozen=True)
class Precision:
    name: str
    dtype: type
    rnd: Callable
    rnd_pv: Callable = None     # rounding of the two operands of the P-bar V product, if not `rnd`
    exp: Callable = np.exp      # the exponential of P-bar, of the rescale factor and of P


def exp_without_subnormals(x):
    """exp in binary32 with results below the smallest normal number (2^-126) replaced by 0 (r7)."""
    y = np.exp(np.asarray(x, dtype=np.float32))
    return np.where(y < np.float32(2.0 ** -126), np.float32(0.0), y)


# Largest shift of the normaliser the optional guard of forward() lets Alg. 3 make (natural-log
# units): the row maximum then still maps to exp(-60) ~ 9e-27, 27 units above the underflow
# threshold of (r7), so every probability within e^-27 of the largest survives.
GUARD_LIMIT = 60.0

FP64 = Precision("fp64", np.float64, lambda x: x)
BF16 = Precision("bf16", np.float32, round_to_bf16, None, exp_without_subnormals)
# The BF16 dataflow with the one product the paper's analysis singles out, P-bar V (Sec. 3.3.2),
# taken in 8-bit floating point: P-bar and V are rounded to E4M3 (rounding point (r1) moves to that
# format, V is quantised without a scale factor), the products are summed in binary32, and
# everything downstream -- (r2) the row sum of the rounded P-bar, (r3), (r4) -- is unchanged.
# Forward only; an exploration of the paper's future-work remark on FP8, not something it specifies.
BF16_PV_E4M3 = Precision("bf16, P-bar V in e4m3", np.float32, round_to_bf16, round_to_e4m3,
                         exp_without_subnormals)


def _tile_scores(Qw, Kj, alpha, causal, k0, prec, shift=0):
    """alpha Q K_j^T for the key tile starting at column k0 (Sec. 2.2), masked entries -inf.
    shift = N_k - N_q: the causal mask is aligned at the bottom right (see oracle.exact)."""
    S = (Qw @ Kj.T) * prec.dtype(alpha)
    if causal:
        r = np.arange(Qw.shape[0])[:, None]
        c = (k0 + np.arange(Kj.shape[0]))[None, :]
        S = np.where(c > r + shift, prec.dtype(-np.inf), S)
    return S.astype(prec.dtype)


def forward(Q, K, V, alpha, causal, variant=STANDARD, beta=2.0, eps=1e-3, Bc=None, prec=BF16,
            round_obar=True, guard=False):
    """One head, Alg. 1 (variant 0) or Alg. 3 (variant 1).

    guard=True is a labelled deviation from Alg. 3, not part of the paper: the rule leaves the
    normaliser at the tile row maximum whenever it would move it by more than GUARD_LIMIT
    ((beta-1) r_m for a positive repeated maximum, -r_m for a negative one), i.e. where Sec. 4's
    "risk of underflow" would otherwise turn the row into 0/0.

    round_obar=False drops rounding point (r3): the unnormalised output stays in working
    precision until after the division (the experiment of Sec. 3.3.2 in which computing only
    O-bar = P-bar V in FP32 is enough to stabilise training); (r4) is kept.

    Returns a dict:
      O      [N,d]  output (bf16-valued in BF16 mode)
      Ohp    [N,d]  Oacc / l with no rounding at (r3) or (r4): the "O computed in high
                    precision" of Sec. 3.2, from which delta_hp = rowsum(dO o Ohp) is formed
      L      [N]    logsumexp  m + log l
      Obar   [N,d]  unnormalised output after rounding point (r3)
      Oacc   [N,d]  unnormalised output before (r3) (working precision)
      ell,m  [N]    final running sum / normaliser
      fired  [N]    number of key tiles in which the Alg. 3 rule changed m' for the row
      ones   [N]    number of entries with (rounded) P-bar exactly 1, counted when produced
    """
    dt = prec.dtype
    Qw = np.asarray(Q, dtype=dt); Kw = np.asarray(K, dtype=dt); Vw = np.asarray(V, dtype=dt)
    N, d = Qw.shape
    Nk = Kw.shape[0]
    Bc = Nk if Bc is None else int(Bc)
    m = np.full(N, -np.inf, dtype=dt)          # running normaliser of every row
    ell = np.zeros(N, dtype=dt)                # running row sum of P-bar
    acc = np.zeros((N, d), dtype=dt)           # running unnormalised output
    fired = np.zeros(N, dtype=np.int64)
    ones = np.zeros(N, dtype=np.int64)
    with np.errstate(invalid="ignore", over="ignore", divide="ignore"):
        for k0 in range(0, Nk, Bc):
            Kj = Kw[k0:k0 + Bc]; Vj = Vw[k0:k0 + Bc]
            S = _tile_scores(Qw, Kj, alpha, causal, k0, prec, Nk - N)
            # normaliser proposed by this tile: the tile row maximum r_m, or Sec. 4's choice
            r_m = np.max(S, axis=1)
            m_prime = r_m
            if variant == MITIGATED:
                # Sec. 4: r_s counts the entries within eps of r_m; more than one of them means
                # several P-bar would be exactly 1, so the normaliser moves off the maximum:
                # to beta r_m when r_m > 0, to 0 when r_m < 0 (every P-bar then stays below 1)
                r_s = np.sum((r_m[:, None] - S) <= dt(eps), axis=1)
                repeated = r_s > 1
                if guard:
                    shift_by = np.where(r_m > 0, (dt(beta) - dt(1.0)) * r_m, -r_m)
                    repeated = repeated & (shift_by <= dt(GUARD_LIMIT))
                m_prime = np.where((r_m > 0) & repeated, dt(beta) * r_m, r_m)
                m_prime = np.where((r_m < 0) & repeated, dt(0.0), m_prime)
                fired += (m_prime != r_m).astype(np.int64)
            m_new = np.maximum(m, m_prime.astype(dt))          # the normaliser only ever grows
            # rows with nothing visible yet have m_new = -inf: they contribute nothing
            safe_m = np.where(np.isneginf(m_new), dt(0.0), m_new)
            Pbar = prec.exp(S - safe_m[:, None]).astype(dt)                # (r7)
            rnd_pv = prec.rnd_pv or prec.rnd
            Phat = rnd_pv(Pbar).astype(dt)                                 # (r1)
            if prec.rnd_pv is not None:
                Vj = prec.rnd_pv(Vj).astype(dt)
            # what was accumulated under the old normaliser is brought to the new one
            corr = np.where(np.isneginf(m), dt(0.0), prec.exp(m - safe_m)).astype(dt)
            ell = (corr * ell + np.sum(Phat, axis=1, dtype=dt)).astype(dt)  # (r2)
            acc = (corr[:, None] * acc + Phat @ Vj).astype(dt)
            ones += np.sum(Phat == dt(1.0), axis=1)
            m = m_new
        Obar = prec.rnd(acc).astype(dt) if round_obar else acc             # (r3)
        seen = ~np.isneginf(m)[:, None]       # a query with no visible key (N_q > N_k) outputs 0, L = -inf
        O = np.where(seen, prec.rnd(Obar / ell[:, None]), dt(0.0)).astype(dt)   # (r4)
        Ohp = np.where(seen, acc / ell[:, None], dt(0.0)).astype(dt)
        L = (m + np.log(ell)).astype(dt)                                    # row logsumexp
    return {"O": O, "L": L, "Obar": Obar, "Oacc": acc, "ell": ell, "m": m,
            "fired": fired, "ones": ones, "Ohp": Ohp}


def backward(Q, K, V, O, dO, L, alpha, causal, Bc=None, Br=None, prec=BF16):
    """One head, Alg. 2.  O and L are the forward pass's outputs (O bf16-valued in BF16 mode).

    O is used for delta = rowsum(dO o O) only and is taken as given: passing the
    forward pass's `Ohp` instead of its bf16 `O` gives delta_hp, the variant of Sec. 3.2 that
    restores stability with everything else unchanged.

    Returns dQ, dK, dV (bf16-valued in BF16 mode) and delta in working precision.
    """
    dt = prec.dtype
    Qw = np.asarray(Q, dtype=dt); Kw = np.asarray(K, dtype=dt); Vw = np.asarray(V, dtype=dt)
    Ow = np.asarray(O, dtype=dt); dOw = np.asarray(dO, dtype=dt); Lw = np.asarray(L, dtype=dt)
    N, d = Qw.shape
    Nk = Kw.shape[0]
    Bc = Nk if Bc is None else int(Bc)
    Br = N if Br is None else int(Br)
    Lw = np.where(np.isneginf(Lw), dt(0.0), Lw)     # queries that see no key: every score is -inf, P = 0
    delta = np.sum(dOw * Ow, axis=1, dtype=dt)        # (r6): from the O handed in
    dQ = np.zeros((N, d), dtype=dt)
    dK = np.zeros((Nk, d), dtype=dt)
    dV = np.zeros((Nk, d), dtype=dt)
    with np.errstate(invalid="ignore", over="ignore"):
        for k0 in range(0, Nk, Bc):                    # key tiles outside, query tiles inside
            Kj = Kw[k0:k0 + Bc]; Vj = Vw[k0:k0 + Bc]
            for q0 in range(0, N, Br):
                Qi = Qw[q0:q0 + Br]; dOi = dOw[q0:q0 + Br]
                S = (Qi @ Kj.T) * dt(alpha)
                if causal:
                    r = (q0 + np.arange(Qi.shape[0]))[:, None]
                    c = (k0 + np.arange(Kj.shape[0]))[None, :]
                    S = np.where(c > r + (Nk - N), dt(-np.inf), S)
                # the probabilities again, from the stored logsumexp (no running statistics)
                P = prec.exp(S.astype(dt) - Lw[q0:q0 + Br, None]).astype(dt)
                dV[k0:k0 + Bc] += prec.rnd(P).astype(dt).T @ dOi          # P rounded as an operand only
                dP = (dOi @ Vj.T).astype(dt)
                dS = (P * (dP - delta[q0:q0 + Br, None])).astype(dt)      # from the unrounded P
                dSr = prec.rnd(dS).astype(dt)                             # rounded once, as an operand
                dQ[q0:q0 + Br] += dSr @ Kj
                dK[k0:k0 + Bc] += dSr.T @ Qi
    # alpha belongs to dS (Eq. 2); applied once to the binary32 sums instead
    dQ = prec.rnd(dQ * dt(alpha)).astype(dt)
    dK = prec.rnd(dK * dt(alpha)).astype(dt)
    dV = prec.rnd(dV).astype(dt)
    return dQ, dK, dV, delta


def delta_recomputed(Q, K, V, dO, L, alpha, causal, Bc=None, prec=BF16):
    """delta = rowsum(P o dP) with P = exp(S - L), dP = dO V^T, accumulated over key tiles in
    working precision, nothing rounded (Sec. 3.2: recomputing the output in the backward pass
    instead of reading the forward's bf16 O; rowsum(P o dP) = rowsum(dO o (P V)))."""
    dt = prec.dtype
    Qw = np.asarray(Q, dtype=dt); Kw = np.asarray(K, dtype=dt); Vw = np.asarray(V, dtype=dt)
    dOw = np.asarray(dO, dtype=dt); Lw = np.asarray(L, dtype=dt)
    N = Qw.shape[0]
    Nk = Kw.shape[0]
    Bc = Nk if Bc is None else int(Bc)
    Lw = np.where(np.isneginf(Lw), dt(0.0), Lw)
    delta = np.zeros(N, dtype=dt)
    with np.errstate(invalid="ignore", over="ignore"):
        for k0 in range(0, Nk, Bc):
            Kj = Kw[k0:k0 + Bc]; Vj = Vw[k0:k0 + Bc]
            S = _tile_scores(Qw, Kj, alpha, causal, k0, prec, Nk - N)
            P = prec.exp(S - Lw[:, None]).astype(dt)
            dP = (dOw @ Vj.T).astype(dt)
            delta = (delta + np.sum(P * dP, axis=1, dtype=dt)).astype(dt)
    return delta


def forward_backward_bh(Q, K, V, dO, alpha, causal, variant=STANDARD, beta=2.0, eps=1e-3,
                        Bc=None, prec=BF16, heads=None):
    """[B,H,N,d] wrapper over forward() then backward(); see oracle.exact.forward_backward_bh."""
    Q = np.asarray(Q); B, H, N, d = Q.shape
    dt = prec.dtype
    out = {k: np.full((B, H, N, d), np.nan, dtype=dt) for k in ("O", "Obar", "dQ", "dK", "dV")}
    for k in ("L", "delta"):
        out[k] = np.full((B, H, N), np.nan, dtype=dt)
    out["fired"] = np.zeros((B, H, N), dtype=np.int64)
    out["ones"] = np.zeros((B, H, N), dtype=np.int64)
    todo = heads if heads is not None else [(b, h) for b in range(B) for h in range(H)]
    for (b, h) in todo:
        f = forward(Q[b, h], K[b, h], V[b, h], alpha, causal, variant, beta, eps, Bc, prec)
        dQ, dK, dV, delta = backward(Q[b, h], K[b, h], V[b, h], f["O"], dO[b, h], f["L"],
                                     alpha, causal, Bc, None, prec)
        out["O"][b, h] = f["O"]; out["Obar"][b, h] = f["Obar"]; out["L"][b, h] = f["L"]
        out["dQ"][b, h] = dQ; out["dK"][b, h] = dK; out["dV"][b, h] = dV
        out["delta"][b, h] = delta
        out["fired"][b, h] = f["fired"]; out["ones"][b, h] = f["ones"]
    return out
