"""GPU tests on the repeated-row-maximum stress inputs: the signed rounding bias of the standard
forward (Sec. 3.3.2, Claim 3) and its removal by the stabilised forward (Sec. 4), measured on
the HIP kernels against the fp64 oracle.

The acceptance criterion of the build target -- the mitigated variant's mean signed error is at
least 10x closer to zero than the standard variant's -- is asserted on `pairs_skew`, the input on
which the paper's mechanism operates (exactly two unit probabilities per row, every other
probability ~1e-6, one-signed V).  On the rank-2 `tied*` inputs both variants sit at the sampling
noise floor (symmetric V: exactly zero expected bias; one-signed V: rows are not peaky enough
unless the scores reach the range where the stabilised normaliser underflows), which is
asserted as such; their numbers are printed.

The stress input AS SPECIFIED (`tied_q1`, `tied_skew_q1`: Q's rank-2 coefficients at 1.0, row
maxima up to ~140) is where Alg. 3 with beta = 2 meets its own limit (Sec. 4: "larger values risk
underflow"): some rows lose every probability.  test_tied_max_stress_as_specified pins what the
kernels do there -- which rows are lost, what that does to the gradients, what the guarded form
does instead -- against the oracle, and states the signed errors as they are.
"""
import numpy as np
import pytest
import torch

from oracle import exact, flash, metrics
from paper_2510_04212_amd import synth
from test_gpu_parity import run_gpu, check_head, head_np, DEV

pytestmark = pytest.mark.gpu


def _signed_stats(lib, name, with_backward_ref=False):
    """Per-variant mean signed errors of O, delta and dV over ALL heads of workload `name`."""
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    got = {v: run_gpu(lib, x, w.causal, w.alpha, v) for v in (0, 1)}
    eO = {0: [], 1: []}; eD = {0: [], 1: []}; eV = {0: [], 1: []}
    for b in range(w.B):
        for h in range(w.H):
            xs = head_np(x, b, h)
            if with_backward_ref:
                O, L, dQ, dK, dV, delta = exact.forward_backward(xs["Q"], xs["K"], xs["V"], xs["dO"], w.alpha, w.causal)
            else:
                O, L = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
                delta = np.sum(xs["dO"] * O, axis=1)
                dV = None
            for v in (0, 1):
                eO[v].append((got[v]["O"][b, h].double().cpu().numpy() - O).ravel())
                eD[v].append(got[v]["delta"][b, h].double().cpu().numpy() - delta)
                if dV is not None:
                    eV[v].append((got[v]["dV"][b, h].double().cpu().numpy() - dV).ravel())
    out = {}
    for v in (0, 1):
        o = np.concatenate(eO[v]); d = np.concatenate(eD[v])
        out[v] = {"O_mean": o.mean(), "O_noise": o.std() / np.sqrt(o.size),
                  "delta_mean": d.mean(), "delta_noise": d.std() / np.sqrt(d.size)}
        if eV[v]:
            dv = np.concatenate(eV[v])
            out[v]["dV_mean"] = dv.mean(); out[v]["dV_noise"] = dv.std() / np.sqrt(dv.size)
    print(f"\n[{name}] mean signed error vs fp64 (all {w.B * w.H} heads)")
    for v in (0, 1):
        s = out[v]
        extra = f"  dV {s['dV_mean']:+.3e} +- {s['dV_noise']:.1e}" if "dV_mean" in s else ""
        print(f"   variant {v}: O {s['O_mean']:+.3e} +- {s['O_noise']:.1e}   "
              f"delta_lp-delta_hp {s['delta_mean']:+.3e} +- {s['delta_noise']:.1e}{extra}")
    return out, x, got, w


def test_bias_and_its_removal_on_paired_keys_one_signed_values(lib):
    st, x, got, w = _signed_stats(lib, "pairs_skew", with_backward_ref=True)
    # standard variant: O biased negative far outside the noise, delta_lp - delta_hp positive (Claim 3)
    assert st[0]["O_mean"] < -50 * st[0]["O_noise"]
    assert st[0]["delta_mean"] > 20 * st[0]["delta_noise"]
    # mitigated variant: at least 10x closer to zero
    assert abs(st[1]["O_mean"]) <= abs(st[0]["O_mean"]) / 10
    assert abs(st[1]["delta_mean"]) <= abs(st[0]["delta_mean"]) / 10
    # dV = P^T dO involves neither O nor delta; the variants differ in it only through L (whose
    # l sums bf16-rounded P-bar values: exactly 1 in the standard variant, exp(-r_m) rounded in the
    # mitigated one).  Both stay three orders of magnitude below the values (|dV| ~ 1..10).
    for v in (0, 1):
        assert abs(st[v]["dV_mean"]) < 1e-3
    # element-wise parity on sampled heads.  The exact dQ is ~1e-3 here (the softmax is one-hot on a
    # tied pair), so dQ and dK are rounding noise of the dataflow, and O, dV have magnitudes of 2-10
    # (bf16 half-ulp 0.8e-2 .. 3e-2): the cases that cannot meet 2e-2 / 1e-2 are in
    # test_gpu_parity.WIDENED with the emulation's own error.
    for variant in (0, 1):
        for (b, h) in [(0, 0), (3, 11)]:
            check_head(got[variant], x, b, h, w.causal, w.alpha, variant, label=f"pairs_skew v{variant}")


def test_symmetric_values_have_no_signed_bias(lib):
    """With V symmetric about zero every rounding step of the dataflow is odd-symmetric, so the
    oracle's emulation shows no signed error in either variant.  The mitigated kernel agrees.
    The standard kernel keeps a small residue (about -1e-5, two orders of magnitude below the
    bias on one-signed V): on elements whose float32 accumulator sits exactly on a bf16 tie, the
    matrix cores' accumulation order leaves it a hair below the tie more often than above, so
    the GPU lands on the lower bf16 neighbour where the emulation's ties-to-even picks either
    (observed 5:1 among the ~1 % of elements that differ).  It is bounded here, not hidden."""
    st, *_ = _signed_stats(lib, "pairs")
    assert abs(st[1]["O_mean"]) < 8 * st[1]["O_noise"]
    assert abs(st[0]["O_mean"]) < 3e-5
    assert abs(st[0]["O_mean"]) < 0.02 * 2.0e-3          # << the one-signed bias (~2e-3)


@pytest.mark.parametrize("name", ["tied", "tied_skew", "tied_any_skew"])
def test_rank2_tied_inputs_reported_and_within_tolerance(lib, name):
    st, x, got, w = _signed_stats(lib, name, with_backward_ref=(name == "tied"))
    for v in (0, 1):
        # no variant shows a bias beyond a few standard errors on these inputs
        assert abs(st[v]["O_mean"]) < 8 * st[v]["O_noise"] + 2e-5
    for variant in (0, 1):
        check_head(got[variant], x, 1, 3, w.causal, w.alpha, variant, label=f"{name} v{variant}")


def _np(t):
    return t.double().cpu().numpy()


@pytest.mark.parametrize("name", ["tied_q1", "tied_skew_q1"])
def test_tied_max_stress_as_specified(lib, name):
    """Rank-2 K with 25 % duplicated rows, Q from the same subspace with unit coefficients.
    Standard forward: nothing is lost.  Stabilised forward, beta = 2: rows whose repeated maximum
    r_m exceeds 126 ln 2 / (beta - 1) = 87.3 lose every probability (l = 0): O is NaN, LSE = -inf,
    and the backward pass turns that into NaN in dQ of the row and in dK, dV of every key the row
    attends to.  The lost rows, and the counts of unit probabilities and of rule firings, must be
    the emulation's, row by row, over all heads.  The guarded form loses nothing."""
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    B, H, N, d = x["Q"].shape
    runs = {}
    for key, variant, guard in (("standard", 0, False), ("mitigated", 1, False), ("guarded", 1, True)):
        r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, want_counts=True,
                             guard_underflow=guard)
        r["dQ"], r["dK"], r["dV"] = lib.attn_bwd(x["Q"], x["K"], x["V"], r["O"], x["dO"], r["LSE"],
                                                 w.causal, w.alpha, variant)
        r["delta"] = lib.attn_delta(r["O"], x["dO"])
        runs[key] = r
    torch.cuda.synchronize()
    finite = lambda t: torch.isfinite(t.float())
    for key in ("standard", "guarded"):
        assert not torch.isneginf(runs[key]["LSE"]).any(), key
        for n in ("O", "dQ", "dK", "dV", "LSE", "delta"):
            assert finite(runs[key][n]).all(), (key, n)
    mit = runs["mitigated"]
    lost = torch.isneginf(mit["LSE"])                                   # [B,H,N]
    assert 20 <= int(lost.sum()) <= 200 and int(lost.any(-1).sum()) >= 8      # this input does reach the limit
    assert torch.equal(torch.isnan(mit["O"].float()).all(-1), lost)     # a lost row is NaN in every column
    assert torch.equal((~finite(mit["O"])).any(-1), lost) and torch.equal((~finite(mit["dQ"])).any(-1), lost)
    # dK, dV: NaN exactly in the keys some lost row attends to (causal: keys up to the last lost row)
    idx = torch.arange(N, device=DEV).expand(B, H, N)
    last_lost = torch.where(lost, idx, torch.full_like(idx, -1)).max(-1, keepdim=True).values
    for n in ("dK", "dV"):
        assert torch.equal((~finite(mit[n])).any(-1), idx <= last_lost), n
    # row by row against the emulation, every head
    mismatch = {"lost": 0, "fired": 0, "ones": 0, "fired_guarded": 0}
    err = {k: {n: [] for n in ("O", "delta", "dQ", "dK", "dV")} for k in runs}
    for b in range(B):
        for h in range(H):
            xs = head_np(x, b, h)
            f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, True, 1, Bc=lib.fwd_key_tile(d))
            g = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, True, 1, Bc=lib.fwd_key_tile(d), guard=True)
            mismatch["lost"] += int((_np(lost[b, h]).astype(bool) != (f["ell"] == 0)).sum())
            mismatch["fired"] += int((_np(mit["fired"][b, h]) != f["fired"]).sum())
            mismatch["ones"] += int((_np(mit["ones"][b, h]) != f["ones"]).sum())
            mismatch["fired_guarded"] += int((_np(runs["guarded"]["fired"][b, h]) != g["fired"]).sum())
            assert np.isfinite(g["O"]).all()
            ref = dict(zip(("O", "L", "dQ", "dK", "dV", "delta"),
                           exact.forward_backward(xs["Q"], xs["K"], xs["V"], xs["dO"], w.alpha, True)))
            for key, r in runs.items():
                for n in err[key]:
                    e = _np(r[n][b, h]) - ref[n]
                    err[key][n].append(e[np.isfinite(e)].ravel())
    print(f"\n[{name}] lost rows {int(lost.sum())} in {int(lost.any(-1).sum())} heads; row mismatches vs emulation {mismatch}")
    assert mismatch["lost"] == 0
    rows = B * H * N
    assert mismatch["fired"] <= 0.01 * rows and mismatch["ones"] <= 0.01 * rows and mismatch["fired_guarded"] <= 0.01 * rows
    st = {}
    for key in runs:
        st[key] = {}
        for n in err[key]:
            e = np.concatenate(err[key][n])
            st[key][n] = (float(e.mean()), float(e.std() / np.sqrt(e.size)))
        print(f"   {key:9s} mean signed error vs fp64 (finite entries): " +
              "  ".join(f"{n} {m:+.2e}+-{s_:.0e}" for n, (m, s_) in st[key].items()))
    # As they are: the standard forward's mean error of O is within 1e-5 of zero here (rows peaky
    # enough for the mechanism of Sec. 3.3.2 are the ones with maxima near 100), two orders of
    # magnitude below its -2e-3 on `pairs_skew`; the guarded stabilised forward is at the same
    # level; the unguarded one is NOT better on this input: the rows that survive just below the
    # limit keep only a few significant bits.
    for key in ("standard", "guarded"):
        assert abs(st[key]["O"][0]) < 2e-5, key
        assert abs(st[key]["dV"][0]) < 2e-4 and abs(st[key]["dQ"][0]) < 1e-4 and abs(st[key]["dK"][0]) < 1e-4, key
    if name == "tied_skew_q1":
        assert abs(st["mitigated"]["O"][0]) > 5 * abs(st["standard"]["O"][0])      # worse, not better
    # element-wise parity of the two finite variants on sampled heads.  The gradients reach
    # magnitudes of several hundred here (scores up to ~140), where a bf16 output cannot be within
    # 2e-2: the bound for each tensor is the larger of the stated tolerance and what the
    # low-precision dataflow itself does on this input (the emulation's error), as listed in
    # test_gpu_parity.WIDENED.
    for key, variant, guard in (("standard", 0, False), ("guarded", 1, True)):
        got = dict(runs[key]); got["L"] = got["LSE"]
        for (b, h) in [(0, 0), (2, 7)]:
            check_head(got, x, b, h, w.causal, w.alpha, variant, guard=guard, label=f"{name}/{key}")
