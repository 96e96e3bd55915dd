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
    # element-wise parity of O and dV on sampled heads (dQ, dK are pure rounding noise here: the exact
    # dQ is ~1e-3 because the softmax is one-hot on a tied pair, so they are compared with the
    # oracle's bf16 emulation of the same dataflow instead)
    for variant in (0, 1):
        for (b, h) in [(0, 0), (3, 11)]:
            xs = head_np(x, b, h)
            ref = exact.forward_backward(xs["Q"], xs["K"], xs["V"], xs["dO"], w.alpha, True)
            f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, True, variant, Bc=lib.fwd_key_tile(w.d))
            g = flash.backward(xs["Q"], xs["K"], xs["V"], f["O"], xs["dO"], f["L"], w.alpha, True, Bc=64)
            for name, r in (("O", ref[0]), ("dV", ref[4])):
                a = got[variant][name][b, h].double().cpu().numpy()
                assert metrics.rel_l2(a, r) <= 1e-2, name
                assert np.max(np.abs(a - r) / np.maximum(1.0, np.abs(r))) <= 2e-2, name
            for name, e, r in (("dQ", g[0], ref[2]), ("dK", g[1], ref[3])):
                a = got[variant][name][b, h].double().cpu().numpy()
                assert np.isfinite(a).all()
                assert metrics.max_abs(a, r) <= 2.0 * metrics.max_abs(e, r) + 2e-2, name


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
        check_head(got[variant], x, 1, 3, w.causal, w.alpha, variant, label=name)
