"""GPU tests of the multi-step harness (paper_2510_04212_amd/harness.py): the HIP kernels driven
over several training steps against the same loop on the CPU oracle (oracle/harness.py), and
the behaviour the paper reports -- a one-signed, accumulating sum of delta_lp - delta_hp with
Alg. 1 (Claim 2, the cumulative curve of Sec. 3.3.1) and its removal by Alg. 3 (Sec. 4) -- at the
full size of the repeated-maximum workload."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import flash
from oracle import harness as oracle_harness
from paper_2510_04212_amd import harness, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("variant", [0, 1])
def test_harness_matches_the_oracle_loop(lib, variant):
    """Small case, every layer, step by step.  Kernel and oracle differ in the summation order
    inside the matrix products (and so in a few of the bf16 roundings that follow), which the
    training loop then carries along: the per-step diagnostics agree to a few percent (Alg. 1;
    with Alg. 3 they are a sum of unbiased rounding errors, compared against its own scale).
    On this input the softmax is saturated, so with Alg. 1 dQ -- and with it the weight update --
    consists of the systematic delta error plus tie-breaking-sized terms; the two weight paths
    share the former and differ in the latter: same direction, lengths within a quarter.
    With Alg. 3 there are no ties to break and the two paths coincide to a fraction of a percent."""
    steps, lr = 4, 1e-4
    w = dataclasses.replace(synth.WORKLOADS["pairs_skew"], B=1, H=3, N=256)
    x = synth.make(w, DEV)
    got = harness.run(x, w.causal, w.alpha, steps, lr, variant)
    for h in range(w.H):
        xs = {k: v[0, h].float().cpu().numpy() for k, v in x.items()}
        ref = oracle_harness.run(xs["Q"], xs["K"], xs["V"], xs["dO"], w.alpha, w.causal, steps, lr, variant)
        s_got = got["sum_delta_diff"][:, 0, h].numpy(); s_ref = ref["sum_delta_diff"]
        u_got = got["update_err"][:, 0, h].numpy(); u_ref = ref["update_err"]
        print(f"\nvariant {variant} layer {h}: sum_T(delta_lp - delta_hp) kernel {np.round(s_got, 3)} oracle {np.round(s_ref, 3)}")
        if variant == 0:
            # (on exact ties of the unnormalised output the matrix cores' summation order falls
            # below the tie more often than the oracle's sequential sum: up to ~10 % more bias)
            assert np.allclose(s_got, s_ref, rtol=0.12, atol=0.2)
            assert (got["rows_tied"][:, 0, h].numpy() == ref["rows_tied"]).all()
        else:
            assert np.abs(s_got - s_ref).max() <= 0.05
            assert (got["rows_tied"][:, 0, h].numpy() == 0).all()
        assert np.allclose(u_got, u_ref, rtol=0.1)
        assert np.allclose(got["loss"][:, 0, h].numpy(), ref["loss"], rtol=1e-4)
        W_got = got["W"][0, h].cpu().numpy().astype(np.float64)
        moved = np.linalg.norm(ref["W"] - np.eye(w.d))
        rel = np.linalg.norm(W_got - ref["W"]) / moved
        a = (W_got - np.eye(w.d)).ravel(); b = (ref["W"] - np.eye(w.d)).ravel().astype(np.float64)
        cos = float(a @ b / (np.linalg.norm(a) * np.linalg.norm(b)))
        print(f"   |W_kernel - W_oracle|_F / |W_oracle - I|_F = {rel:.3e}, cosine of the two displacements {cos:.4f}")
        assert moved > 0 and cos >= 0.97 and rel <= (0.25 if variant == 0 else 0.02)


def test_bias_accumulates_over_steps_with_alg1_not_with_alg3(lib):
    """All 48 layers of the repeated-maximum workload, 12 steps."""
    w = synth.WORKLOADS["pairs_skew"]
    x = synth.make(w, DEV)
    steps = 12
    r0 = harness.run(x, w.causal, w.alpha, steps, 1e-4, 0)
    r1 = harness.run(x, w.causal, w.alpha, steps, 1e-4, 1)
    s0 = r0["sum_delta_diff"].sum((1, 2)).numpy(); s1 = r1["sum_delta_diff"].sum((1, 2)).numpy()
    print(f"\ncumulative sum_T(delta_lp - delta_hp) over {steps} steps: Alg. 1 {s0.sum():+.1f}, Alg. 3 {s1.sum():+.1f}")
    assert (s0 > 0).all()                                     # positive at every step, as in the paper's curve
    assert (r0["sum_delta_diff"].numpy() > 0).all()           # ... in every layer
    assert abs(s1.sum()) * 10 <= abs(s0.sum())
    assert (r0["rows_tied"].numpy() > 0.9 * w.N).all() and (r1["rows_tied"].numpy() == 0).all()
    # the error of the weight update keeps its direction with Alg. 1 (its sum over steps grows
    # like the step count), and is several times smaller with Alg. 3
    e0 = r0["cum_update_err"][-1].numpy(); tot0 = r0["update_err"].sum(0).numpy()
    assert (e0 >= 0.98 * tot0).all()
    assert r1["cum_update_err"][-1].sum().item() * 5 <= e0.sum()


def test_high_precision_delta_removes_the_update_error(lib):
    """With delta_hp in the backward pass (Sec. 3.2) the trained weights follow a different path
    from the delta_lp run; the diagnostics of the first step, taken at identical weights, are
    identical."""
    w = dataclasses.replace(synth.WORKLOADS["pairs_skew"], B=1, H=2, N=512)
    x = synth.make(w, DEV)
    a = harness.run(x, w.causal, w.alpha, 3, 1e-4, 0, "lp")
    b = harness.run(x, w.causal, w.alpha, 3, 1e-4, 0, "hp")
    assert torch.equal(a["sum_delta_diff"][0], b["sum_delta_diff"][0])
    assert torch.equal(a["update_err"][0], b["update_err"][0])
    assert (a["W"] - b["W"]).abs().max().item() > 0
