"""GPU tests of the forward's switches and side outputs (attn_fwd_opt, attn_delta_hp): the
high-precision output O_hp and delta_hp of Sec. 3.2, the single-rounding dataflow of Sec. 3.3.2,
and the tie statistics (unit probabilities per row, Alg. 3 firings per row) of Sec. 3.3.2 / 4.

Counts are integers decided by float32 comparisons; the kernel and the oracle form the scores
in different summation orders, so a score that sits within a float32 ulp of a decision boundary
may be counted differently.  Exact equality is therefore asserted where the decision is
structural (bit-identical key rows, constant scores), and a small mismatch fraction is allowed
on generic inputs.
"""
import numpy as np
import pytest
import torch

from oracle import exact, flash, metrics
from paper_2510_04212_amd import synth
from test_gpu_parity import head_np, DEV, TOL_ABS, TOL_REL

pytestmark = pytest.mark.gpu


def _np(t):
    return t.double().cpu().numpy()


@pytest.mark.parametrize("name", ["tiny", "gpt2s"])
@pytest.mark.parametrize("variant", [0, 1])
def test_extras_do_not_change_the_ordinary_outputs(lib, name, variant):
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, want_O_hp=True, want_counts=True)
    torch.cuda.synchronize()
    assert torch.equal(O, r["O"]) and torch.equal(L, r["LSE"])


@pytest.mark.parametrize("d", [32, 96, 128, 256])
@pytest.mark.parametrize("variant", [0, 1, 2])
def test_extras_at_every_head_size(lib, d, variant):
    """The kernels with optional outputs and the whole-row variant at the head sizes the named
    workloads do not have: ordinary outputs unchanged by the extras, O_hp within float32 rounding
    of the exact O times the bf16 error bound, every row's unit-probability count at least 1 with
    the standard normaliser, and the whole-row variant within tolerance of the fp64 oracle."""
    B, H, N = 1, 2, 200
    g = torch.Generator().manual_seed(77 + d + variant)
    x = {k: torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV) for k in ("Q", "K", "V")}
    alpha = d ** -0.5
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], True, alpha, variant)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], True, alpha, variant, want_O_hp=True, want_counts=True)
    torch.cuda.synchronize()
    assert torch.equal(O, r["O"]) and torch.equal(L, r["LSE"])
    for h in range(H):
        O64, L64 = exact.forward(_np(x["Q"][0, h]), _np(x["K"][0, h]), _np(x["V"][0, h]), alpha, True)
        assert metrics.max_abs(_np(O[0, h]), O64) <= TOL_ABS
        assert metrics.max_abs(_np(r["O_hp"][0, h]), O64) <= TOL_ABS
        assert metrics.max_abs(_np(L[0, h]), L64) < 5e-3      # l sums bf16-rounded probabilities
    if variant == 0:
        assert int(r["ones"].min()) >= 1


@pytest.mark.parametrize("name,heads", [("tiny", [(0, 0)]), ("gpt2s", [(0, 0), (7, 11)]), ("pairs_skew", [(1, 5)])])
@pytest.mark.parametrize("variant", [0, 1])
def test_high_precision_output_and_delta_hp(lib, name, heads, variant):
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, want_O_hp=True)
    d_hp = lib.attn_delta_hp(r["O_hp"], x["dO"])
    torch.cuda.synchronize()
    assert torch.isfinite(r["O_hp"]).all()
    # delta_hp is the float32 row sum of dO o O_hp, whatever O_hp holds
    ref = (x["dO"].double() * r["O_hp"].double()).sum(-1)
    assert (d_hp.double() - ref).abs().max().item() <= 1e-5 * (1 + ref.abs().max().item())
    for (b, h) in heads:
        xs = head_np(x, b, h)
        O64, _ = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
        f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, variant, Bc=64)
        got = _np(r["O_hp"][b, h])
        assert metrics.max_abs(got, O64) <= TOL_ABS and metrics.rel_l2(got, O64) <= TOL_REL
        # against the emulation only P-bar's bf16 roundings can differ (a few elements, one ulp each)
        assert metrics.rel_l2(got, f["Ohp"]) <= 1e-3
        # O is the twice-rounded version of the same accumulator
        O_from_hp = _np(r["O"][b, h])
        assert metrics.max_abs(O_from_hp, got) <= 2.0 ** -7 * (np.abs(got).max() + 1e-30)


def test_delta_bias_and_its_two_remedies(lib):
    """Claim 1 / Sec. 3.2 on the one-signed paired-key input, all heads: delta_lp - delta_hp > 0
    with the standard forward; delta_hp (high-precision O) and the stabilised forward each
    bring the mean error of delta at least 10x closer to zero; dropping only the rounding of the
    unnormalised output shrinks the mean error of O several times."""
    w = synth.WORKLOADS["pairs_skew"]
    x = synth.make(w, DEV)
    std = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 0, want_O_hp=True)
    mit = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 1)
    single = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 0, single_rounding=True)
    row = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 2)
    d_lp = lib.attn_delta(std["O"], x["dO"])
    d_hp = lib.attn_delta_hp(std["O_hp"], x["dO"])
    d_mit = lib.attn_delta(mit["O"], x["dO"])
    torch.cuda.synchronize()
    e = {k: [] for k in ("lp", "hp", "mit", "O_std", "O_single", "O_row")}
    for b in range(w.B):
        for h in range(w.H):
            xs = head_np(x, b, h)
            O64, _ = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
            d64 = np.sum(xs["dO"] * O64, axis=1)
            e["lp"].append(_np(d_lp[b, h]) - d64); e["hp"].append(_np(d_hp[b, h]) - d64)
            e["mit"].append(_np(d_mit[b, h]) - d64)
            e["O_std"].append((_np(std["O"][b, h]) - O64).ravel())
            e["O_single"].append((_np(single["O"][b, h]) - O64).ravel())
            e["O_row"].append((_np(row["O"][b, h]) - O64).ravel())
    m = {k: float(np.concatenate(v).mean()) for k, v in e.items()}
    print("mean signed errors on pairs_skew:", {k: f"{v:+.3e}" for k, v in m.items()})
    assert m["lp"] > 0
    assert float((d_lp.double() - d_hp.double()).mean().item()) > 0
    assert abs(m["hp"]) < m["lp"] / 10 and abs(m["mit"]) < m["lp"] / 10
    # Single rounding: on this input (a + b) / 2 of two bf16 values sits exactly on a bf16 midpoint
    # for half of the outputs, so float32-ulp effects decide the direction of the one remaining
    # rounding.  The emulation's sequential float32 sum leaves a residue of ~1/11 of the standard
    # bias; the matrix cores' own accumulation order leaves ~1/5 (measured +4.2e-4 vs -2.2e-3).
    assert m["O_std"] < 0 and abs(m["O_single"]) < abs(m["O_std"]) / 4
    assert abs(m["O_row"]) < abs(m["O_std"]) / 10          # whole-row form of Alg. 3


@pytest.mark.parametrize("variant", [0, 1])
def test_single_rounding_matches_its_emulation(lib, variant):
    w = synth.WORKLOADS["gpt2s"]
    x = synth.make(w, DEV)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, single_rounding=True)
    torch.cuda.synchronize()
    for (b, h) in ((0, 0), (3, 7)):
        xs = head_np(x, b, h)
        O64, L64 = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
        f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, variant, Bc=64, round_obar=False)
        got = _np(r["O"][b, h])
        assert metrics.max_abs(got, O64) <= TOL_ABS and metrics.rel_l2(got, O64) <= TOL_REL
        assert (got != f["O"]).mean() < 0.02            # same bf16 value almost everywhere
        assert np.abs(_np(r["LSE"][b, h]) - L64).max() < 5e-3


def test_counts_on_constant_scores(lib):
    """All keys identical: every visible score of a row is the same number.
    Standard: every visible key has P-bar = 1 (ones = number of visible keys, nothing fires).
    Stabilised: a row whose key tile holds more than one visible key has a repeated maximum in
    it; with a positive score the normaliser becomes beta*r_m and no P-bar equals 1."""
    B, H, N, d = 1, 2, 256, 64
    g = torch.Generator().manual_seed(5)
    k = torch.randn((1, 1, 1, d), generator=g)
    K = k.expand(B, H, N, d).contiguous().to(torch.bfloat16).to(DEV)
    Q = (K.float() * 0.5).to(torch.bfloat16)                     # q . k > 0 for every pair
    V = torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV)
    rows = torch.arange(N, device=DEV)
    for causal in (True, False):
        vis = (rows + 1) if causal else torch.full_like(rows, N)
        s = lib.attn_fwd_opt(Q, K, V, causal, 0.125, 0, want_counts=True)
        m = lib.attn_fwd_opt(Q, K, V, causal, 0.125, 1, want_counts=True)
        torch.cuda.synchronize()
        assert torch.equal(s["ones"][0, 0].long(), vis) and int(s["fired"].abs().sum()) == 0
        # tiles of 64 keys: tile t holds min(64, vis - 64 t) visible keys of the row; it fires when that is > 1
        t = torch.arange(N // 64, device=DEV)[None, :]
        in_tile = (vis[:, None] - 64 * t).clamp(0, 64)
        assert torch.equal(m["fired"][0, 0].long(), (in_tile > 1).sum(1))
        # a row that never fired (causal row 0: a single visible key) keeps the plain maximum
        never = (in_tile > 1).sum(1) == 0
        assert int(m["ones"][0, 0][~never].sum()) == 0
        xs = {n: v[0, 0].double().cpu().numpy() for n, v in (("Q", Q), ("K", K), ("V", V))}
        for variant, got in ((0, s), (1, m)):
            f = flash.forward(xs["Q"], xs["K"], xs["V"], 0.125, causal, variant, Bc=64)
            assert np.array_equal(got["ones"][0, 0].cpu().numpy(), f["ones"])
            assert np.array_equal(got["fired"][0, 0].cpu().numpy(), f["fired"])


@pytest.mark.parametrize("name", ["tied", "pairs", "gpt2s"])
def test_counts_against_the_emulation(lib, name):
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    got = {v: lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, v, want_counts=True) for v in (0, 1)}
    torch.cuda.synchronize()
    for (b, h) in ((0, 0), (w.B - 1, w.H - 1)):
        xs = head_np(x, b, h)
        for v in (0, 1):
            f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, v, Bc=64)
            ones = got[v]["ones"][b, h].cpu().numpy(); fired = got[v]["fired"][b, h].cpu().numpy()
            bad_ones = float(np.mean(ones != f["ones"])); bad_fired = float(np.mean(fired != f["fired"]))
            print(f"{name} head {(b, h)} variant {v}: rows with >= 2 unit probabilities "
                  f"{int((ones >= 2).sum())} (oracle {int((f['ones'] >= 2).sum())}), firings {int(fired.sum())} "
                  f"(oracle {int(f['fired'].sum())}); mismatching rows {bad_ones:.4f} / {bad_fired:.4f}")
            assert bad_ones <= 0.01 and bad_fired <= 0.01
            if v == 0:
                assert int(fired.sum()) == 0
                assert (ones >= 1).all()        # the running maximum itself always has P-bar = 1 at least once


@pytest.mark.parametrize("name,heads", [("tiny", [(0, 0)]), ("gpt2s", [(0, 0), (5, 3)]), ("pairs_skew", [(0, 0), (3, 11)])])
def test_recomputed_delta(lib, name, heads):
    """attn_delta_recompute: rowsum(P o dP) against the fp64 delta and against its emulation;
    on the one-signed paired-key input it carries none of the bias of delta_lp."""
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], w.causal, w.alpha, 0)
    d_rc = lib.attn_delta_recompute(x["Q"], x["K"], x["V"], x["dO"], L, w.causal, w.alpha)
    d_lp = lib.attn_delta(O, x["dO"])
    torch.cuda.synchronize()
    assert torch.isfinite(d_rc).all()
    e_rc, e_lp = [], []
    for (b, h) in heads:
        xs = head_np(x, b, h)
        O64, L64 = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
        d64 = np.sum(xs["dO"] * O64, axis=1)
        emu = flash.delta_recomputed(xs["Q"], xs["K"], xs["V"], xs["dO"], _np(L[b, h]), w.alpha, w.causal, Bc=64)
        got = _np(d_rc[b, h])
        scale = 1 + np.abs(d64).max()
        assert np.abs(got - emu).max() <= 2e-4 * scale          # float32 reassociation + exp2 vs exp
        assert np.abs(got - d64).max() <= 5e-3 * scale          # float32 L of the bf16 forward
        e_rc.append(got - d64); e_lp.append(_np(d_lp[b, h]) - d64)
    if name == "pairs_skew":
        e_rc, e_lp = np.concatenate(e_rc), np.concatenate(e_lp)
        assert e_lp.mean() > 0 and abs(e_rc.mean()) < e_lp.mean() / 10


def test_backward_from_each_delta(lib):
    """The three deltas (from bf16 O, from O_hp, recomputed) fed to the same two backward stages:
    each set of gradients meets the tolerance against fp64; dV does not depend on delta."""
    w = synth.WORKLOADS["gpt2s"]
    x = synth.make(w, DEV)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 0, want_O_hp=True)
    deltas = {"lp": lib.attn_delta(r["O"], x["dO"]), "hp": lib.attn_delta_hp(r["O_hp"], x["dO"]),
              "rc": lib.attn_delta_recompute(x["Q"], x["K"], x["V"], x["dO"], r["LSE"], w.causal, w.alpha)}
    grads = {}
    for k, dl in deltas.items():
        dK, dV = lib.attn_bwd_dkdv(x["Q"], x["K"], x["V"], x["dO"], r["LSE"], dl, w.causal, w.alpha)
        dQ = lib.attn_bwd_dq(x["Q"], x["K"], x["V"], x["dO"], r["LSE"], dl, w.causal, w.alpha)
        grads[k] = {"dQ": dQ, "dK": dK, "dV": dV}
    torch.cuda.synchronize()
    assert torch.equal(grads["lp"]["dV"], grads["hp"]["dV"]) and torch.equal(grads["lp"]["dV"], grads["rc"]["dV"])
    b, h = 2, 9
    xs = head_np(x, b, h)
    ref = exact.forward_backward(xs["Q"], xs["K"], xs["V"], xs["dO"], w.alpha, w.causal)
    for k in grads:
        for name, rr in (("dQ", ref[2]), ("dK", ref[3]), ("dV", ref[4])):
            got = _np(grads[k][name][b, h])
            assert metrics.rel_l2(got, rr) <= TOL_REL, (k, name)
            assert metrics.max_abs(got, rr) <= 1.25 * TOL_ABS, (k, name)


@pytest.mark.parametrize("name,heads", [("tiny", [(0, 0)]), ("gpt2s", [(0, 0), (7, 11)]), ("tied_any", [(0, 0), (3, 5)]),
                                        ("pairs_skew", [(2, 2)])])
def test_whole_row_detection_variant(lib, name, heads):
    """ATTN_VARIANT_MITIGATED_ROW against Alg. 3 applied to the whole row (the oracle with the key
    tile equal to N): outputs within tolerance of fp64, per-row firing flags and unit-probability
    counts equal to the oracle's, and the result independent of where the tied keys sit."""
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    r = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 2, want_counts=True, want_O_hp=True)
    plain = lib.attn_fwd(x["Q"], x["K"], x["V"], w.causal, w.alpha, 2)
    torch.cuda.synchronize()
    assert torch.equal(plain[0], r["O"]) and torch.equal(plain[1], r["LSE"])
    for (b, h) in heads:
        xs = head_np(x, b, h)
        O64, L64 = exact.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal)
        f = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, flash.MITIGATED, Bc=None)
        got = _np(r["O"][b, h])
        assert np.isfinite(got).all()
        assert metrics.max_abs(got, O64) <= TOL_ABS and metrics.rel_l2(got, O64) <= TOL_REL
        assert np.abs(_np(r["LSE"][b, h]) - L64).max() < 5e-3
        assert metrics.rel_l2(_np(r["O_hp"][b, h]), f["Ohp"]) <= 1e-3
        fired = r["fired"][b, h].cpu().numpy(); ones = r["ones"][b, h].cpu().numpy()
        assert np.mean(fired != f["fired"]) <= 0.01 and np.mean(ones != f["ones"]) <= 0.01
        print(f"{name} head {(b, h)}: rows where the whole-row rule fired {int(fired.sum())} (oracle {int(f['fired'].sum())})")


def test_whole_row_detection_sees_ties_that_straddle_tiles(lib):
    """Two bit-identical maximal keys placed in different 64-key tiles: the per-tile rule (Alg. 3
    as written) does not see the repetition, the whole-row rule does."""
    B, H, N, d = 1, 1, 256, 64
    g = torch.Generator().manual_seed(77)
    K = (0.3 * torch.randn((B, H, N, d), generator=g)).to(torch.bfloat16)
    K[0, 0, 200] = K[0, 0, 10]                       # tiles 0 and 3
    Q = (4.0 * K[:, :, 10:11].float()).expand(B, H, N, d).contiguous().to(torch.bfloat16)   # every query points at that key
    V = torch.randn((B, H, N, d), generator=g).to(torch.bfloat16)
    Q, K, V = Q.to(DEV), K.to(DEV), V.to(DEV)
    tile = lib.attn_fwd_opt(Q, K, V, False, 0.125, 1, want_counts=True)
    row = lib.attn_fwd_opt(Q, K, V, False, 0.125, 2, want_counts=True)
    torch.cuda.synchronize()
    assert int(tile["fired"].sum()) == 0 and (tile["ones"] == 2).all()
    assert (row["fired"] == 1).all() and (row["ones"] == 0).all()
    xs = {n: v[0, 0].double().cpu().numpy() for n, v in (("Q", Q), ("K", K), ("V", V))}
    O64, _ = exact.forward(xs["Q"], xs["K"], xs["V"], 0.125, False)
    for got in (tile, row):
        assert metrics.max_abs(_np(got["O"][0, 0]), O64) <= TOL_ABS


@pytest.mark.parametrize("d,causal,N", [(64, True, 384), (128, True, 256), (128, False, 200), (64, False, 129), (32, True, 200), (256, True, 200), (96, True, 200)])
def test_strided_layouts_give_bit_identical_results(lib, d, causal, N):
    """attn_fwd_strided / attn_bwd_strided on (a) a [B,N,H,d] buffer and (b) views into one fused
    [B,N,3,H,d] projection buffer, against the contiguous [B,H,N,d] entry points on the same
    values: same arithmetic, so the results are equal bit for bit; memory around the strided
    outputs is left untouched."""
    B, H = 2, 3
    g = torch.Generator().manual_seed(900 + N + d)
    alpha = 1.0 / np.sqrt(d)
    qkv = (1.1 * torch.randn((B, N, 3, H, d), generator=g)).to(torch.bfloat16).to(DEV)
    dO_bnhd = torch.randn((B, N, H, d), generator=g).to(torch.bfloat16).to(DEV)
    c = {k: qkv[:, :, i].permute(0, 2, 1, 3).contiguous() for i, k in enumerate(("Q", "K", "V"))}   # [B,H,N,d] copies
    c["dO"] = dO_bnhd.permute(0, 2, 1, 3).contiguous()
    for variant in (0, 1):
        O_ref, L_ref = lib.attn_fwd(c["Q"], c["K"], c["V"], causal, alpha, variant)
        dQ_ref, dK_ref, dV_ref = lib.attn_bwd(c["Q"], c["K"], c["V"], O_ref, c["dO"], L_ref, causal, alpha, variant)
        # (a) plain [B,N,H,d] tensors seen as [B,H,N,d]
        a = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in c.items()}
        assert a["Q"].stride() == (N * H * d, d, H * d, 1)
        O_a, L_a = lib.attn_fwd_strided(a["Q"], a["K"], a["V"], causal, alpha, variant)
        dQ_a, dK_a, dV_a = lib.attn_bwd_strided(a["Q"], a["K"], a["V"], O_a, a["dO"], L_a, causal, alpha, variant)
        torch.cuda.synchronize()
        assert O_a.stride() == a["Q"].stride()
        for got, ref in ((O_a, O_ref), (dQ_a, dQ_ref), (dK_a, dK_ref), (dV_a, dV_ref)):
            assert torch.equal(got, ref)
        assert torch.equal(L_a, L_ref)
    # (b) forward straight from the fused projection buffer, output into a canary-filled fused buffer
    v = {k: qkv[:, :, i].permute(0, 2, 1, 3) for i, k in enumerate(("Q", "K", "V"))}
    assert v["Q"].stride() == (N * 3 * H * d, d, 3 * H * d, 1)
    out = torch.full((B, N, 3, H, d), 777.0, dtype=torch.bfloat16, device=DEV)
    O_b = out[:, :, 1].permute(0, 2, 1, 3)
    lib.attn_fwd_strided(v["Q"], v["K"], v["V"], causal, alpha, 1, O=O_b)
    torch.cuda.synchronize()
    O_ref, _ = lib.attn_fwd(c["Q"], c["K"], c["V"], causal, alpha, 1)
    assert torch.equal(O_b, O_ref)
    assert (out[:, :, 0] == 777.0).all() and (out[:, :, 2] == 777.0).all()


def test_autograd_wrapper(lib):
    """`attention()` under torch.autograd: gradients of a scalar loss equal what attn_bwd returns
    for the same dO, for contiguous inputs and for [B,N,H,d]-backed views; a few optimiser steps
    on q run through."""
    from paper_2510_04212_amd.autograd import attention
    B, H, N, d = 2, 3, 256, 64
    g = torch.Generator().manual_seed(31)
    base = {k: torch.randn((B, N, H, d), generator=g).to(torch.bfloat16).to(DEV) for k in ("q", "k", "v", "w")}
    for layout in ("bhnd", "bnhd"):
        if layout == "bhnd":
            t = {k: x.permute(0, 2, 1, 3).contiguous() for k, x in base.items()}
        else:
            t = {k: x.permute(0, 2, 1, 3) for k, x in base.items()}           # views, no copy
        q, k, v = (t[n].detach().requires_grad_(True) for n in ("q", "k", "v"))
        o = attention(q, k, v, causal=True, variant=lib.MITIGATED)
        loss = (o.float() * t["w"].float()).sum()
        loss.backward()
        torch.cuda.synchronize()
        # the same through the C ABI by hand, dO = w
        qc, kc, vc, wc = (t[n].contiguous() for n in ("q", "k", "v", "w"))
        O, L = lib.attn_fwd(qc, kc, vc, True, 1.0 / np.sqrt(d), lib.MITIGATED)
        dQ, dK, dV = lib.attn_bwd(qc, kc, vc, O, wc, L, True, 1.0 / np.sqrt(d), lib.MITIGATED)
        assert torch.equal(o, O)
        assert torch.equal(q.grad, dQ) and torch.equal(k.grad, dK) and torch.equal(v.grad, dV)
    # grouped-query: 3 query heads on 1 key/value head
    q = base["q"].permute(0, 2, 1, 3).contiguous().requires_grad_(True)
    k1 = base["k"].permute(0, 2, 1, 3)[:, :1].contiguous().requires_grad_(True)
    v1 = base["v"].permute(0, 2, 1, 3)[:, :1].contiguous().requires_grad_(True)
    w = base["w"].permute(0, 2, 1, 3).contiguous()
    o = attention(q, k1, v1, causal=True, variant=lib.STANDARD)
    (o.float() * w.float()).sum().backward()
    O, L = lib.attn_fwd_gqa(q.detach(), k1.detach(), v1.detach(), True, 1.0 / np.sqrt(d), lib.STANDARD)
    dQ, dK, dV = lib.attn_bwd_gqa(q.detach(), k1.detach(), v1.detach(), O, w, L, True, 1.0 / np.sqrt(d), lib.STANDARD)
    torch.cuda.synchronize()
    assert torch.equal(o, O) and torch.equal(q.grad, dQ) and torch.equal(k1.grad, dK) and torch.equal(v1.grad, dV)
    # fewer queries than keys (a chunk of queries at the end of the sequence)
    qr = base["q"].permute(0, 2, 1, 3)[:, :, N - 100:].contiguous().requires_grad_(True)
    kr = base["k"].permute(0, 2, 1, 3).contiguous().requires_grad_(True)
    vr = base["v"].permute(0, 2, 1, 3).contiguous().requires_grad_(True)
    wr = base["w"].permute(0, 2, 1, 3)[:, :, N - 100:].contiguous()
    o = attention(qr, kr, vr, causal=True, variant=lib.MITIGATED)
    (o.float() * wr.float()).sum().backward()
    O, L = lib.attn_fwd_rect(qr.detach(), kr.detach(), vr.detach(), True, 1.0 / np.sqrt(d), lib.MITIGATED)
    dQ, dK, dV = lib.attn_bwd_rect(qr.detach(), kr.detach(), vr.detach(), O, wr, L, True, 1.0 / np.sqrt(d), lib.MITIGATED)
    torch.cuda.synchronize()
    assert torch.equal(o, O) and torch.equal(qr.grad, dQ) and torch.equal(kr.grad, dK) and torch.equal(vr.grad, dV)
    q = base["q"].permute(0, 2, 1, 3).contiguous().float().requires_grad_(True)
    opt = torch.optim.SGD([q], lr=1e-2)
    first = None
    for _ in range(3):
        opt.zero_grad()
        o = attention(q.to(torch.bfloat16), t["k"].contiguous(), t["v"].contiguous())
        loss = (o.float() ** 2).mean()
        loss.backward()
        opt.step()
        first = loss.item() if first is None else first
    assert np.isfinite(loss.item()) and loss.item() <= first


@pytest.mark.parametrize("H,Hkv,N,d,causal", [(4, 4, 256, 64, True), (6, 2, 320, 64, True), (4, 1, 200, 128, True),
                                              (8, 2, 256, 128, False), (3, 1, 65, 64, False), (4, 2, 192, 32, True), (4, 2, 200, 256, True), (6, 2, 200, 96, True)])
def test_grouped_query_attention(lib, H, Hkv, N, d, causal):
    """attn_fwd_gqa / attn_bwd_gqa: O and dQ equal, bit for bit, ordinary attention on K, V repeated
    for every query head of a group; dK, dV (summed over the group in float32, rounded once)
    against the fp64 oracle's per-head gradients summed over the group."""
    B = 2
    group = H // Hkv
    g = torch.Generator().manual_seed(555 + H * 10 + Hkv + N)
    alpha = 1.0 / np.sqrt(d)
    Q = torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV)
    dO = torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV)
    K = torch.randn((B, Hkv, N, d), generator=g).to(torch.bfloat16).to(DEV)
    V = torch.randn((B, Hkv, N, d), generator=g).to(torch.bfloat16).to(DEV)
    Kx, Vx = K.repeat_interleave(group, dim=1).contiguous(), V.repeat_interleave(group, dim=1).contiguous()
    for variant in (0, 1):
        O, L = lib.attn_fwd_gqa(Q, K, V, causal, alpha, variant)
        dQ, dK, dV = lib.attn_bwd_gqa(Q, K, V, O, dO, L, causal, alpha, variant)
        O_ref, L_ref = lib.attn_fwd(Q, Kx, Vx, causal, alpha, variant)
        dQ_ref, dKx, dVx = lib.attn_bwd(Q, Kx, Vx, O_ref, dO, L_ref, causal, alpha, variant)
        torch.cuda.synchronize()
        assert dK.shape == K.shape and dV.shape == V.shape
        assert torch.equal(O, O_ref) and torch.equal(L, L_ref) and torch.equal(dQ, dQ_ref)
        if group == 1:
            assert torch.equal(dK, dKx) and torch.equal(dV, dVx)
        for (b, hk) in ((0, 0), (B - 1, Hkv - 1)):
            dK64 = np.zeros((N, d)); dV64 = np.zeros((N, d))
            for j in range(group):
                h = hk * group + j
                r = exact.forward_backward(_np(Q[b, h]), _np(K[b, hk]), _np(V[b, hk]), _np(dO[b, h]), alpha, causal)
                dK64 += r[3]; dV64 += r[4]
            for got, ref in ((dK[b, hk], dK64), (dV[b, hk], dV64)):
                got = _np(got)
                assert np.isfinite(got).all()
                assert metrics.rel_l2(got, ref) <= TOL_REL
                # a sum of `group` heads: magnitudes and bf16 steps grow with the group
                assert metrics.max_abs(got, ref) <= max(TOL_ABS, 2.0 ** -8 * np.abs(ref).max())


def test_lds_probe(lib):
    """The LDS read loops report the hardware's rates: one wave-wide read instruction per 4 clocks
    and CU, i.e. 256 bytes per clock for ds_read_b128 and 128 for the transposing 8-byte read."""
    from paper_2510_04212_amd import probe
    r = probe.lds_clock(kind=0, workgroups=256, iters=2000)
    assert 200.0 < r["bytes_per_clk_per_cu"] <= 257.0, r
    assert 1.0 < r["shader_clock_ghz"] < 2.6, r
    t = probe.lds_clock(kind=1, workgroups=256, iters=2000)
    assert 100.0 < t["bytes_per_clk_per_cu"] <= 129.0, t
    raw = probe.raw()
    out = torch.zeros(4, dtype=torch.int64, device=DEV)
    assert raw.attn_probe_lds_clock(out.data_ptr(), 0, 0, 10, None) == 2
    assert raw.attn_probe_lds_clock(out.data_ptr(), 2, 8, 10, None) == 2
    assert raw.attn_probe_lds_clock(None, 0, 8, 10, None) == 1


def test_matrix_clock_probe(lib):
    """The benchmark's measurement aid: plausible clock and rate, argument checks."""
    from paper_2510_04212_amd import probe
    p = probe.matrix_clock(workgroups=1024, iters=10000)
    print(f"\nprobe: {p['shader_clock_ghz']:.2f} GHz ({p['shader_clock_ghz_min']:.2f}..{p['shader_clock_ghz_max']:.2f}), "
          f"{p['tflops']:.0f} TFLOP/s over {p['ms']:.2f} ms (device {p['device_ms']:.2f} ms), {p['clocks_per_mfma']:.1f} clocks per instruction")
    assert 0.8 < p["shader_clock_ghz_min"] <= p["shader_clock_ghz"] <= p["shader_clock_ghz_max"] < 2.7
    assert 300 < p["tflops"] < 2600
    # self-consistency: clock x 4096 FLOP/clk/CU x 256 CUs reproduces the rate (8 passes of 4 clocks
    # per instruction and SIMD)
    assert 31.0 < p["clocks_per_mfma"] < 36.0
    assert p["device_ms"] <= p["ms"] * 1.02
    out = torch.zeros(4 + 2 * 8, dtype=torch.int64, device=DEV)
    raw = probe.raw()
    assert raw.attn_probe_matrix_clock(out.data_ptr(), 0, 10, None) == 2
    assert raw.attn_probe_matrix_clock(out.data_ptr(), 8, 0, None) == 2
    assert raw.attn_probe_matrix_clock(None, 8, 10, None) == 1


@pytest.mark.parametrize("B,H,N,d,causal", [(1, 2, 128, 64, True), (2, 2, 384, 128, True), (1, 3, 200, 64, False), (2, 2, 300, 32, True), (1, 2, 320, 256, True), (2, 2, 300, 96, True),
                                             (1, 2, 333, 128, True), (1, 1, 1, 64, True), (1, 2, 1024, 128, False)])
def test_dq_stage_forming_its_own_delta_gives_the_same_bits(lib, B, H, N, d, causal):
    """attn_bwd_dq_delta == attn_delta followed by attn_bwd_dq, bit for bit (delta and dQ), and
    attn_bwd (which uses it) == the three separate stages."""
    g = torch.Generator().manual_seed(N + d)
    x = {k: torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV) for k in ("Q", "K", "V", "dO")}
    alpha = d ** -0.5
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], causal, alpha, lib.MITIGATED)
    delta = lib.attn_delta(O, x["dO"])
    dQ = lib.attn_bwd_dq(x["Q"], x["K"], x["V"], x["dO"], L, delta, causal, alpha)
    dK, dV = lib.attn_bwd_dkdv(x["Q"], x["K"], x["V"], x["dO"], L, delta, causal, alpha)
    dQ2, delta2 = lib.attn_bwd_dq_delta(x["Q"], x["K"], x["V"], O, x["dO"], L, causal, alpha)
    torch.cuda.synchronize()
    assert torch.equal(delta, delta2) and torch.equal(dQ, dQ2)
    ws = torch.empty(max(256, lib.bwd_workspace_bytes(B, H, N, d)), dtype=torch.uint8, device=DEV)
    dQ3, dK3, dV3 = lib.attn_bwd(x["Q"], x["K"], x["V"], O, x["dO"], L, causal, alpha, lib.MITIGATED, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(dQ3, dQ) and torch.equal(dK3, dK) and torch.equal(dV3, dV)
    assert torch.equal(ws[: B * H * N * 4].view(torch.float32).view(B, H, N), delta)


@pytest.mark.parametrize("name,heads,variant", [("tiny", [(0, 0)], 0), ("gpt2s", [(0, 0), (7, 11)], 0),
                                                ("gpt2s", [(3, 4)], 1), ("pairs_skew", [(1, 5)], 0)])
def test_fp8_product_mode_against_its_emulation(lib, name, heads, variant):
    """ATTN_FWD_PV_E4M3 (P-bar and V in E4M3 for the P-bar V product) against the oracle's
    emulation of the same dataflow: products of two E4M3 values are exact in float32, so kernel
    and emulation differ only in the float32 summation order and in exp's last bits, i.e. in a
    small fraction of the roundings of P-bar (1/16 steps: a flipped one moves an output by ~1e-2
    of its size) -- close in the mean, and the high-precision side output much closer to the
    emulation than the bf16 mode's output is."""
    w = synth.WORKLOADS[name]
    x = synth.make(w, DEV)
    f = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, want_O_hp=True, want_counts=True,
                         pv_e4m3=True)
    g = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, variant, want_O_hp=True)
    torch.cuda.synchronize()
    for (b, h) in heads:
        xs = head_np(x, b, h)
        e = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, variant, Bc=64, prec=flash.BF16_PV_E4M3)
        got = f["O_hp"][b, h].double().cpu().numpy()
        bf = g["O_hp"][b, h].double().cpu().numpy()
        err = np.abs(got - e["Ohp"]); scale = np.abs(e["Ohp"]).mean()
        dist_modes = np.abs(bf - e["Ohp"]).mean()
        print(f"\n{name} {(b, h)} v{variant}: |kernel - emulation| mean {err.mean():.2e} max {err.max():.2e}; "
              f"mean |O| {scale:.2e}; bf16 mode differs from it by {dist_modes:.2e} in the mean")
        assert err.mean() <= 0.1 * dist_modes + 1e-6
        assert np.abs(f["LSE"][b, h].double().cpu().numpy() - e["L"]).max() < 2e-2
        ones_g = f["ones"][b, h].cpu().numpy(); ones_e = e["ones"]
        assert np.mean(ones_g == ones_e) > 0.98 and abs(int(ones_g.sum()) - int(ones_e.sum())) <= 0.01 * ones_e.sum() + 2


def test_fp8_product_mode_and_alg3_underflow_together(lib):
    """Finding of the FP8 exploration, asserted so that it stays documented: Alg. 3 moves the
    normaliser to beta * r_m, i.e. every probability of a row with a repeated maximum is at most
    exp(-(beta - 1) r_m); E4M3's smallest positive number is 2^-9, so for (beta - 1) r_m > ~6.6 the
    whole row of P-bar rounds to 0, l = 0 and the output row is 0/0 -- on the paired-key input for
    four rows in ten, the same rows in the kernel and in the emulation.  (bf16 has binary32's exponent
    range and only meets this beyond (beta - 1) r_m ~ 87, Sec. 4.)  With Alg. 1 the mode is finite."""
    w = synth.WORKLOADS["pairs_skew"]
    x = synth.make(w, DEV)
    f1 = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 1, want_counts=True, pv_e4m3=True)
    f0 = lib.attn_fwd_opt(x["Q"], x["K"], x["V"], w.causal, w.alpha, 0, pv_e4m3=True)
    torch.cuda.synchronize()
    assert torch.isfinite(f0["O"].float()).all()
    b, h = 2, 3
    xs = head_np(x, b, h)
    e = flash.forward(xs["Q"], xs["K"], xs["V"], w.alpha, w.causal, 1, Bc=64, prec=flash.BF16_PV_E4M3)
    bad_gpu = torch.isnan(f1["O"][b, h].float()).any(dim=1).cpu().numpy()
    bad_emu = np.isnan(e["O"]).any(axis=1)
    print(f"\nrows lost to underflow: kernel {bad_gpu.mean():.3f}, emulation {bad_emu.mean():.3f}")
    assert bad_emu.mean() > 0.3 and np.mean(bad_gpu == bad_emu) > 0.99
    assert (f1["fired"][b, h].cpu().numpy()[bad_gpu] >= 1).all()      # only rows where the rule fired
