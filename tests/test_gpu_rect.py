"""GPU parity for different numbers of queries and keys (attn_fwd_rect / attn_bwd_rect): against
the fp64 oracle element by element, and against the square problem the rectangular one is a
part of."""
import numpy as np
import pytest
import torch

from paper_2510_04212_amd import synth
from test_gpu_parity import check_head, DEV, V_SCALE, DO_SCALE

pytestmark = pytest.mark.gpu


def _inputs(seed, B, H, Nq, Nk, d, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    r = lambda n, sc: (sc * torch.randn(B, H, n, d, generator=g)).to(torch.bfloat16).to(DEV)
    # V and dO at the scales of the other shape-coverage tests (outputs stay below 4 in magnitude)
    return {"Q": r(Nq, scale), "K": r(Nk, scale), "V": r(Nk, V_SCALE), "dO": r(Nq, DO_SCALE)}


def _run(lib, x, causal, alpha, variant):
    B, H, Nq, d = x["Q"].shape
    O, L = lib.attn_fwd_rect(x["Q"], x["K"], x["V"], causal, alpha, variant)
    ws = torch.empty(max(256, lib.bwd_workspace_bytes(B, H, Nq, d)), dtype=torch.uint8, device=DEV)
    dQ, dK, dV = lib.attn_bwd_rect(x["Q"], x["K"], x["V"], O, x["dO"], L, causal, alpha, variant, workspace=ws)
    torch.cuda.synchronize()
    delta = ws[: B * H * Nq * 4].view(torch.float32).view(B, H, Nq).clone()
    return {"O": O, "L": L, "dQ": dQ, "dK": dK, "dV": dV, "delta": delta}


SHAPES = [(128, 256), (256, 128), (100, 333), (333, 100), (64, 1024), (1024, 64), (1, 257), (257, 1),
          (200, 264), (129, 130), (448, 384)]


@pytest.mark.parametrize("Nq,Nk", SHAPES)
@pytest.mark.parametrize("d", [32, 64, 96, 128, 256])
@pytest.mark.parametrize("causal", [False, True])
def test_rectangular_against_the_oracle(lib, Nq, Nk, d, causal):
    x = _inputs(Nq * 7 + Nk, 1, 2, Nq, Nk, d, scale=1.25)
    alpha = d ** -0.5
    for variant in (0, 1):
        got = _run(lib, x, causal, alpha, variant)
        for h in range(2):
            check_head(got, x, 0, h, causal, alpha, variant, label=f"rect {Nq}x{Nk} d{d} c{causal} v{variant}")
        if causal and Nq > Nk:       # the first Nq - Nk queries see no key
            e = Nq - Nk
            assert (got["O"][:, :, :e] == 0).all() and (got["dQ"][:, :, :e] == 0).all()
            assert torch.isneginf(got["L"][:, :, :e]).all()


def test_whole_row_variant_and_side_entry_points_reject_nothing_new(lib):
    """The whole-row normaliser (two passes) on a rectangular causal problem with unseen rows."""
    x = _inputs(5, 1, 2, 300, 172, 64, scale=1.5)
    got = _run(lib, x, True, 0.125, 2)
    for h in range(2):
        check_head(got, x, 0, h, True, 0.125, 2, label="rect whole-row")


def test_chunk_of_queries_equals_the_tail_of_the_square_problem(lib):
    """Nq < Nk, causal: the same numbers as the last Nq rows of self-attention over Nk tokens
    (forward), and the same dK / dV as self-attention whose upstream gradient is zero on the
    other rows (both to rounding: the two paths accumulate over the same tiles in the same order)."""
    B, H, Nk, Nq, d = 2, 3, 512, 192, 64
    xs = _inputs(77, B, H, Nk, Nk, d)
    xs["dO"][:, :, : Nk - Nq] = 0
    alpha = d ** -0.5
    O_sq, L_sq = lib.attn_fwd(xs["Q"], xs["K"], xs["V"], True, alpha, 1)
    dQ_sq, dK_sq, dV_sq = lib.attn_bwd(xs["Q"], xs["K"], xs["V"], O_sq, xs["dO"], L_sq, True, alpha, 1)
    xr = {"Q": xs["Q"][:, :, Nk - Nq:].contiguous(), "K": xs["K"], "V": xs["V"],
          "dO": xs["dO"][:, :, Nk - Nq:].contiguous()}
    got = _run(lib, xr, True, alpha, 1)
    assert torch.equal(got["O"], O_sq[:, :, Nk - Nq:])
    assert torch.equal(got["L"], L_sq[:, :, Nk - Nq:])
    assert torch.equal(got["dQ"], dQ_sq[:, :, Nk - Nq:])
    assert torch.equal(got["dK"], dK_sq) and torch.equal(got["dV"], dV_sq)


def test_equal_lengths_is_the_ordinary_entry_point(lib):
    w = synth.WORKLOADS["tiny"]
    x = synth.make(w, DEV)
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], True, w.alpha, 1)
    O2, L2 = lib.attn_fwd_rect(x["Q"], x["K"], x["V"], True, w.alpha, 1)
    assert torch.equal(O, O2) and torch.equal(L, L2)
    g = lib.attn_bwd(x["Q"], x["K"], x["V"], O, x["dO"], L, True, w.alpha, 1)
    g2 = lib.attn_bwd_rect(x["Q"], x["K"], x["V"], O, x["dO"], L, True, w.alpha, 1)
    assert all(torch.equal(a, b) for a, b in zip(g, g2))


def test_rect_rejects_bad_arguments(lib):
    x = _inputs(1, 1, 1, 64, 128, 64)
    with pytest.raises(ValueError):
        lib.attn_fwd_rect(x["Q"], x["K"][:, :, :, :32].contiguous(), x["V"], False, 0.125)
    raw = lib.raw()
    p = lambda t: t.data_ptr()
    O = torch.empty_like(x["Q"]); L = torch.empty(1, 1, 64, device=DEV)
    assert raw.attn_fwd_rect(p(x["Q"]), p(x["K"]), p(x["V"]), p(O), p(L), 1, 1, 64, 0, 64, 0, 0.125, 0, 2.0, 1e-3, None) == 3
    assert raw.attn_fwd_rect(p(x["Q"]), p(x["K"]), p(x["V"]), p(O), p(L), 1, 1, -1, 128, 64, 0, 0.125, 0, 2.0, 1e-3, None) == 2
