"""attn_bwd_noalloc (the backward pass for callers that cannot allocate: delta lives in a device
array inside the library) against attn_bwd, through the C ABI: same kernels, so the same bits.
Two calls in a row on the same GPU, the second with a smaller input, so that what the first call
left in the shared array would show if anything stale were read."""
import ctypes

import pytest
import torch

from paper_2510_04212_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _inputs(B, H, N, d, seed):
    g = torch.Generator().manual_seed(seed)
    return {k: torch.randn((B, H, N, d), generator=g).to(torch.bfloat16).to(DEV) for k in ("Q", "K", "V", "dO")}


def _both(lib, x, causal, alpha):
    O, L = lib.attn_fwd(x["Q"], x["K"], x["V"], causal, alpha, lib.MITIGATED)
    want = lib.attn_bwd(x["Q"], x["K"], x["V"], O, x["dO"], L, causal, alpha, lib.MITIGATED)
    got = [torch.full_like(x["Q"], float("nan")) for _ in range(3)]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    lib.attn_bwd_noalloc(x["Q"], x["K"], x["V"], O, x["dO"], L, causal, alpha, *got, variant=lib.MITIGATED)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # torch's allocator was not touched either
    return got, want


def test_noalloc_backward_matches_attn_bwd_twice_in_a_row(lib):
    assert lib.raw().attn_bwd_noalloc_max_rows() == 1 << 20
    # first call: a ragged shape with several heads; second call: a smaller input
    for (B, H, N, d, causal) in ((2, 3, 1000, 128, True), (1, 2, 200, 64, False)):
        x = _inputs(B, H, N, d, seed=31 + N)
        got, want = _both(lib, x, causal, d ** -0.5)
        for name, g, w in zip(("dQ", "dK", "dV"), got, want):
            assert torch.isfinite(g.float()).all(), name
            assert torch.equal(g, w), (name, (B, H, N, d))
    # the headline shape fits the array (B*H*N = 2^19 rows) and gives the same bits as well
    w = synth.WORKLOADS["mid"]
    x = synth.make(w, DEV)
    got, want = _both(lib, x, w.causal, w.alpha)
    for g, wv in zip(got, want):
        assert torch.equal(g, wv)


def test_noalloc_backward_rejects_what_does_not_fit(lib):
    raw = lib.raw()
    p = ctypes.c_void_p(0x1000)
    # 2^20 + 128 rows: one tile too many for the array
    st = raw.attn_bwd_noalloc(p, p, p, p, p, p, ctypes.c_void_p(0x2000), ctypes.c_void_p(0x3000),
                              ctypes.c_void_p(0x4000), 1, 1, (1 << 20) + 128, 64, 1, 0.125, 0, None)
    assert st == 4 and "noalloc" in lib.status_string(st)
    # an empty batch is a no-op, bad shapes are reported as by attn_bwd
    assert raw.attn_bwd_noalloc(None, None, None, None, None, None, None, None, None, 0, 4, 128, 64, 1, 0.125, 0, None) == 0
    assert raw.attn_bwd_noalloc(p, p, p, p, p, p, p, p, p, 1, 1, 128, 80, 1, 0.125, 0, None) == 3
