"""Multi-step harness around the attention kernels: does the rounding bias of Sec. 3.3 add up
over training steps, and does the stabilised forward of Sec. 4 stop it?

The paper tracks, over the training steps before the loss explodes, the sum over tokens of
delta_lp - delta_hp (delta_lp = rowsum(dO o O) from the bf16 output, delta_hp from the
unrounded one) and finds it positive step after step, so that the error it puts into the
gradient of the query projection,

    dW^Q_hp - dW^Q_lp = alpha * sum_T (delta_lp - delta_hp)[T] * (P K)[T]^T X[T]        (Sec. 3.3.1)

accumulates (Claim 2).  Its curve comes from GPT-2 training on OpenWebText, which is not
available here; this harness reproduces the mechanism on synthetic data.  Every (batch, head)
slice is an independent attention layer with fixed input features X, fixed K, V and upstream
gradient G, and a query projection W^Q (d x d, initialised to the identity) trained by plain
gradient descent on the linear loss <O, G>:

    Q    = bf16(X bf16(W^Q))        (projection: torch, binary64 sums of exact products)
    O, LSE, O_hp, unit-probability counts = attn_fwd_opt
    delta_lp = attn_delta(O, G),  delta_hp = attn_delta_hp(O_hp, G)
    dQ   = attn_bwd_dq with the chosen delta
    dW^Q = X^T dQ,  W^Q <- W^Q - lr dW^Q    (torch)

The attention work runs in the HIP kernels; torch only does the two d x d projections and the
bookkeeping.  Usage:  python -m paper_2510_04212_amd.harness [--workload pairs_skew] [--steps 20]
"""
import argparse
import json
import time

import torch

from . import binding, synth


def run(x, causal, alpha, steps, lr, variant=binding.STANDARD, delta_mode="lp", beta=None, eps=None,
        track_update_error=True):
    """x: dict of bf16 CUDA tensors [B,H,N,d]: "Q" serves as the fixed features X, "K", "V" are
    fixed, "dO" is the fixed upstream gradient G.  delta_mode: "lp" | "hp" (which delta the
    backward pass uses).  Returns a dict of float64 CPU tensors [steps, B, H]:
      sum_delta_diff   sum over tokens of delta_lp - delta_hp
      loss             <O, G>
      rows_tied        rows with at least two unit probabilities (the precondition of Claim 3)
      update_err       Frobenius norm of dW^Q_lp - dW^Q_hp of the step           (track_update_error)
      cum_update_err   Frobenius norm of that difference summed over the steps so far
    and "W": the final W^Q, float32 [B,H,d,d] on the device."""
    X, K, V, G = x["Q"], x["K"], x["V"], x["dO"]
    B, H, N, d = X.shape
    X64 = X.double()
    Xt64 = X64.transpose(-1, -2).contiguous()
    W = torch.eye(d, dtype=torch.float32, device=X.device).repeat(B, H, 1, 1)
    cumD = torch.zeros((B, H, d, d), dtype=torch.float64, device=X.device)
    keys = ["sum_delta_diff", "loss", "rows_tied"] + (["update_err", "cum_update_err"] if track_update_error else [])
    rec = {k: [] for k in keys}
    for _ in range(steps):
        Wb = W.to(torch.bfloat16)
        Q = (X64 @ Wb.double()).float().to(torch.bfloat16).contiguous()
        f = binding.attn_fwd_opt(Q, K, V, causal, alpha, variant, beta, eps, want_O_hp=True, want_counts=True)
        d_lp = binding.attn_delta(f["O"], G)
        d_hp = binding.attn_delta_hp(f["O_hp"], G)
        dQ = {}
        for mode, delta in (("lp", d_lp), ("hp", d_hp)):
            if mode == delta_mode or track_update_error:
                dQ[mode] = binding.attn_bwd_dq(Q, K, V, G, f["LSE"], delta, causal, alpha)
        dW = Xt64 @ dQ[delta_mode].double()
        if track_update_error:
            D = Xt64 @ dQ["lp"].double() - Xt64 @ dQ["hp"].double()
            cumD += D
            rec["update_err"].append(torch.linalg.matrix_norm(D).cpu())
            rec["cum_update_err"].append(torch.linalg.matrix_norm(cumD).cpu())
        W = W - lr * dW.float()
        rec["sum_delta_diff"].append((d_lp.double() - d_hp.double()).sum(-1).cpu())
        rec["loss"].append((f["O"].double() * G.double()).sum((-1, -2)).cpu())
        rec["rows_tied"].append((f["ones"] >= 2).sum(-1).double().cpu())
    out = {k: torch.stack(v) for k, v in rec.items()}
    out["W"] = W
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="pairs_skew", choices=sorted(synth.WORKLOADS))
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--lr", type=float, default=1e-4)
    ap.add_argument("--delta", default="lp", choices=["lp", "hp"])
    a = ap.parse_args()
    w = synth.WORKLOADS[a.workload]
    x = synth.make(w, "cuda:0")
    summary = {"workload": w.name, "steps": a.steps, "lr": a.lr, "delta": a.delta}
    run(x, w.causal, w.alpha, 1, a.lr)               # untimed: loads the library, warms the allocator
    for name, variant in (("standard", binding.STANDARD), ("mitigated", binding.MITIGATED)):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        r = run(x, w.causal, w.alpha, a.steps, a.lr, variant, a.delta)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        s = r["sum_delta_diff"].sum((1, 2))          # all layers together, per step
        cum = torch.cumsum(s, 0)
        print(f"{name}: {w.B * w.H} layers x {a.steps} steps in {dt * 1e3:.1f} ms")
        print("  step  sum_T(delta_lp - delta_hp)  cumulative   tied rows   |cum. update error|")
        for t in range(a.steps):
            print(f"  {t:4d}  {s[t].item():+26.4f}  {cum[t].item():+10.3f}  {int(r['rows_tied'][t].sum().item()):10d}"
                  f"  {r['cum_update_err'][t].sum().item():12.4f}")
        summary[name] = {"cumulative_sum_delta_diff": cum[-1].item(), "steps_per_s": a.steps / dt,
                         "positive_steps": int((s > 0).sum().item()),
                         "cum_update_err": r["cum_update_err"][-1].sum().item()}
    print(json.dumps(summary))


if __name__ == "__main__":
    main()
