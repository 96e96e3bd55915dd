"""CPU oracle for bf16 flash attention (forward + backward).

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and its
Python binding) may import this package; only the test-suite, the smoke check and
the benchmark's CPU-baseline leg do.  It shares no code with the GPU path.

Modules
-------
bf16        software bfloat16 rounding (round-to-nearest, ties-to-even) on numpy arrays
exact       fp64 attention forward/backward written from the plain definitions
            (Sec. 2.2 of the paper: O = softmax(alpha Q K^T) V, delta, dS, dQ/dK/dV)
flash       the tiled algorithms (Alg. 1, Alg. 2, Alg. 3 of the paper: online softmax over key
            tiles, the recomputing backward, the stabilised normaliser of Sec. 4), with a
            pluggable working precision and explicit bf16 rounding points
metrics     error measures used by the parity tests (max-abs, relative L2, mean signed)

Pin status (see tests/test_oracle_*.py, all CPU-only):
  bf16.round_to_bf16 .......... pinned (worked addition example of Sec. 3.3.2, exhaustive
                                16-bit neighbourhood checks, torch's own conversion)
  exact.forward / backward .... pinned (finite differences, brute-force loops, closed forms,
                                identities of Sec. 3.2 / Eq. 2)
  flash.forward (fp64 mode) ... pinned (equals exact.forward for any tile size and both
                                variants: shift invariance, Sec. 4)
  flash.backward (fp64 mode) .. pinned (equals exact.backward)
  flash.forward (bf16 mode) ... pinned: a hand evaluation of one tile through the rounding
                                points (r1)-(r4) (the E4M3 product test walks the same lines),
                                bf16 ties reproduced exactly, P-bar == 1 at a row maximum and
                                max P-bar < 1 once the rule fires, the sign of the bias of
                                Sec. 3.3.2 and its removal, the underflow threshold of (r7)
  flash.backward (bf16 mode) .. pinned: an explicit-loop evaluation of one tile with the rounding
                                points of (r6) written out, bit for bit on inputs whose sums are
                                exact in any order; four planted mistakes each change a result
  Bit-exact agreement of the GPU kernels with the bf16 emulation on general inputs is NOT
  claimed: parity unpinned at bit level, because matrix-core summation order and the hardware
  exp2 differ from numpy's; the kernels are held to tolerances against the fp64 functions.
"""
