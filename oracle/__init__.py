"""CPU oracle for the DART drafting step -- TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct implementation (numpy, fp64 unless the step
fixes fp32 arithmetic) of what the hot path computes: the draft forward pass
(Sec. 3.2), per-position top-k with log-softmax scores (Alg. 1 steps "Top-k_i"
and "s_logit", App. D) and continuity-aware tree pruning (Alg. 1, App. D).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package.  The product path (the HIP library and its Python binding) never does,
and this package imports nothing from the product path.  The two share no code;
they meet only at the seeded input generators.

Parity status: every function here is pinned by CPU tests to something other
than itself (library routines on special cases, closed forms, brute force on
tiny inputs, a hand-derived worked example).  The beam cut of Alg. 1 at finite
beam width is a heuristic defined only by its steps; `tree_prune` with finite
`beam_w` is pinned by brute force on tiny inputs (every path of the full tree
scored by the enumerator, Alg. 1 then read as sets: children of the previous
beam, all into T, the w best kept), by the hand-derived tie-break example and by
invariants.  At sizes where all paths cannot be enumerated it has no other pin.
"""
