"""CPU oracle for the DepCap denoising-step hot path.  TEST INFRASTRUCTURE ONLY.

Plain numpy, fp64 arithmetic (inputs widened exactly), one function per
definition in the paper, no blocking / fusion / reordering.  It shares no code
with the HIP path and imports nothing from the product package; only tests, the
smoke check and the benchmark's cpu_baseline leg may call it.

Parity status of each function against something other than itself
(tests/test_oracle_*.py):

  forward.matmul_nt / rmsnorm / swiglu   pinned (triple loops, closed forms)
  forward.rope                           pinned (identity at 0, isometry, relative-position)
  forward.attention                      pinned (scalar loops, one-key, equal-keys, permutation, GQA)
  forward.forward_span + KV cache        pinned (replay invariant, full-recompute equivalence)
  stats.vocab_stats (softmax, H, KL)     pinned (closed forms, MI identity of Sec. 4.4)
  boundary.block_boundary                pinned for the scan/clip rule of Sec. 4.2 (exhaustive scan,
                                         invariants); the smoothing and normalisation the paper
                                         leaves undefined are this build's reading:
                                         "parity unpinned" against the authors' behaviour
  select.select_parallel                 pinned (independent set-recursive Alg. 1, invariants)
  decode.decode_full                     pinned: structural invariants (Eq. 1, Eq. 2, Sec. 3), and every boundary
                                         decision's KL / entropy rows rebuilt from the trace's pass records by
                                         absolute position with scipy's KL and entropy, with the pairing of Sec. 4.2
                                         checked (p^prev from the pass taken while the block just decoded was all
                                         masks, p^curr from the pass right after it was finished); planted mistakes
                                         in the schedule arithmetic fail that check.  The schedule itself is this
                                         build's reading of Sec. 4.2 / App. A.3: "parity unpinned" against the
                                         authors' behaviour
"""
