"""CPU oracle for the sparse-drafter hot path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 NumPy definitions of what the HIP library computes, written
from the paper's problem statement (Sec. 2.1: a pruned draft model proposes k
tokens, the target keeps the longest greedy-matching prefix; Sec. 2.3-2.4: the
draft model's decoder linears carry a fixed binary weight mask).

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the HIP path and
never imports it; the only common dependency is the seeded input generator.

Pins (see tests, all runnable without a GPU):
  linear   -- masked-dense matmul vs explicit per-row loop over kept columns;
              zero sparsity vs numpy.matmul; exact rational brute force on 8x8;
              one-hot inputs return columns of the masked matrix; linearity.
  packing  -- decoded (row, col, value) list equals argwhere(W != 0); unpack(pack(W)) == W;
              byte-identical to the C++ packer.
  stack    -- k = 1 collapses attention to a copy of v; zero layers is the identity;
              all-zero weights leave the residual stream untouched.
  verify   -- hand-worked examples of Eq. 2, all 2^k match patterns, closed-form mean.
  macs     -- reproduces the abstract's MAC reduction for the 3B drafter.
  lm_head  -- identity weights return the normalised input; duplicated rows: lowest index wins; triple loop.
Model quality (accepted length on real prompts, task accuracy) is parity unpinned
and out of scope: it needs trained weights and evaluation suites.
"""
