"""CPU oracle for Self Speculative Decoding on masked-diffusion LLMs.

TEST INFRASTRUCTURE ONLY.  A plain, slow, obviously-correct CPU statement of
what the HIP path computes, written from the paper.  Only tests, the smoke
check and the benchmark's cpu_baseline leg may import it; the product path
never does.  It shares no code with the HIP library and imports nothing from
the package.

  model.py   the bidirectional transformer f_theta (Section 3.1, Eq. 2) with an
             exact block-causal prefix KV cache, written as explicit formulas
             over torch CPU matmuls.
  decode.py  greedy stepwise decoding (the result SSD must reproduce), SSD
             itself (Section 3.2, Algorithm 1) and a cache-free brute force; the
             mix-order tree (Section 5.2), a round across the block boundary
             (Section 3.2.2) and the dual cache with periodic refresh of the
             paper's experiments (Section 4.1).

Parity pins (tests/test_oracle_*.py): SSD == stepwise token for token;
cache-free brute force == cached stepwise; the zero-attention closed form
(every verification accepts N_eff+1 drafts, reaching the N/(N+1) bound of
Tables 2-3); the dual cache refreshed before every token == cache-free
full-attention decoding, and a block computed right after a refresh
reproduces the refresh's logits; torch's own attention / norm / activation routines; RoPE shift
invariance; softmax identities; hand-made acceptance cases.
Parity unpinned: absolute token values on random weights (the paper prints no
worked numeric example), beyond the invariants above.
"""
