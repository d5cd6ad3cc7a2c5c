"""fp64 CPU oracle for the RPO suffix-rollout path.

TEST INFRASTRUCTURE ONLY.  This package is the slow, plain definition of what
the rollout hot path computes, written from the paper (RPO, arXiv 2601.19404):
Sec. 3.2 "Rollout" (Eq. 3: the response is the kept prefix of the cached answer
followed by a fresh continuation sampled from the policy) and the
group-relative advantage of Eq. 7.  Nothing in the product package imports it;
only tests, the smoke check and the benchmark's cpu_baseline leg do.  It shares
no code with the HIP library: arrays go in, arrays come out.

Parity pins (tests/test_oracle_*.py, all CPU):
  transformer forward   -> Hugging Face Qwen2/Llama reference modules in fp64,
                           torch SDPA, scipy log_softmax, brute-force loops,
                           RoPE relative-position property, incremental == full
  Philox4x32-10         -> published known-answer vectors (tests/golden)
  sampler               -> exhaustive threshold enumeration on tiny vocabularies,
                           chi-square against the fp64 softmax, T -> 0+ arg-max
  advantages            -> closed form for 0/1 rewards, affine invariance
Parity unpinned: whole-model numerics at the 1.5B / 7B shapes have no printed
values anywhere; they rest on the same code that the pins above cover at small
shapes.
"""
