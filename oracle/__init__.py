"""CPU oracle for one SpecDiff draft-then-verify round (arxiv 2408.05636).

TEST INFRASTRUCTURE ONLY.  Plain numpy in fp64, slow on purpose, written from the
paper's Algorithm 1 and Sections 3-4.  Nothing in the product path may import this
package; only the tests, the smoke check and the benchmark's cpu_baseline leg do.
It shares no code with the HIP implementation.

Pins (tests/test_oracle_*.py):
  philox        known-answer vectors of Philox4x32-10 (Salmon et al., SC'11)
  transformer   independent composition of torch CPU fp64 library ops; causal /
                bidirectional dependence properties; RoPE shift invariance
  specdiff      brute-force enumeration: output law == target law (Sec. 1, 3);
                alpha = sum min(p,q) (Appendix A, Corollary); expected tokens
                (Appendix A, Eq. 2); unmasking schedule closed form; fixed point
Parity unpinned: behaviour on the paper's trained models and datasets (acceptance
rates of Tables 2-4) -- those weights and prompts are not available.
"""
