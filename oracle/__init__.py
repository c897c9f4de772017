"""CPU oracle for the population step of Population Based Training (PBT).

TEST INFRASTRUCTURE ONLY.  This package is a plain, slow, double-precision
restatement of what the method computes (Jaderberg et al., Population Based
Training of Neural Networks, Section 3, Algorithm 1, Section 4.1.1 and
Appendix A.1).  It exists so that the GPU library can be checked against
something that can be read next to the paper.  Only the test-suite, the smoke
check and the benchmark's reported CPU baseline may import it; the GPU library
and its Python binding never do, and it imports nothing from them.

Precision: every quantity is float64 except where the method itself fixes a
narrower type: hyperparameters and scores are float32 values (so that ranking
and the explore multiply are decided in the precision the population store
holds them in), and random words are uint32.

Parity status.  The paper prints no numeric trace of a population step, so the
end-to-end numbers of `train` are "parity unpinned" against the paper; every
building block is pinned separately (finite differences, closed forms, library
cross-checks, brute force, published known-answer vectors, the toy example of
Figure 2).
"""
