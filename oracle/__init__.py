"""CPU oracle for the DAB-Net binarized-layer hot path.

TEST INFRASTRUCTURE ONLY.  Everything in this package is a plain, slow,
float64 CPU statement of what the method computes, written from the paper
(arXiv 1804.02941).  It exists so that the HIP library can be checked against
something that does not share a single line with it.  Only the test-suite,
the smoke check and the ``cpu_baseline`` leg of the benchmark may import it;
the product path never does, and it has no fallback that lands here.

Modules
-------
estimate   Theorem 2 / Algorithm 1: per-filter split search, alpha, beta, K, mask e.
layers     Sign binarization of activations, the two-valued filter of Corollary 1,
           the direct float64 convolution / fully-connected product, the integer
           side channel (s1, sA) and the popcount form of the same dot product.
packing    Reference bit packers that pin the bit order of the packed operands.

Parity status: every function here is pinned by the CPU tests (exact rational
brute force over all masks, closed forms, library cross-checks); none is
"parity unpinned".
"""
