"""CPU oracle for the dKV-Cache hot path (arxiv 2505.15781).

TEST INFRASTRUCTURE ONLY. A plain, slow, double-precision numpy statement of
what one denoising run computes: the active-set schedule, the partial
transformer forward over a position-indexed K/V store, the vocabulary softmax
and the confidence / fixed-order unmasking step. It shares no code with the
HIP library and is imported only by tests, by the smoke check and by the
`cpu_baseline` leg of the benchmark; the product path never calls it.

Pins (see tests marked "not gpu"): the worked index example of Appendix A,
refresh-every-step == cache-free recomputation, one-layer exactness of the
one-step delay, agreement of the position-indexed store with the
concat/reorder formulation of Algorithm 1, a literal Eq. 4 reconstruction from
full K/V history, closed-form set sizes, stamps and cache ratio, and textbook
properties of softmax, attention, RoPE and RMSNorm.

Parity unpinned: the numeric logits of a random-weight model have no value
outside this oracle; they are fixed only through the pins above.
"""
