"""CPU oracle for the ADPSGD hot path (TEST INFRASTRUCTURE ONLY).

A slow, plain numpy restatement of what one ADPSGD iteration computes
(Algorithm 1 / Eq. 2 of the paper with the fixed-ring, random-ring and
delay-by-one choices of Section III, the synchronous baseline of Section
III-A (Algorithm 2), and a stacked (bi)directional LSTM
acoustic model with a softmax cross-entropy output, Section IV).

Nothing in the product package imports this; only the tests, the smoke check
and the CPU-baseline leg of the benchmark do.  It shares no code with the HIP
library: the schedule generator, the parameter layout and the arithmetic are
written a second time here, from the paper.

Parity status of the pieces (what pins each one is listed in the test files):
  schedule      pinned by invariants + the paper's closed forms (TRI mixing)
  mix / update  pinned by dense-matrix brute force, mean preservation,
                consensus in one step for T = 11'/L, L=1 -> plain SGD
  synchronous baseline  pinned by the dense product (W - a G) 11'/L, exact
                model-averaging = gradient-averaging on dyadic data, and
                L learners of batch B = one learner of batch L*B
  LSTM fwd/bwd  pinned by finite differences, hand-computed special cases
                and a stock CPU LSTM (test only)
  exact partner sequence for a given seed: the paper defines none, so it is
                pinned only by stored vectors of this generator ("parity
                unpinned" with respect to the paper).
"""
