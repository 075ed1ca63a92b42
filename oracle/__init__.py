"""CPU oracle for the PosS draft-and-verify round.  TEST INFRASTRUCTURE ONLY.

A plain, slow NumPy (float64) statement of what the hot path computes, written
from the paper (arXiv 2506.03566).  Only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import it; the HIP library never does, and it
shares no code with the HIP library (inputs come from synth/, which holds none
of the method's arithmetic).

Modules
  numerics  RMSNorm, rotary embedding, masked softmax attention, storage rounding
  model     Llama-style target rows (features, Head) and one specialist pass (Eq. 1, 2, 7, 9)
  greedy    vanilla autoregressive greedy decoding: the plain definition the
            committed stream must equal under greedy verification (section 2.1)
  tree      top-k expansion tree, position ids, ancestor mask, acceptance walk,
            brute-force path enumeration (section 4.1 "Implementations": width,
            depth, total tokens)
  poss      the round: draft -> verify -> accept/commit; tau and pos-acc (Eq. 3, 4)
  sampling  verification at a temperature: the target's token drawn from softmax(logits / T) by
            inverse CDF with a uniform number per position (section 2.1 asks only that the
            target's distribution is kept)

Pins (tests/test_oracle_*.py): layer parameter count of section 3.3,
specialist indexing example below Eq. 7, draft-layer counts of appendix D,
Eq. 3/4 identities, losslessness against `greedy`, brute-force acceptance,
brute-force top-N, perfect-drafter and S-identical-specialists special cases,
textbook reductions (softmax rows, RoPE relativity, norm invariants).
Parity unpinned: the specialist used beyond depth S*n (clamped to the last
one); whether the paper's printed tau counts the bonus token; whether "total
tokens" counts the root; which acceptance rule the paper's temperature-1 runs used.
"""
