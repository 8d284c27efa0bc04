"""CPU oracle for the decoding rule the paper times: temperature + top-k sampling.
TEST INFRASTRUCTURE ONLY (same rules as first_oracle.py: the HIP library never imports it
and shares no code with it).

Appendix, "Inference settings": every task is decoded with temperature 0.8 and top-k
sampling over 10 tokens.  The paper gives no formula; the reading taken is the usual one,
written out plainly:

  1. candidates = the k tokens with the largest logits; equal logits are ordered by token
     index, lowest first (the same tie rule as the greedy argmax);
  2. p_j = exp((l_j - l_max) / T) / sum over the candidates  (softmax of logits / T
     restricted to the candidates);
  3. the draw is a uniform number u in [0, 1) SUPPLIED BY THE CALLER (neither side owns a
     random number generator): candidates are walked in descending-logit order and the
     first one whose cumulative probability exceeds u is returned.

Step 3 turns floating point into an integer, so it exists in two precisions: fp64 (the
definition) and fp32 (`dtype=numpy.float32`: the arithmetic type of the GPU kernel, same
operation order), which is the one a parity test must compare decisions with.

Pins (tests/test_oracle_pins.py): a hand-worked example with exact probabilities 4/7, 2/7,
1/7; k = 1 and T -> 0 reduce to argmax; shift invariance; tie order; agreement with a
brute-force implementation via a full sort; the measure of the u-interval of each token
equals its softmax probability.
"""
from __future__ import annotations

import numpy as np


def top_k_candidates(logits: np.ndarray, k: int):
    """Indices of the k largest logits, descending by logit, ties by ascending index (step 1)."""
    logits = np.asarray(logits)
    taken = np.zeros(logits.shape[0], dtype=bool)
    chosen = []
    for _ in range(min(int(k), logits.shape[0])):
        rest = np.flatnonzero(~taken)
        j = int(rest[np.argmax(logits[rest])])       # argmax returns the first maximum: lowest index among equals
        taken[j] = True
        chosen.append(j)
    return chosen


def candidate_probabilities(logits: np.ndarray, cand, temperature: float, dtype=np.float64):
    """Step 2 for the candidate list `cand` (descending), in the given arithmetic type."""
    l = np.asarray(logits, dtype=dtype)
    t = dtype(temperature)
    lmax = l[cand[0]]
    w = np.array([np.exp((l[j] - lmax) / t) for j in cand], dtype=dtype)
    total = dtype(0)
    for x in w:                      # summed in candidate order
        total = dtype(total + x)
    return w, total


def sample_top_k(logits: np.ndarray, u: float, temperature: float, k: int, dtype=np.float64) -> int:
    """Steps 1-3.  Returns the sampled token index."""
    cand = top_k_candidates(np.asarray(logits, dtype=dtype), k)
    w, total = candidate_probabilities(logits, cand, temperature, dtype)
    target = dtype(dtype(u) * total)
    cum = dtype(0)
    for j, x in zip(cand, w):
        cum = dtype(cum + x)
        if cum > target:
            return int(j)
    return int(cand[-1])             # u * total rounded up to the total itself


def decision_margin(logits: np.ndarray, u: float, temperature: float, k: int) -> float:
    """Distance (in probability) from u to the nearest boundary of the cumulative distribution:
    a draw with a margin far above the rounding error has one correct answer in any precision."""
    cand = top_k_candidates(np.asarray(logits, dtype=np.float64), k)
    w, total = candidate_probabilities(logits, cand, temperature, np.float64)
    edges = np.cumsum(w) / total
    return float(np.min(np.abs(edges[:-1] - u))) if len(edges) > 1 else 1.0
