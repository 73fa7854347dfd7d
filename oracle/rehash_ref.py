"""Step Rehash reference: similarity test, key-step search, replay (float64).

TEST INFRASTRUCTURE ONLY -- see the package docstring.

The paper speaks of the "similarity" between the features of two steps
(Sec. 4.3.1, Appendix B) without naming the measure; this build fixes cosine
similarity over the whole flattened feature.  The key-step search follows the
steps of Algorithm 1 (Appendix B).
"""
from __future__ import annotations

import math
from typing import Callable, List, Sequence

import numpy as np


def cosine_terms_ref(a, b):
    """(sum a*b, sum a*a, sum b*b) in float64 over all elements."""
    a = np.asarray(a, np.float64).ravel()
    b = np.asarray(b, np.float64).ravel()
    return float(np.dot(a, b)), float(np.dot(a, a)), float(np.dot(b, b))


def cosine_ref(a, b) -> float:
    """cos = <a,b> / (|a| |b|).  Both all-zero -> 1 (identical); exactly one
    all-zero -> 0; any non-finite term -> NaN."""
    dot, na, nb = cosine_terms_ref(a, b)
    if not (math.isfinite(dot) and math.isfinite(na) and math.isfinite(nb)):
        return float("nan")
    if na == 0.0 and nb == 0.0:
        return 1.0
    if na == 0.0 or nb == 0.0:
        return 0.0
    return dot / math.sqrt(na * nb)


def rehash_decision_ref(a, b, gamma: float) -> int:
    """1 = reuse the cached feature (similarity >= gamma), 0 = recompute.

    Decided without the division: dot >= gamma * sqrt(na*nb) in float64, gamma
    taken as the float32 value the C-ABI receives.  Non-finite terms -> 0."""
    dot, na, nb = cosine_terms_ref(a, b)
    g = float(np.float32(gamma))
    if not (math.isfinite(dot) and math.isfinite(na) and math.isfinite(nb)) or math.isnan(g):
        return 0
    if na == 0.0 and nb == 0.0:
        return 1 if 1.0 >= g else 0
    if na == 0.0 or nb == 0.0:
        return 1 if 0.0 >= g else 0
    return 1 if dot >= g * math.sqrt(na * nb) else 0


def key_step_search_ref(S, gamma: float, K: int) -> List[int]:
    """Algorithm 1 (Appendix B): walk i upward with anchor j = last key step.

    Step i similar to the anchor (S[i][j] >= gamma) is skipped; otherwise i
    becomes a key step and the new anchor.  Step 0 and step K-1 are always key
    steps.  Returned as a sorted list without duplicates.  Requires the
    diagonal to pass the test (gamma <= S[i][i]), else the walk cannot end."""
    S = np.asarray(S, np.float64)
    if K < 1 or S.shape[0] < K or S.shape[1] < K or not (gamma <= 1.0):
        raise ValueError("bad arguments")
    i = 0
    j = 0
    G = [0]
    while i < K:
        if S[i][j] >= gamma:
            i += 1
        else:
            if not (S[i][i] >= gamma):
                raise ValueError("diagonal fails the threshold: walk cannot terminate")
            G.append(i)
            j = i
    G.append(K - 1)
    return sorted(set(G))


def rehash_replay_ref(compute: Callable[[int], np.ndarray], key_steps: Sequence[int], K: int):
    """Sec. 4.3.2 hand-back rule at the block output: at a key step the feature
    is computed and cached; at any other step the cached feature of the most
    recent key step is returned.  Yields (t, feature, recomputed)."""
    keys = set(key_steps)
    cache = None
    for t in range(K):
        if t in keys or cache is None:
            cache = compute(t)
            yield t, cache, True
        else:
            yield t, cache, False


def rehash_causal_ref(inputs: Sequence[np.ndarray], compute: Callable[[np.ndarray], np.ndarray], gamma: float):
    """One-pass (causal) variant of the Sec. 4.3.2 hand-back rule: the decision
    for step t is taken from what is known when step t starts.  The block's
    input x_t is compared with the input of the last recomputed step (the
    anchor, as in Algorithm 1's walk: always the last key step, never simply
    the previous step); similar (>= gamma) -> the anchor's output is handed
    back, over as many consecutive steps as the test keeps passing; otherwise
    the block is computed on x_t, which becomes the new anchor.  The first
    step always computes.  Yields (t, feature, recomputed, cos) with cos = NaN
    where no test was taken."""
    anchor_x = None
    anchor_y = None
    for t, x in enumerate(inputs):
        if anchor_x is not None and rehash_decision_ref(x, anchor_x, gamma) == 1:
            yield t, anchor_y, False, cosine_ref(x, anchor_x)
            continue
        c = float("nan") if anchor_x is None else cosine_ref(x, anchor_x)
        anchor_y = compute(x)
        anchor_x = x
        yield t, anchor_y, True, c
