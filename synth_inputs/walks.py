"""Walk policy: how a synthetic request picks its next token from a mask.

The policy stands in for a language model's sampler.  It sees only the
allowed-token bits and the token bytes; it knows nothing about grammars.
"""

from __future__ import annotations

import numpy as np

# A model closes strings and brackets far more often than a uniform draw over
# the allowed tokens would; the biased policy below restores that behaviour.
STRUCTURAL_BYTES = frozenset(b'"{}[],:;()')


def pick_token(rng: np.random.Generator, allowed: np.ndarray, first_bytes: np.ndarray,
               stop_ids, structural_bias: float = 0.0) -> int:
    """Pick a token id among the allowed ones.

    ``allowed``: bool [V]; ``first_bytes``: int16 [V] (first byte of each
    token, -1 for zero-length tokens).  Stop tokens are chosen only when they
    are the sole allowed tokens.  With probability ``structural_bias`` the
    draw is restricted to allowed tokens whose first byte is structural
    (if there are any); otherwise it is uniform over all allowed non-stop
    tokens.  Returns -1 if nothing is allowed.
    """
    cand = np.flatnonzero(allowed)
    if cand.size == 0:
        return -1
    stop = np.isin(cand, np.asarray(stop_ids))
    non_stop = cand[~stop]
    if non_stop.size == 0:
        return int(cand[0])
    if structural_bias > 0.0 and rng.random() < structural_bias:
        fb = first_bytes[non_stop]
        m = np.isin(fb, np.fromiter(STRUCTURAL_BYTES, dtype=np.int16))
        if m.any():
            non_stop = non_stop[m]
    return int(non_stop[int(rng.integers(0, non_stop.size))])
