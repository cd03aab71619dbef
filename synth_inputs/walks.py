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


def pick_tokens(rng: np.random.Generator, allowed: np.ndarray, structural: np.ndarray, is_stop: np.ndarray,
                structural_bias: float = 0.0) -> np.ndarray:
    """Batched version of :func:`pick_token` for ``allowed`` of shape [B, V].

    One vector of random priorities is drawn per call and shared by all rows
    (rows are independent requests with different masks); each row takes its
    allowed token of highest priority.  ``structural`` / ``is_stop``: bool [V].
    Returns int64 [B]; -1 where nothing is allowed; a stop token only where
    nothing else is allowed.
    """
    B, V = allowed.shape
    keys = rng.random(V, dtype=np.float32) + np.float32(1e-6)
    use_struct = rng.random(B) < structural_bias
    out = np.full(B, -1, dtype=np.int64)
    non_stop = allowed & ~is_stop[None, :]
    score = non_stop * keys[None, :]
    if structural_bias > 0.0:
        s_score = score * structural[None, :]
        s_best = s_score.argmax(axis=1)
        s_ok = s_score[np.arange(B), s_best] > 0
    best = score.argmax(axis=1)
    ok = score[np.arange(B), best] > 0
    for b in range(B):
        if structural_bias > 0.0 and use_struct[b] and s_ok[b]:
            out[b] = s_best[b]
        elif ok[b]:
            out[b] = best[b]
        else:
            stops = np.flatnonzero(allowed[b] & is_stop)
            if stops.size:
                out[b] = stops[0]
    return out
