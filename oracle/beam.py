"""CPU oracle for the beam-search selection step -- TEST INFRASTRUCTURE ONLY.

Section 4.5.1 ("Beam Search Optimization") selects, out of beam_width * top_k candidate continuations,
the beam_width best in descending order.  The result has a plain definition, written out here: score
every candidate, sort ALL of them, keep the first beam_width.  No heap, no early exit.

Reading fixed here (the paper does not order equal scores): "score descending, then sequence index
ascending, then candidate index ascending".  Scores are added in float32, the precision of the log-probs
handed to the selection, so that the order is decided on the same numbers as in the product.
"""
from __future__ import annotations

import numpy as np


def beam_select(beam_lp: np.ndarray, cand_lp: np.ndarray, cand_tok: np.ndarray | None = None):
    """beam_lp [R, W] float32, cand_lp [R, W, K] float32, cand_tok [R, W, K] int32 or None (token = k).
    Returns (scores [R, W] float32, parent [R, W] int32, token [R, W] int32)."""
    beam_lp = np.asarray(beam_lp, dtype=np.float32)
    cand_lp = np.asarray(cand_lp, dtype=np.float32)
    R, W, K = cand_lp.shape
    score = (beam_lp[:, :, None] + cand_lp).astype(np.float32)          # float32 + float32 -> float32
    out_s = np.empty((R, W), np.float32)
    out_p = np.empty((R, W), np.int32)
    out_t = np.empty((R, W), np.int32)
    for r in range(R):
        flat = score[r].reshape(W * K)                                   # index = w * K + k
        order = np.argsort(-flat.astype(np.float64), kind="stable")[:W]  # stable: equal scores keep (w, k) order
        out_s[r] = flat[order]
        out_p[r] = order // K
        k = order % K
        out_t[r] = k if cand_tok is None else np.asarray(cand_tok)[r].reshape(W * K)[order]
    return out_s, out_p, out_t
