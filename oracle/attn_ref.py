"""Decode attention over ragged contexts, plain fp64 (test infrastructure, not product code).

The paper names an `attn` compute uop that performs the fused attention score computation
(Section 4.1, "Abstraction of GPU Hardware") in the manner of FlashAttention (Section 4.3,
"Virtual Memory Core") and evaluates decoding with one query per request over contexts of
uneven length (Section 6.2, "Dynamic Attention Length"); it prints no formula.  The reading
taken by this build is the textbook one: for every request s with context rows
row_off[s] .. row_off[s + 1] of the key and value caches,

    score_r = scale * sum_j Q[s][j] * K[r][j]
    p_r     = exp(score_r - max_r score_r) / sum_r exp(score_r - max_r score_r)
    O[s][t] = sum_r p_r * V[r][t]

The definition is written out directly: all scores of a request first, then the softmax, then the
weighted sum, in fp64 from the fp32 inputs.  The tiled, running-maximum evaluation order of the
uop is not used here.
"""
import numpy as np


def attn_decode(Q, K, V, row_off, scale):
    """Q: [n_seg][d]; K, V: [rows][d]; row_off: n_seg + 1 offsets into the rows; scale: float.
    Returns (O, A, S): O[n_seg][d] in fp64; A[n_seg][d] = sum_r p_r |V[r][t]|, the scale of O's rounding
    error; S[n_seg] = max_r scale * sum_j |Q[s][j] K[r][j]|, the scale of a score's rounding error."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    n_seg, d = Q.shape
    O = np.zeros((n_seg, d))
    A = np.zeros((n_seg, d))
    S = np.zeros(n_seg)
    for s in range(n_seg):
        r0, r1 = int(row_off[s]), int(row_off[s + 1])
        if r1 <= r0:
            raise ValueError("a request needs at least one context row")
        score = np.zeros(r1 - r0)
        for r in range(r0, r1):
            score[r - r0] = scale * np.sum(Q[s] * K[r])
            S[s] = max(S[s], scale * np.sum(np.abs(Q[s] * K[r])))
        e = np.exp(score - score.max())
        p = e / e.sum()
        for r in range(r0, r1):
            O[s] += p[r - r0] * V[r]
            A[s] += p[r - r0] * np.abs(V[r])
    return O, A, S
