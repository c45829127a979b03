"""Reference for the score reductions over the mass tensor (TEST INFRASTRUCTURE ONLY; shares no
code with the GPU library).  Section 2.2 (analyzer: aggregate the recomputed attention over each
prompt's token ranges and turn it into a score), Section 2 (config: average or weighted sum),
Section 3 (focus score; per-document relevance).  The paper elides the formula itself, so the
three readings below are this project's options and "parity" means agreement with these
definitions, written as plain fp64 loops; which of them matches the paper's own code is unpinned.
"""
from typing import Optional, Sequence

import numpy as np

SPAN_MEAN, RATIO_MEAN, RATIO_OF_SUMS = 0, 1, 2


def valid_slots(i: int, NQ: int, query_sel, cu_q_lens) -> range:
    """Slots of mass[i, p, :, r] that hold a selected row: slot = t - begin for chunk-local rows
    t in [max(begin, 0), min(end, n_i, begin + NQ))."""
    if query_sel is None:
        return range(NQ)
    qb, qe = int(query_sel[i][0]), int(query_sel[i][1])
    hi = min(qe, qb + NQ)
    if cu_q_lens is not None:
        hi = min(hi, int(cu_q_lens[i + 1]) - int(cu_q_lens[i]))
    lo = max(qb, 0)
    return range(lo - qb, max(hi, lo) - qb)


def reduce_mass(mass, mode: int, span_a: int = 0, span_b: int = 1, query_sel=None, cu_q_lens=None,
                head_weights: Optional[Sequence[float]] = None, scores_in=None) -> np.ndarray:
    """Returns scores ([num_seqs, S] for SPAN_MEAN, else [num_seqs]) in fp64; when scores_in is
    given the result is added to it (the accumulate option)."""
    m = np.asarray(mass, dtype=np.float64)
    num_seqs, P, NQ, S = m.shape
    w = [1.0 / P] * P if head_weights is None else [float(x) for x in head_weights]
    out = np.zeros((num_seqs, S) if mode == SPAN_MEAN else (num_seqs,), dtype=np.float64)
    for i in range(num_seqs):
        slots = valid_slots(i, NQ, query_sel, cu_q_lens)
        nv = len(slots)
        if nv == 0:
            continue
        if mode == SPAN_MEAN:
            for r in range(S):
                out[i, r] = sum(w[p] * sum(m[i, p, t, r] for t in slots) / nv for p in range(P))
        elif mode == RATIO_MEAN:
            tot = 0.0
            for p in range(P):
                acc = 0.0
                for t in slots:
                    a, b = m[i, p, t, span_a], m[i, p, t, span_b]
                    acc += a / (a + b) if (a + b) != 0.0 else 0.0
                tot += w[p] * acc / nv
            out[i] = tot
        elif mode == RATIO_OF_SUMS:
            A = sum(w[p] * sum(m[i, p, t, span_a] for t in slots) / nv for p in range(P))
            B = sum(w[p] * sum(m[i, p, t, span_b] for t in slots) / nv for p in range(P))
            out[i] = A / (A + B) if (A + B) != 0.0 else 0.0
        else:
            raise ValueError("unknown mode")
    if scores_in is not None:
        out = out + np.asarray(scores_in, dtype=np.float64)
    return out
