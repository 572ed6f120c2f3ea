"""Plain fp64 CPU oracle of sampling-based acceptance (TEST INFRASTRUCTURE, not a product path).

The paper's core loop (section 4.1) is stated for greedy decoding; a footnote there says it extends
to sampling-based decoding by standard rejection sampling and gives no further text.  The reading
taken here is the textbook speculative-sampling rule, with every random number passed in:

  p_j = softmax(target_row_j / T)   the full-KV distribution for drafted position j
  q_j = softmax(draft_row_j / T)    the distribution the drafted token t_j was sampled from
  position j is accepted iff  u_accept[j] * q_j(t_j) < p_j(t_j)        (i.e. with probability
                                                                         min(1, p_j(t_j) / q_j(t_j)))
  a = first rejected position, else w
  a < w : next token ~ normalised max(0, p_a - q_a), drawn by inverse CDF with u_resample:
          the smallest v whose running sum of max(0, p_a - q_a) exceeds u_resample * (total sum)
  a = w : the bonus token, drawn the same way from p_w when that row is supplied, else -1
u values lie in [0, 1).  All arithmetic is IEEE double in the order written; results that hinge on
a comparison also return how far from a tie the comparison was, so that a test can insist on a
margin before it asks another implementation for the identical integer.
"""
from __future__ import annotations

import numpy as np


def softmax_t(row, temperature: float) -> np.ndarray:
    z = np.asarray(row, dtype=np.float64) / float(temperature)
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def inverse_cdf(weights: np.ndarray, u: float):
    """Smallest index whose running sum exceeds u * total; also the relative distance of the
    threshold from the nearest running-sum boundary."""
    c = np.cumsum(weights)
    total = c[-1]
    thr = float(u) * total
    idx = int(np.searchsorted(c, thr, side="right"))
    idx = min(idx, len(c) - 1)
    lo = c[idx - 1] if idx > 0 else 0.0
    margin = min(thr - lo, c[idx] - thr) / total if total > 0 else 0.0
    return idx, float(margin)


def accept_sample(target_logits, draft_logits, cu_rows, draft_ids, cu_win, temperature, u_accept, u_resample):
    """Returns (accept_len [B], next_token [B], margins) where margins = (accept margins [sum w],
    resample margin [B]): |u*q - p| / p of every accept test that was evaluated (inf for the
    others) and the inverse-CDF margin of every drawn token (inf when none was drawn)."""
    target_logits = np.asarray(target_logits, dtype=np.float64)
    draft_logits = np.asarray(draft_logits, dtype=np.float64)
    nseq = len(cu_rows) - 1
    acc = np.zeros(nseq, dtype=np.int32)
    nxt = np.zeros(nseq, dtype=np.int32)
    m_acc = np.full(len(draft_ids), np.inf)
    m_res = np.full(nseq, np.inf)
    for b in range(nseq):
        r0, r1 = int(cu_rows[b]), int(cu_rows[b + 1])
        w0, w1 = int(cu_win[b]), int(cu_win[b + 1])
        w = w1 - w0
        a = w
        for j in range(w):
            p = softmax_t(target_logits[r0 + j], temperature)
            q = softmax_t(draft_logits[w0 + j], temperature)
            t = int(draft_ids[w0 + j])
            lhs = float(u_accept[w0 + j]) * q[t]
            m_acc[w0 + j] = abs(lhs - p[t]) / max(p[t], 1e-300)
            if not (lhs < p[t]):
                a = j
                break
        acc[b] = a
        if a < w:
            p = softmax_t(target_logits[r0 + a], temperature)
            q = softmax_t(draft_logits[w0 + a], temperature)
            nxt[b], m_res[b] = inverse_cdf(np.maximum(p - q, 0.0), u_resample[b])
        elif r0 + w < r1:
            nxt[b], m_res[b] = inverse_cdf(softmax_t(target_logits[r0 + w], temperature), u_resample[b])
        else:
            nxt[b] = -1
    return acc, nxt, (m_acc, m_res)
