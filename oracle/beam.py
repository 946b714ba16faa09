"""Plain reference of the beam bookkeeping around the decode step (Introduction, "Beam expansion";
Table 1, row "Hidden states reorder").  TEST INFRASTRUCTURE: imported only by tests/ (and by the
smoke check); the product path never touches it.  Python loops over tiny inputs, numpy for storage.

The paper describes beam search only in passing; the conventions here are the usual ones and are
listed as a reading of their own in the design notes:
  * slot b of a sentence continues parent out_beam[b] with word out_word[b]; the recurrent state
    rows are gathered by parent (an empty slot, parent -1, gets zeros);
  * a slot whose word is `eos` is finished: it keeps its score in the history and its next-step
    score is -inf (never expanded again); empty slots also get -inf;
  * the result is the finished hypothesis with the highest score (then earliest step, then lowest
    slot); if none finished, the best slot of the last recorded step; words are read by walking
    the parent pointers back to step 0.
"""
from __future__ import annotations

import numpy as np


def advance(out_beam, out_word, out_score, states, eos):
    """One step for one sentence.  out_* are length-B arrays, states a list of [B, D] arrays.
    Returns (new_states, next_scores)."""
    B = len(out_beam)
    new_states = []
    for st in states:
        new = np.zeros_like(st)
        for b in range(B):
            p = int(out_beam[b])
            if 0 <= p < B:
                for j in range(st.shape[1]):
                    new[b, j] = st[p, j]
        new_states.append(new)
    nxt = np.empty(B, dtype=np.float32)
    for b in range(B):
        p, w = int(out_beam[b]), int(out_word[b])
        nxt[b] = -np.inf if (p < 0 or p >= B or w == eos) else np.float32(out_score[b])
    return new_states, nxt


def backtrace(backptr, words, scores, eos):
    """History arrays [n_steps, B] of one sentence -> (tokens list, score)."""
    n_steps, B = backptr.shape if backptr.ndim == 2 else (0, 0)
    best = None  # (score, -step, -slot) compared lexicographically, larger is better
    for finished_only in (True, False):
        steps = range(n_steps) if finished_only else range(max(n_steps - 1, 0), n_steps)
        for t in steps:
            for b in range(B):
                if not (0 <= backptr[t, b] < B):
                    continue
                if finished_only and words[t, b] != eos:
                    continue
                sc = float(scores[t, b])
                if np.isnan(sc) or sc == -np.inf:
                    continue
                key = (sc, -t, -b)
                if best is None or key > best[0]:
                    best = (key, t, b)
        if best is not None:
            break
    if best is None:
        return [], -np.inf
    _, t_end, cur = best
    toks = [0] * (t_end + 1)
    for t in range(t_end, -1, -1):
        toks[t] = int(words[t, cur])
        cur = int(backptr[t, cur])
    return toks, best[0][0]
