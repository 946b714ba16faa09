"""Pins of the beam-bookkeeping reference (oracle/beam.py): numpy fancy indexing for the state
gather, exhaustive enumeration of every root-to-leaf path for the backtrace, and hand-made cases."""
import itertools

import numpy as np

from oracle import beam


def test_state_gather_is_fancy_indexing_and_finished_slots_die():
    rng = np.random.default_rng(0)
    B, D = 6, 5
    states = [rng.standard_normal((B, D)).astype(np.float32) for _ in range(3)]
    parents = np.array([2, 2, 0, 5, -1, 1], dtype=np.int32)
    words = np.array([7, 9, 3, 9, -1, 4], dtype=np.int32)        # eos = 9
    scores = rng.standard_normal(B).astype(np.float32)
    new, nxt = beam.advance(parents, words, scores, states, eos=9)
    for st, nw in zip(states, new):
        want = st[np.maximum(parents, 0)]
        want[parents < 0] = 0
        assert np.array_equal(nw, want)
    assert np.array_equal(np.isneginf(nxt), [False, True, False, True, True, False])
    assert np.array_equal(nxt[[0, 2, 5]], scores[[0, 2, 5]])
    # identity parents leave the states alone
    same, _ = beam.advance(np.arange(B, dtype=np.int32), words, scores, states, eos=-1)
    assert all(np.array_equal(a, b) for a, b in zip(same, states))


def all_paths(backptr, words):
    """Every (step, slot) entry with its word sequence, by following parents (tiny inputs only)."""
    n, B = backptr.shape
    out = {}
    for t, b in itertools.product(range(n), range(B)):
        seq, cur, ok = [], b, True
        for tt in range(t, -1, -1):
            if not (0 <= backptr[tt, cur] < B):
                ok = False
                break
            seq.append(int(words[tt, cur]))
            cur = int(backptr[tt, cur])
        if ok:
            out[(t, b)] = seq[::-1]
    return out


def test_backtrace_equals_exhaustive_search_over_all_hypotheses():
    rng = np.random.default_rng(1)
    for trial in range(200):
        n, B, eos = int(rng.integers(1, 6)), int(rng.integers(1, 5)), 0
        backptr = rng.integers(-1 if trial % 3 == 0 else 0, B, size=(n, B)).astype(np.int32)
        words = rng.integers(0, 4, size=(n, B)).astype(np.int32)
        scores = np.round(rng.standard_normal((n, B)) * 2, 1).astype(np.float32)   # ties happen
        # a slot can only have a valid parent chain if the parent entry itself is valid
        paths = all_paths(backptr, words)
        # the reference only looks at its own entry's validity; make histories well-formed:
        for t in range(1, n):
            for b in range(B):
                p = backptr[t, b]
                if p >= 0 and (t - 1, int(p)) not in paths:
                    backptr[t, b] = -1
        paths = all_paths(backptr, words)
        fin = [(float(scores[t, b]), -t, -b, t, b) for (t, b) in paths if words[t, b] == eos]
        if not fin:
            fin = [(float(scores[t, b]), -t, -b, t, b) for (t, b) in paths if t == n - 1]
        toks, sc = beam.backtrace(backptr, words, scores, eos)
        if not fin:
            assert toks == [] and sc == -np.inf
            continue
        s, _, _, t, b = max(fin)
        assert sc == s and toks == paths[(t, b)]


def test_hand_made_search_tree():
    # step 0: slots continue the single start hypothesis with words 5, 6
    # step 1: slot 0 = (parent 1, word 7), slot 1 = (parent 0, word 9 = eos)  -> "5 9" finishes, -1.0
    # step 2: slot 0 = (parent 0, word 9) -> "6 7 9" finishes with -0.5: the winner
    backptr = np.array([[0, 0], [1, 0], [0, -1]], dtype=np.int32)
    words = np.array([[5, 6], [7, 9], [9, -1]], dtype=np.int32)
    scores = np.array([[-0.1, -0.2], [-0.3, -1.0], [-0.5, -np.inf]], dtype=np.float32)
    toks, sc = beam.backtrace(backptr, words, scores, eos=9)
    assert toks == [6, 7, 9] and sc == np.float32(-0.5)
    # without an end-of-sentence word nothing finishes: best slot of the last step
    toks, sc = beam.backtrace(backptr, words, scores, eos=-2)
    assert toks == [6, 7, 9]
    toks, sc = beam.backtrace(backptr[:2], words[:2], scores[:2], eos=-2)
    assert toks == [6, 7] and sc == np.float32(-0.3)
    # equal scores: the earlier step wins
    scores2 = scores.copy()
    scores2[1, 1] = -0.5
    toks, _ = beam.backtrace(backptr, words, scores2, eos=9)
    assert toks == [5, 9]
