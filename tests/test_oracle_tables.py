"""Pins for the oracle's bucket tables (T_w), hit matrix (Eq. 9, Algorithm 1) and candidate list
(Eq. 10, Eq. 3).  The comparison side is the definition evaluated with numpy on the code arrays,
with no tables at all, plus the structural invariants the definition implies."""
import numpy as np
import pytest

import oracle
import workloads


@pytest.fixture(scope="module")
def tiny():
    cfg = workloads.CONFIGS["tiny"]
    E, perms, topfreq, H = workloads.make_all(cfg, seed=0)
    return cfg, E, perms, topfreq, H, oracle.Index(E, perms, cfg.W)


def _np_band_codes(X, perms, W):
    """Definition written with numpy only: argmax over the gathered window, packed big-endian."""
    P, K = perms.shape
    bits = int(np.ceil(np.log2(K)))
    codes = np.argmax(X[:, perms], axis=2).reshape(X.shape[0], W, P // W)
    out = np.zeros((X.shape[0], W), dtype=np.int64)
    for i in range(P // W):
        out = (out << bits) | codes[:, :, i]
    return out


def test_buckets_partition_the_vocabulary(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    bandE = _np_band_codes(E, perms, cfg.W)
    for w in range(cfg.W):
        keys = ix.bucket_keys(w)
        assert len(set(keys.tolist())) == len(keys) == ix.num_buckets(w)
        seen = np.zeros(cfg.V, dtype=np.int32)
        for code in keys:
            words = ix.bucket(w, code)
            assert np.all(np.diff(words) > 0)               # ascending, no repeats
            assert np.all(bandE[words, w] == code)          # every member carries the key
            seen[words] += 1
        assert np.all(seen == 1)                            # disjoint, union = 0..V-1
        assert set(keys.tolist()) == set(bandE[:, w].tolist())


def test_absent_code_has_no_bucket(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    present = set(ix.bucket_keys(0).tolist())
    absent = next(c for c in range(1 << 12) if c not in present)
    assert ix.bucket(0, absent) is None


def test_hit_matrix_equals_definition(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    bandE = _np_band_codes(E, perms, cfg.W)
    for step in range(3):
        Hs = H[step]
        bandH = _np_band_codes(Hs, perms, cfg.W)
        assert np.array_equal(ix.hidden_band_codes(Hs), bandH)
        L_def = (bandH[:, None, :] == bandE[None, :, :]).sum(axis=2)     # Eq. 9, O(B V W)
        assert np.array_equal(ix.hit_counts(Hs), L_def)


@pytest.mark.parametrize("t", [1, 2, 3])
def test_candidates_equal_definition(tiny, t):
    cfg, E, perms, topfreq, H, ix = tiny
    bandE = _np_band_codes(E, perms, cfg.W)
    for step in range(5):
        Hs = H[step]
        bandH = _np_band_codes(Hs, perms, cfg.W)
        L_def = (bandH[:, None, :] == bandE[None, :, :]).sum(axis=2)
        want = np.union1d(topfreq, np.nonzero((L_def >= t).any(axis=0))[0])
        got = ix.candidates(Hs, topfreq, t=t)
        assert np.array_equal(got, want)
        assert np.all(np.diff(got) > 0)


def test_candidate_invariants(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    Hs = H[0]
    got = ix.candidates(Hs, topfreq)
    assert set(topfreq.tolist()) <= set(got.tolist())
    # every word sharing a band code with a hidden row is a candidate
    bandH = ix.hidden_band_codes(Hs)
    per_row = 0
    for i in range(cfg.B):
        mine = set()
        for w in range(cfg.W):
            b = ix.bucket(w, bandH[i, w])
            if b is not None:
                assert set(b.tolist()) <= set(got.tolist())
                mine |= set(b.tolist())
        per_row += len(mine)
    assert len(got) <= cfg.T + per_row
    # nothing else is: remove top-freq and bucket members, nothing may remain
    rest = set(got.tolist()) - set(topfreq.tolist())
    for i in range(cfg.B):
        for w in range(cfg.W):
            b = ix.bucket(w, bandH[i, w])
            if b is not None:
                rest -= set(b.tolist())
    assert not rest


def test_embedding_row_collides_with_itself(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    words = np.array([77, 500, 999, 123])
    got = ix.candidates(E[words], np.zeros(0, dtype=np.int32))
    assert set(words.tolist()) <= set(got.tolist())
    L = ix.hit_counts(E[words])
    assert all(L[i, w] == cfg.W for i, w in enumerate(words))     # all W bands agree


def test_threshold_above_band_count_leaves_only_topfreq(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    got = ix.candidates(H[0], topfreq, t=cfg.W + 1)
    assert np.array_equal(got, np.sort(topfreq))


def test_topfreq_duplicates_and_order_do_not_matter(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    tf = np.array([5, 3, 5, 900, 3], dtype=np.int32)
    a = ix.candidates(H[1], tf)
    b = ix.candidates(H[1], np.array([3, 5, 900], dtype=np.int32))
    assert np.array_equal(a, b)


def test_bf16_index_matches_definition_on_stored_values():
    cfg = workloads.CONFIGS["tiny"]
    E = workloads.f32_to_bf16_bits(workloads.make_embeddings(cfg, seed=3))
    perms = workloads.make_perms(cfg, seed=3)
    ix = oracle.Index(E, perms, cfg.W)
    bandE = _np_band_codes(workloads.bf16_bits_to_f32(E), perms, cfg.W)
    for w in range(cfg.W):
        for code in ix.bucket_keys(w):
            assert np.array_equal(ix.bucket(w, code), np.nonzero(bandE[:, w] == code)[0])
