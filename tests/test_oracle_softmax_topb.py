"""Pins for the oracle's logits (Eq. 2), log-softmax (Eq. 1 over the candidate list) and heap
beam expansion, against torch's CPU float64 library routines, closed-form cases and invariants."""
import numpy as np
import pytest
import torch

import oracle
import workloads


@pytest.fixture(scope="module")
def tiny():
    cfg = workloads.CONFIGS["tiny"]
    E, perms, topfreq, H = workloads.make_all(cfg, seed=0)
    return cfg, E, perms, topfreq, H, oracle.Index(E, perms, cfg.W)


def _lib_logprobs(H, E, cand):
    logits = torch.from_numpy(H.astype(np.float64)) @ torch.from_numpy(E[cand].astype(np.float64)).T
    return torch.log_softmax(logits, dim=1).numpy(), logits.numpy()


def test_logprobs_match_library_log_softmax(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    cand = ix.candidates(H[0], topfreq)
    lp, lg = ix.logprobs(H[0], cand, want_logits=True)
    want_lp, want_lg = _lib_logprobs(H[0], E, cand)
    np.testing.assert_allclose(lg, want_lg, rtol=0, atol=1e-12)
    np.testing.assert_allclose(lp, want_lp, rtol=0, atol=1e-12)
    np.testing.assert_allclose(np.exp(lp).sum(axis=1), 1.0, atol=1e-12)


def test_logits_are_not_transposed_or_misindexed():
    # E rows are one-hot scaled: logit[i, c] must be exactly H[i, hot(cand[c])] * scale(cand[c])
    V, d = 37, 11
    E = np.zeros((V, d), dtype=np.float32)
    hot = (np.arange(V) * 7) % d
    E[np.arange(V), hot] = 1.0 + np.arange(V, dtype=np.float32)
    perms = np.arange(d, dtype=np.int32)[None, :4].repeat(2, axis=0)
    ix = oracle.Index(E, perms, 1)
    H = np.arange(3 * d, dtype=np.float32).reshape(3, d) / 8.0
    cand = np.array([36, 2, 19, 5], dtype=np.int32)
    _, lg = ix.logprobs(H, cand, want_logits=True)
    want = H[:, hot[cand]].astype(np.float64) * (1.0 + cand)
    assert np.array_equal(lg, want)


def test_uniform_logits_closed_form():
    V, d = 50, 8
    E = np.ones((V, d), dtype=np.float32)
    perms = np.arange(4, dtype=np.int32)[None, :]
    ix = oracle.Index(E, perms, 1)
    H = np.full((2, d), 0.25, dtype=np.float32)
    cand = np.arange(0, 50, 5, dtype=np.int32)
    lp = ix.logprobs(H, cand)
    np.testing.assert_allclose(lp, -np.log(len(cand)), atol=1e-15)


def test_large_logits_do_not_overflow():
    V, d = 20, 4
    rng = np.random.default_rng(0)
    E = (rng.standard_normal((V, d)) * 300).astype(np.float32)
    ix = oracle.Index(E, np.arange(4, dtype=np.int32)[None, :], 1)
    H = (rng.standard_normal((3, d)) * 30).astype(np.float32)
    lp = ix.logprobs(H, None)
    assert np.all(np.isfinite(lp))
    want, _ = _lib_logprobs(H, E, np.arange(V))
    np.testing.assert_allclose(lp, want, rtol=1e-13, atol=1e-9)


def test_row_shift_leaves_logprobs_unchanged(tiny):
    # append a dimension where every E row holds 1 and H row i holds c_i: all logits of row i
    # shift by c_i, which a softmax must cancel
    cfg, E, perms, topfreq, H, ix = tiny
    cand = ix.candidates(H[2], topfreq)
    base = ix.logprobs(H[2], cand)
    E2 = np.concatenate([E, np.ones((cfg.V, 1), dtype=np.float32)], axis=1)
    H2 = np.concatenate([H[2], np.array([[3.0], [-7.0], [0.5], [100.0]], dtype=np.float32)], axis=1)
    ix2 = oracle.Index(E2, perms, cfg.W)            # perms never index the new dimension
    assert np.array_equal(ix2.candidates(H2, topfreq), cand)
    np.testing.assert_allclose(ix2.logprobs(H2, cand), base, atol=1e-10)


def test_full_vocab_step_equals_library_topk(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    rng = np.random.default_rng(7)
    for step in range(4):
        bs = rng.standard_normal(cfg.B).astype(np.float32)
        ob, ow, osc, cnt = ix.decode_step(H[step], bs, topfreq, 1, cfg.B, full_vocab=True)
        assert cnt[0] == cfg.V
        lp, _ = _lib_logprobs(H[step], E, np.arange(cfg.V))
        scores = torch.from_numpy(bs.astype(np.float64)[:, None] + lp).reshape(-1)
        top = torch.topk(scores, cfg.B)
        assert np.array_equal(ob[0], (top.indices // cfg.V).numpy())
        assert np.array_equal(ow[0], (top.indices % cfg.V).numpy())
        np.testing.assert_allclose(osc[0], top.values.numpy(), atol=1e-12)
        assert np.all(np.diff(osc[0]) <= 0)


def test_lsh_step_equals_library_topk_over_candidates(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    bs = np.array([0.0, -1.0, -0.5, -3.0], dtype=np.float32)
    ob, ow, osc, cnt = ix.decode_step(H[5], bs, topfreq, 1, cfg.B)
    cand = ix.candidates(H[5], topfreq)
    assert cnt[0] == len(cand)
    lp, _ = _lib_logprobs(H[5], E, cand)
    scores = torch.from_numpy(bs.astype(np.float64)[:, None] + lp).reshape(-1)
    top = torch.topk(scores, cfg.B)
    assert np.array_equal(ob[0], (top.indices // len(cand)).numpy())
    assert np.array_equal(ow[0], cand[(top.indices % len(cand)).numpy()])
    np.testing.assert_allclose(osc[0], top.values.numpy(), atol=1e-12)


def test_single_beam_top1_is_argmax_of_dot_products(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    h = H[3][:1]
    cand = ix.candidates(h, topfreq)
    ob, ow, osc, _ = ix.decode_step(h, np.zeros(1, dtype=np.float32), topfreq, 1, 1)
    dots = E[cand].astype(np.float64) @ h[0].astype(np.float64)
    assert ob[0, 0] == 0 and ow[0, 0] == cand[np.argmax(dots)]


def test_topb_tie_order_and_padding():
    lp = np.array([[-1.0, -2.0, -1.0], [-1.0, -5.0, -2.0]])
    cand = np.array([4, 9, 11], dtype=np.int32)
    ob, ow, osc = oracle.topb(np.zeros(2), lp, cand, 5)
    # three pairs tie at -1: lower beam first, then lower word id; then the two at -2
    assert list(zip(ob.tolist(), ow.tolist())) == [(0, 4), (0, 11), (1, 4), (0, 9), (1, 11)]
    assert osc.tolist() == [-1.0, -1.0, -1.0, -2.0, -2.0]
    # a dead beam (-inf) can never be selected; missing entries are padded
    ob, ow, osc = oracle.topb(np.array([-np.inf, 0.0]), lp, cand, 5)
    assert ob.tolist() == [1, 1, 1, -1, -1] and ow.tolist() == [4, 11, 9, -1, -1]
    assert osc[3] == -np.inf and osc[4] == -np.inf


def test_beam_scores_select_across_beams():
    lp = np.log(np.array([[0.7, 0.2, 0.1], [0.6, 0.3, 0.1]]))
    ob, ow, osc = oracle.topb(np.array([0.0, np.log(2.0)]), lp, None, 3)
    # scores: beam0: .7 .2 .1 ; beam1 doubled: 1.2 .6 .2
    assert list(zip(ob.tolist(), ow.tolist())) == [(1, 0), (0, 0), (1, 1)]
    np.testing.assert_allclose(np.exp(osc), [1.2, 0.7, 0.6], rtol=1e-12)


def test_sentences_are_independent(tiny):
    cfg, E, perms, topfreq, H, ix = tiny
    Hcat = np.concatenate([H[0], H[1], H[2]], axis=0)
    bs = np.linspace(-2, 0, 3 * cfg.B).astype(np.float32)
    ob, ow, osc, cnt = ix.decode_step(Hcat, bs, topfreq, 3, cfg.B)
    for s in range(3):
        b1, w1, s1, c1 = ix.decode_step(H[s], bs[s * cfg.B:(s + 1) * cfg.B], topfreq, 1, cfg.B)
        assert np.array_equal(ob[s], b1[0]) and np.array_equal(ow[s], w1[0])
        assert np.array_equal(osc[s], s1[0]) and cnt[s] == c1[0]


def test_bf16_embeddings_are_read_exactly():
    cfg = workloads.CONFIGS["tiny"]
    Ef = workloads.make_embeddings(cfg, seed=2)
    bits = workloads.f32_to_bf16_bits(Ef)
    perms = workloads.make_perms(cfg, seed=2)
    ix = oracle.Index(bits, perms, cfg.W)
    H = workloads.make_hidden(cfg, Ef, seed=2, steps=1)[0]
    cand = np.arange(0, cfg.V, 3, dtype=np.int32)
    lp = ix.logprobs(H, cand)
    want, _ = _lib_logprobs(H, workloads.bf16_bits_to_f32(bits), cand)
    np.testing.assert_allclose(lp, want, atol=1e-12)
