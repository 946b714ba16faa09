"""GPU parity of the beam bookkeeping calls (lsh_beam_advance, lsh_beam_backtrace) against
oracle/beam.py, bit-exact (copies, integers, scores passed through), and the whole multi-step
loop -- decode step, bookkeeping, a stand-in recurrent update -- eager and as one HIP graph."""
import numpy as np
import pytest

import oracle
import workloads
from oracle import beam as obeam
from gpu_harness import GpuCase, assert_topb_matches, to_dev

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("S,B,D,n_states", [(3, 5, 37, 3), (1, 12, 1000, 4), (2, 4, 64, 0), (4, 20, 8, 1)])
def test_advance_matches_reference(S, B, D, n_states):
    import torch
    from paper_1806_00588_amd import binding
    rng = np.random.default_rng(S * 100 + B)
    R, eos, L = S * B, 3, 4
    hist = binding.BeamHistory(S, B, L, n_states, D, eos)
    states = [rng.standard_normal((R, max(D, 1))).astype(np.float32) for _ in range(n_states)]
    ob = rng.integers(-1, B, size=(S, B)).astype(np.int32)
    ow = rng.integers(0, 6, size=(S, B)).astype(np.int32)
    osc = rng.standard_normal((S, B)).astype(np.float32)
    sin = [to_dev(x) for x in states]
    sout = [torch.full_like(x, 7.0) for x in sin]
    nxt = torch.full((R,), 5.0, device="cuda")
    for t in (0, 2):
        binding.beam_advance(hist, t, to_dev(ob), to_dev(ow), to_dev(osc), sin, sout, nxt)
    torch.cuda.synchronize()
    for s in range(S):
        want_states, want_next = obeam.advance(ob[s], ow[s], osc[s], [x[s * B:(s + 1) * B] for x in states], eos)
        for k in range(n_states):
            assert np.array_equal(sout[k].cpu().numpy()[s * B:(s + 1) * B], want_states[k])
        assert np.array_equal(nxt.cpu().numpy()[s * B:(s + 1) * B], want_next)
    for t in (0, 2):
        assert np.array_equal(hist.backptr[t].cpu().numpy(), ob)
        assert np.array_equal(hist.words[t].cpu().numpy(), ow)
        assert np.array_equal(hist.scores[t].cpu().numpy(), osc)


def well_formed_history(rng, n, B, with_empty):
    backptr = rng.integers(-1 if with_empty else 0, B, size=(n, B)).astype(np.int32)
    for t in range(1, n):
        for b in range(B):
            if backptr[t, b] >= 0 and backptr[t - 1, backptr[t, b]] < 0:
                backptr[t, b] = -1                          # a parent must itself be a real slot
    return backptr


@pytest.mark.parametrize("S,B,n", [(1, 12, 50), (5, 3, 7), (3, 70, 4), (2, 1, 1)])
def test_backtrace_matches_reference(S, B, n):
    import torch
    from paper_1806_00588_amd import binding
    rng = np.random.default_rng(n)
    eos, L = 0, n + 3
    hist = binding.BeamHistory(S, B, L, eos=eos)
    bp = np.stack([well_formed_history(rng, n, B, s % 2 == 1) for s in range(S)], axis=1)   # [n,S,B]
    words = rng.integers(0, 5, size=(n, S, B)).astype(np.int32)
    scores = np.round(rng.standard_normal((n, S, B)) * 2, 1).astype(np.float32)             # ties
    hist.backptr[:n] = to_dev(bp)
    hist.words[:n] = to_dev(words)
    hist.scores[:n] = to_dev(scores)
    for steps in (n, max(1, n // 2), 0):
        tokens, length, score = binding.beam_backtrace(hist, steps)
        torch.cuda.synchronize()
        tokens, length, score = tokens.cpu().numpy(), length.cpu().numpy(), score.cpu().numpy()
        for s in range(S):
            toks, sc = ([], -np.inf) if steps == 0 else \
                obeam.backtrace(bp[:steps, s], words[:steps, s], scores[:steps, s], eos)
            assert length[s] == len(toks) and tokens[s, :len(toks)].tolist() == toks
            assert (score[s] == np.float32(sc)) or (np.isneginf(score[s]) and sc == -np.inf)


def test_whole_search_loop_eager_and_as_one_graph():
    import torch
    from paper_1806_00588_amd import binding
    import paper_1806_00588_amd as lsh
    cfg = workloads.CONFIGS["tiny"]
    gc = GpuCase.from_config(cfg)
    S, B, steps, eos = 2, 4, 8, 3
    R, d = S * B, cfg.d
    X = workloads.make_hidden(cfg, gc.E, seed=3, steps=steps * S).reshape(steps, R, d)
    X_dev = to_dev(X)
    sp = binding.step_params(S, B, cfg.T)
    ws = torch.empty(lsh.step_workspace_bytes(gc.tables, sp), dtype=torch.uint8, device="cuda")
    hist = binding.BeamHistory(S, B, steps, n_states=2, state_dim=d, eos=eos)
    st = [[torch.zeros(R, d, device="cuda") for _ in range(2)] for _ in range(2)]   # double buffer
    scores = [torch.zeros(R, device="cuda") for _ in range(2)]
    ob = torch.empty(R, dtype=torch.int32, device="cuda")
    ow = torch.empty(R, dtype=torch.int32, device="cuda")
    osc = torch.empty(R, device="cuda")

    def reset():
        st[0][0].copy_(X_dev[0]); st[0][1].zero_(); scores[0].zero_()
        scores[0].view(S, B)[:, 1:] = -float("inf")          # one live hypothesis per sentence at the start

    def one_step(t, check):
        a, b = t & 1, (t + 1) & 1
        H = st[a][0]                                         # state 0 is what the softmax layer sees
        lsh.decode_step(gc.tables, H, scores[a], gc.topfreq_dev, sp, ws, ob, ow, osc)
        if check:
            torch.cuda.synchronize()
            Hn, bsn = H.cpu().numpy(), scores[a].cpu().numpy()
            for s in range(S):
                ref = gc.oracle_sentence(Hn[s * B:(s + 1) * B], bsn[s * B:(s + 1) * B], B)
                sl = slice(s * B, (s + 1) * B)
                assert_topb_matches(ob.cpu().numpy()[sl], ow.cpu().numpy()[sl], osc.cpu().numpy()[sl], ref,
                                    bsn[sl])
        binding.beam_advance(hist, t, ob, ow, osc, st[a], st[b], scores[b])
        if check:
            torch.cuda.synchronize()
            for s in range(S):
                sl = slice(s * B, (s + 1) * B)
                want, nxt = obeam.advance(ob.cpu().numpy()[sl], ow.cpu().numpy()[sl], osc.cpu().numpy()[sl],
                                          [x.cpu().numpy()[sl] for x in st[a]], eos)
                for k in range(2):
                    assert np.array_equal(st[b][k].cpu().numpy()[sl], want[k])
                assert np.array_equal(scores[b].cpu().numpy()[sl], nxt)
        # stand-in recurrent update (the LSTM layers are not part of this library)
        if t + 1 < steps:
            st[b][0].mul_(0.5).add_(X_dev[t + 1])
        st[b][1].add_(1.0)

    reset()
    for t in range(steps):
        one_step(t, check=True)
    tokens, length, best = binding.beam_backtrace(hist, steps)
    torch.cuda.synchronize()
    eager = [x.cpu().numpy().copy() for x in (tokens, length, best, hist.backptr, hist.words, hist.scores)]
    for s in range(S):
        toks, sc = obeam.backtrace(eager[3][:, s], eager[4][:, s], eager[5][:, s], eos)
        assert eager[1][s] == len(toks) and eager[0][s, :len(toks)].tolist() == toks
        assert eager[2][s] == np.float32(sc)
    assert np.all(eager[1] >= 1)
    # path-length counter carried in state 1: every live slot has been advanced `steps` times
    live = eager[3][steps - 1].reshape(-1) >= 0
    assert np.all(st[steps & 1][1].cpu().numpy()[live] == steps)

    # the same loop captured once and replayed
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        reset()
        for t in range(steps):
            one_step(t, check=False)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        reset()
        for t in range(steps):
            one_step(t, check=False)
        gt, gl, gb = binding.beam_backtrace(hist, steps)
    for _ in range(3):
        hist.backptr.fill_(-5); hist.words.fill_(-5)
        g.replay()
        torch.cuda.synchronize()
        got = [x.cpu().numpy() for x in (gl, gb, hist.backptr, hist.words, hist.scores)]
        for x, y in zip(got, eager[1:]):
            assert np.array_equal(x, y)
        for s in range(S):
            assert np.array_equal(gt.cpu().numpy()[s, :eager[1][s]], eager[0][s, :eager[1][s]])
