"""The recall/speedup sweep (stand-in for Figs. 6-8 and Tables 7-8) runs on the HIP path; its
three figures -- recall@B against the full-vocabulary step, top-1 agreement, mean |V_LSH| -- are
checked here against the same figures computed by the CPU oracle on the same inputs, and against
two limits that hold by construction."""
import dataclasses

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


def _inputs(cfg, B, T, S, steps):
    c = dataclasses.replace(cfg, S=S, B=B, T=T)
    E = workloads.make_embeddings(cfg, 0)
    return E, workloads.make_hidden(c, E, seed=0, steps=steps), workloads.make_topfreq(c)


@pytest.fixture(scope="module")
def tiny():
    from paper_1806_00588_amd import sweep
    cfg = workloads.CONFIGS["tiny"]
    E = workloads.make_embeddings(cfg, 0)
    perms = workloads.make_perms(cfg, 0)
    return cfg, E, perms, sweep.Sweeper(E, perms, cfg.W), oracle.Index(E, perms, cfg.W)


@pytest.mark.parametrize("B,T,t,S", [(4, 50, 1, 1), (4, 50, 1, 2), (4, 0, 1, 1), (4, 50, 2, 1),
                                     (12, 20, 1, 1), (4, 50, 3, 3)])
def test_sweep_figures_equal_the_oracles(tiny, B, T, t, S):
    """recall@B, top-1 and mean |V_LSH| from oracle.Index.decode_step (LSH list against the list
    forced to all of V) on the same hidden states, beam scores and top-frequent list.  The
    id sets may differ only where the oracle's own scores tie within the fp32 tolerance; on these
    inputs they do not, so the figures must be equal."""
    from paper_1806_00588_amd import sweep
    cfg, E, perms, sw, ix = tiny
    steps = 6
    _, H, tf = _inputs(cfg, B, T, S, steps)
    got = sw.measure(H, tf, B, t, S=S, time_it=False)
    bs = sweep.beam_scores_for(S * B, 0)
    lb, lw, fb, fw, counts = [], [], [], [], []
    for i in range(steps):
        b1, w1, _, cnt = ix.decode_step(H[i], bs, tf, S, B, t=t)
        b2, w2, _, _ = ix.decode_step(H[i], bs, tf, S, B, t=t, full_vocab=True)
        lb.append(b1); lw.append(w1); fb.append(b2); fw.append(w2)
        counts += list(np.asarray(cnt).reshape(-1))
    recall, top1 = sweep.recall_stats(np.stack(lb).reshape(steps, S, B), np.stack(lw).reshape(steps, S, B),
                                      np.stack(fb).reshape(steps, S, B), np.stack(fw).reshape(steps, S, B))
    assert got["mean_candidates"] == round(float(np.mean(counts)), 1)
    assert got["recall_at_B"] == round(recall, 4)
    assert got["top1"] == round(top1, 4)
    # and the HIP results themselves are the oracle's, pair for pair
    assert np.array_equal(got["lsh_results"][0], np.stack(lb).reshape(steps, S, B))
    assert np.array_equal(got["lsh_results"][1], np.stack(lw).reshape(steps, S, B))
    assert np.array_equal(got["full_results"][0], np.stack(fb).reshape(steps, S, B))
    assert np.array_equal(got["full_results"][1], np.stack(fw).reshape(steps, S, B))


def test_sweep_limits_on_the_tiny_shape(tiny):
    from paper_1806_00588_amd import sweep
    cfg, E, perms, sw, ix = tiny
    _, H, tf_all = _inputs(cfg, 4, cfg.V, 1, 5)
    everything = sw.measure(H, tf_all, 4, 1)
    assert everything["recall_at_B"] == 1.0 and everything["top1"] == 1.0
    assert everything["mean_candidates"] == cfg.V
    _, H, tf = _inputs(cfg, 4, 50, 1, 5)
    top_only = sw.measure(H, tf, 4, cfg.W + 1)
    assert top_only["mean_candidates"] == 50.0
    _, H2, _ = _inputs(cfg, 4, 50, 2, 5)
    lsh = sw.measure(H2, tf, 4, 1, S=2)
    assert 50 <= lsh["mean_candidates"] <= cfg.V and 0.0 <= lsh["recall_at_B"] <= 1.0
    assert lsh["lsh_us"] > 0 and lsh["full_us"] > 0
    assert sweep.default_settings(dataclasses.replace(cfg, W=32))[4][2] == 2   # t sweep needs bands
