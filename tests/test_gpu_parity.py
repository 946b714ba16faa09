"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bit-exact on band codes, bucket contents and candidate lists; log-probabilities and
scores within 1e-5 * max(1, |lp|, |logit|, |lse|) (the magnitudes entering the fp32 subtraction,
see gpu_harness); top-B ids equal except inside score ties (gpu_harness.assert_topb_matches)."""
import numpy as np
import pytest

import oracle
import workloads
from gpu_harness import GpuCase, assert_close_logprobs, assert_topb_matches, to_dev

pytestmark = pytest.mark.gpu

_CASES = {}


def case(name):
    if name not in _CASES:
        _CASES[name] = (workloads.CONFIGS[name], GpuCase.from_config(workloads.CONFIGS[name]))
    return _CASES[name]


def hidden(cfg, gc, steps):
    return workloads.make_hidden(cfg, gc.E, seed=0, steps=steps)


@pytest.fixture
def force():
    """force(gc, name=value, ...): launch-plan options (lsh_set_option) on a case's tables for the
    rest of the test; every option is restored to the library's own rule afterwards."""
    touched = []

    def _force(gc, **opts):
        touched.append(gc)
        gc.tables.set_options(**opts)
    yield _force
    for gc in touched:
        gc.tables.reset_options()


# ---------------------------------------------------------------------------------------------
# build: codes, buckets, cuckoo
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "paper", "widebeam", "largevocab"])
def test_embedding_band_codes_bit_exact(name):
    cfg, gc = case(name)
    got = gc.tables.debug_embedding_codes()                      # every row of E
    assert got.shape == (cfg.V, cfg.W)
    for r0 in range(0, cfg.V, 50000):                            # (the oracle, a slab at a time)
        r1 = min(cfg.V, r0 + 50000)
        want = oracle.band_codes(oracle.wta_codes(gc.E[r0:r1], gc.perms), cfg.W, cfg.K)
        assert np.array_equal(got[r0:r1], want), (r0, r1)


@pytest.mark.parametrize("name", ["tiny", "paper", "widebeam", "largevocab"])
def test_hidden_band_codes_bit_exact(name):
    cfg, gc = case(name)
    H = hidden(cfg, gc, 2).reshape(-1, cfg.d)
    assert np.array_equal(gc.tables.debug_codes(to_dev(H)), gc.index.hidden_band_codes(H))


@pytest.mark.parametrize("name,max_keys", [("tiny", None), ("paper", None), ("widebeam", 300),
                                           ("largevocab", 150)])
def test_buckets_through_cuckoo_bit_exact(name, max_keys):
    cfg, gc = case(name)
    rng = np.random.default_rng(0)
    for w in range(cfg.W):
        okeys = np.sort(gc.index.bucket_keys(w))
        keys, offs, words = gc.tables.debug_csr(w)
        assert np.array_equal(keys, okeys)                       # distinct codes, ascending
        assert offs[0] == 0 and offs[-1] == cfg.V and np.all(np.diff(offs) > 0)
        # the whole flat array, span by span: the oracle's buckets concatenated in key order
        obuckets = [gc.index.bucket(w, int(code)) for code in okeys]
        assert np.array_equal(np.diff(offs), [len(b) for b in obuckets])
        assert np.array_equal(words, np.concatenate(obuckets))
        cap, nk = gc.tables.debug_cuckoo_shape(w)
        assert nk == len(keys) and cap >= 2 * nk and cap & (cap - 1) == 0
        probe = okeys if max_keys is None else rng.choice(okeys, size=min(max_keys, len(okeys)),
                                                          replace=False)
        for code in probe:
            got = gc.tables.debug_bucket(w, int(code))
            assert got is not None and np.array_equal(got, gc.index.bucket(w, int(code)))
            i = np.searchsorted(keys, code)
            assert np.array_equal(words[offs[i]:offs[i + 1]], got)
        present = set(okeys.tolist())
        limit = 1 << (cfg.u * int(np.ceil(np.log2(cfg.K))))
        absent = [c for c in rng.integers(0, limit, size=300).tolist() if c not in present]
        for code in absent[:100]:
            assert gc.tables.debug_bucket(w, code) is None


@pytest.mark.parametrize("env", [{"LSHBEAM_HOST_BUILD": "1"}, {"LSHBEAM_CUCKOO_CHAIN": "4"},
                                 {"LSHBEAM_CUCKOO_CHAIN": "8"}, {"LSHBEAM_CUCKOO_CHAIN": "1"}])
@pytest.mark.parametrize("name", ["tiny", "paper"])
def test_table_build_paths_agree(name, env, monkeypatch):
    # default: sort + parallel cuckoo insertion on the device.  Host build, device build with
    # eviction chains so short that bands must be redone with new hash parameters, and chains of
    # one (any collision fails the band: on the tiny shape the host path takes over after all
    # attempts; on the paper shape multiplicative hashing of 12-bit codes into 2^14 slots happens
    # to be collision-free) must all give the same bucket layout and the same answers through
    # their own cuckoo tables.
    cfg, gc = case(name)
    for k, v in env.items():
        monkeypatch.setenv(k, v)
    other = GpuCase.from_config(cfg)
    assert gc.tables.debug_build_info() == (True, 1)               # load <= 1/3: first attempt
    on_device, attempts = other.tables.debug_build_info()
    if "LSHBEAM_HOST_BUILD" in env:
        assert (on_device, attempts) == (False, 0)
    else:
        # short chains: bands are redone with new hash parameters until all fit (or, after 24
        # rounds, the host takes over)
        assert (on_device and 1 <= attempts <= 24) or (not on_device and attempts == 24)
        print(name, env, "on_device", on_device, "attempts", attempts)
    for w in range(cfg.W):
        k0, o0, w0 = gc.tables.debug_csr(w)
        k1, o1, w1 = other.tables.debug_csr(w)
        assert np.array_equal(k0, k1) and np.array_equal(o0, o1) and np.array_equal(w0, w1)
        for i in range(len(k0)):
            assert np.all(np.diff(w0[o0[i]:o0[i + 1]]) > 0)          # ids ascending inside a span
        cap, nk = other.tables.debug_cuckoo_shape(w)
        assert nk == len(k1) and cap >= 2 * nk and cap & (cap - 1) == 0
        for code in k0[:: max(1, len(k0) // 64)]:
            assert np.array_equal(other.tables.debug_bucket(w, int(code)), w0[o0[np.searchsorted(k0, code)]:
                                                                            o0[np.searchsorted(k0, code) + 1]])
    H = hidden(cfg, gc, 1)[0]
    bs = np.zeros(cfg.R, np.float32)
    a = gc.step(H, bs, cfg.S, cfg.B)
    b = other.step(H, bs, cfg.S, cfg.B)
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x, y)


def test_cuckoo_with_wide_band_codes():
    # 24-bit band codes (K=64, u=4): far too many possible codes for direct addressing
    rng = np.random.default_rng(11)
    V, d, K, P, W = 5000, 96, 64, 8, 2
    E = rng.standard_normal((V, d)).astype(np.float32)
    E[1000:2000] = E[:1000]                                       # force multi-word buckets
    perms = np.stack([rng.permutation(d)[:K] for _ in range(P)]).astype(np.int32)
    gc = GpuCase(E, perms, np.zeros(0, dtype=np.int32), W)
    want = oracle.band_codes(oracle.wta_codes(E, perms), W, K)
    assert want.max() >= 1 << 20
    assert np.array_equal(gc.tables.debug_embedding_codes(), want)
    for w in range(W):
        for code in gc.index.bucket_keys(w):
            assert np.array_equal(gc.tables.debug_bucket(w, int(code)), gc.index.bucket(w, int(code)))
    H = E[[5, 1005, 4000]] * 2.0
    _, _, _, sp, ws = gc.step(H, np.zeros(3, np.float32), 1, 3)
    assert np.array_equal(gc.tables.debug_candidates(ws, sp, 0),
                          gc.index.candidates(H, np.zeros(0, np.int32)))


# ---------------------------------------------------------------------------------------------
# decode step
# ---------------------------------------------------------------------------------------------

def run_and_check(cfg, gc, H, bs, S, B, full_vocab=False, check_lp=True, threshold=1):
    gb, gw, gs, sp, ws = gc.step(H, bs, S, B, full_vocab=full_vocab, threshold=threshold)
    swaps = 0
    for s in range(S):
        Hs, bss = H[s * B:(s + 1) * B], bs[s * B:(s + 1) * B]
        ref = gc.oracle_sentence(Hs, bss, B, full_vocab=full_vocab, threshold=threshold)
        if not full_vocab:
            assert np.array_equal(gc.tables.debug_candidates(ws, sp, s), ref.cand)   # bit-exact list
        if check_lp:
            assert_close_logprobs(gc.tables.debug_logprobs(ws, sp, s, cap=len(ref.cand)), ref)
        swaps += assert_topb_matches(gb[s], gw[s], gs[s], ref, bss)
    return gb, gw, gs, swaps


def test_tiny_all_steps_with_score_feedback():
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, cfg.steps)
    bs = np.zeros(cfg.R, dtype=np.float32)
    for step in range(cfg.steps):
        # each step is checked with the oracle's previous scores fed to both sides (no drift)
        run_and_check(cfg, gc, H[step], bs, cfg.S, cfg.B)
        bs = gc.oracle_sentence(H[step], bs, cfg.B).score.astype(np.float32)


def test_tiny_full_vocab_equals_oracle_brute_force():
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 3)
    rng = np.random.default_rng(1)
    for step in range(3):
        run_and_check(cfg, gc, H[step], rng.standard_normal(cfg.R).astype(np.float32), 1, cfg.B,
                      full_vocab=True)


def test_tiny_many_sentences_and_other_beam_counts():
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)          # 80 rows
    rng = np.random.default_rng(2)
    # few (sentence, 16-row group) pairs -> fused kernel; many -> one wave per tile with 1..4
    # row groups; more than 64 beams -> split-k kernel with several row groups
    H = np.concatenate([H, H[::-1] * 0.5 + 0.1], axis=0)      # 160 rows
    for S, B in [(5, 16), (2, 17), (80, 1), (3, 20), (1, 33), (9, 17), (4, 40), (3, 50), (2, 70)]:
        bs = (rng.standard_normal(S * B) * 2).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B)
    run_and_check(cfg, gc, H[:34], np.zeros(34, np.float32), 2, 17, full_vocab=True)
    run_and_check(cfg, gc, H[:153], np.zeros(153, np.float32), 9, 17, full_vocab=True)


def test_maximum_beam_and_sentence_counts():
    # the largest B (256) and S (4096) the step accepts, and the first values it refuses
    from paper_1806_00588_amd import binding
    cfg, gc = case("tiny")
    base = hidden(cfg, gc, 20).reshape(-1, cfg.d)                 # 80 rows
    rng = np.random.default_rng(256)
    mix = rng.standard_normal((4096, 80)).astype(np.float32) / 4
    H = (mix @ base).astype(np.float32)                           # 4096 rows in the span of the 80
    H[:80] = base
    for S, B in [(1, 256), (2, 256), (1, 128), (3, 100)]:
        bs = (rng.standard_normal(S * B) * 2).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B, check_lp=(S == 1 and B == 128))
    run_and_check(cfg, gc, H[:256], np.zeros(256, np.float32), 1, 256, full_vocab=True, check_lp=False)
    run_and_check(cfg, gc, H[:256], np.zeros(256, np.float32), 1, 256, threshold=2, check_lp=False)
    # 4096 sentences of one beam: every output checked against the oracle for a sample of the
    # sentences, and for all of them that the word is the row's best candidate by the oracle
    S = 4096
    bs = rng.standard_normal(S).astype(np.float32)
    gb, gw, gs, sp, ws = gc.step(H, bs, S, 1)
    assert np.all(gb == 0)
    for s in list(range(0, S, 97)) + [S - 1]:
        ref = gc.oracle_sentence(H[s:s + 1], bs[s:s + 1], 1)
        assert np.array_equal(gc.tables.debug_candidates(ws, sp, s), ref.cand)
        assert_topb_matches(gb[s], gw[s], gs[s], ref, bs[s:s + 1])
    for S_bad, B_bad in [(1, 257), (4097, 1), (0, 4), (4, 0)]:
        assert gc.lsh.step_workspace_bytes(gc.tables, binding.step_params(S_bad, B_bad, 0, 1, False)) == 0


# Shapes between the named configurations, chosen to sit on the launch plans' boundaries (16/17,
# 32/33, 64/65 beams; one, a few and many sentences; 1-, 2- and 4-bit codes; one code per band
# and five; hidden sizes that are tiny, not a multiple of four, or above 1024; bf16 rows; hit
# thresholds), each with every sentence checked in full against the oracle, plan left to the
# library.  (V, d, K, P, W, T, centres, bf16, [(S, B, t), ...])
_SWEEP = [
    (5000, 200, 4, 24, 6, 300, 250, False, [(1, 12, 1), (1, 16, 1), (2, 16, 1), (1, 17, 1), (1, 32, 1),
                                            (1, 33, 1), (1, 48, 1), (1, 64, 1), (1, 65, 1), (6, 12, 1),
                                            (24, 8, 1), (3, 12, 2), (1, 40, 2)]),
    (3000, 6, 2, 20, 4, 0, 40, False, [(1, 5, 1), (7, 3, 1), (1, 70, 1)]),
    (9000, 1001, 3, 12, 12, 128, 300, False, [(1, 12, 1), (2, 33, 1), (12, 6, 1)]),
    (20000, 1000, 8, 30, 6, 700, 500, False, [(1, 12, 1), (3, 12, 1), (1, 50, 1), (1, 12, 3)]),
    (7000, 1500, 16, 8, 2, 64, 200, False, [(1, 8, 1), (2, 36, 1), (9, 9, 1)]),
    (6000, 256, 8, 32, 8, 500, 300, True, [(1, 12, 1), (8, 16, 1), (2, 40, 1), (20, 4, 1), (2, 10, 2)]),
    (4100, 1024, 8, 16, 4, 1000, 100, True, [(1, 16, 1), (5, 24, 1)]),
    # four buckets per band over 37 words: every span is long for its size, the last one ends with
    # the word array, and no span starts on a multiple of four
    (37, 8, 2, 4, 2, 5, 4, False, [(1, 3, 1), (2, 2, 1), (1, 40, 1), (30, 1, 1)]),
]


@pytest.mark.parametrize("shape", _SWEEP, ids=lambda sh: "V%d-d%d-K%d-P%d-W%d-T%d%s" % (
    sh[0], sh[1], sh[2], sh[3], sh[4], sh[5], "-bf16" if sh[7] else ""))
def test_shapes_between_the_named_configurations(shape):
    V, d, K, P, W, T, nc, bf16, runs = shape
    sd = 1.0 / np.sqrt(d)
    cfg = workloads.Config("sweep", d, V, 1, 1, K, P, W, T, nc, sd, 0.3 * sd, 0.8, 0.3 * sd, 1,
                           workloads.BF16 if bf16 else workloads.F32, 0.05)
    gc = GpuCase.from_config(cfg, seed=V + d)
    rng = np.random.default_rng(V * 31 + d)
    for S, B, t in runs:
        import dataclasses
        c = dataclasses.replace(cfg, S=S, B=B)
        H = workloads.make_hidden(c, gc.E, seed=S * 1000 + B, steps=1)[0]
        bs = (rng.standard_normal(S * B) * 1.5).astype(np.float32)
        run_and_check(c, gc, H, bs, S, B, threshold=t)
    S, B, _ = runs[0]
    run_and_check(c, gc, H[:S * B], bs[:S * B], S, B, full_vocab=True, check_lp=V <= 6000)


def test_paper_shape_steps():
    cfg, gc = case("paper")
    H = hidden(cfg, gc, cfg.steps)
    bs = np.zeros(cfg.R, dtype=np.float32)
    for step in range(0, cfg.steps, 5):
        run_and_check(cfg, gc, H[step], bs, cfg.S, cfg.B)
        bs = gc.oracle_sentence(H[step], bs, cfg.B).score.astype(np.float32)


def test_paper_shape_as_the_benchmark_runs_it():
    """The launch configuration bench.py times: a 50-step sentence, steps chained through the
    returned scores, captured once as a HIP graph and replayed; sampled steps are checked
    against the oracle (fed with the scores the GPU itself produced for the previous step)."""
    import torch
    import paper_1806_00588_amd as lsh
    from paper_1806_00588_amd import binding
    cfg, gc = case("paper")
    n = cfg.steps
    H = hidden(cfg, gc, n)
    H_dev = to_dev(H)
    sp = binding.step_params(cfg.S, cfg.B, cfg.T)
    ws = torch.empty(lsh.step_workspace_bytes(gc.tables, sp), dtype=torch.uint8, device="cuda")
    call = binding.make_step_caller(gc.tables, sp, ws, gc.topfreq_dev)
    zero = torch.zeros(cfg.R, device="cuda")
    ob = torch.empty((n, cfg.R), dtype=torch.int32, device="cuda")
    ow = torch.empty((n, cfg.R), dtype=torch.int32, device="cuda")
    osc = torch.empty((n, cfg.R), device="cuda")

    def run(stream):
        for i in range(n):
            prev = zero if i == 0 else osc[i - 1]
            call(H_dev[i].data_ptr(), prev.data_ptr(), ob[i].data_ptr(), ow[i].data_ptr(),
                 osc[i].data_ptr(), stream)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = (ob.clone(), ow.clone(), osc.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        ob.fill_(-9); ow.fill_(-9); osc.fill_(0)
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ob, eager[0]) and torch.equal(ow, eager[1]) and torch.equal(osc, eager[2])
    b, w, sc = ob.cpu().numpy(), ow.cpu().numpy(), osc.cpu().numpy()
    for i in (0, 1, 7, 23, 38, n - 1):
        bs = np.zeros(cfg.R, np.float32) if i == 0 else sc[i - 1]
        ref = gc.oracle_sentence(H[i], bs, cfg.B)
        assert_topb_matches(b[i], w[i], sc[i], ref, bs)


@pytest.mark.parametrize("name,S,B,t", [("paper", 16, 10, 1),     # candidates, wave-per-tile contraction
                                        ("paper", 2, 40, 1),      # parts, union, candidate rows through LDS
                                        ("paper", 1, 24, 1),      # the larger hashing stage, fused
                                        ("paper", 3, 12, 3),      # hit counts, union inside the contraction
                                        ("largevocab", 8, 10, 1)])  # bf16 rows, bf16 planes
def test_other_launch_plans_replayed_as_a_graph(name, S, B, t):
    """Four chained steps of the launch plans the paper shape does not take, captured as one HIP
    graph: three replays (with eager work and synchronisations between them) equal the eager
    run bit for bit, and the eager run's first step matches the oracle."""
    import dataclasses
    import torch
    import paper_1806_00588_amd as lsh
    from paper_1806_00588_amd import binding
    cfg, gc = case(name)
    n = 4
    H = workloads.make_hidden(dataclasses.replace(cfg, S=S, B=B), gc.E, seed=3, steps=n)
    H_dev = to_dev(H)
    R = S * B
    sp = binding.step_params(S, B, gc.topfreq.size, t)
    ws = torch.empty(lsh.step_workspace_bytes(gc.tables, sp), dtype=torch.uint8, device="cuda")
    call = binding.make_step_caller(gc.tables, sp, ws, gc.topfreq_dev)
    zero = torch.zeros(R, device="cuda")
    ob = torch.empty((n, R), dtype=torch.int32, device="cuda")
    ow = torch.empty((n, R), dtype=torch.int32, device="cuda")
    osc = torch.empty((n, R), device="cuda")

    def run(stream):
        for i in range(n):
            prev = zero if i == 0 else osc[i - 1]
            call(H_dev[i].data_ptr(), prev.data_ptr(), ob[i].data_ptr(), ow[i].data_ptr(),
                 osc[i].data_ptr(), stream)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    eager = (ob.clone(), ow.clone(), osc.clone())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        ob.fill_(-9); ow.fill_(-9); osc.fill_(0)
        ws.fill_(0xA5)                                   # eager work between the replays
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(ob, eager[0]) and torch.equal(ow, eager[1]) and torch.equal(osc, eager[2])
    b, w, sc = (x.cpu().numpy().reshape(n, S, B) for x in eager)
    for s in range(min(S, 3)):
        Hs = H[0].reshape(S, B, -1)[s]
        ref = gc.oracle_sentence(Hs, np.zeros(B), B, threshold=t)
        assert_topb_matches(b[0, s], w[0, s], sc[0, s], ref, np.zeros(B))


def test_paper_shape_full_vocab():
    cfg, gc = case("paper")
    H = hidden(cfg, gc, 1)
    run_and_check(cfg, gc, H[0], np.linspace(-3, 0, cfg.R).astype(np.float32), 1, cfg.B,
                  full_vocab=True)


def test_tiny_hit_thresholds():
    """Eq. 10 with t > 1: a word needs t colliding bands with one row; t > W leaves V_T only."""
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    rng = np.random.default_rng(5)
    sizes = {}
    for t in [2, 3, 4, 5]:
        for S, B in [(1, 4), (3, 7), (2, 20)]:
            bs = rng.standard_normal(S * B).astype(np.float32)
            run_and_check(cfg, gc, H[:S * B], bs, S, B, threshold=t)
        sizes[t] = len(gc.index.candidates(H[:4], gc.topfreq, t))
    assert sizes[2] >= sizes[3] >= sizes[4] >= sizes[5]
    assert sizes[5] == len(np.unique(gc.topfreq))          # cfg.W == 4 bands: nothing reaches 5
    # without top-frequent words and out of reach: an empty list, all outputs padded
    gb, gw, gs, sp, ws = gc.step(H[:4], np.zeros(4, np.float32), 1, 4, T=0, threshold=5)
    assert len(gc.tables.debug_candidates(ws, sp, 0)) == 0
    assert np.all(gb == -1) and np.all(gw == -1) and np.all(np.isneginf(gs))


def test_large_vocabulary_hit_threshold():
    # V = 200000 bf16: 16 bands, t = 2..3; the hit counters of a row are spread over four workgroups
    cfg, gc = case("largevocab")
    H = hidden(cfg, gc, 1)[0][:30]
    for t, S, B in [(2, 3, 10), (3, 1, 10)]:
        run_and_check(cfg, gc, H[:S * B], np.zeros(S * B, np.float32), S, B, threshold=t, check_lp=False)
    # K = 16 (windows longer than the eight entries the kernel preloads), V = 100000
    cfg, gc = case("widebeam")
    H = hidden(cfg, gc, 1)[0][:10]
    run_and_check(cfg, gc, H, np.zeros(10, np.float32), 2, 5, threshold=2, check_lp=False)


def test_paper_banding_with_hit_threshold():
    """{K, u, W} = {8, 3, 500} on the Table 1 shape: thousands of hits per row, t selects."""
    cfg, gc = case("paperscale")
    H = hidden(cfg, gc, 3)
    bs = np.zeros(cfg.R, dtype=np.float32)
    for step in range(3):
        run_and_check(cfg, gc, H[step], bs, cfg.S, cfg.B, threshold=cfg.threshold)
        bs = gc.oracle_sentence(H[step], bs, cfg.B, threshold=cfg.threshold).score.astype(np.float32)
    n5 = len(gc.index.candidates(H[0], gc.topfreq, cfg.threshold))
    assert cfg.T < n5 < cfg.V // 4
    run_and_check(cfg, gc, H[1], bs, cfg.S, cfg.B, threshold=2, check_lp=False)
    run_and_check(cfg, gc, H[2], bs, cfg.S, cfg.B, threshold=40)
    # the same tables with t = 1 (500 probes per row through the one-kernel candidate path)
    run_and_check(cfg, gc, H[0], bs, cfg.S, cfg.B, check_lp=False)
    # several sentences
    H3 = np.concatenate([H[0], H[1], H[2]])[:30]
    run_and_check(cfg, gc, H3, np.zeros(30, np.float32), 3, 10, threshold=cfg.threshold, check_lp=False)


def test_batched_shape():
    cfg, gc0 = case("paper")                       # same E / perms / top-freq as the paper shape
    cfg = workloads.CONFIGS["batched"]
    H = workloads.make_hidden(cfg, gc0.E, seed=0, steps=3)
    rng = np.random.default_rng(3)
    # every sentence of two steps in full (candidate lists, log-probabilities, top-B) ...
    for step in (1, 2):
        run_and_check(cfg, gc0, H[step], -rng.random(cfg.R).astype(np.float32), cfg.S, cfg.B)


def test_widebeam_shape():
    cfg, gc = case("widebeam")
    H = hidden(cfg, gc, 2)
    run_and_check(cfg, gc, H[0], np.zeros(cfg.R, np.float32), cfg.S, cfg.B)
    # a second step with spread-out beam scores: candidate lists and top-B of every sentence
    rng = np.random.default_rng(50)
    run_and_check(cfg, gc, H[1], (rng.standard_normal(cfg.R) * 3).astype(np.float32), cfg.S, cfg.B,
                  check_lp=False)


def test_largevocab_bf16_shape():
    cfg, gc = case("largevocab")
    H = hidden(cfg, gc, 1)
    gb, gw, gs, sp, ws = gc.step(H[0], np.zeros(cfg.R, np.float32), cfg.S, cfg.B)
    counts = gc.tables.debug_counts(ws, sp)
    # candidate lists: all 64 sentences, bit for bit (cheap for the oracle)
    for s in range(cfg.S):
        Hs = H[0][s * cfg.B:(s + 1) * cfg.B]
        want = gc.index.candidates(Hs, gc.topfreq)
        assert counts[s] == len(want)
        assert np.array_equal(gc.tables.debug_candidates(ws, sp, s), want), s
    # log-probabilities and top-B: 12 of the 64 sentences (the oracle's fp64 products take time)
    for s in list(range(11)) + [cfg.S - 1]:
        Hs = H[0][s * cfg.B:(s + 1) * cfg.B]
        ref = gc.oracle_sentence(Hs, np.zeros(cfg.B), cfg.B)
        assert_close_logprobs(gc.tables.debug_logprobs(ws, sp, s, cap=len(ref.cand)), ref)
        assert_topb_matches(gb[s], gw[s], gs[s], ref, np.zeros(cfg.B))


@pytest.mark.parametrize("planes", ["1", "0"])
def test_bf16_rows_with_hidden_rows_as_three_bf16_planes(planes, force):
    # bf16 rows, up to 16 beams, many tiles: the hidden rows are staged as hi + mid + lo bf16
    # planes (an exact split of every fp32 value) and contracted with bf16 matrix instructions;
    # option logits_planes = 0 widens the rows to fp32 instead.  Hidden values span 40 binades,
    # with full 24-bit significands, signed zeros and tiny values; d = 264 leaves a last k-step
    # of which only a quarter lies inside the row.
    rng = np.random.default_rng(264)
    V, d, K, P, W = 3000, 264, 8, 16, 4
    E32 = (rng.standard_normal((V, d)) / np.sqrt(d)).astype(np.float32)
    E = workloads.f32_to_bf16_bits(E32)
    perms = np.stack([rng.permutation(d)[:K] for _ in range(P)]).astype(np.int32)
    gc = GpuCase(E, perms, np.arange(100, dtype=np.int32), W)
    force(gc, fused=0, logits_waves=1, logits_planes=int(planes))
    H = rng.standard_normal((64, d)).astype(np.float32)
    H *= np.exp2(rng.integers(-20, 21, size=(64, 1))).astype(np.float32)   # per-row scale
    H[:, ::7] *= np.float32(1.0 + 2.0 ** -23)                               # low significand bits set
    H[3, :40] = 0.0
    H[4, :40] = -0.0
    H[5, 100:140] = 1e-30
    cfg = None
    for S, B in [(3, 10), (2, 16), (5, 1), (2, 20), (4, 7)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B)


# ---------------------------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------------------------

def test_no_topfreq_and_empty_candidate_list():
    cfg, gc = case("tiny")
    from paper_1806_00588_amd import binding
    H = hidden(cfg, gc, 2)
    gb, gw, gs, sp, ws = gc.step(H[0], np.zeros(4, np.float32), 1, 4, T=0)
    ref = gc.oracle_sentence(H[0], np.zeros(4), 4, topfreq=np.zeros(0, np.int32))
    assert np.array_equal(gc.tables.debug_candidates(ws, sp, 0), ref.cand)
    assert_topb_matches(gb[0], gw[0], gs[0], ref, np.zeros(4))
    # a hidden row whose band codes hit no bucket, and no top-freq list: zero candidates
    Hz = np.zeros((1, cfg.d), dtype=np.float32)      # all-tie windows: every code is 0
    codes = gc.index.hidden_band_codes(Hz)[0]
    if all(gc.index.bucket(w, int(codes[w])) is None for w in range(cfg.W)):
        gb, gw, gs, sp, ws = gc.step(Hz, np.zeros(1, np.float32), 1, 1, T=0)
        assert gc.tables.debug_candidates(ws, sp, 0).size == 0
        assert gb[0, 0] == -1 and gw[0, 0] == -1 and np.isneginf(gs[0, 0])


def test_dead_beams_and_padding():
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 1)[0]
    bs = np.array([-np.inf, -1.0, -np.inf, -2.0], dtype=np.float32)
    gb, gw, gs, _ = run_and_check(cfg, gc, H, bs, 1, 4)
    assert set(gb[0].tolist()) <= {1, 3}
    bs[:] = -np.inf
    gb, gw, gs, sp, ws = gc.step(H, bs, 1, 4)
    assert np.all(gb == -1) and np.all(gw == -1) and np.all(np.isneginf(gs))


def test_fewer_candidates_than_beams():
    rng = np.random.default_rng(5)
    V, d = 6, 32
    E = rng.standard_normal((V, d)).astype(np.float32)
    perms = np.stack([rng.permutation(d)[:4] for _ in range(4)]).astype(np.int32)
    gc = GpuCase(E, perms, np.array([0, 3], dtype=np.int32), 2)
    H = rng.standard_normal((3, d)).astype(np.float32)
    cfg = None
    run_and_check(cfg, gc, H, np.zeros(3, np.float32), 1, 3)            # <= 6 candidates, B*C >= B
    run_and_check(cfg, gc, H[:1], np.zeros(1, np.float32), 1, 1)
    # B = 8 beams over at most 6 words with 1 live beam: fewer than B finite pairs -> padded tail
    H8 = rng.standard_normal((8, d)).astype(np.float32)
    bs = np.full(8, -np.inf, dtype=np.float32)
    bs[2] = 0.0
    gb, gw, gs, _ = run_and_check(cfg, gc, H8, bs, 1, 8, full_vocab=True)
    assert (gb[0] >= 0).sum() == 6


def test_all_logits_tie_orders_by_beam_then_word():
    cfg, gc = case("tiny")
    Hz = np.zeros((4, cfg.d), dtype=np.float32)
    gb, gw, gs, sp, ws = gc.step(Hz, np.zeros(4, np.float32), 1, 4)
    cand = gc.index.candidates(Hz, gc.topfreq)
    assert np.array_equal(gc.tables.debug_candidates(ws, sp, 0), cand)
    assert gb[0].tolist() == [0, 0, 0, 0] and gw[0].tolist() == cand[:4].tolist()
    np.testing.assert_allclose(gs[0], -np.log(len(cand)), rtol=1e-6)
    # all 1000 words tie in full-vocabulary mode: far more ties than the short list of the
    # selection holds, so its exact radix fallback decides
    gb, gw, gs, sp, ws = gc.step(Hz, np.array([0, 0, 1, 0], np.float32), 1, 4, full_vocab=True)
    assert gb[0].tolist() == [2, 2, 2, 2] and gw[0].tolist() == [0, 1, 2, 3]
    np.testing.assert_allclose(gs[0], 1 - np.log(cfg.V), rtol=1e-6)
    gb, gw, gs, sp, ws = gc.step(Hz, np.zeros(4, np.float32), 1, 4, full_vocab=True)
    assert gb[0].tolist() == [0, 0, 0, 0] and gw[0].tolist() == [0, 1, 2, 3]


def test_many_beams_ties_dead_beams_and_padding():
    # 33..64 beams take the contraction that leaves one tile record per group of tiles and the
    # selection that reads them 16 lanes per row: its degenerate inputs
    cfg, gc = case("tiny")
    B = 40
    rng = np.random.default_rng(40)
    Hz = np.zeros((2 * B, cfg.d), dtype=np.float32)
    # every score of a sentence ties: more qualifying tiles than the selection lists, the exact
    # radix select decides: lowest beam first, then lowest word
    bs = np.zeros(2 * B, np.float32)
    bs[B + 7] = 1.0                                   # second sentence: one beam ahead of the rest
    gb, gw, gs, sp, ws = gc.step(Hz, bs, 2, B)
    cand = gc.index.candidates(Hz[:B], gc.topfreq)
    assert np.array_equal(gc.tables.debug_candidates(ws, sp, 0), cand) and len(cand) >= B
    assert gb[0].tolist() == [0] * B and gw[0].tolist() == cand[:B].tolist()
    assert gb[1].tolist() == [7] * B and gw[1].tolist() == cand[:B].tolist()
    np.testing.assert_allclose(gs[0], -np.log(len(cand)), rtol=1e-6)
    np.testing.assert_allclose(gs[1], 1 - np.log(len(cand)), rtol=1e-6)
    # two live beams among 40, then none
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)[:B]
    bs = np.full(B, -np.inf, dtype=np.float32)
    bs[3], bs[38] = -0.5, 0.25
    gb, gw, gs, _ = run_and_check(cfg, gc, H, bs, 1, B)
    assert set(gb[0].tolist()) <= {3, 38}
    bs[:] = -np.inf
    gb, gw, gs, sp, ws = gc.step(H, bs, 1, B)
    assert np.all(gb == -1) and np.all(gw == -1) and np.all(np.isneginf(gs))
    # fewer finite pairs than beams: one live beam, no LSH hits, five top-frequent words
    bs[11] = 0.0
    gb, gw, gs, sp, ws = gc.step(H, bs, 1, B, T=5, threshold=cfg.W + 1)
    assert (gb[0] >= 0).sum() == 5 and np.all(gb[0][:5] == 11) and np.all(gb[0][5:] == -1)
    assert sorted(gw[0][:5].tolist()) == sorted(gc.topfreq[:5].tolist()) and np.all(np.isneginf(gs[0][5:]))


def test_topfreq_out_of_range_ids_and_duplicates_are_harmless():
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 1)[0]
    tf = np.array([3, 3, -5, cfg.V, cfg.V + 100, 999, 0, 3], dtype=np.int32)
    gb, gw, gs, sp, ws = gc.step(H, np.zeros(4, np.float32), 1, 4, T=len(tf), topfreq_dev=to_dev(tf))
    want = gc.index.candidates(H, np.array([0, 3, 999], dtype=np.int32))
    assert np.array_equal(gc.tables.debug_candidates(ws, sp, 0), want)


def test_unaligned_hidden_size_uses_scalar_loads():
    rng = np.random.default_rng(9)
    for d, V, dt in [(50, 333, np.float32), (77, 200, np.float32), (52, 300, np.uint16)]:
        E = rng.standard_normal((V, d)).astype(np.float32)
        if dt == np.uint16:
            E = workloads.f32_to_bf16_bits(E)
        perms = np.stack([rng.permutation(d)[:8] for _ in range(8)]).astype(np.int32)
        gc = GpuCase(E, perms, np.arange(20, dtype=np.int32), 2)
        H = rng.standard_normal((2 * 5, d)).astype(np.float32)
        run_and_check(None, gc, H, rng.standard_normal(10).astype(np.float32), 2, 5)
        run_and_check(None, gc, H, np.zeros(10, np.float32), 2, 5, full_vocab=True)


@pytest.mark.parametrize("pad,off,bf16", [(8, 0, False), (3, 0, False), (4, 1, False), (0, 4, False),
                                          (16, 0, True), (5, 3, True)])
def test_pitched_and_offset_embedding_rows(pad, off, bf16):
    # E handed over as a view [:, off : off + d] of a wider matrix: row pitch d + pad + off, base
    # pointer off elements into an allocation.  Pitches and offsets that keep 16-byte alignment
    # take the vector loads, the others the element-wise path; all agree with the oracle.
    import torch
    rng = np.random.default_rng(pad * 16 + off)
    V, d, K, P, W = 1200, 96, 8, 16, 4
    E = (rng.standard_normal((V, d)) / np.sqrt(d)).astype(np.float32)
    if bf16:
        E = workloads.f32_to_bf16_bits(E)
    wide = np.zeros((V, d + pad + off), dtype=E.dtype)
    wide[:] = 77 if bf16 else 1e30                 # what lies between the rows must never be read as data
    wide[:, off:off + d] = E
    wide_dev = to_dev(wide)
    E_dev = wide_dev[:, off:off + d]
    assert int(E_dev.stride(0)) == d + pad + off and not E_dev.is_contiguous() or pad + off == 0
    perms = np.stack([rng.permutation(d)[:K] for _ in range(P)]).astype(np.int32)
    gc = GpuCase(E, perms, np.arange(60, dtype=np.int32), W, E_dev=E_dev)
    want = oracle.band_codes(oracle.wta_codes(E, perms), W, K)
    assert np.array_equal(gc.tables.debug_embedding_codes(), want)
    H = rng.standard_normal((64, d)).astype(np.float32)
    for S, B in [(1, 4), (2, 12), (1, 40), (16, 4)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(None, gc, H[:S * B], bs, S, B)
    run_and_check(None, gc, H[:8], np.zeros(8, np.float32), 2, 4, full_vocab=True)
    run_and_check(None, gc, H[:8], np.zeros(8, np.float32), 2, 4, threshold=2)


@pytest.mark.parametrize("name", ["tiny", "paper"])
def test_hidden_rows_not_16_byte_aligned(name):
    # H starting 4 (12) bytes into its allocation: no 16-byte loads of hidden rows anywhere
    cfg, gc = case(name)
    H = hidden(cfg, gc, 4).reshape(-1, cfg.d)
    rng = np.random.default_rng(4)
    for S, B, t in [(1, cfg.B, 1), (3, 4, 1), (1, 40, 1), (2, 3, 2)]:
        if S * B > len(H):
            continue
        bs = rng.standard_normal(S * B).astype(np.float32)
        gb, gw, gs, sp, ws = gc.step(H[:S * B], bs, S, B, threshold=t, h_misalign=1)
        for s in range(S):
            ref = gc.oracle_sentence(H[s * B:(s + 1) * B], bs[s * B:(s + 1) * B], B, threshold=t)
            assert np.array_equal(gc.tables.debug_candidates(ws, sp, s), ref.cand)
            assert_topb_matches(gb[s], gw[s], gs[s], ref, bs[s * B:(s + 1) * B])
    gb, gw, gs, sp, ws = gc.step(H[:8], np.zeros(8, np.float32), 2, 4, full_vocab=True, h_misalign=3)
    for s in range(2):
        ref = gc.oracle_sentence(H[s * 4:(s + 1) * 4], np.zeros(4), 4, full_vocab=True)
        assert_topb_matches(gb[s], gw[s], gs[s], ref, np.zeros(4))


def test_step_is_deterministic():
    cfg, gc = case("paper")
    H = hidden(cfg, gc, 1)[0]
    a = gc.step(H, np.zeros(cfg.R, np.float32), 1, cfg.B)
    ca = gc.tables.debug_candidates(a[4], a[3], 0)
    la = gc.tables.debug_logprobs(a[4], a[3], 0, cap=len(ca))
    b = gc.step(H, np.zeros(cfg.R, np.float32), 1, cfg.B)
    cb = gc.tables.debug_candidates(b[4], b[3], 0)
    lb = gc.tables.debug_logprobs(b[4], b[3], 0, cap=len(cb))
    assert np.array_equal(ca, cb) and np.array_equal(la, lb)
    for x, y in zip(a[:3], b[:3]):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("name,S,B,t", [("paper", 1, 12, 1), ("tiny", 2, 4, 1), ("tiny", 1, 20, 1),
                                        ("tiny", 2, 4, 2), ("paperscale", 1, 12, 5),
                                        ("paper", 1, 30, 1), ("paper", 4, 12, 1), ("tiny", 8, 16, 1)])
def test_one_launch_two_launch_and_three_kernel_plans_agree_bit_for_bit(name, S, B, t, force):
    # few sentences: candidates are regenerated inside the logits kernel, whose last workgroup per
    # sentence also runs the selection (one launch).  Option one_launch = 0 ends the step with a
    # selection kernel instead; option fused = 0 forces the general three-kernel path.  Same
    # arithmetic, same order: every output must be identical.
    from paper_1806_00588_amd import binding
    cfg, gc = case(name)
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    if len(H) < S * B:
        H = np.concatenate([H, H[::-1] * 0.5 + 0.1], axis=0)
    H = H[:S * B]
    bs = np.linspace(-1, 0, S * B).astype(np.float32)
    res = {}
    # (the "narrow" runs cut the list into tiles of 7 instead of 16: the per-tile softmax partials
    # are then summed in other groups, so they are compared with each other and with the oracle)
    for mode, opts in (("one", dict(fused=1, one_launch=1)), ("two", dict(fused=1, one_launch=0)),
                       ("three", dict(fused=0)), ("one-narrow", dict(fused=1, one_launch=1, fused_tile=7)),
                       ("two-narrow", dict(fused=1, one_launch=0, fused_tile=7))):
        gc.tables.reset_options()
        force(gc, **opts)
        gc.tables.profile_begin(4)
        gb, gw, gs, sp, ws = gc.step(H, bs, S, B, threshold=t)
        launches = {k: n for k, (_, n) in gc.tables.profile_end().items()}
        assert binding.step_is_fused(gc.tables, sp) == (mode != "three")
        assert launches["k_select"] == (0 if mode.startswith("one") else 1), (mode, launches)
        if mode.endswith("narrow"):
            for s_ in range(S):
                ref = gc.oracle_sentence(H[s_ * B:(s_ + 1) * B], bs[s_ * B:(s_ + 1) * B], B, threshold=t)
                assert_topb_matches(gb[s_], gw[s_], gs[s_], ref, bs[s_ * B:(s_ + 1) * B])
        cands = [gc.tables.debug_candidates(ws, sp, s) for s in range(S)]
        lps = [gc.tables.debug_logprobs(ws, sp, s, cap=len(cands[s])) for s in range(S)]
        res[mode] = (gb, gw, gs, cands, lps)
    for a, other in (("one", "two"), ("one", "three"), ("one-narrow", "two-narrow")):
        for x, y in zip(res[a][:3], res[other][:3]):
            assert np.array_equal(x, y), other
        for s in range(S):
            assert np.array_equal(res[a][3][s], res[other][3][s])
            assert np.array_equal(res[a][4][s], res[other][4][s])
    for s in range(S):
        assert np.array_equal(res["one"][3][s], gc.index.candidates(H[s * B:(s + 1) * B], gc.topfreq, t))


@pytest.mark.parametrize("width", [1, 2, 3, 5, 9, 13, 16])
def test_fused_kernel_with_every_tile_width(width, force):
    # option fused_tile makes the fused kernels cut the candidate list into tiles narrower than the
    # 16 columns of the matrix instruction.  Lists that are not a multiple of the
    # width, one and several tiles per workgroup (small grids), one and two row groups.
    cfg, gc = case("tiny")
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    rng = np.random.default_rng(width)
    for grid in (256, 8, 3):
        for one_launch in (0, 1):
            force(gc, fused=1, fused_tile=width, fused_grid=grid, one_launch=one_launch)
            for S, B in [(1, 4), (2, 12), (1, 20), (3, 5)]:
                bs = rng.standard_normal(S * B).astype(np.float32)
                run_and_check(cfg, gc, H[:S * B], bs, S, B)
    cfg, gc = case("paper")
    force(gc, fused=1, fused_tile=width)
    H = hidden(cfg, gc, 2)
    run_and_check(cfg, gc, H[1], np.linspace(-2, 0, cfg.R).astype(np.float32), cfg.S, cfg.B)


@pytest.mark.parametrize("V", [640, 6400])
@pytest.mark.parametrize("one_launch", [1, 0])
def test_winners_that_share_a_tile(one_launch, V, force):
    # The selection of the fused plans works from per-tile records (largest and second largest
    # logit of each row and tile) and must notice when a tile hides a third winner.  Here the
    # candidate list is all of V in id order (every id is "top-frequent"), so tile = id / 16, and
    # the words of one tile are near copies of the hidden direction: for the dominant beam all B
    # winners sit in that one tile; other steps put two winners into one tile, or one per tile.
    # (40 tiles, or 400: the selection's code for four, or for eight, records per lane)
    rng = np.random.default_rng(16)
    d, K, P, W = 32, 4, 8, 2
    E = rng.standard_normal((V, d)).astype(np.float32)
    base = rng.standard_normal(d).astype(np.float32)
    for k in range(16):
        E[96 + k] = base * np.float32(1.0 - 0.01 * k)          # tile 6: scores fall slowly with k
    E[200] = base * np.float32(0.97)                             # lone near-winners in other tiles
    E[333] = base * np.float32(0.955)
    perms = np.stack([rng.permutation(d)[:K] for _ in range(P)]).astype(np.int32)
    gc = GpuCase(E, perms, np.arange(V, dtype=np.int32), W)
    force(gc, fused=1, one_launch=one_launch)
    for B in (4, 6, 12, 16, 20):
        H = rng.standard_normal((B, d)).astype(np.float32) * 0.05
        H[0] += base * 3.0
        if B > 4:
            H[3] += base * 2.9
        for bs0 in (0.0, -50.0):
            bs = np.full(B, -60.0, np.float32)
            bs[0] = 0.0
            if B > 4:
                bs[3] = bs0
            gb, gw, gs, swaps = run_and_check(None, gc, H, bs, 1, B)
            assert swaps == 0
            assert gb[0, 0] == 0 and gw[0, 0] == 96
        # and with every beam alive: winners spread over rows
        run_and_check(None, gc, H, np.zeros(B, np.float32), 1, B)


@pytest.mark.parametrize("part_rows", [1, 3, 5])
def test_sentence_hashed_in_parts(part_rows, force):
    # sentences with many beams are hashed by several workgroups, each leaving a bitmap that the
    # consumer ORs; option part_rows forces small parts so that the tiny shape takes this plan
    cfg, gc = case("tiny")
    force(gc, part_rows=part_rows)
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    H = np.concatenate([H, H[::-1] * 0.5 + 0.1], axis=0)
    rng = np.random.default_rng(part_rows)
    for S, B in [(1, 4), (2, 17), (9, 17), (1, 40), (3, 20)]:      # fused and separate plans
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B)
    gb, gw, gs, sp, ws = gc.step(H[:8], np.zeros(8, np.float32), 2, 4, T=0)
    for s in range(2):
        assert np.array_equal(gc.tables.debug_candidates(ws, sp, s),
                              gc.index.candidates(H[4 * s:4 * s + 4], gc.topfreq[:0]))


def test_paper_shape_wide_beams():
    # the beam sizes of Table 8: more rows than one chunk of hashing holds
    cfg, gc = case("paper")
    H = hidden(cfg, gc, 8).reshape(-1, cfg.d)                     # 96 rows
    rng = np.random.default_rng(8)
    for S, B in [(1, 24), (1, 48), (2, 36), (3, 30)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B, check_lp=(B == 24))


@pytest.mark.parametrize("hlds,rows", [("0", "0"), ("1", "0"), ("1", "32"), ("1", "16")])
def test_contraction_with_hidden_rows_in_lds_or_in_global_memory(hlds, rows, force):
    # many-tile steps stage the sentence's hidden rows in LDS (more than 32 beams: in groups of 16
    # rows, a workgroup each; option hlds_rows forces a group size); option logits_hlds = 0 reads
    # them from global memory
    cfg, gc = case("tiny")
    force(gc, fused=0, logits_waves=1, logits_hlds=int(hlds), hlds_rows=int(rows))
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    H = np.concatenate([H, H[::-1] * 0.5 + 0.1], axis=0)
    rng = np.random.default_rng(3)
    for grid in ("1", "3", "512"):
        force(gc, logits_grid=int(grid))
        for S, B in [(5, 16), (2, 17), (3, 40), (2, 70), (1, 33), (7, 4)]:
            bs = rng.standard_normal(S * B).astype(np.float32)
            run_and_check(cfg, gc, H[:S * B], bs, S, B)
    run_and_check(cfg, gc, H[:80], np.zeros(80, np.float32), 2, 40, full_vocab=True)


@pytest.mark.parametrize("union", ["inside", "before"])
@pytest.mark.parametrize("grid", ["256", "4", "1"])
def test_contraction_with_hidden_rows_in_registers_and_candidate_rows_through_lds(grid, union, force):
    # 33..64 beams, fp32 rows: the workgroup keeps the hidden rows in registers and double-buffers
    # the tiles' candidate rows through LDS.  Small grids give a workgroup many tiles (both
    # buffers in use, the last tile ragged); d = 1000 leaves 24 zeroed pad columns, d = 64 leaves 960.
    # Sentences this wide are hashed in parts; the kernel ORs the parts' bitmaps and makes the
    # candidate list itself (more than 16 tiles per workgroup: ids read back from the list), or
    # option estage_union = 0 puts a union kernel before it.  One record per row and workgroup
    # for the selection either way.
    cfg, gc = case("paper")
    force(gc, logits_grid=int(grid), estage_union=int(union == "inside"))
    H = hidden(cfg, gc, 12).reshape(-1, cfg.d)                    # 144 rows
    rng = np.random.default_rng(int(grid))
    for S, B in [(2, 50), (1, 33), (2, 64), (3, 48)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B, check_lp=(B == 33))
    if union == "inside":   # all of V: 2500 tiles, many groups of records per workgroup
        run_and_check(cfg, gc, H[:80], rng.standard_normal(80).astype(np.float32), 2, 40, full_vocab=True,
                      check_lp=False)
    cfg, gc = case("tiny")
    force(gc, logits_grid=int(grid), estage_union=int(union == "inside"))
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    H = np.concatenate([H, H[::-1] * 0.5 + 0.1, H * 0.25 - 0.1], axis=0)
    for S, B in [(3, 40), (2, 64), (1, 33), (4, 49)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B)
    run_and_check(cfg, gc, H[:80], np.zeros(80, np.float32), 2, 40, full_vocab=True)
    # no candidates at all (no top-frequent words, threshold above the number of bands)
    gb, gw, gs, sp, ws = gc.step(H[:80], np.zeros(80, np.float32), 2, 40, T=0, threshold=cfg.W + 1)
    assert gc.tables.debug_candidates(ws, sp, 1).size == 0
    assert np.all(gb == -1) and np.all(gw == -1) and np.all(np.isneginf(gs))


@pytest.mark.parametrize("rem", ["4", "0"])
@pytest.mark.parametrize("grid", [1, 2, 3, 5, 8, 16])
def test_wave_kernel_remainder_tiles_split_over_workgroups(grid, rem, force):
    # one wave per tile for whole rounds of the (here artificially small) grid; a short last
    # round (at most a quarter of the waves; option hlds_rem = 0: any) is dealt to whole
    # workgroups that split k.  Every grid size moves the boundary.
    cfg, gc = case("tiny")
    force(gc, fused=0, logits_waves=1, hlds_rem=int(rem), logits_grid=grid)
    H = hidden(cfg, gc, 20).reshape(-1, cfg.d)
    rng = np.random.default_rng(grid)
    for S, B in [(3, 4), (2, 20), (1, 40), (4, 7)]:
        bs = rng.standard_normal(S * B).astype(np.float32)
        run_and_check(cfg, gc, H[:S * B], bs, S, B)
    run_and_check(cfg, gc, H[:8], np.zeros(8, np.float32), 2, 4, full_vocab=True)


def test_argument_validation_returns_codes_and_leaves_outputs_untouched():
    import torch
    import paper_1806_00588_amd as lsh
    from paper_1806_00588_amd import binding
    cfg, gc = case("tiny")
    H = to_dev(hidden(cfg, gc, 1)[0])
    bs = torch.zeros(4, device="cuda")
    ob = torch.full((1, 4), 42, dtype=torch.int32, device="cuda")
    ow = ob.clone()
    osc = torch.full((1, 4), 42.0, device="cuda")
    sp = binding.step_params(1, 4, 50)
    ws = torch.empty(lsh.step_workspace_bytes(gc.tables, sp), dtype=torch.uint8, device="cuda")
    with pytest.raises(lsh.LshBeamError) as e:
        lsh.decode_step(gc.tables, H, bs, gc.topfreq_dev, binding.step_params(1, 4, 50, threshold=0),
                        ws, ob, ow, osc)
    assert e.value.status == 1                                  # t < 1
    with pytest.raises(lsh.LshBeamError) as e:
        lsh.decode_step(gc.tables, H, bs, gc.topfreq_dev, sp, ws[:1024], ob, ow, osc)
    assert e.value.status == 6                                  # workspace too small
    with pytest.raises(lsh.LshBeamError) as e:
        lsh.decode_step(gc.tables, H, bs, None, sp, ws, ob, ow, osc)
    assert e.value.status == 1                                  # T > 0 without a list
    torch.cuda.synchronize()
    assert torch.all(ob == 42) and torch.all(ow == 42) and torch.all(osc == 42.0)
    assert lsh.step_workspace_bytes(gc.tables, binding.step_params(0, 4, 0)) == 0
    assert lsh.step_workspace_bytes(gc.tables, binding.step_params(1, 257, 0)) == 0
    # t > 1 keeps a quarter of V as 16-bit hit counters in LDS: 400000 words do not fit
    rng = np.random.default_rng(0)
    Eb = to_dev(rng.standard_normal((400000, 16)).astype(np.float32))
    pb = to_dev(np.stack([rng.permutation(16)[:4] for _ in range(4)]).astype(np.int32))
    big = lsh.build_tables(Eb, pb, 4, 2)
    Hb = torch.zeros(3, 16, device="cuda")
    spb = binding.step_params(1, 3, 0, threshold=2)
    wsb = torch.empty(lsh.step_workspace_bytes(big, spb), dtype=torch.uint8, device="cuda")
    with pytest.raises(lsh.LshBeamError) as e:
        lsh.decode_step(big, Hb, torch.zeros(3, device="cuda"), None, spb, wsb,
                        torch.zeros(1, 3, dtype=torch.int32, device="cuda"),
                        torch.zeros(1, 3, dtype=torch.int32, device="cuda"),
                        torch.zeros(1, 3, device="cuda"))
    assert e.value.status == 2
    # build-time validation
    for K, W in [(1, 4), (8, 3), (8, 0), (8, 1)]:          # (8, 1): u * bits = 48 > 30
        with pytest.raises(lsh.LshBeamError):
            lsh.build_tables(gc.E_dev, gc.perms_dev[:, :K].contiguous(), K, W)
    bad = gc.perms_dev.clone()
    bad[0, 0] = cfg.d
    with pytest.raises(lsh.LshBeamError):
        lsh.build_tables(gc.E_dev, bad, cfg.K, cfg.W)
