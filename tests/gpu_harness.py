"""Shared plumbing of the GPU parity tests: upload synthetic inputs, run the HIP path through the
C ABI, run the CPU oracle on the same bytes, and compare under the stated tolerances."""
from __future__ import annotations

import numpy as np

import oracle
import workloads

import collections

# |gpu - oracle| <= TOL * max(1, magnitudes entering the result).  A log-probability is the
# difference logit - lse of two fp32 numbers; when they nearly cancel, the error is set by THEIR
# size (one ulp of 80.0 is 7.6e-6), so the bound scales with max(|lp|, |logit|, |lse|).
TOL_F32 = 1e-5

Ref = collections.namedtuple("Ref", "cand lp logits beam word score")


def to_dev(a: np.ndarray):
    import torch
    if a.dtype == np.uint16:                     # bf16 bit patterns travel as int16
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class GpuCase:
    """Inputs of one configuration resident on the device + tables + the oracle index."""

    def __init__(self, E, perms, topfreq, W, seed=0, E_dev=None):
        """E_dev: the device tensor to hand to the library instead of a plain upload of E (a
        pitched or offset view holding the same values)."""
        import torch
        import paper_1806_00588_amd as lsh
        self.lsh = lsh
        self.torch = torch
        self.E, self.perms, self.topfreq = E, perms, np.ascontiguousarray(topfreq, dtype=np.int32)
        self.V, self.d = E.shape
        self.P, self.K = perms.shape
        self.W = W
        self.E_dev = to_dev(E) if E_dev is None else E_dev
        self.perms_dev = to_dev(perms)
        self.topfreq_dev = to_dev(self.topfreq) if self.topfreq.size else None
        self.tables = lsh.build_tables(self.E_dev, self.perms_dev, self.K, W, seed=seed)
        self.index = oracle.Index(E, perms, W)
        self._ws = {}

    @classmethod
    def from_config(cls, cfg: workloads.Config, seed=0):
        return cls(workloads.make_embeddings(cfg, seed), workloads.make_perms(cfg, seed),
                   workloads.make_topfreq(cfg), cfg.W, seed)

    def step(self, H: np.ndarray, beam_scores: np.ndarray, S: int, B: int, full_vocab=False,
             T=None, topfreq_dev=None, threshold=1, h_misalign=0):
        """One lsh_decode_step; returns (beam, word, score) numpy [S,B] plus (sp, workspace).
        h_misalign: the hidden rows start that many floats into their allocation."""
        from paper_1806_00588_amd import binding
        torch = self.torch
        T = self.topfreq.size if T is None else T
        sp = binding.step_params(S, B, T, threshold, full_vocab)
        nbytes = self.lsh.step_workspace_bytes(self.tables, sp)
        assert nbytes > 0
        key = (S, B, bool(full_vocab), threshold > 1)
        if key not in self._ws or self._ws[key].numel() < nbytes:
            self._ws[key] = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        ws = self._ws[key]
        H_dev = to_dev(np.ascontiguousarray(H, dtype=np.float32))
        if h_misalign:
            buf = torch.zeros(H_dev.numel() + h_misalign, dtype=torch.float32, device="cuda")
            buf[h_misalign:] = H_dev.reshape(-1)
            H_dev = buf[h_misalign:].view(H_dev.shape)
        bs_dev = to_dev(np.ascontiguousarray(beam_scores, dtype=np.float32))
        ob = torch.full((S, B), -7, dtype=torch.int32, device="cuda")
        ow = torch.full((S, B), -7, dtype=torch.int32, device="cuda")
        osc = torch.full((S, B), 123.0, dtype=torch.float32, device="cuda")
        tf = self.topfreq_dev if topfreq_dev is None else topfreq_dev
        self.lsh.decode_step(self.tables, H_dev, bs_dev, tf, sp, ws, ob, ow, osc)
        torch.cuda.synchronize()
        return ob.cpu().numpy(), ow.cpu().numpy(), osc.cpu().numpy(), sp, ws

    def oracle_sentence(self, Hs, bs, B, full_vocab=False, topfreq=None, threshold=1):
        """Oracle for one sentence: Ref(cand, lp fp64 [B,C], logits fp64 [B,C], beam, word, score)."""
        tf = self.topfreq if topfreq is None else topfreq
        cand = np.arange(self.V, dtype=np.int32) if full_vocab else self.index.candidates(Hs, tf, threshold)
        lp, lg = self.index.logprobs(Hs, cand, want_logits=True)
        ob, ow, osc = oracle.topb(np.asarray(bs, dtype=np.float64), lp, cand, B)
        return Ref(cand, lp, lg, ob, ow, osc)


def logprob_bound(ref: Ref, tol=TOL_F32) -> np.ndarray:
    lse = ref.logits - ref.lp
    return tol * np.maximum.reduce([np.ones_like(ref.lp), np.abs(ref.lp), np.abs(ref.logits),
                                    np.abs(lse)])


def assert_close_logprobs(got: np.ndarray, ref: Ref, tol=TOL_F32):
    err = np.abs(got.astype(np.float64) - ref.lp)
    bound = logprob_bound(ref, tol)
    worst = np.unravel_index(np.argmax(err - bound), err.shape)
    assert np.all(err <= bound), f"log-prob error {err[worst]:.3e} > bound {bound[worst]:.3e} at {worst}"


def assert_topb_matches(gb, gw, gs, ref: Ref, bs, tol=TOL_F32):
    """GPU top-B (gb, gw, gs) against the oracle's for one sentence.

    Scores must agree position by position.  Ids must agree wherever the oracle's ranking is
    unique beyond the tolerance; inside a group of scores tied within tolerance any member of the
    group is valid, so there the check is: a real (beam, candidate) pair, no duplicates, and the
    oracle's own score for that pair equals the reported score within tolerance."""
    cand, lp, ob, ow, osc = ref.cand, ref.lp, ref.beam, ref.word, ref.score
    lpb = logprob_bound(ref, tol)
    bs = np.asarray(bs, dtype=np.float64)
    n_valid = int((ob >= 0).sum())
    assert int((gb >= 0).sum()) == n_valid, (gb, ob)
    assert np.all(gb[n_valid:] == -1) and np.all(gw[n_valid:] == -1)
    assert np.all(np.isneginf(gs[n_valid:]))
    pos = {int(w): i for i, w in enumerate(cand)}
    seen = set()
    for r in range(n_valid):
        b, w = int(gb[r]), int(gw[r])
        assert 0 <= b < lp.shape[0] and w in pos, (b, w)
        assert (b, w) not in seen
        seen.add((b, w))
        mine = bs[b] + lp[b, pos[w]]
        # the score inherits the log-probability's error, which scales with |lp| (and the fp32
        # addition's with the operands), not with the possibly cancelling sum
        bound = max(lpb[b, pos[w]], tol * max(abs(osc[r]), abs(bs[b])))
        assert abs(float(gs[r]) - mine) <= bound, (r, float(gs[r]), mine)
        assert abs(float(gs[r]) - osc[r]) <= bound, (r, float(gs[r]), osc[r])
        if (b, w) != (int(ob[r]), int(ow[r])):
            # only acceptable inside a near-tie: the pair the oracle put here scores the same
            assert abs(mine - osc[r]) <= 2 * bound, (r, (b, w), (int(ob[r]), int(ow[r])), mine, osc[r])
    assert np.all(np.diff(gs[:n_valid].astype(np.float64)) <= 0)
    return sum(1 for r in range(n_valid) if (int(gb[r]), int(gw[r])) != (int(ob[r]), int(ow[r])))
