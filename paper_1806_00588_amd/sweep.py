"""Recall / speedup sweep of the LSH decode step against the full-vocabulary step.

A synthetic stand-in for the paper's parameter studies (Figs. 6-8, Tables 7-8): for every
setting of {T, t, banding, beam size} it runs the same decode steps twice through the HIP path --
once with the LSH candidate list, once with the candidate list forced to all of V (Eq. 1-2 as
printed) -- and reports

  recall@B   fraction of the full-vocabulary top-B (beam, word) pairs that the LSH step returns,
  top1       fraction of steps whose best pair agrees,
  |V_LSH|    mean candidate-list length,
  speedup    full-vocabulary step time / LSH step time (HIP-graph replay of the step sequence).

The "TOP" rows use a hit threshold above the number of bands, which leaves V_LSH = V_T: the
paper's top-frequent-words-only baseline.  Inputs are the seeded synthetic workloads of
the repository's generator (no corpus, no trained model), so recall here says how well the hashing finds the
large inner products of THOSE inputs, not BLEU.  The library part (Sweeper) takes arrays; only
the command line below fetches them from the generator.

    python -m paper_1806_00588_amd.sweep [--config paper] [--steps 20] [--out file.jsonl]
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def _graph_time(run, reps: int) -> float:
    """Seconds per call of run(stream_ptr) under HIP-graph replay."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(side.cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run(torch.cuda.current_stream().cuda_stream)
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        g.replay()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps


def beam_scores_for(R: int, seed: int = 0) -> np.ndarray:
    """The accumulated scores every setting of the sweep starts its steps from: R seeded normal
    draws (scale 2), descending."""
    rng = np.random.default_rng(seed + 17)
    return np.sort(rng.standard_normal(R).astype(np.float32) * 2)[::-1].copy()


def recall_stats(lsh_beam, lsh_word, full_beam, full_word) -> tuple:
    """(recall@B, top-1 agreement) of LSH results against full-vocabulary results, arrays
    [steps, S, B] of beam / word ids (-1 = padding)."""
    steps, S, _ = full_beam.shape
    hit = top1 = total = 0
    for i in range(steps):
        for s in range(S):
            want = {(int(b), int(w)) for b, w in zip(full_beam[i, s], full_word[i, s]) if b >= 0}
            got = {(int(b), int(w)) for b, w in zip(lsh_beam[i, s], lsh_word[i, s]) if b >= 0}
            hit += len(want & got)
            total += len(want)
            top1 += int((lsh_beam[i, s, 0], lsh_word[i, s, 0]) == (full_beam[i, s, 0], full_word[i, s, 0]))
    return hit / max(total, 1), top1 / (steps * S)


class Sweeper:
    """Tables for one (E, perms, bands) plus the step plumbing shared by all settings on them.
    E: numpy [V, d] fp32 or bf16 bit patterns (uint16); perms: numpy int32 [P, K]."""

    def __init__(self, E: np.ndarray, perms: np.ndarray, bands: int, seed: int = 0):
        import torch
        import paper_1806_00588_amd as lsh
        self.torch, self.lsh = torch, lsh
        self.E = E
        self.V, self.d = E.shape
        self.P, self.K = perms.shape
        self.W = bands
        self.E_dev = torch.from_numpy(E.view(np.int16) if E.dtype == np.uint16 else E).cuda()
        self.tables = lsh.build_tables(self.E_dev, torch.from_numpy(perms).cuda(), self.K, bands, seed=seed)
        self.seed = seed

    def measure(self, H: np.ndarray, topfreq: np.ndarray, B: int, t: int, S: int = 1, time_it: bool = True) -> dict:
        """One setting: the decode steps H [steps, S*B, d] of S sentences x B beams with the
        top-frequent list `topfreq` and hit threshold t, LSH and full-vocabulary."""
        from . import binding
        torch, lsh = self.torch, self.lsh
        steps, R = H.shape[0], S * B
        assert H.shape[1] == R and H.shape[2] == self.d
        T = int(len(topfreq))
        H = torch.from_numpy(np.ascontiguousarray(H, dtype=np.float32)).cuda()
        tf = torch.from_numpy(np.ascontiguousarray(topfreq, dtype=np.int32)).cuda() if T > 0 else None
        bs = torch.from_numpy(beam_scores_for(R, self.seed)).cuda()
        res = {}
        for mode, full in (("lsh", False), ("full", True)):
            sp = binding.step_params(S, B, T, t, full)
            ws = torch.empty(lsh.step_workspace_bytes(self.tables, sp), dtype=torch.uint8, device="cuda")
            ob = torch.empty((steps, R), dtype=torch.int32, device="cuda")
            ow = torch.empty((steps, R), dtype=torch.int32, device="cuda")
            osc = torch.empty((steps, R), dtype=torch.float32, device="cuda")
            call = binding.make_step_caller(self.tables, sp, ws, tf)

            def run(stream, call=call, ob=ob, ow=ow, osc=osc):
                for i in range(steps):
                    call(H[i].data_ptr(), bs.data_ptr(), ob[i].data_ptr(), ow[i].data_ptr(),
                         osc[i].data_ptr(), stream)
            sec = _graph_time(run, reps=10) / steps if time_it else 0.0
            counts = None
            if not full or not time_it:   # candidate-list lengths, one eager step at a time
                counts = []
                for i in range(steps):
                    lsh.decode_step(self.tables, H[i], bs, tf, sp, ws, ob[i], ow[i], osc[i])
                    torch.cuda.synchronize()
                    if not full:
                        counts += [len(self.tables.debug_candidates(ws, sp, s)) for s in range(S)]
            torch.cuda.synchronize()
            res[mode] = (ob.cpu().numpy().reshape(steps, S, B), ow.cpu().numpy().reshape(steps, S, B), sec, counts)
        (lb, lw, lsec, counts), (fb, fw, fsec, _) = res["lsh"], res["full"]
        recall, top1 = recall_stats(lb, lw, fb, fw)
        return {"S": S, "B": B, "T": T, "t": t, "K": self.K, "u": self.P // self.W, "W": self.W,
                "recall_at_B": round(recall, 4), "top1": round(top1, 4),
                "mean_candidates": round(float(np.mean(counts)), 1), "V": self.V,
                "lsh_us": round(lsec * 1e6, 2), "full_us": round(fsec * 1e6, 2),
                "speedup": round(fsec / lsec, 3) if lsec > 0 else None, "steps": steps,
                "lsh_results": (lb, lw), "full_results": (fb, fw)}


def default_settings(cfg) -> list:
    """(B, T, t) triples: T sweep, t sweep (where the banding has enough bands), beam sweep
    (Table 8's sizes), and the top-frequent-only baseline."""
    W = cfg.W
    out = [(cfg.B, T, cfg.threshold) for T in (0, 250, 1000, 4000)]
    if W >= 16:
        out += [(cfg.B, cfg.T, t) for t in (2, 3, 5, 8, 12, 20, 40) if t != cfg.threshold and t <= W]
    out += [(B, cfg.T, cfg.threshold) for B in (24, 36, 48)]
    out += [(cfg.B, T, W + 1) for T in (1000, 4000)]          # TOP: V_LSH = V_T
    return out


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--config", default="paper")
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--out", default=None, help="also append one JSON line per setting to this file")
    args = ap.parse_args(argv)
    import torch
    import workloads   # the seeded synthetic inputs of this repository (tests and bench share them)
    assert torch.cuda.is_available(), "the sweep runs on the GPU path only"
    cfg = workloads.CONFIGS[args.config]
    E = workloads.make_embeddings(cfg, 0)
    sw = Sweeper(E, workloads.make_perms(cfg, 0), cfg.W)
    rows = []
    print(f"# {cfg.name}: d={cfg.d} V={cfg.V} K={cfg.K} u={cfg.u} W={cfg.W}; {args.steps} steps per setting")
    print(f"{'B':>3} {'T':>5} {'t':>4} {'|V_LSH|':>9} {'recall@B':>9} {'top1':>6} {'lsh us':>8} {'full us':>8} {'speedup':>8}")
    for B, T, t in default_settings(cfg):
        c = dataclasses.replace(cfg, S=1, B=B, T=T, threshold=t)
        r = sw.measure(workloads.make_hidden(c, E, seed=0, steps=args.steps), workloads.make_topfreq(c), B, t)
        del r["lsh_results"], r["full_results"]
        r["config"] = cfg.name
        r["baseline"] = "TOP" if t > cfg.W else "LSH"
        rows.append(r)
        tag = "TOP" if t > cfg.W else str(t)
        print(f"{B:3d} {T:5d} {tag:>4} {r['mean_candidates']:9.1f} {r['recall_at_B']:9.4f} {r['top1']:6.3f} "
              f"{r['lsh_us']:8.2f} {r['full_us']:8.2f} {r['speedup']:8.3f}", flush=True)
        if args.out:
            with open(args.out, "a") as f:
                f.write(json.dumps(r) + "\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
