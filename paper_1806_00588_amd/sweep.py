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
workloads.py (no corpus, no trained model), so recall here says how well the hashing finds the
large inner products of THOSE inputs, not BLEU.

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


class Sweeper:
    """Tables for one (E, perms, bands) plus the step plumbing shared by all settings on them."""

    def __init__(self, cfg, seed: int = 0):
        import torch
        import workloads
        import paper_1806_00588_amd as lsh
        self.torch, self.lsh, self.cfg = torch, lsh, cfg
        self.E = workloads.make_embeddings(cfg, seed)
        perms = workloads.make_perms(cfg, seed)
        self.E_dev = torch.from_numpy(self.E.view(np.int16) if self.E.dtype == np.uint16 else self.E).cuda()
        self.tables = lsh.build_tables(self.E_dev, torch.from_numpy(perms).cuda(), cfg.K, cfg.W, seed=seed)
        self.workloads = workloads
        self.seed = seed

    def measure(self, B: int, T: int, t: int, steps: int, S: int = 1) -> dict:
        """One setting: `steps` decode steps of S sentences x B beams, LSH and full-vocabulary."""
        from . import binding
        torch, lsh = self.torch, self.lsh
        cfg = dataclasses.replace(self.cfg, S=S, B=B, T=T, threshold=t)
        H = torch.from_numpy(self.workloads.make_hidden(cfg, self.E, seed=self.seed, steps=steps)).cuda()
        tf = torch.from_numpy(self.workloads.make_topfreq(cfg)).cuda() if T > 0 else None
        R = S * B
        rng = np.random.default_rng(self.seed + 17)
        bs = torch.from_numpy(np.sort(rng.standard_normal(R).astype(np.float32) * 2)[::-1].copy()).cuda()
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
            sec = _graph_time(run, reps=10) / steps
            counts = None
            if not full:   # candidate-list lengths, one eager step at a time
                counts = []
                for i in range(steps):
                    lsh.decode_step(self.tables, H[i], bs, tf, sp, ws, ob[i], ow[i], osc[i])
                    torch.cuda.synchronize()
                    counts += [len(self.tables.debug_candidates(ws, sp, s)) for s in range(S)]
            torch.cuda.synchronize()
            res[mode] = (ob.cpu().numpy().reshape(steps, S, B), ow.cpu().numpy().reshape(steps, S, B), sec, counts)
        (lb, lw, lsec, counts), (fb, fw, fsec, _) = res["lsh"], res["full"]
        hit = top1 = total = 0
        for i in range(steps):
            for s in range(S):
                want = {(int(b), int(w)) for b, w in zip(fb[i, s], fw[i, s]) if b >= 0}
                got = {(int(b), int(w)) for b, w in zip(lb[i, s], lw[i, s]) if b >= 0}
                hit += len(want & got)
                total += len(want)
                top1 += int((lb[i, s, 0], lw[i, s, 0]) == (fb[i, s, 0], fw[i, s, 0]))
        return {"S": S, "B": B, "T": T, "t": t, "K": cfg.K, "u": cfg.u, "W": cfg.W,
                "recall_at_B": round(hit / max(total, 1), 4), "top1": round(top1 / (steps * S), 4),
                "mean_candidates": round(float(np.mean(counts)), 1), "V": cfg.V,
                "lsh_us": round(lsec * 1e6, 2), "full_us": round(fsec * 1e6, 2),
                "speedup": round(fsec / lsec, 3), "steps": steps}


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
    import workloads
    assert torch.cuda.is_available(), "the sweep runs on the GPU path only"
    cfg = workloads.CONFIGS[args.config]
    sw = Sweeper(cfg)
    rows = []
    print(f"# {cfg.name}: d={cfg.d} V={cfg.V} K={cfg.K} u={cfg.u} W={cfg.W}; {args.steps} steps per setting")
    print(f"{'B':>3} {'T':>5} {'t':>4} {'|V_LSH|':>9} {'recall@B':>9} {'top1':>6} {'lsh us':>8} {'full us':>8} {'speedup':>8}")
    for B, T, t in default_settings(cfg):
        r = sw.measure(B, T, t, args.steps)
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
