#!/usr/bin/env python3
"""Decode-step throughput of the LSH reduced-vocabulary softmax + beam expansion on one MI355X.

A "step" is one lsh_decode_step call: hash the hidden rows, probe the cuckoo tables, build the
candidate list, gathered logits, log-softmax, top-B -- for one batch of synthetic hidden states,
with every input already resident in HBM.  Steps of a synthetic "sentence" are chained: the
scores a step returns are the next step's beam scores.

Prints ONE JSON line.  The headline (`value`, `roofline`, `full_vocab`, `with_bookkeeping`,
`cpu_baseline`) is the workload named by --config (default: the paper shape); `other_configs`
carries the same measurement, shorter, for the other shapes of the metric.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
FP32_MATRIX_PEAK_TFLOPS = 157.3
OTHER_CONFIGS = ("tiny", "batched", "widebeam", "largevocab")


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def committed_traffic(workload: str):
    """(HBM bytes per launch of the dominant kernel, file) from the committed rocprofv3 --pmc
    summary of that workload; measured by hand with the counters, not during this run."""
    for kernel in ("k_cand_logits", "k_union_logits", "k_logits_hlds", "k_logits_estage", "k_logits_wave"):
        name = f"{kernel}_{workload}_pmc.md"
        try:
            for line in open(os.path.join(ROOT, "profiles", name)):
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0]), "profiles/" + name
        except OSError:
            pass
    return None, None


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


class Workload:
    """One configuration resident on the device: embeddings, tables, hidden states of a sentence."""

    def __init__(self, cfg, E=None, options=()):
        import numpy as np
        import torch
        import workloads
        import paper_1806_00588_amd as lsh
        self.cfg, self.np, self.torch, self.lsh = cfg, np, torch, lsh
        t0 = time.time()
        self.E = workloads.make_embeddings(cfg, 0) if E is None else E
        self.perms = workloads.make_perms(cfg, 0)
        self.topfreq = workloads.make_topfreq(cfg)
        self.H = workloads.make_hidden(cfg, self.E, seed=0)
        log(f"[bench] generated {cfg.name}: E {self.E.shape} {self.E.dtype}, H {self.H.shape} in {time.time()-t0:.1f}s")
        self.E_dev = torch.from_numpy(self.E.view(np.int16) if self.E.dtype == np.uint16 else self.E).cuda()
        self.tf_dev = torch.from_numpy(self.topfreq).cuda()
        self.H_dev = torch.from_numpy(self.H).cuda()
        t0 = time.time()
        self.tables = lsh.build_tables(self.E_dev, torch.from_numpy(self.perms).cuda(), cfg.K, cfg.W, seed=0)
        torch.cuda.synchronize()
        log(f"[bench] lsh_build_tables: {time.time()-t0:.2f}s")
        for name, value in options:
            self.tables.set_option(name, value)
        R = cfg.R
        self.zero = torch.zeros(R, dtype=torch.float32, device="cuda")
        self.score = [torch.empty(R, dtype=torch.float32, device="cuda") for _ in range(2)]
        self.ob = torch.empty(R, dtype=torch.int32, device="cuda")
        self.ow = torch.empty(R, dtype=torch.int32, device="cuda")
        self.h_ptrs = [self.H_dev[i].data_ptr() for i in range(cfg.steps)]
        self.e_bytes = 2 if cfg.e_dtype == workloads.BF16 else 4

    def stream_ptr(self):
        return int(self.torch.cuda.current_stream().cuda_stream)

    def runner(self, full_vocab: bool):
        """(sp, workspace, run_steps(first, n, stream)): steps first .. first+n-1 of the endless
        sequence of sentences, chained through the returned scores."""
        from paper_1806_00588_amd import binding
        cfg, nst = self.cfg, self.cfg.steps
        sp = binding.step_params(cfg.S, cfg.B, cfg.T, cfg.threshold, full_vocab)
        ws = self.torch.empty(self.lsh.step_workspace_bytes(self.tables, sp), dtype=self.torch.uint8, device="cuda")
        call = binding.make_step_caller(self.tables, sp, ws, self.tf_dev)
        zp, sps = self.zero.data_ptr(), [self.score[0].data_ptr(), self.score[1].data_ptr()]
        obp, owp, h_ptrs = self.ob.data_ptr(), self.ow.data_ptr(), self.h_ptrs

        def run_steps(first: int, n: int, stream_ptr: int):
            for i in range(first, first + n):
                st = i % nst
                call(h_ptrs[st], zp if st == 0 else sps[(st - 1) & 1], obp, owp, sps[st & 1], stream_ptr)
        return sp, ws, run_steps

    def capture(self, run_steps, first: int, n: int):
        """A HIP graph of steps first .. first+n-1 (warmed on a side stream first)."""
        torch = self.torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run_steps(first, n, int(side.cuda_stream))
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run_steps(first, n, self.stream_ptr())
        return g

    def results(self, upto_step: int):
        return (self.ob.clone(), self.ow.clone(), self.score[upto_step & 1].clone())

    def time_steps(self, run_steps, n_steps: int, warmup: int, mode: str):
        """Exactly n_steps timed steps after `warmup` untimed ones -> (seconds, mode taken).
        graph: a graph of one sentence (or of all n_steps if that is fewer) is replayed, a second
        graph covers what is left over; every graph is first replayed and compared with the
        eager result of the same steps, bit for bit."""
        torch, nst = self.torch, self.cfg.steps
        if mode == "graph":
            unit = min(nst, n_steps)
            q, r = divmod(n_steps, unit)
            graphs = [(self.capture(run_steps, 0, unit), unit)]
            if r:
                graphs.append((self.capture(run_steps, 0, r), r))
            for g, n in graphs:           # replay == eager, every time
                run_steps(0, n, self.stream_ptr())
                torch.cuda.synchronize()
                ref = self.results(n - 1)
                for _ in range(2):
                    self.ob.fill_(-9); self.ow.fill_(-9)
                    g.replay()
                    torch.cuda.synchronize()
                    got = self.results(n - 1)
                    assert all(torch.equal(a, b) for a, b in zip(ref, got)), "graph replay differs from the eager result"

            def go(count):
                qq, rr = divmod(count, unit)
                for _ in range(qq):
                    graphs[0][0].replay()
                if rr:
                    if len(graphs) > 1 and rr == graphs[1][1]:
                        graphs[1][0].replay()
                    else:
                        run_steps(0, rr, self.stream_ptr())
        else:
            def go(count):
                run_steps(0, count, self.stream_ptr())
        go(warmup)
        torch.cuda.synchronize()
        done = torch.cuda.Event()
        t = time.perf_counter()
        go(n_steps)
        # (the host polls for the end of the work before it synchronizes: a blocking wait is woken
        # tens of microseconds late, which a 20-step run would book as step time)
        done.record()
        while not done.query():
            pass
        torch.cuda.synchronize()
        return time.perf_counter() - t, mode

    def kernel_times(self, run_steps, n_steps: int):
        """{kernel: (us per step, launches)} from HIP events around every kernel of n_steps steps
        (lsh_decode_step_timed, events on the launch stream)."""
        self.tables.profile_begin(n_steps)
        run_steps(0, n_steps, self.stream_ptr())
        return {name: (ms * n / n_steps * 1e3, n) for name, (ms, n) in self.tables.profile_end().items()}

    def step_traffic(self, sp, ws, run_steps):
        """Per step of the sentence: candidate counts [steps, S] and the ids read from the hit
        spans (sum over rows and bands of the bucket size of the row's band code)."""
        np, cfg = self.np, self.cfg
        counts = np.zeros((cfg.steps, cfg.S), dtype=np.int64)
        for st in range(cfg.steps):
            run_steps(st, 1, self.stream_ptr())
            counts[st] = self.tables.debug_counts(ws, sp)
        span_ids = np.zeros(cfg.steps, dtype=np.int64)
        ecodes = self.tables.debug_embedding_codes()          # bucket sizes: a histogram per band
        sizes = [np.bincount(ecodes[:, w]) for w in range(cfg.W)]
        for st in range(cfg.steps):
            hc = self.tables.debug_codes(self.H_dev[st])
            for w in range(cfg.W):
                c = hc[:, w]
                ok = c < len(sizes[w])
                span_ids[st] += int(sizes[w][c[ok]].sum())
        return counts, span_ids

    def measure(self, n_steps: int, warmup: int, mode: str):
        """The LSH step: time, per-kernel durations, algorithmic bytes, roofline of the dominant kernel."""
        from paper_1806_00588_amd import binding
        np, cfg = self.np, self.cfg
        sp, ws, run = self.runner(False)
        counts, span_ids = self.step_traffic(sp, ws, run)
        secs, mode_taken = self.time_steps(run, n_steps, warmup, mode)
        run(0, min(warmup, cfg.steps), self.stream_ptr())
        self.torch.cuda.synchronize()
        prof = self.kernel_times(run, n_steps)
        fused = binding.step_is_fused(self.tables, sp)
        pre_hashed = prof["k_hit_rows"][1] > 0 or prof["k_part_bitmaps"][1] > 0
        one_launch = fused and prof["k_select"][1] == 0
        fused_name = "k_union_logits" if pre_hashed else "k_cand_logits"
        names = {"k_logits": fused_name if fused else "k_logits"}
        kernels_us = {names.get(k, k): round(v[0], 3) for k, v in prof.items() if v[1]}

        # algorithmic bytes per step: what the method has to move (no padding, no cache refills)
        R, S, B, d, e = cfg.R, cfg.S, cfg.B, cfg.d, self.e_bytes
        mean_rows = float(counts.sum(axis=1).mean())               # gathered E rows per step
        gather = mean_rows * d * e
        list_bytes = mean_rows * 4 * (1 if fused else 2)           # the fused plan writes the list once, for inspection
        step_bytes = (R * d * 4 + cfg.P * cfg.K * 4 + R * cfg.W * 2 * 16 + float(span_ids.mean()) * 4 +
                      cfg.T * 4 + list_bytes + gather + R * 4 + S * B * 12)
        k_us = prof["k_logits"][0]
        achieved = gather / (k_us * 1e-6) / 1e9 if k_us > 0 else 0.0
        flops = 2.0 * B * mean_rows * d
        traffic, src = committed_traffic(cfg.name)
        dominant = fused_name + (" (candidate generation, contraction, log-softmax and top-B in one launch)"
                                 if one_launch else " (candidate generation fused into the logits kernel)") \
            if fused else "k_logits"
        us_step = secs / n_steps * 1e6
        roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": traffic, "traffic_source": (src + " (rocprofv3 --pmc run of this command, committed; not measured in this run)") if src else None,
                    "algorithmic_bytes_per_launch": gather, "kernel_us": round(k_us, 3),
                    "step_bytes": round(step_bytes, 1),
                    "step_frac": round(step_bytes / (us_step * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                    "mfma_tflops": round(flops / (k_us * 1e-6) / 1e12, 2) if k_us > 0 else 0.0,
                    "mfma_frac_of_fp32_peak": round(flops / (k_us * 1e-6) / 1e12 / FP32_MATRIX_PEAK_TFLOPS, 4) if k_us > 0 else 0.0}
        log(f"[bench] {cfg.name} LSH: {n_steps} steps in {secs*1e3:.2f} ms -> {n_steps/secs:,.0f} steps/s "
            f"({us_step:.2f} us/step, mode={mode_taken}); kernels {kernels_us}")
        return {"secs": secs, "mode": mode_taken, "us_per_step": us_step, "kernels_us": kernels_us,
                "roofline": roofline, "mean_rows": mean_rows, "sp": sp, "ws": ws, "run": run,
                "one_launch": one_launch}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default="paper")
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph",
                    help="graph: replay captured HIP graphs of the steps; stream: launch every step from the host")
    ap.add_argument("--option", action="append", default=[], metavar="NAME=VALUE",
                    help="launch-plan option for the tables (lsh_set_option), e.g. one_launch=0")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-vocab", action="store_true")
    ap.add_argument("--no-bookkeeping", action="store_true",
                    help="skip the extra measurement of the step followed by lsh_beam_advance")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the shorter measurements of the other shapes (tiny, batched, widebeam, largevocab)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (for scaling rocprofv3 --pmc "
                         "FETCH_SIZE / WRITE_SIZE readings to bytes)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-GPU kernel "
              "sequence; how it would shard is described in the design notes). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    import paper_1806_00588_amd as lsh
    from paper_1806_00588_amd import binding, build as hip_build

    if not os.path.exists(lsh.library_path()):
        hip_build.build()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    cfg = workloads.CONFIGS[args.config]
    K, Wm = args.steps, args.warmup
    options = [(o.split("=")[0], int(o.split("=")[1])) for o in args.option]
    wl = Workload(cfg, options=options)
    R, S, B, nst = cfg.R, cfg.S, cfg.B, cfg.steps

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- LSH step: the headline ---------------------------------------------------------------
    head = wl.measure(K, Wm, args.mode)
    secs = head["secs"]

    # ---- full-vocabulary step on the same kernels (Eq. 1-2 as printed): the speedup's base ----
    full = None
    if not args.no_full_vocab:
        _, _, run_full = wl.runner(True)
        kf = max(1, min(K, 400))
        fsecs, _ = wl.time_steps(run_full, kf, min(Wm, nst), args.mode)
        fprof = wl.kernel_times(run_full, kf)
        full = {"steps": kf, "ms_per_step": round(fsecs / kf * 1e3, 5),
                "kernels_us": {k: round(v[0], 3) for k, v in fprof.items() if v[1]},
                "steps_per_s": round(kf / fsecs, 1),
                "lsh_speedup": round((fsecs / kf) / (secs / K), 3),
                "algorithmic_bytes_per_step": float(S) * cfg.V * cfg.d * wl.e_bytes}
        log(f"[bench] {cfg.name} full-vocab: {fsecs/kf*1e6:.2f} us/step -> LSH speedup {full['lsh_speedup']}x")

    # ---- the step followed by the beam bookkeeping (state reorder of a 2-layer LSTM: h and c of
    #      both layers, history, next scores): what a decoder loop adds around the hot path -------
    book = None
    if not args.no_bookkeeping:
        hist = binding.BeamHistory(S, B, nst, n_states=4, state_dim=cfg.d, eos=-1)
        st_bufs = [[torch.randn(R, cfg.d, device="cuda") for _ in range(4)] for _ in range(2)]
        call = binding.make_step_caller(wl.tables, head["sp"], head["ws"], wl.tf_dev)

        def run_book(first: int, n: int, stream_ptr_: int):
            for i in range(first, first + n):
                st = i % nst
                a, b2 = st & 1, (st + 1) & 1
                call(wl.h_ptrs[st], wl.zero.data_ptr() if st == 0 else wl.score[a].data_ptr(), wl.ob.data_ptr(),
                     wl.ow.data_ptr(), wl.score[b2].data_ptr(), stream_ptr_)
                # scores for the next step are written by the bookkeeping call (in place: the
                # kernel reads out_score[r] and writes next_scores[r] in the same thread)
                binding.beam_advance(hist, st, wl.ob, wl.ow, wl.score[b2], st_bufs[a], st_bufs[b2], wl.score[b2],
                                     stream=stream_ptr_)
        kb = max(1, min(K, 1000))
        # (the replay check of time_steps compares score[(n - 1) & 1]; run_book alternates the other way)
        torch.cuda.synchronize()
        g = wl.capture(run_book, 0, min(nst, kb)) if args.mode == "graph" else None
        unit = min(nst, kb)
        reps = max(1, kb // unit)
        for _ in range(2):
            g.replay() if g else run_book(0, unit, wl.stream_ptr())
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            g.replay() if g else run_book(0, unit, wl.stream_ptr())
        torch.cuda.synchronize()
        bsecs, kb = time.perf_counter() - t0, reps * unit
        book = {"steps": kb, "ms_per_step": round(bsecs / kb * 1e3, 6),
                "steps_per_s": round(kb / bsecs, 1), "state_arrays": 4, "state_dim": cfg.d,
                "extra_us_per_step": round((bsecs / kb - secs / K) * 1e6, 2)}
        log(f"[bench] {cfg.name} step + lsh_beam_advance (4 state arrays): {bsecs/kb*1e6:.2f} us/step")

    # ---- the other shapes of the metric, shorter: steps/s, dominant kernel, its roofline fraction
    others = None
    if not args.no_other_configs and args.config == "paper":
        others = {}
        for name in OTHER_CONFIGS:
            ocfg = workloads.CONFIGS[name]
            same_E = ocfg.V == cfg.V and ocfg.d == cfg.d and name == "batched"   # batched: the paper shape's E
            ow_ = Workload(ocfg, E=wl.E if same_E else None, options=options)
            n = max(1, min(K, 4 * ocfg.steps))
            m = ow_.measure(n, min(Wm, ocfg.steps), args.mode)
            rf = m["roofline"]
            others[name] = {
                "workload": f"d={ocfg.d} V={ocfg.V} S={ocfg.S} B={ocfg.B} K={ocfg.K} P={ocfg.P} W={ocfg.W} "
                            f"T={ocfg.T} t={ocfg.threshold}" + (", E in bf16" if ow_.e_bytes == 2 else ""),
                "steps": n, "mode": m["mode"], "steps_per_s": round(n / m["secs"], 1),
                "us_per_step": round(m["us_per_step"], 2), "kernels_us": m["kernels_us"],
                "mean_candidates_per_sentence": round(m["mean_rows"] / ocfg.S, 1),
                "dominant_kernel": rf["kernel"], "kernel_us": rf["kernel_us"],
                "algorithmic_bytes_per_launch": rf["algorithmic_bytes_per_launch"],
                "achieved_GBps": rf["achieved"], "frac": rf["frac"], "step_bytes": rf["step_bytes"],
                "step_frac": rf["step_frac"], "traffic": rf["traffic"], "traffic_source": rf["traffic_source"],
                "mfma_tflops": rf["mfma_tflops"], "mfma_frac_of_fp32_peak": rf["mfma_frac_of_fp32_peak"],
                "bound": "mfma (fp32 matrix peak %.1f TFLOP/s on the %d real rows per sentence)" % (FP32_MATRIX_PEAK_TFLOPS, ocfg.B)
                         if name == "widebeam" else "hbm"}
            del ow_
            torch.cuda.empty_cache()

    # ---- the oracle on the host cores, bounded sample -----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ix = oracle.Index(wl.E, wl.perms, cfg.W)
        n_done, t0 = 0, time.perf_counter()
        bs = np.zeros(R, dtype=np.float32)
        while True:
            st = n_done % nst
            if st == 0:
                bs[:] = 0
            _, _, osc, _ = ix.decode_step(wl.H[st], bs, wl.topfreq, S, B, t=cfg.threshold)
            bs = osc.reshape(-1).astype(np.float32)
            n_done += 1
            el = time.perf_counter() - t0
            if el >= args.cpu_seconds and (n_done % nst == 0 or el >= 2.5 * args.cpu_seconds):
                break
        cpu = {"value": round(n_done / el, 3), "unit": "steps/s", "cores": 1, "kind": "oracle",
               "host_cores": os.cpu_count(), "cpu_model": cpu_model(),
               "sample": f"{n_done} consecutive steps of the same workload ({el:.1f} s, "
                         f"single thread, g++ -O2)"}
        log(f"[bench] oracle: {n_done} steps in {el:.1f}s -> {cpu['value']} steps/s on 1 core "
            f"of {os.cpu_count()} ({cpu['cpu_model']})")

    out = {
        "metric": "LSH decode steps/sec (d=%d,V=%d,B=%d)" % (cfg.d, cfg.V, cfg.B),
        "value": round(K / secs, 1), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(secs / K * 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16xf32" if wl.e_bytes == 2 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: d={cfg.d} V={cfg.V} S={S} B={B} K={cfg.K} P={cfg.P} "
                               f"W={cfg.W} T={cfg.T} t={cfg.threshold}, {nst}-step sentences, seed 0",
                   "mode": head["mode"], "launches_per_step": len(head["kernels_us"]),
                   "options": dict(options),
                   "mean_candidates_per_sentence": round(head["mean_rows"] / S, 1)},
        "roofline": head["roofline"],
        "kernels_us": head["kernels_us"],
        "full_vocab": full,
        "with_bookkeeping": book,
        "other_configs": others,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
