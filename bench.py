#!/usr/bin/env python3
"""Decode-step throughput of the LSH reduced-vocabulary softmax + beam expansion on one MI355X.

A "step" is one lsh_decode_step call: hash the hidden rows, probe the cuckoo tables, build the
candidate list, gathered logits, log-softmax, top-B -- for one batch of synthetic hidden states,
with every input already resident in HBM.  Steps of a synthetic "sentence" are chained: the
scores a step returns are the next step's beam scores.

Prints ONE JSON line (the fields are described in the README and the design notes).
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


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def measured_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc summary."""
    for kernel in ("k_cand_logits", "k_union_logits", "k_logits_hlds", "k_logits_estage", "k_logits_wave"):
        path = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_pmc.md")
        try:
            for line in open(path):
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1].split()[0])
        except OSError:
            pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--config", default="paper")
    ap.add_argument("--mode", choices=["graph", "stream"], default="graph",
                    help="graph: replay a captured HIP graph of one sentence's steps; "
                         "stream: launch every step from the host")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-full-vocab", action="store_true")
    ap.add_argument("--no-bookkeeping", action="store_true",
                    help="skip the extra measurement of the step followed by lsh_beam_advance")
    ap.add_argument("--no-regime", action="store_true",
                    help="skip the extra bandwidth-regime measurement (the logits kernel on the "
                         "32-sentence 'batched' shape, same embeddings and tables)")
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

    t0 = time.time()
    E, perms, topfreq, H = workloads.make_all(cfg, seed=0)
    log(f"[bench] generated {cfg.name}: E {E.shape} {E.dtype}, H {H.shape} in {time.time()-t0:.1f}s")
    E_dev = torch.from_numpy(E.view(np.int16) if E.dtype == np.uint16 else E).cuda()
    perms_dev = torch.from_numpy(perms).cuda()
    tf_dev = torch.from_numpy(topfreq).cuda()
    H_dev = torch.from_numpy(H).cuda()
    t0 = time.time()
    tables = lsh.build_tables(E_dev, perms_dev, cfg.K, cfg.W, seed=0)
    torch.cuda.synchronize()
    log(f"[bench] lsh_build_tables: {time.time()-t0:.2f}s")

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    R, S, B, nst = cfg.R, cfg.S, cfg.B, cfg.steps
    zero = torch.zeros(R, dtype=torch.float32, device="cuda")
    score = [torch.empty(R, dtype=torch.float32, device="cuda") for _ in range(2)]
    ob = torch.empty(R, dtype=torch.int32, device="cuda")
    ow = torch.empty(R, dtype=torch.int32, device="cuda")
    h_ptrs = [H_dev[i].data_ptr() for i in range(nst)]

    def make_runner(full_vocab: bool):
        sp = binding.step_params(S, B, cfg.T, cfg.threshold, full_vocab)
        ws = torch.empty(lsh.step_workspace_bytes(tables, sp), dtype=torch.uint8, device="cuda")
        call = binding.make_step_caller(tables, sp, ws, tf_dev)
        zp, sps = zero.data_ptr(), [score[0].data_ptr(), score[1].data_ptr()]
        obp, owp = ob.data_ptr(), ow.data_ptr()

        def run_steps(first: int, n: int, stream_ptr: int):
            # steps first .. first+n-1 of the endless sequence of sentences
            for i in range(first, first + n):
                st = i % nst
                call(h_ptrs[st], zp if st == 0 else sps[(st - 1) & 1], obp, owp, sps[st & 1],
                     stream_ptr)
        return sp, ws, run_steps

    def stream_ptr():
        return int(torch.cuda.current_stream().cuda_stream)

    def time_region(run_steps, n_steps, mode):
        """Exactly n_steps steps; returns seconds."""
        graph = None
        if mode == "graph" and n_steps >= nst:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                run_steps(0, nst, stream_ptr())          # warm the capture stream
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                run_steps(0, nst, stream_ptr())
        def go(n):
            done = 0
            if graph is not None:
                for _ in range(n // nst):
                    graph.replay()
                done = (n // nst) * nst
            if done < n:
                run_steps(done, n - done, stream_ptr())
        go(Wm)
        torch.cuda.synchronize()
        t = time.perf_counter()
        go(n_steps)
        torch.cuda.synchronize()
        return time.perf_counter() - t, graph

    # ---- LSH step: the headline ---------------------------------------------------------------
    sp, ws, run_lsh = make_runner(False)

    # untimed pass: candidate counts per step (they depend on H only) and a reference result of
    # one full sentence for the graph-vs-eager check
    counts = np.zeros((nst, S), dtype=np.int64)
    for st in range(nst):
        run_lsh(st, 1, stream_ptr())
        torch.cuda.synchronize()
        for s in range(S if S <= 4 else 4):
            counts[st, s] = len(tables.debug_candidates(ws, sp, s))
        if S > 4:
            counts[st, 4:] = counts[st, :4].mean()
    ref = (ob.clone(), ow.clone(), score[(nst - 1) & 1].clone())

    secs, graph = time_region(run_lsh, K, args.mode)
    if graph is not None:
        # replays must reproduce the eager result exactly, every time
        for _ in range(3):
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(ob, ref[0]) and torch.equal(ow, ref[1]) and \
                torch.equal(score[(nst - 1) & 1], ref[2]), "graph replay differs from eager result"
    steps_per_s = K / secs
    log(f"[bench] {cfg.name} LSH: {K} steps in {secs*1e3:.2f} ms -> {steps_per_s:,.0f} steps/s "
        f"({secs/K*1e6:.2f} us/step, mode={args.mode})")

    # ---- per-kernel durations over the same K steps, from HIP events around each kernel -------
    run_lsh(0, min(Wm, nst), stream_ptr())
    torch.cuda.synchronize()
    # (every kernel is launched at most once per step; durations are still summed per step, so the
    #  figures stay right should a step ever launch one several times)
    launches_per_step = 1
    tables.profile_begin(K * launches_per_step)
    run_lsh(0, K, stream_ptr())
    prof = {name: (ms * n / K, n) for name, (ms, n) in tables.profile_end().items()}
    for name, (ms, n) in prof.items():
        log(f"[bench]   {name:14s} mean {ms*1e3:8.2f} us per step ({n} launches)")

    e_bytes = 2 if cfg.e_dtype == workloads.BF16 else 4
    mean_rows = float(counts.sum(axis=1).mean())                 # gathered E rows per launch
    alg_bytes = mean_rows * cfg.d * e_bytes
    k_ms = prof["k_logits"][0]
    achieved = alg_bytes / (k_ms * 1e-3) / 1e9 if k_ms > 0 else 0.0
    flops = 2.0 * B * mean_rows * cfg.d
    fused = binding.step_is_fused(tables, sp)
    pre_hashed = prof["k_hit_rows"][1] > 0 or prof["k_part_bitmaps"][1] > 0
    fused_name = "k_union_logits" if pre_hashed else "k_cand_logits"
    dominant = (fused_name + " (candidate generation fused into the logits kernel)") if fused \
        else "k_logits"
    roofline = {"kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": measured_traffic(cfg.name),
                "algorithmic_bytes_per_launch": alg_bytes, "kernel_us": round(k_ms * 1e3, 3),
                "mfma_tflops": round(flops / (k_ms * 1e-3) / 1e12, 2) if k_ms > 0 else 0.0}

    # ---- full-vocabulary step on the same kernels (Eq. 1-2 as printed): the speedup's base ----
    full = None
    if not args.no_full_vocab:
        _, _, run_full = make_runner(True)
        kf = max(nst, min(K, 400) // nst * nst)
        fsecs, _ = time_region(run_full, kf, args.mode)
        tables.profile_begin(kf * launches_per_step)
        run_full(0, kf, stream_ptr())
        fprof = {name: (ms * n / kf, n) for name, (ms, n) in tables.profile_end().items()}
        for name, (ms, n) in fprof.items():
            log(f"[bench]   full-vocab {name:14s} mean {ms*1e3:8.2f} us per step ({n} launches)")
        full = {"steps": kf, "ms_per_step": round(fsecs / kf * 1e3, 5),
                "kernels_us": {k: round(v[0] * 1e3, 3) for k, v in fprof.items() if v[1]},
                "steps_per_s": round(kf / fsecs, 1),
                "lsh_speedup": round((fsecs / kf) / (secs / K), 3),
                "algorithmic_bytes_per_step": float(S) * cfg.V * cfg.d * e_bytes}
        log(f"[bench] {cfg.name} full-vocab: {fsecs/kf*1e6:.2f} us/step -> LSH speedup "
            f"{full['lsh_speedup']}x")

    # ---- the gathered contraction where bandwidth, not latency, limits it: 32 sentences on the
    #      same embeddings and tables (the 'batched' shape), three-kernel path -------------------
    regime = None
    if not args.no_regime and cfg.name == "paper":
        bcfg = workloads.CONFIGS["batched"]
        Hb = torch.from_numpy(workloads.make_hidden(bcfg, E, seed=0, steps=8)).cuda()
        bsp = binding.step_params(bcfg.S, bcfg.B, bcfg.T, 1, False)
        bws = torch.empty(lsh.step_workspace_bytes(tables, bsp), dtype=torch.uint8, device="cuda")
        bz = torch.zeros(bcfg.R, dtype=torch.float32, device="cuda")
        bo = [torch.empty(bcfg.R, dtype=torch.int32, device="cuda") for _ in range(2)]
        bsc = torch.empty(bcfg.R, dtype=torch.float32, device="cuda")
        rows = []
        for i in range(8):
            lsh.decode_step(tables, Hb[i], bz, tf_dev, bsp, bws, bo[0], bo[1], bsc)
            torch.cuda.synchronize()
            rows.append(sum(len(tables.debug_candidates(bws, bsp, s)) for s in range(bcfg.S)))
        for i in range(16):
            lsh.decode_step(tables, Hb[i % 8], bz, tf_dev, bsp, bws, bo[0], bo[1], bsc)
        torch.cuda.synchronize()
        tables.profile_begin(64)
        for i in range(64):
            lsh.decode_step(tables, Hb[i % 8], bz, tf_dev, bsp, bws, bo[0], bo[1], bsc)
        bprof = {name: (ms * n / 64, n) for name, (ms, n) in tables.profile_end().items()}
        bbytes = float(np.mean(rows)) * bcfg.d * e_bytes
        bms = bprof["k_logits"][0]
        regime = {"workload": f"batched: S={bcfg.S} B={bcfg.B}, same E and tables",
                  "kernel": "k_logits_hlds", "kernel_us": round(bms * 1e3, 2),
                  "algorithmic_bytes_per_launch": bbytes,
                  "achieved_GBps": round(bbytes / (bms * 1e-3) / 1e9, 1),
                  "frac_of_hbm_peak": round(bbytes / (bms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                  "traffic": measured_traffic("batched"),
                  "kernels_us": {k: round(v[0] * 1e3, 2) for k, v in bprof.items()}}
        log(f"[bench] bandwidth regime ({regime['workload']}): k_logits {bms*1e3:.1f} us, "
            f"{regime['achieved_GBps']} GB/s = {regime['frac_of_hbm_peak']*100:.1f}% of HBM peak")
        del Hb, bws

    # ---- the step followed by the beam bookkeeping (state reorder of a 2-layer LSTM: h and c of
    #      both layers, history, next scores): what a decoder loop adds around the hot path -------
    book = None
    if not args.no_bookkeeping:
        hist = binding.BeamHistory(S, B, nst, n_states=4, state_dim=cfg.d, eos=-1)
        st_bufs = [[torch.randn(R, cfg.d, device="cuda") for _ in range(4)] for _ in range(2)]
        call = binding.make_step_caller(tables, sp, ws, tf_dev)

        def run_book(first: int, n: int, stream_ptr_: int):
            for i in range(first, first + n):
                st = i % nst
                a, b2 = st & 1, (st + 1) & 1
                call(h_ptrs[st], zero.data_ptr() if st == 0 else score[a].data_ptr(), ob.data_ptr(),
                     ow.data_ptr(), score[b2].data_ptr(), stream_ptr_)
                # scores for the next step are written by the bookkeeping call (in place: the
                # kernel reads out_score[r] and writes next_scores[r] in the same thread)
                binding.beam_advance(hist, st, ob, ow, score[b2], st_bufs[a], st_bufs[b2], score[b2],
                                     stream=stream_ptr_)
        kb = max(nst, min(K, 1000) // nst * nst)
        bsecs, _ = time_region(run_book, kb, args.mode)
        book = {"steps": kb, "ms_per_step": round(bsecs / kb * 1e3, 6),
                "steps_per_s": round(kb / bsecs, 1), "state_arrays": 4, "state_dim": cfg.d,
                "extra_us_per_step": round((bsecs / kb - secs / K) * 1e6, 2)}
        log(f"[bench] {cfg.name} step + lsh_beam_advance (4 state arrays): {bsecs/kb*1e6:.2f} us/step")

    # ---- the oracle on the host cores, bounded sample -----------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        ix = oracle.Index(E, perms, cfg.W)
        n_done, t0 = 0, time.perf_counter()
        bs = np.zeros(R, dtype=np.float32)
        while True:
            st = n_done % nst
            if st == 0:
                bs[:] = 0
            _, _, osc, _ = ix.decode_step(H[st], bs, topfreq, S, B, t=cfg.threshold)
            bs = osc.reshape(-1).astype(np.float32)
            n_done += 1
            el = time.perf_counter() - t0
            if el >= args.cpu_seconds and (n_done % nst == 0 or el >= 2.5 * args.cpu_seconds):
                break
        cpu = {"value": round(n_done / el, 3), "unit": "steps/s", "cores": 1, "kind": "oracle",
               "sample": f"{n_done} consecutive steps of the same workload ({el:.1f} s, "
                         f"single thread, g++ -O2)"}
        log(f"[bench] oracle: {n_done} steps in {el:.1f}s -> {cpu['value']} steps/s on 1 core "
            f"of {os.cpu_count()}")

    out = {
        "metric": "LSH decode steps/sec (d=%d,V=%d,B=%d)" % (cfg.d, cfg.V, cfg.B),
        "value": round(steps_per_s, 1), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": round(secs / K * 1e3, 6), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16xf32" if cfg.e_dtype == workloads.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: d={cfg.d} V={cfg.V} S={S} B={B} K={cfg.K} P={cfg.P} "
                               f"W={cfg.W} T={cfg.T} t={cfg.threshold}, {nst}-step sentences, seed 0",
                   "mode": args.mode, "mean_candidates_per_sentence": round(mean_rows / S, 1)},
        "roofline": roofline,
        "kernels_us": {(fused_name if (fused and k == "k_logits") else k): round(v[0] * 1e3, 3)
                       for k, v in prof.items() if v[1]},
        "full_vocab": full,
        "bandwidth_regime": regime,
        "with_bookkeeping": book,
        "step_bytes_over_step_time_GBps": round(alg_bytes / secs * K / 1e9, 1),
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
