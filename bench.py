#!/usr/bin/env python3
"""Benchmark of the Col-Bandit scoring hot path on one MI355X.

One step = one pass of the whole hot path over one synthetic query batch that is already
resident in HBM: exhaustive Full-MaxSim with top-K (colbandit_full_maxsim) followed by the
Col-Bandit estimator of the same top-K (colbandit_topk).  The default workload is the
large text configuration: N=500,000 documents, lengths U[32,180], d=128, bf16, 128 queries
of T=32 tokens, K=5, alpha_ef=0.2, delta=0.01, M=5.

Prints ONE JSON line.  `value` is queries per second through the whole step; the
`full_maxsim` and `colbandit` objects give each path's own rate, MaxSim cells/s, coverage
and Overlap@K against the exhaustive result; `roofline` is the dense Full-MaxSim kernel
against the bf16 MFMA peak; `cpu_baseline` is the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0        # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch of the dominant kernels come from hardware-counter runs of this very
# command (FETCH_SIZE, then WRITE_SIZE, each scaled by the same counter's reading for the 1 GiB
# calibration copy below).  Their summary, profiles/hbm_traffic_counters.txt, records for every
# kernel the raw readings, the calibration factors, the workload and a hash of the kernel sources
# it was taken from; the figure is reported only when workload and hash match this run, else null.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_counters.txt")
KERNEL_SOURCES = ["cb_dense.hip", "cb_kernels.hip", "cb_device.h", "cb_launch.h"]
CALIBRATION_COPY_BYTES = 1 << 30


def kernel_source_hash():
    """Hash of the kernel sources with comments and white space removed (a comment may change
    without making a counter reading stale; code may not)."""
    import hashlib
    import re
    h = hashlib.sha256()
    for f in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2602_02827_amd", "csrc", f), "r") as fh:
            text = fh.read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        text = re.sub(r"//[^\n]*", "", text)
        h.update(re.sub(r"\s+", "", text).encode())
    return h.hexdigest()[:16]


def measured_traffic(workload_key, field="calibrated"):
    """{kernel label: HBM bytes per launch} from the counter summary, or {} if it was taken on
    other kernel sources or another workload.  Line format of the file:
    record <label> workload=<key> sources=<hash> fetch_kib=<x> write_kib=<y> fetch_scale=<a> write_scale=<b>
        [rd32=<n> rd64=<n> rd128=<n> wr32=<n> wr64=<n>]
    field "calibrated": FETCH_SIZE and WRITE_SIZE readings times their copy-kernel factors;
    field "by_request_size": the L2's read and write requests to memory counted by size (the
    optional fields), bytes = 32 / 64 / 128 per request."""
    out = {}
    if not os.path.exists(TRAFFIC_FILE):
        return out
    have = kernel_source_hash()
    for line in open(TRAFFIC_FILE):
        f = line.split()
        if len(f) < 3 or f[0] != "record" or not all("=" in x for x in f[2:]):
            continue
        kv = dict(x.split("=", 1) for x in f[2:])
        if kv.get("workload") != workload_key or kv.get("sources") != have:
            continue
        if field == "calibrated":
            out[f[1]] = 1024.0 * (float(kv["fetch_kib"]) * float(kv["fetch_scale"]) +
                                  float(kv["write_kib"]) * float(kv["write_scale"]))
        elif all(k in kv for k in ("rd32", "rd64", "rd128", "wr32", "wr64")):
            out[f[1]] = (32.0 * float(kv["rd32"]) + 64.0 * float(kv["rd64"]) + 128.0 * float(kv["rd128"]) +
                         32.0 * float(kv["wr32"]) + 64.0 * float(kv["wr64"]))
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=2, help="index into the five configurations")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink N (for quick checks)")
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--K", type=int, default=5)
    ap.add_argument("--alpha", type=float, default=0.2)
    ap.add_argument("--no-int8", action="store_true", help="skip the int8 coarse-pass leg")
    ap.add_argument("--no-baselines", action="store_true",
                    help="skip the Doc-Uniform / Ball-carving operating points")
    ap.add_argument("--no-k10", action="store_true", help="skip the K = 10 leg")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample-docs", type=int, default=60000)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 (sharding by query or by "
              "document is a design note only, not built)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2602_02827_amd import binding as B, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    B.lib()
    torch.cuda.set_device(0)
    dev = "cuda"

    t0 = time.time()
    w = synth.config(args.config, device=dev, scale=args.scale, nq=args.nq)
    torch.cuda.synchronize()
    gen_s = time.time() - t0
    K, M, delta, alpha = args.K, w.M, w.delta, args.alpha
    nq, T, d, N, total = w.nq, w.T, w.d, w.N, w.total_tokens

    ws = B.new_workspace(nq, T, d, N, total, dev)
    out_full = {"topk_ids": torch.empty((nq, K), dtype=torch.int64, device=dev),
                "topk_scores": torch.empty((nq, K), dtype=torch.float32, device=dev),
                "scores": torch.empty((nq, N), dtype=torch.float32, device=dev)}
    out_cb = {"topk_ids": torch.empty((nq, K), dtype=torch.int64, device=dev),
              "topk_scores": torch.empty((nq, K), dtype=torch.float32, device=dev)}

    # a plain copy kernel of known size (reads 1 GiB, writes 1 GiB): the yardstick that the
    # hardware-counter runs use to turn FETCH_SIZE / WRITE_SIZE readings into bytes
    cal_src = torch.ones(CALIBRATION_COPY_BYTES // 4, dtype=torch.float32, device=dev)
    cal_dst = torch.empty_like(cal_src)
    torch.mul(cal_src, 1.0, out=cal_dst)
    torch.cuda.synchronize()
    del cal_src, cal_dst

    def run_full(phases=False):
        return B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws, out=out_full,
                                       want_phase_ms=phases)

    def run_cb(stats=False):
        return B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, delta, M, w.seed, workspace=ws,
                                out=out_cb, want_stats=stats)

    for _ in range(args.warmup):
        run_full()
        run_cb()
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ms_kernel = []
    for s in range(args.steps):
        ev[s][0].record()
        ms_kernel.append(run_full(phases=True)["phase_ms"])   # events on the launch stream
        ev[s][1].record()
        run_cb()
        ev[s][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_full = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    ms_cb = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
    ms_step = wall * 1e3 / args.steps

    # fidelity and cost of the Col-Bandit path (outside the timed region)
    res = run_cb(stats=True)
    torch.cuda.synchronize()
    ids_full = out_full["topk_ids"].cpu().numpy()
    ids_cb = res["topk_ids"].cpu().numpy()
    overlap = float(np.mean([len(set(ids_full[q]) & set(ids_cb[q])) / K for q in range(nq)]))

    def tolerant_overlap(ids):
        """A returned document also counts as a hit when its exhaustive score is within the
        bf16 score tolerance (2e-3 relative) of the K-th exhaustive score: near-ties at the
        boundary are not errors of the estimator."""
        kth = out_full["topk_scores"][:, K - 1:K]
        got = torch.gather(out_full["scores"], 1, ids.clamp(min=0))
        ok = (got >= kth - 2e-3 * kth.abs()) & (ids >= 0)
        return float(ok.float().mean().item())

    overlap_tol = tolerant_overlap(res["topk_ids"])
    st = res["stats"]
    cells_total = float(nq) * N * T
    cells_touched = float(sum(s["cells_elim"] + s["cells_rescore"] for s in st))
    cells_unique = float(sum(s["cells_unique"] for s in st))
    coverage = cells_unique / cells_total
    rounds = [s["rounds"] for s in st]
    surv1 = float(np.mean([s["survivors"][1] if s["rounds"] >= 1 else N for s in st]))
    max_r = max(rounds)
    surv_by_round = [round(float(np.mean([s["survivors"][min(r, s["rounds"])] for s in st])), 1)
                     for r in range(max_r + 1)]
    same_bits = bool(all(
        torch.equal(res["topk_scores"][q], out_full["scores"][q][res["topk_ids"][q]]) for q in range(nq)))

    # the same estimator with its elimination rounds on int8 codes (the paper's deployed
    # layout); reported beside the step, not part of `value`.  Coding the corpus is an
    # index-time step and is timed on its own.
    int8 = None
    if not args.no_int8:
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        d8, dscale = B.colbandit_quantize_i8(w.docs)
        e1.record()
        torch.cuda.synchronize()
        ms_quant = e0.elapsed_time(e1)
        out8 = {"topk_ids": torch.empty((nq, K), dtype=torch.int64, device=dev),
                "topk_scores": torch.empty((nq, K), dtype=torch.float32, device=dev)}

        def run_cb8(stats=False):
            return B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, delta, M, w.seed, workspace=ws,
                                    out=out8, want_stats=stats, docs_i8=d8, docs_scale=dscale)

        for _ in range(max(1, args.warmup)):
            run_cb8()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(args.steps):
            run_cb8()
        e1.record()
        torch.cuda.synchronize()
        ms_cb8 = e0.elapsed_time(e1) / args.steps
        r8 = run_cb8(stats=True)
        torch.cuda.synchronize()
        ids8 = r8["topk_ids"].cpu().numpy()
        st8 = r8["stats"]
        int8 = {"ms": round(ms_cb8, 3), "queries_per_s": round(nq / (ms_cb8 * 1e-3), 1),
                "effective_cells_per_s": round(cells_total / (ms_cb8 * 1e-3), 1),
                "coverage": round(float(sum(s["cells_unique"] for s in st8)) / cells_total, 4),
                "overlap_at_k": round(float(np.mean([len(set(ids_full[q]) & set(ids8[q])) / K
                                                     for q in range(nq)])), 4),
                "overlap_at_k_within_score_tolerance": round(tolerant_overlap(r8["topk_ids"]), 4),
                "mean_rounds": round(float(np.mean([s["rounds"] for s in st8])), 2),
                "speedup_vs_full": round(ms_full / ms_cb8, 2),
                "ms_phases": {k[3:]: round(st8[0][k], 3) for k in
                              ("ms_first_reveal", "ms_later_reveals", "ms_select_prune", "ms_rescore_topk")},
                "survivor_scores_bit_identical_to_full": bool(all(
                    torch.equal(r8["topk_scores"][q], out_full["scores"][q][r8["topk_ids"][q]])
                    for q in range(nq))),
                "corpus_coding_ms_index_time": round(ms_quant, 2),
                "corpus_codes_gb": round(total * d / 1e9, 2)}
        del d8

    # the configuration's second setting, K = 10 (same corpus, same knobs otherwise)
    k10 = None
    if args.K != 10 and N > 15 and not args.no_k10:
        K10 = 10
        out10 = {"topk_ids": torch.empty((nq, K10), dtype=torch.int64, device=dev),
                 "topk_scores": torch.empty((nq, K10), dtype=torch.float32, device=dev)}
        f10 = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K10, workspace=ws, want_scores=False, out=dict(out10))

        def run_cb10(stats=False):
            return B.colbandit_topk(w.Q, w.docs, w.offsets, K10, alpha, delta, M, w.seed, workspace=ws,
                                    want_stats=stats)

        for _ in range(max(1, args.warmup)):
            run_cb10()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            run_cb10()
        e1.record()
        torch.cuda.synchronize()
        ms10 = e0.elapsed_time(e1) / args.steps
        r10 = run_cb10(stats=True)
        torch.cuda.synchronize()
        idf, idc = f10["topk_ids"].cpu().numpy(), r10["topk_ids"].cpu().numpy()
        st10 = r10["stats"]
        k10 = {"K": K10, "ms": round(ms10, 3), "queries_per_s": round(nq / (ms10 * 1e-3), 1),
               "effective_cells_per_s": round(cells_total / (ms10 * 1e-3), 1),
               "coverage": round(float(sum(s["cells_unique"] for s in st10)) / cells_total, 4),
               "overlap_at_k": round(float(np.mean([len(set(idf[q]) & set(idc[q])) / K10 for q in range(nq)])), 4),
               "mean_rounds": round(float(np.mean([s["rounds"] for s in st10])), 2),
               "speedup_vs_full": round(ms_full / ms10, 2),
               "survivor_scores_bit_identical_to_full": bool(torch.equal(
                   r10["topk_scores"], torch.gather(out_full["scores"], 1, r10["topk_ids"].clamp(min=0))))}
        del f10, r10

    # the paper's two non-adaptive baselines at one operating point each (appendix "Compared
    # Methods"): Doc-Uniform at Col-Bandit's own coverage, Ball-carving at tau = 0.8; reported
    # beside the step, not part of `value`
    baselines = None
    if not args.no_baselines and T <= 64:
        def timed_ms(fn):
            fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                r = fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps, r

        overlap_of = lambda ids: round(float(np.mean([len(set(ids_full[q]) & set(ids[q])) / K
                                                      for q in range(nq)])), 4)
        m = B.colbandit_cells_per_doc(coverage, T)
        wsu = torch.empty(int(B.lib().colbandit_doc_uniform_workspace_bytes(nq, T, d, N, total)),
                          dtype=torch.uint8, device=dev)
        ms_u, ru = timed_ms(lambda: B.colbandit_doc_uniform(w.Q, w.docs, w.offsets, K, m, seed=w.seed,
                                                            want_scores=False, workspace=wsu))
        ids_u = ru["topk_ids"].cpu().numpy()
        del wsu, ru
        tau = 0.8
        wsb = torch.empty(int(B.lib().colbandit_ball_carving_workspace_bytes(nq, T, d, B._dt(w.Q), N, total)),
                          dtype=torch.uint8, device=dev)
        ms_b, rb = timed_ms(lambda: B.colbandit_ball_carving(w.Q, w.docs, w.offsets, K, tau,
                                                             want_scores=False, workspace=wsb))
        kq = rb["n_clusters"].cpu().numpy()
        baselines = {
            "doc_uniform": {"cells_per_doc": m, "coverage": round(m / T, 4), "ms": round(ms_u, 3),
                            "overlap_at_k": overlap_of(ids_u), "speedup_vs_full": round(ms_full / ms_u, 2)},
            "ball_carving": {"tau": tau, "mean_clusters": round(float(kq.mean()), 2),
                             "coverage": round(float(kq.mean()) / T, 4), "ms": round(ms_b, 3),
                             "overlap_at_k": overlap_of(rb["topk_ids"].cpu().numpy()),
                             "speedup_vs_full": round(ms_full / ms_b, 2)}}
        del wsb, rb

    flops_full = 2.0 * nq * T * d * total
    tflops = flops_full / (ms_full * 1e-3) / 1e12
    ms_dense = float(np.mean([m[0] for m in ms_kernel]))
    ms_topk = float(np.mean([m[1] for m in ms_kernel]))
    tflops_kernel = flops_full / (ms_dense * 1e-3) / 1e12
    traffic = measured_traffic("%s/nq%d/N%d/tok%d" % (w.name, nq, N, total))
    traffic_rs = measured_traffic("%s/nq%d/N%d/tok%d" % (w.name, nq, N, total), "by_request_size")
    dense = w.dtype == "bf16"
    elem = 2 if dense else 4
    roofline = {"bound": "mfma" if dense else "alu",
                "kernel": "k_dense (Full-MaxSim scoring kernel, bf16 16x16x32 MFMA)" if dense
                          else "k_gather (fp32 inputs)",
                "achieved": round(tflops_kernel, 2), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": round(tflops_kernel / PEAK_BF16_TFLOPS, 4), "traffic": traffic.get("full_maxsim"),
                "traffic_by_request_size": traffic_rs.get("full_maxsim"),
                "ms_per_launch": round(ms_dense, 3),
                "flops_per_launch": flops_full,
                "note": "algorithmic flops 2*T*d per (query, document token) x nq x tokens per "
                        "launch, over the kernel's own duration taken by the library with events "
                        "on the launch stream inside the timed steps; the whole call (kernel + "
                        "chunk table + top-K, %.3f ms) runs at %.1f TFLOP/s; traffic = HBM bytes "
                        "per launch from hardware counters (profiles/hbm_traffic_counters.txt: "
                        "FETCH_SIZE and WRITE_SIZE scaled by their readings for a 1 GiB copy; "
                        "traffic_by_request_size = the L2's memory requests counted by size), "
                        "null unless taken on these kernel sources and this workload"
                        % (ms_full, tflops)}

    # round 1 of Col-Bandit: one pass over the whole corpus that multiplies B query rows per query.
    # Two bounds apply, HBM (the corpus once + the (sum, M2) pair of every (query, document)) and the
    # matrix pipes (2*B*d flops per (query, token)); the larger lower bound on the time is the binding one
    ms_r1 = st[0]["ms_first_reveal"]
    nb1 = min(w.B, T)
    bytes_r1 = float(total) * d * elem + 8.0 * nq * N
    flops_r1 = 2.0 * nq * nb1 * d * total
    t_hbm, t_mfma = bytes_r1 / (PEAK_HBM_GBS * 1e9), flops_r1 / (PEAK_BF16_TFLOPS * 1e12)
    reveal1 = {"kernel": "k_dense<..., REVEAL> (round-1 reveal, corpus-streaming)",
               "ms": round(ms_r1, 3),
               "bound": "mfma" if t_mfma >= t_hbm else "hbm",
               "frac": round(max(t_hbm, t_mfma) * 1e3 / ms_r1, 4) if ms_r1 > 0 else None,
               "hbm": {"achieved": round(bytes_r1 / (ms_r1 * 1e-3) / 1e9, 1) if ms_r1 > 0 else None,
                       "peak": PEAK_HBM_GBS, "unit": "GB/s",
                       "frac": round(t_hbm * 1e3 / ms_r1, 4) if ms_r1 > 0 else None,
                       "bytes": bytes_r1, "traffic": traffic.get("reveal_round1"),
                       "traffic_by_request_size": traffic_rs.get("reveal_round1")},
               "mfma": {"achieved": round(flops_r1 / (ms_r1 * 1e-3) / 1e12, 1) if ms_r1 > 0 else None,
                        "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                        "frac": round(t_mfma * 1e3 / ms_r1, 4) if ms_r1 > 0 else None,
                        "flops": flops_r1},
               "note": "ms = the whole first-reveal phase of the statistics call (k_init, chunk table "
                       "and the reveal kernel; events on the launch stream); frac = the larger of the "
                       "two lower bounds on the time over the measured time"} if dense else None

    # round 2 against the HBM roofline: every (query, document) pair that survives round 1 is
    # streamed once (visit-once cell cache).  Bytes = the tokens of exactly those documents, added
    # up on the device by the prune kernel; ms = the reveal launches of round 2 alone.  The figure
    # over all rounds >= 2 (which adds the launches that find nothing left to gather) is given too.
    pairs2 = float(st[0]["pairs_round2"])
    gather_bytes = float(st[0]["tokens_round2"]) * d * elem
    ms_r2, ms_later = st[0]["ms_reveal_round2"], st[0]["ms_later_reveals"]
    # if round 2 streamed the corpus instead of gathering, or the queries' survivors overlap so
    # much that most gathered bytes come from cache, HBM is not the bound
    gather_valid = ms_r2 > 0 and 2 not in st[0]["corpus_pass_rounds"] and gather_bytes <= 4.0 * total * d * elem
    gbs = lambda ms: round(gather_bytes / (ms * 1e-3) / 1e9, 1) if gather_valid and ms > 0 else None
    gather = {"bound": "hbm", "kernel": "k_gather (round 2: reveal + cell cache fill)",
              "achieved": gbs(ms_r2), "peak": PEAK_HBM_GBS, "unit": "GB/s",
              "frac": round(gbs(ms_r2) / PEAK_HBM_GBS, 4) if gather_valid else None,
              "traffic": traffic.get("gather_round2"),
              "traffic_by_request_size": traffic_rs.get("gather_round2"),
              "pairs": pairs2, "bytes": gather_bytes, "ms": round(ms_r2, 3),
              "all_rounds_ge2": {"ms": round(ms_later, 3), "achieved": gbs(ms_later)},
              "corpus_pass_rounds": st[0]["corpus_pass_rounds"],
              "note": "bytes = document tokens of the (query, document) pairs that entered round 2 x "
                      "row bytes (summed on the device); ms = the reveal launches of round 2 (events, "
                      "statistics call); null when round 2 took the corpus pass or the gathered bytes "
                      "exceed 4x the corpus (then caches serve most of them and HBM is not the bound)"}

    line = {
        "metric": "queries/s through one step = Full-MaxSim top-K + Col-Bandit top-K at N=%d,T=%d,"
                  "d=%d,K=%d (MaxSim cells/s and Overlap@%d vs exhaustive in full_maxsim / "
                  "colbandit)" % (N, T, d, K, K),
        "value": round(nq / (ms_step * 1e-3), 2), "unit": "queries/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "recipe": w.recipe, "n_queries": nq, "N": N, "T": T, "d": d,
                   "total_tokens": total, "K": K, "alpha_ef": alpha, "delta": delta, "M": M, "B": w.B,
                   "workspace_bytes": int(ws.numel()), "corpus_bytes": int(total) * d * elem},
        "full_maxsim": {"ms": round(ms_full, 3), "queries_per_s": round(nq / (ms_full * 1e-3), 1),
                        "cells_per_s": round(cells_total / (ms_full * 1e-3), 1),
                        "tflops": round(tflops, 2), "ms_scoring_kernel": round(ms_dense, 3),
                        "ms_topk": round(ms_topk, 3)},
        "colbandit": {"ms": round(ms_cb, 3), "queries_per_s": round(nq / (ms_cb * 1e-3), 1),
                      "revealed_cells_per_s": round(cells_touched / (ms_cb * 1e-3), 1),
                      "effective_cells_per_s": round(cells_total / (ms_cb * 1e-3), 1),
                      "coverage": round(coverage, 4),
                      "computed_cells_over_all_cells": round(float(sum(s["cells_computed"] for s in st)) / cells_total, 4),
                      "overlap_at_k": round(overlap, 4),
                      "overlap_at_k_within_score_tolerance": round(overlap_tol, 4),
                      "mean_rounds": round(float(np.mean(rounds)), 2),
                      "mean_survivors_after_round1": round(surv1, 1),
                      "mean_survivors_by_round": surv_by_round,
                      "speedup_vs_full": round(ms_full / ms_cb, 2),
                      "ms_phases": {k[3:]: round(st[0][k], 3) for k in
                                    ("ms_first_reveal", "ms_later_reveals", "ms_select_prune",
                                     "ms_rescore_topk")},
                      "survivor_scores_bit_identical_to_full": same_bits},
        "colbandit_k10": k10,
        "colbandit_int8": int8,
        "baselines": baselines,
        "roofline": roofline,
        "roofline_reveal1": reveal1,
        "roofline_gather": gather,
        "paper_context": "paper (CPU, real embeddings): up to ~8x fewer MaxSim FLOPs, up to ~13x "
                         "single-thread CPU speedup at Overlap@5 >= 0.9; no GPU kernel reported",
        "setup_s": round(gen_s, 1),
    }

    if not args.no_cpu_baseline:
        import oracle
        nthreads = oracle.num_threads()
        nq_s = min(nq, nthreads)
        n_s = min(N, args.cpu_sample_docs)
        # a seeded uniform sample of the documents (in index order), not a prefix of the corpus
        sample = np.sort(np.random.default_rng(2602).choice(N, size=n_s, replace=False))
        E, off = w.host_docs(sample.tolist())
        Qh = w.host_queries(list(range(nq_s)))
        pi = np.stack([oracle.permutation(w.seed, q, T) for q in range(nq_s)])
        t0 = time.perf_counter()
        oracle.full_batch(Qh, E, off, min(K, n_s))
        t_full = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.colbandit_batch(Qh, E, off, min(K, n_s), M, w.B, alpha, delta, pi)
        t_cb = time.perf_counter() - t0
        # the same on ONE thread (one query; the oracle threads only across queries)
        t0 = time.perf_counter()
        oracle.full_batch(Qh[:1], E, off, min(K, n_s))
        t_full1 = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.colbandit_batch(Qh[:1], E, off, min(K, n_s), M, w.B, alpha, delta, pi[:1])
        t_cb1 = time.perf_counter() - t0
        scale = n_s / float(N)
        line["cpu_baseline"] = {
            "value": round(nq_s / (t_full + t_cb) * scale, 5), "unit": "queries/s",
            "cores": nthreads, "kind": "oracle",
            "sample": "%d queries x a seeded uniform sample of %d documents of the same corpus, one thread per query; "
                      "%.1f s Full + %.1f s Col-Bandit measured, rate scaled by %d/%d to the full N"
                      % (nq_s, n_s, t_full, t_cb, n_s, N),
            "full_s": round(t_full, 2), "colbandit_s": round(t_cb, 2),
            "single_thread": {"value": round(1.0 / (t_full1 + t_cb1) * scale, 6), "unit": "queries/s",
                              "full_s": round(t_full1, 2), "colbandit_s": round(t_cb1, 2),
                              "colbandit_speedup_vs_full": round(t_full1 / t_cb1, 2)}}
    print(json.dumps(line))


if __name__ == "__main__":
    main()
