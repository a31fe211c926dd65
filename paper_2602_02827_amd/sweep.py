"""Knob sweeps of the two scoring paths on one synthetic configuration.

    python -m paper_2602_02827_amd.sweep --config 4 --alpha 0.05 0.1 0.2 0.5 1.0 --K 1 5 10 50
    python -m paper_2602_02827_amd.sweep --config 4 --alpha 1.0 --K 1 5 10 50 --interval-miss 8
    python -m paper_2602_02827_amd.sweep --config 2 --K 100 500 1000 --M 0 5 10
    python -m paper_2602_02827_amd.sweep --config 2 --nq 1            # single-query latency
    python -m paper_2602_02827_amd.sweep --config 2 --nq 1 --int8     # ... with int8 elimination rounds
    python -m paper_2602_02827_amd.sweep --config 2 --alpha 0.05 0.1 0.2 0.5 1.0 \
        --gamma 0.05 0.1 0.2 0.3 0.5 0.7 0.9 1.0 --tau 0.4 0.5 0.6 0.7 0.8 0.9  # quality-coverage frontier
    python -m paper_2602_02827_amd.sweep --doc-length 16 32 48 106 512 4096 65536  # cost of document ends

Prints one JSON line per (K, alpha_ef, M): batch latency of colbandit_full_maxsim and of
colbandit_topk (events around `--reps` back-to-back asynchronous calls), coverage
(unique revealed cells / (N*T), Sec. 3.1 Eq. (6)), Overlap@K against the exhaustive top-K, mean
rounds and survivors entering the rescore.  `--gamma` / `--tau` add one line per setting of the
paper's two non-adaptive baselines, Doc-Uniform and Ball-carving (appendix "Compared Methods"),
with the same Overlap@K and their coverage (ceil(gamma T)/T, mean k/T).  `--interval-miss Q`
traces the first Q queries of every Col-Bandit setting and counts how often the exhaustive score
of a live document lies outside its decision interval [LCB, UCB] (Theorem 1 and the remark on its
scope: at alpha_ef = 1 the intervals hold jointly with probability 1 - delta only up to the
simplified radius; at alpha_ef < 1 misses are expected).  `--doc-length L ...` runs nothing of
the above: it times the exhaustive scoring kernel on 53 M random bf16 tokens (the token count of
configuration 3, 128 queries x 32 tokens, d = 128) cut into documents of one length L each, one
JSON line per L; the work per token is the same for every L, so the differences are the cost of
the document boundaries.  The grid of alpha_ef x K follows the knob sweeps of
the paper's evaluation (Sec. 5, implementation appendix "Default parameter setting").
"""
from __future__ import annotations

import argparse
import json
import sys


def doc_length_sweep(lengths, reps, d):
    """Exhaustive scoring kernel (Eq. (1)-(3)) against the document length at a fixed token count."""
    import torch
    from . import binding as B

    nq, T, total = 128, 32, 53_000_000
    g = torch.Generator(device="cuda").manual_seed(1)
    docs = torch.empty((total, d), dtype=torch.bfloat16, device="cuda")
    for i in range(0, total, 1 << 22):
        n = min(1 << 22, total - i)
        docs[i:i + n] = torch.randn((n, d), generator=g, device="cuda").to(torch.bfloat16)
    Q = torch.randn((nq, T, d), generator=g, device="cuda").to(torch.bfloat16)
    for L in lengths:
        N = total // L
        off = torch.arange(N + 1, dtype=torch.int64, device="cuda") * L
        tok = N * L
        ws = B.new_workspace(nq, T, d, N, tok, "cuda")
        out = {"scores": torch.empty((nq, N), dtype=torch.float32, device="cuda"),
               "topk_ids": torch.empty((nq, 5), dtype=torch.int64, device="cuda"),
               "topk_scores": torch.empty((nq, 5), dtype=torch.float32, device="cuda")}
        for _ in range(2):
            B.colbandit_full_maxsim(Q, docs[:tok], off, K=5, workspace=ws, out=out)
        torch.cuda.synchronize()
        ms = [B.colbandit_full_maxsim(Q, docs[:tok], off, K=5, workspace=ws, out=out,
                                      want_phase_ms=True)["phase_ms"][0] for _ in range(max(reps, 1))]
        mean = sum(ms) / len(ms)
        flops = 2.0 * nq * T * d * tok
        print(json.dumps({"doc_length": L, "N": N, "tokens": tok, "nq": nq, "T": T, "d": d,
                          "ms_scoring_kernel": [round(m, 3) for m in ms],
                          "tflops": round(flops / mean / 1e9, 1),
                          "frac_of_bf16_mfma_peak": round(flops / mean / 1e9 / 2500.0, 4)}), flush=True)
        del ws, out
    return 0


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=4)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--nq", type=int, default=None)
    ap.add_argument("--d", type=int, default=128, help="embedding width (128, or 64)")
    ap.add_argument("--alpha", type=float, nargs="+", default=[0.2])
    ap.add_argument("--K", type=int, nargs="+", default=[5])
    ap.add_argument("--M", type=int, nargs="+", default=[5])
    ap.add_argument("--B", type=int, default=4)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--gamma", type=float, nargs="*", default=[],
                    help="Doc-Uniform budgets (fraction of the T cells revealed per document)")
    ap.add_argument("--tau", type=float, nargs="*", default=[],
                    help="Ball-carving cosine thresholds")
    ap.add_argument("--int8", action="store_true",
                    help="run the elimination rounds on int8 codes of the corpus (coded once, untimed)")
    ap.add_argument("--interval-miss", type=int, default=0, metavar="Q",
                    help="trace the first Q queries and count live documents whose exhaustive score "
                         "leaves [LCB, UCB]")
    ap.add_argument("--doc-length", type=int, nargs="+", default=[], metavar="L",
                    help="time the exhaustive kernel on 53 M random tokens cut into documents of L tokens")
    args = ap.parse_args(argv)

    import numpy as np
    import torch
    from . import binding as B, synth

    assert torch.cuda.is_available(), "sweep needs a GPU"
    B.lib()
    if args.doc_length:
        return doc_length_sweep(args.doc_length, args.reps, args.d)
    w = synth.config(args.config, device="cuda", scale=args.scale, nq=args.nq, d=args.d)
    nq, T, d, N, total = w.nq, w.T, w.d, w.N, w.total_tokens
    ws = B.new_workspace(nq, T, d, N, total, "cuda")

    ckw = {}
    if args.int8:
        d8, ds = B.colbandit_quantize_i8(w.docs)
        ckw = {"docs_i8": d8, "docs_scale": ds}

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.reps

    nmiss = min(args.interval_miss, nq)
    S_traced = None
    if nmiss > 0:       # exhaustive scores of the traced queries (the bounds are about these)
        S_traced = B.colbandit_full_maxsim(w.Q[:nmiss].contiguous(), w.docs, w.offsets, K=0)["scores"].cpu().numpy()

    def interval_misses(K, alpha, M):
        """Theorem 1's event on the traced queries: per (round, live document), is the exhaustive
        score inside [LCB, UCB]?  The bounds are fp32 on the device: 1e-4 of slack."""
        r = B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, w.delta, M, w.seed, B=args.B,
                             workspace=ws, trace=True, trace_queries=list(range(nmiss)))
        tr = r["trace"]
        checks = misses = q_miss = below = 0
        for q in range(nmiss):
            any_miss = False
            for rr in range(r["stats"][q]["rounds"]):
                live = ~np.isnan(tr.lcb[rr, q])
                lo = S_traced[q][live] < tr.lcb[rr, q][live] - 1e-4
                hi = S_traced[q][live] > tr.ucb[rr, q][live] + 1e-4
                checks += int(live.sum())
                misses += int(lo.sum() + hi.sum())
                below += int(lo.sum())
                any_miss |= bool(lo.any() or hi.any())
            q_miss += any_miss
        return {"traced_queries": nmiss, "interval_checks": checks, "misses": misses,
                "misses_score_below_lcb": below, "miss_rate": round(misses / max(1, checks), 6),
                "queries_with_a_miss": q_miss, "delta": w.delta}

    for K in args.K:
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws, want_scores=False)
        ms_full = timed(lambda: B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws,
                                                        want_scores=False, out=full))
        ids_full = full["topk_ids"].cpu().numpy()
        overlap_of = lambda ids: float(np.mean([len(set(ids_full[q]) & set(ids[q])) / K for q in range(nq)]))
        # the scoring kernel alone (the library's own events), mean of `reps` launches
        nrep = max(args.reps, 1)
        ms_kernel = sum(B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws, want_scores=False,
                                                out=full, want_phase_ms=True)["phase_ms"][0]
                        for _ in range(nrep)) / nrep
        head = {"workload": w.name, "n_queries": nq, "N": N, "T": T, "d": d, "K": K,
                "full_ms": round(ms_full, 3), "full_kernel_ms": round(ms_kernel, 3)}
        if args.gamma:
            wsu = torch.empty(int(B.lib().colbandit_doc_uniform_workspace_bytes(nq, T, d, N, total)),
                              dtype=torch.uint8, device="cuda")
            for gamma in args.gamma:
                m = B.colbandit_cells_per_doc(gamma, T)
                run = lambda: B.colbandit_doc_uniform(w.Q, w.docs, w.offsets, K, m, seed=w.seed,
                                                      want_scores=False, workspace=wsu)
                ms = timed(run)
                ids = run()["topk_ids"].cpu().numpy()
                print(json.dumps({**head, "method": "doc_uniform", "gamma": gamma, "cells_per_doc": m,
                                  "ms": round(ms, 3), "speedup": round(ms_full / ms, 2),
                                  "coverage": round(m / T, 4), "overlap_at_k": round(overlap_of(ids), 4)}),
                      flush=True)
            del wsu
        if args.tau:
            wsb = torch.empty(int(B.lib().colbandit_ball_carving_workspace_bytes(nq, T, d, B._dt(w.Q), N, total)),
                              dtype=torch.uint8, device="cuda")
            for tau in args.tau:
                run = lambda: B.colbandit_ball_carving(w.Q, w.docs, w.offsets, K, tau,
                                                       want_scores=False, workspace=wsb)
                ms = timed(run)
                r = run()
                ids = r["topk_ids"].cpu().numpy()
                kq = r["n_clusters"].cpu().numpy()
                print(json.dumps({**head, "method": "ball_carving", "tau": tau, "ms": round(ms, 3),
                                  "speedup": round(ms_full / ms, 2),
                                  "coverage": round(float(kq.mean()) / T, 4),
                                  "mean_clusters": round(float(kq.mean()), 2),
                                  "columns_scored": int((4 * ((kq + 3) // 4)).sum()),
                                  "overlap_at_k": round(overlap_of(ids), 4)}), flush=True)
            del wsb
        for alpha in args.alpha:
            for M in args.M:
                run = lambda stats=False: B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, w.delta, M,
                                                           w.seed, B=args.B, workspace=ws, want_stats=stats, **ckw)
                ms_cb = timed(run)
                res = run(True)
                torch.cuda.synchronize()
                ids = res["topk_ids"].cpu().numpy()
                st = res["stats"]
                overlap = float(np.mean([len(set(ids_full[q]) & set(ids[q])) / K for q in range(nq)]))
                cov = sum(s["cells_unique"] for s in st) / (float(nq) * N * T)
                extra = {"interval_miss": interval_misses(K, alpha, M)} if nmiss > 0 else {}
                print(json.dumps({
                    "workload": w.name, "n_queries": nq, "N": N, "T": T, "d": d, "K": K,
                    "method": "colbandit", "alpha_ef": alpha,
                    "M": M, "B": args.B, "reveals": "int8" if args.int8 else w.dtype, "full_ms": round(ms_full, 3), "full_kernel_ms": round(ms_kernel, 3), "colbandit_ms": round(ms_cb, 3),
                    "speedup": round(ms_full / ms_cb, 2), "coverage": round(cov, 4),
                    "computed_cells_over_all_cells": round(sum(s["cells_computed"] for s in st) / (float(nq) * N * T), 4),
                    "overlap_at_k": round(overlap, 4),
                    "mean_rounds": round(float(np.mean([s["rounds"] for s in st])), 2),
                    "mean_rescored": round(float(np.mean([s["survivors"][s["rounds"]] for s in st])), 1),
                    "ms_phases": {k[3:]: round(st[0][k], 3) for k in
                                  ("ms_first_reveal", "ms_later_reveals", "ms_select_prune", "ms_rescore_topk")},
                    "corpus_pass_rounds": st[0]["corpus_pass_rounds"], **extra,
                }), flush=True)


if __name__ == "__main__":
    sys.exit(main())
