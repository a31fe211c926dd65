"""GPU <-> oracle parity through the C-ABI (run with -m gpu on an MI355X).

Tolerances (relative, on scores): 1e-5 for fp32 inputs, 2e-3 for bf16 inputs with fp32
accumulation; the oracle reads the same storage-rounded values.  Index results are exact
wherever the deciding gap exceeds the tolerance.  The Col-Bandit rounds are compared by
feeding the oracle the GPU's own MaxSim cells, so that only the bookkeeping differs; a
document may then differ only if its UCB lies within EPS_BAND of the round's threshold.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}
EPS_BAND = 2e-4          # fp32 bound arithmetic vs the oracle's double, on values of size <= T


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2602_02827_amd import binding
    binding.lib()          # raises if the HIP library is not built: no fallback
    return binding


@pytest.fixture(scope="module")
def S():
    from paper_2602_02827_amd import synth
    return synth


def _custom(S, lengths, nq, T, d, dtype, seed):
    """Corpus with prescribed document lengths (iid unit tokens), on the GPU."""
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    L = torch.tensor(lengths, dtype=torch.int64)
    off = torch.zeros(len(lengths) + 1, dtype=torch.int64); off[1:] = torch.cumsum(L, 0)
    E = torch.randn((int(off[-1]), d), generator=g)
    E = E / E.norm(dim=1, keepdim=True)
    Q = torch.randn((nq, T, d), generator=g)
    Q = Q / Q.norm(dim=2, keepdim=True)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    return S.Workload(f"custom-{dtype}", dtype, Q.to(td).cuda(), E.to(td).cuda(), off.cuda(), seed=seed)


def _oracle_scores(oracle_mod, w, qs=None):
    E, off = w.host_docs()
    Qh = w.host_queries()
    qs = range(w.nq) if qs is None else qs
    H = np.stack([oracle_mod.maxsim_cells(Qh[q], E, off) for q in qs])
    return H, H.sum(axis=2)


def _check_topk(ids, scores, S_or, K, tol):
    """ids/scores: GPU top-K of one query; S_or: oracle scores of all docs."""
    order = np.lexsort((np.arange(len(S_or)), -S_or))
    kth = S_or[order[K - 1]]
    band = tol * max(1.0, abs(kth))
    assert len(set(ids.tolist())) == K
    assert np.all(np.diff(scores) <= 0)                       # returned in score order
    assert np.all(S_or[ids] >= kth - band)                    # nothing clearly below the cut
    must = order[:K][S_or[order[:K]] > kth + band]            # clearly above the cut
    assert set(must.tolist()) <= set(ids.tolist())
    np.testing.assert_allclose(scores, S_or[ids], rtol=tol, atol=tol)
    gaps = -np.diff(S_or[order[:K + 1]]) if len(S_or) > K else -np.diff(S_or[order[:K]])
    if np.all(gaps > 2 * band):                                # no near-ties: exact order
        np.testing.assert_array_equal(ids, order[:K])


# ------------------------------------------------------------------ Full-MaxSim
def test_full_maxsim_fp32_config1(B, S, oracle_mod):
    w = S.config(0, device="cuda")                              # N=1000, fp32, 1 query
    H, Sor = _oracle_scores(oracle_mod, w)
    r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=5, want_cells=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(r["cells"].cpu().numpy(), H, rtol=1e-5, atol=1e-6)
    np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=1e-5, atol=1e-6)
    _check_topk(r["topk_ids"][0].cpu().numpy(), r["topk_scores"][0].cpu().numpy(), Sor[0], 5, 1e-5)
    assert set(w.planted[0]) == set(r["topk_ids"][0].tolist())  # the planted docs are the top-5


@pytest.mark.parametrize("nq,T,d", [(1, 32, 128), (3, 32, 128), (6, 24, 128), (20, 32, 128),
                                     (5, 7, 128), (3, 40, 128), (2, 100, 128), (4, 32, 64),
                                     (40, 16, 64), (4, 32, 96), (3, 24, 32), (2, 100, 96)])
def test_full_maxsim_bf16_dense_ragged(B, S, oracle_mod, nq, T, d):
    # lengths span 1 token, block edges (15/16/17), stage edges (63/64/65), ring wrap (>256)
    # and documents longer than a workgroup's token chunk (4096)
    rng = np.random.default_rng(nq * 1000 + T)
    lengths = [1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 127, 129, 255, 257, 700, 1030, 4500, 1] + \
        rng.integers(1, 200, 150).tolist() + [5000, 3] + rng.integers(30, 181, 100).tolist()
    w = _custom(S, lengths, nq, T, d, "bf16", 7)
    H, Sor = _oracle_scores(oracle_mod, w)
    r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=7, want_cells=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(r["cells"].cpu().numpy(), H, rtol=TOL["bf16"], atol=1e-5)
    np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=TOL["bf16"], atol=1e-4)
    # fp32 accumulation of exact bf16 products is far tighter than the stated tolerance
    assert np.abs(r["scores"].cpu().numpy() - Sor).max() < 5e-5 * T
    for q in range(nq):
        _check_topk(r["topk_ids"][q].cpu().numpy(), r["topk_scores"][q].cpu().numpy(), Sor[q], 7,
                    TOL["bf16"])


def test_documents_much_longer_than_a_token_chunk(B, S, oracle_mod):
    """Documents of several chunks leave runs of empty chunks behind them (a chunk belongs to the
    document that starts in it); every workgroup with an empty chunk must exit and the others
    must cover the long rows - exhaustive cells for a wide and a narrow batch, and the reveal
    pass through Col-Bandit's first round."""
    lengths = [20000, 3, 9000, 1, 1, 4096, 4097, 8192, 17, 12289, 40]
    for nq in (1, 2, 20):       # one query: the wavefronts of a workgroup split the documents
        w = _custom(S, lengths, nq, 32, 128, "bf16", 5 + nq)
        H, Sor = _oracle_scores(oracle_mod, w)
        r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=3, want_cells=True)
        torch.cuda.synchronize()
        np.testing.assert_allclose(r["cells"].cpu().numpy(), H, rtol=TOL["bf16"], atol=1e-5)
        np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=TOL["bf16"], atol=1e-4)
    w = _custom(S, lengths, 3, 32, 128, "bf16", 9)
    _run_colbandit_case(B, oracle_mod, w, 2, 1, 4, 0.5, seed=3)


def test_full_maxsim_fp32_ragged_and_d64(B, S, oracle_mod):
    rng = np.random.default_rng(5)
    lengths = [1, 16, 17, 300] + rng.integers(1, 90, 120).tolist()
    for d, T in [(128, 32), (64, 24), (128, 50), (96, 32), (32, 40)]:
        w = _custom(S, lengths, 3, T, d, "f32", 11)
        H, Sor = _oracle_scores(oracle_mod, w)
        r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=4, want_cells=True)
        torch.cuda.synchronize()
        np.testing.assert_allclose(r["cells"].cpu().numpy(), H, rtol=1e-5, atol=1e-6)
        np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=1e-5, atol=1e-6)


def test_documents_without_tokens_get_minus_infinity_and_disturb_nothing(B, S, oracle_mod):
    """Empty documents violate the input contract (colbandit_validate_offsets reports them), but
    the scoring kernels must stay in bounds: such a document scores -inf and its neighbours,
    which share 16-token blocks with it, keep their exact scores."""
    rng = np.random.default_rng(41)
    lengths = rng.integers(1, 40, 400).tolist()
    for i in (0, 1, 7, 8, 9, 100, 250, 251, 252, 399):
        lengths[i] = 0
    for nq in (3, 1):
        w = _custom(S, lengths, nq, 32, 128, "bf16", 43)
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=0)
        torch.cuda.synchronize()
        got = full["scores"].cpu().numpy()
        keep = [i for i, n in enumerate(lengths) if n > 0]
        E, off = w.host_docs(keep)
        Qh = w.host_queries()
        for q in range(w.nq):
            want = oracle_mod.row_sums(oracle_mod.maxsim_cells(Qh[q], E, off))
            np.testing.assert_allclose(got[q][keep], want, rtol=TOL["bf16"], atol=1e-4)
            assert np.all(np.isneginf(got[q][[i for i, n in enumerate(lengths) if n == 0]]))


def test_nan_rows_and_token_less_documents_do_not_damage_other_documents(B, S, oracle_mod):
    """Inputs outside the contract: one document whose embeddings are NaN, one without tokens.
    Their own scores are meaningless, but they must neither enter a top-K nor wipe out a query's
    threshold: every other document keeps its exact score, the exhaustive top-K is the ordered
    head of the valid scores, and Col-Bandit returns K valid documents with those scores."""
    rng = np.random.default_rng(61)
    lengths = rng.integers(20, 90, 1200).tolist()
    p_nan, r_empty = 333, 700
    lengths[r_empty] = 0
    w = _custom(S, lengths, 4, 32, 128, "bf16", 67)
    off = w.offsets.cpu().numpy()
    w.docs[int(off[p_nan]):int(off[p_nan + 1])] = float("nan")
    K = 6
    full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K)
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.3, 0.01, 5, 8, trace=True)
    plain = B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.3, 0.01, 5, 8)       # untraced code paths
    gathered = B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.3, 0.01, 5, 8, force_gather=True,
                                no_cell_cache=True)
    torch.cuda.synchronize()
    for other in (plain, gathered):
        assert torch.equal(other["topk_ids"], res["topk_ids"])
        assert torch.equal(other["topk_scores"], res["topk_scores"])
    sc = full["scores"].cpu().numpy()
    bad = np.array([p_nan, r_empty])
    good = np.setdiff1d(np.arange(w.N), bad)
    # the hardware maximum drops a NaN operand, so the NaN document scores -inf (NaN would do too)
    assert np.all(np.isnan(sc[:, p_nan]) | np.isneginf(sc[:, p_nan])) and np.all(np.isneginf(sc[:, r_empty]))
    E, offg = w.host_docs(good.tolist())
    for q in range(w.nq):
        want = oracle_mod.row_sums(oracle_mod.maxsim_cells(w.host_queries()[q], E, offg))
        np.testing.assert_allclose(sc[q][good], want, rtol=TOL["bf16"], atol=1e-4)
        order = good[np.lexsort((good, -sc[q][good]))][:K]
        np.testing.assert_array_equal(full["topk_ids"][q].cpu().numpy(), order)
        ids = res["topk_ids"][q].cpu().numpy()
        assert len(set(ids.tolist())) == K and not (set(ids.tolist()) & set(bad.tolist())) and ids.min() >= 0
        np.testing.assert_array_equal(res["topk_scores"][q].cpu().numpy(), sc[q][ids])
        st = res["stats"][q]
        assert st["rounds"] >= 1 and st["survivors"][st["rounds"]] >= K
        assert not res["trace"].alive[0, q][bad].any()          # both dropped in the first round
        assert not np.isnan(res["trace"].tau[0, q])


def test_topk_ties_resolve_to_lower_index(B, S):
    # documents 10.. are exact copies of documents 0..9 -> exact score ties
    base = _custom(S, [20] * 10, 2, 32, 128, "bf16", 3)
    docs = torch.cat([base.docs, base.docs, base.docs])
    off = (torch.arange(31, dtype=torch.int64) * 20).cuda()
    r = B.colbandit_full_maxsim(base.Q, docs, off, K=12)
    torch.cuda.synchronize()
    sc = r["scores"].cpu().numpy()
    np.testing.assert_array_equal(sc[:, :10], sc[:, 10:20])
    for q in range(2):
        order = np.lexsort((np.arange(30), -sc[q]))[:12]
        np.testing.assert_array_equal(r["topk_ids"][q].cpu().numpy(), order)


def test_mid_text_config2_scaled(B, S, oracle_mod):
    w = S.config(1, device="cuda", scale=0.06, nq=8)            # N=3000, bf16, planted docs
    H, Sor = _oracle_scores(oracle_mod, w)
    r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=5)
    torch.cuda.synchronize()
    np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=TOL["bf16"], atol=1e-4)
    for q in range(w.nq):
        _check_topk(r["topk_ids"][q].cpu().numpy(), r["topk_scores"][q].cpu().numpy(), Sor[q], 5,
                    TOL["bf16"])


# ------------------------------------------------------------------ Col-Bandit
def _compare_rounds(oracle_mod, tr, q, Hq, K, M, Bsz, alpha, delta, pi, a=-1.0, b=1.0, Hexact=None):
    """Oracle on the GPU's cells vs the GPU trace, EVERY executed round of query column q.

    Each round's live set, LCB, UCB (within EPS_BAND) and threshold are compared; the survivor
    sets may differ only at documents whose UCB lies within 2*EPS_BAND of the threshold.  When
    such a band document makes the two survivor sets differ, the oracle is entered again at the
    next round with the GPU's own active set (oracle.colbandit_resume) and the comparison goes
    on to the last round, so no later round escapes.  Returns (number of re-entries, the oracle
    result that the last rounds were compared with); its final_ids are the GPU's final set.
    Hexact: the rounds decide on Hq (coarse cells) and the rescore reads Hexact."""
    N, T = Hq.shape
    if Hexact is None:
        orc = oracle_mod.colbandit_from_H(Hq, K, M, Bsz, alpha, delta, pi, a, b)
    else:
        orc = oracle_mod.colbandit_coarse(Hq, Hexact, K, M, Bsz, alpha, delta, pi, a, b)
    reentries = 0
    r = 0
    while r < orc.rounds:
        assert tr.count[r, q] == orc.counts[r], (q, r)
        live = ~np.isnan(orc.lcb[r])
        g_live = ~np.isnan(tr.lcb[r, q])
        np.testing.assert_array_equal(g_live, live)
        np.testing.assert_allclose(tr.lcb[r, q][live], orc.lcb[r][live], rtol=0, atol=EPS_BAND)
        np.testing.assert_allclose(tr.ucb[r, q][live], orc.ucb[r][live], rtol=0, atol=EPS_BAND)
        assert abs(tr.tau[r, q] - orc.tau[r]) <= EPS_BAND, (q, r)
        assert not np.any(tr.alive[r, q] & ~live), (q, r)         # nobody comes back
        mism = np.flatnonzero(tr.alive[r, q] != orc.alive[r])
        if len(mism):
            assert np.all(np.abs(orc.ucb[r][mism] - orc.tau[r]) <= 2 * EPS_BAND), (q, r, mism)
            reentries += 1
            orc = oracle_mod.colbandit_resume(Hq, K, M, Bsz, alpha, delta, pi,
                                              np.flatnonzero(tr.alive[r, q]), r + 2, a, b,
                                              H_exact=Hexact)
        r += 1
    # the GPU ran exactly these rounds, and its last active set is the oracle's final set
    assert tr.count[orc.rounds, q] == orc.counts[orc.rounds], q
    if orc.rounds < tr.tau.shape[0]:
        assert np.isnan(tr.tau[orc.rounds, q]), q                  # no further round ran
    if orc.rounds >= 1:
        np.testing.assert_array_equal(np.flatnonzero(tr.alive[orc.rounds - 1, q]), orc.final_ids)
    return reentries, orc


def _run_colbandit_case(B, oracle_mod, w, K, M, Bsz, alpha, delta=0.01, seed=0, a=0.0, b=0.0,
                        force_gather=False, later_rounds=0, coarse=None, **kw):
    """coarse = (docs_i8, docs_scale): the rounds run on int8 codes; the oracle then decides on
    the GPU's coarse cells and rescored from its exact ones.  Every round of every query is
    compared (see _compare_rounds); the number of queries that needed a re-entry at a band
    document is bounded as a sanity check on the band's width."""
    full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=0, want_cells=True)
    ckw = {} if coarse is None else {"docs_i8": coarse[0], "docs_scale": coarse[1]}
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, delta, M, seed, B=Bsz, a=a, b=b,
                           trace=True, force_gather=force_gather, later_rounds=later_rounds, **ckw, **kw)
    Hc = None
    if coarse is not None:
        cm = B.colbandit_coarse_maxsim(w.Q, coarse[0], coarse[1], w.offsets, want_cells=True)
        torch.cuda.synchronize()
        Hc = cm["cells"].cpu().numpy().astype(np.float64)
    torch.cuda.synchronize()
    H = full["cells"].cpu().numpy().astype(np.float64)
    Sfull = full["scores"].cpu().numpy()
    ids = res["topk_ids"].cpu().numpy()
    sc = res["topk_scores"].cpu().numpy()
    tr = res["trace"]
    aa, bb = (-1.0, 1.0) if a == 0.0 and b == 0.0 else (a, b)
    diverged = 0
    for q in range(w.nq):
        pi = B.colbandit_permutation(seed, q, w.T)
        np.testing.assert_array_equal(pi, oracle_mod.permutation(seed, q, w.T))
        if Hc is None:
            div, orc = _compare_rounds(oracle_mod, tr, q, H[q], K, M, Bsz, alpha, delta, pi, aa, bb)
        else:
            div, orc = _compare_rounds(oracle_mod, tr, q, Hc[q], K, M, Bsz, alpha, delta, pi, aa, bb,
                                       Hexact=H[q])
        st = res["stats"][q]
        # survivor scores carry the same bits as the exhaustive path
        ok = ids[q] >= 0
        np.testing.assert_array_equal(sc[q][ok], Sfull[q][ids[q][ok]])
        # accounting identity (cells touched) from the GPU's own survivor counts
        T = w.T
        cells = sum((min((r + 1) * Bsz, T) - r * Bsz) * st["survivors"][r] for r in range(st["rounds"]))
        assert st["cells_elim"] == cells
        assert st["cells_rescore"] == T * st["survivors"][st["rounds"]]
        n_last = min(st["rounds"] * Bsz, T)
        assert st["cells_unique"] == cells + (T - n_last) * st["survivors"][st["rounds"]]
        assert st["survivors"] == [int(x) for x in tr.count[: st["rounds"] + 1, q]]
        # rounds, final set and top-K against the oracle that saw the GPU's active sets
        assert st["rounds"] == orc.rounds
        kk = min(K, len(orc.final_ids))
        fin_scores = Sfull[q][orc.final_ids].astype(np.float64)
        order = orc.final_ids[np.lexsort((orc.final_ids, -fin_scores))][:kk]
        np.testing.assert_array_equal(ids[q][:kk], order)
        assert np.all(ids[q][kk:] == -1)
        assert st["cells_rescore"] == orc.cells_rescore
        if div == 0:
            assert (st["cells_elim"], st["cells_unique"]) == (orc.cells_elim, orc.cells_unique)
        else:
            diverged += 1
    assert diverged <= max(1, int(0.15 * w.nq)), diverged
    # what a gathered round 2 has to read: the pairs that entered it and their document tokens
    if tr.count.shape[0] >= 3:
        L = np.diff(w.offsets.cpu().numpy())
        goes_on = [q for q in range(w.nq) if res["stats"][q]["rounds"] >= 1 and tr.count[1, q] > K + M]
        assert res["stats"][0]["pairs_round2"] == sum(int(tr.count[1, q]) for q in goes_on)
        assert res["stats"][0]["tokens_round2"] == sum(int(L[tr.alive[0, q]].sum()) for q in goes_on)
    return res, tr


def test_colbandit_fp32_config1(B, S, oracle_mod):
    w = S.config(0, device="cuda")
    res, tr = _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 0.2)
    # end to end against the oracle working from the embeddings themselves
    E, off = w.host_docs()
    pi = oracle_mod.permutation(0, 0, w.T)
    orc = oracle_mod.colbandit_lazy(w.host_queries()[0], E, off, 5, 5, 4, 0.2, 0.01, pi)
    np.testing.assert_array_equal(res["topk_ids"][0].cpu().numpy(), orc.topk_ids)
    np.testing.assert_allclose(res["topk_scores"][0].cpu().numpy(), orc.topk_scores, rtol=1e-5)
    assert res["stats"][0]["cells_unique"] == orc.cells_unique
    assert set(w.planted[0]) == set(orc.topk_ids.tolist())


@pytest.mark.parametrize("alpha,K,M,Bsz", [(0.2, 5, 5, 4), (1.0, 5, 5, 4), (0.05, 1, 0, 4),
                                           (0.2, 50, 5, 4), (0.5, 10, 5, 3), (0.2, 5, 5, 16),
                                           (0.2, 5, 0, 1), (1.0, 3, 2, 5)])
def test_colbandit_bf16_rounds_match_oracle(B, S, oracle_mod, alpha, K, M, Bsz):
    w = S.config(1, device="cuda", scale=0.04, nq=6)            # N=2000, planted docs
    _run_colbandit_case(B, oracle_mod, w, K, M, Bsz, alpha)


def test_colbandit_topic_corpus_and_pages(B, S, oracle_mod):
    w = S.config(2, device="cuda", scale=0.008, nq=10)          # N=4000 topic mixture
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 0.2)
    _run_colbandit_case(B, oracle_mod, w, 10, 5, 4, 0.2, seed=9)
    w = S.config(3, device="cuda", scale=0.01, nq=5)            # 200 pages x 1030 tokens, T=24
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 0.2)
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 1.0)


def test_colbandit_gather_and_dense_first_round_agree(B, S, oracle_mod):
    w = S.config(1, device="cuda", scale=0.03, nq=5)
    r1 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 3, trace=True)
    r2 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 3, trace=True, force_gather=True)
    torch.cuda.synchronize()
    for f in ("count", "tau", "lcb", "ucb", "alive"):
        np.testing.assert_array_equal(getattr(r1["trace"], f), getattr(r2["trace"], f))
    assert torch.equal(r1["topk_ids"], r2["topk_ids"]) and torch.equal(r1["topk_scores"], r2["topk_scores"])


def _same_run(r1, r2):
    for f in ("count", "tau", "lcb", "ucb", "alive"):
        np.testing.assert_array_equal(getattr(r1["trace"], f), getattr(r2["trace"], f))
    assert torch.equal(r1["topk_ids"], r2["topk_ids"]) and torch.equal(r1["topk_scores"], r2["topk_scores"])
    # which path computed a round's cells may differ between the runs; nothing else may
    counts = lambda st: {k: v for k, v in st.items() if not k.startswith("ms_")
                         and k not in ("corpus_pass_rounds", "cells_computed")}
    assert [counts(a) for a in r1["stats"]] == [counts(b) for b in r2["stats"]]


@pytest.mark.parametrize("alpha,Bsz,T", [(0.2, 4, 32), (1.0, 4, 32), (0.5, 3, 24), (0.2, 8, 40), (1.0, 16, 100)])
def test_cell_cache_and_regather_give_identical_runs(B, S, alpha, Bsz, T):
    """Caching a visited document's cells must not change a single decision or bit."""
    rng = np.random.default_rng(T)
    w = _custom(S, rng.integers(1, 120, 1500).tolist(), 4, T, 128, "bf16", 5)
    r1 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, alpha, 0.01, 5, 3, B=Bsz, trace=True)
    r2 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, alpha, 0.01, 5, 3, B=Bsz, trace=True,
                          no_cell_cache=True)
    torch.cuda.synchronize()
    assert max(s["rounds"] for s in r1["stats"]) >= 2
    _same_run(r1, r2)


@pytest.mark.parametrize("alpha,Bsz,T,nq", [(1.0, 4, 32, 4), (0.5, 3, 24, 9), (1.0, 16, 100, 2), (0.2, 4, 32, 40)])
def test_later_rounds_by_corpus_pass_or_by_gather_are_identical(B, S, oracle_mod, alpha, Bsz, T, nq):
    """Rounds >= 2 revealed by the corpus-streaming pass (merged into the running statistics by
    the prune kernel), by per-pair gathers, or by the device-side choice between them: the
    same cells, the same merge, so every bound, threshold, survivor and output bit agrees."""
    rng = np.random.default_rng(100 + T)
    w = _custom(S, rng.integers(1, 90, 3000).tolist(), nq, T, 128, "bf16", 17)
    runs = [B.colbandit_topk(w.Q, w.docs, w.offsets, 5, alpha, 0.01, 5, 4, B=Bsz, trace=True,
                             later_rounds=m) for m in (2, 1, 0)]
    torch.cuda.synchronize()
    assert max(s["rounds"] for s in runs[0]["stats"]) >= 3
    _same_run(runs[0], runs[1])
    _same_run(runs[0], runs[2])
    # the statistics name the rounds that streamed the corpus: none when gathers are forced,
    # every round >= 2 that still had an ids-mode query when the pass is forced
    assert all(s["corpus_pass_rounds"] == [] for s in runs[0]["stats"])
    forced = runs[1]["stats"][0]["corpus_pass_rounds"]
    assert forced and forced[0] == 2 and forced == list(range(2, 2 + len(forced)))
    assert set(runs[2]["stats"][0]["corpus_pass_rounds"]) <= set(forced)
    # the streaming pass also under the cache-free mode, and against the oracle
    r3 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, alpha, 0.01, 5, 4, B=Bsz, trace=True,
                          later_rounds=1, no_cell_cache=True)
    torch.cuda.synchronize()
    _same_run(runs[0], r3)
    _run_colbandit_case(B, oracle_mod, w, 5, 5, Bsz, alpha, seed=4, later_rounds=1)


def test_device_side_choice_takes_the_corpus_pass_for_large_active_sets(B, S):
    """A conservative radius on a topic corpus keeps thousands of documents per query alive:
    the automatic mode must then not fall behind the exhaustive path by gathering them all."""
    w = S.config(4, device="cuda", scale=0.2, nq=64)                 # N=20,000, 64 queries
    ws = B.new_workspace(w.nq, w.T, w.d, w.N, w.total_tokens, "cuda")
    res = {}
    for m in (0, 2):
        r = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 1.0, 0.01, 5, w.seed, workspace=ws,
                             later_rounds=m)
        res[m] = r
    torch.cuda.synchronize()
    assert torch.equal(res[0]["topk_ids"], res[2]["topk_ids"])
    assert torch.equal(res[0]["topk_scores"], res[2]["topk_scores"])
    c = lambda st: {k: v for k, v in st.items() if not k.startswith("ms_")
                    and k not in ("corpus_pass_rounds", "cells_computed")}
    assert [c(a) for a in res[0]["stats"]] == [c(b) for b in res[2]["stats"]]
    assert 2 in res[0]["stats"][0]["corpus_pass_rounds"] and res[2]["stats"][0]["corpus_pass_rounds"] == []
    print("later reveals: auto %.3f ms, gather %.3f ms" %
          (res[0]["stats"][0]["ms_later_reveals"], res[2]["stats"][0]["ms_later_reveals"]))


def test_cells_computed_counts_what_the_kernels_multiply(B, S):
    """cells_computed against the path each round took: per-pair gathers without the cache
    compute exactly the revealed cells; with the cache the first gathered round computes all T
    cells of its documents and nothing afterwards; a corpus pass computes the batch for all N."""
    rng = np.random.default_rng(12)
    w = _custom(S, rng.integers(1, 90, 3000).tolist(), 4, 32, 128, "bf16", 19)
    N, T, Bsz = w.N, w.T, 4
    plain = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.5, 0.01, 5, 4, no_cell_cache=True, later_rounds=2)
    cached = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.5, 0.01, 5, 4, later_rounds=2)
    passes = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.5, 0.01, 5, 4, later_rounds=1, no_cell_cache=True)
    torch.cuda.synchronize()
    assert max(s["rounds"] for s in plain["stats"]) >= 3
    for sp, sc, sd in zip(plain["stats"], cached["stats"], passes["stats"]):
        assert sp["survivors"] == sc["survivors"] == sd["survivors"]
        surv, R = sp["survivors"], sp["rounds"]
        assert sp["cells_computed"] == sp["cells_elim"] + sp["cells_rescore"]
        want = Bsz * N + (T * surv[1] if R >= 2 else T * surv[R])      # round 1, then one visit
        assert sc["cells_computed"] == want
        assert sd["cells_computed"] == Bsz * N * R + T * surv[R]       # every round a pass, then the rescore
        assert sd["corpus_pass_rounds"] == list(range(2, 2 + len(sd["corpus_pass_rounds"])))


def test_active_sets_larger_than_the_cell_cache(B, S, oracle_mod):
    """N above the cache capacity with a conservative radius: the first gathered rounds
    run uncached and a query switches to its cache only once its active set fits."""
    rng = np.random.default_rng(8)
    w = _custom(S, rng.integers(2, 9, 40000).tolist(), 3, 32, 128, "bf16", 21)
    r1 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 1.0, 0.01, 5, 1, trace=True)
    r2 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 1.0, 0.01, 5, 1, trace=True, no_cell_cache=True)
    torch.cuda.synchronize()
    surv = [s["survivors"] for s in r1["stats"]]
    assert any(len(x) > 2 and x[1] > 16384 for x in surv), surv     # really started above capacity
    _same_run(r1, r2)
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 1.0, seed=1)


@pytest.mark.parametrize("K", [5, 300])
def test_long_lists_take_the_sampled_prefilter(B, S, oracle_mod, K):
    """Lists far longer than the selection kernels' sample: the threshold of a strided sample
    pre-filters candidates before the exact selection.  Checked against the oracle (rounds,
    survivors, top-K) and against a full sort of the GPU's own scores."""
    rng = np.random.default_rng(77)
    w = _custom(S, rng.integers(1, 4, 150000).tolist(), 2, 32, 128, "bf16", 31)
    full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K)
    torch.cuda.synchronize()
    sc = full["scores"].cpu().numpy()
    for q in range(w.nq):
        order = np.lexsort((np.arange(w.N), -sc[q]))[:K]
        np.testing.assert_array_equal(full["topk_ids"][q].cpu().numpy(), order)
        np.testing.assert_array_equal(full["topk_scores"][q].cpu().numpy(), sc[q][order])
    _run_colbandit_case(B, oracle_mod, w, K, 5, 4, 0.2, seed=2)


@pytest.mark.parametrize("nq", [1, 3])
def test_long_lists_stay_long_under_a_conservative_radius(B, S, oracle_mod, nq):
    """alpha_ef = 1 keeps most of 150,000 documents alive for several rounds: explicit lists
    longer than the pre-filter limit, cut down by several workgroups per query, revealed by the
    corpus pass (statistics merged for the candidates only) or by gathers - same decisions."""
    rng = np.random.default_rng(78)
    w = _custom(S, rng.integers(1, 4, 150000).tolist(), nq, 32, 128, "bf16", 37)
    runs = [B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 1.0, 0.01, 5, 6, trace=True, later_rounds=m)
            for m in (1, 2)]
    torch.cuda.synchronize()
    surv = runs[0]["stats"][0]["survivors"]
    assert len(surv) > 3 and surv[2] > 131072, surv          # long lists beyond round 1
    _same_run(runs[0], runs[1])
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 1.0, seed=6, later_rounds=1)


def test_long_lists_with_massive_ties(B, S):
    """150,000 documents that are copies of 40 distinct ones: the K-th score is shared by
    thousands; ties resolve to the lowest indices."""
    base = _custom(S, [3] * 40, 2, 32, 128, "bf16", 13)
    reps = 3750
    docs = base.docs.repeat(reps, 1)
    off = (torch.arange(40 * reps + 1, dtype=torch.int64) * 3).cuda()
    r = B.colbandit_full_maxsim(base.Q, docs, off, K=100)
    torch.cuda.synchronize()
    sc = r["scores"].cpu().numpy()
    for q in range(2):
        order = np.lexsort((np.arange(40 * reps), -sc[q]))[:100]
        np.testing.assert_array_equal(r["topk_ids"][q].cpu().numpy(), order)


def test_colbandit_support_wider_than_default(B, S, oracle_mod):
    w = S.config(1, device="cuda", scale=0.02, nq=3)
    _run_colbandit_case(B, oracle_mod, w, 5, 5, 4, 0.2, a=-1.5, b=1.25)


def test_colbandit_small_candidate_sets(B, S, oracle_mod):
    # N <= K+M: no round runs and the answer is the exhaustive top-K; also N == K and N == 1
    for N, K, M in [(9, 4, 5), (10, 5, 5), (5, 5, 0), (1, 1, 0), (11, 5, 5)]:
        w = _custom(S, [33] * N, 2, 32, 128, "bf16", N)
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K)
        res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.2, 0.01, M, 0)
        torch.cuda.synchronize()
        if N <= K + M:
            assert all(s["rounds"] == 0 and s["cells_elim"] == 0 and s["cells_rescore"] == 32 * N
                       for s in res["stats"])
            assert torch.equal(res["topk_ids"], full["topk_ids"])
            assert torch.equal(res["topk_scores"], full["topk_scores"])


@pytest.mark.parametrize("nq,T,d,N,K,M,Bsz,alpha,coarse", [
    (2, 1, 128, 300, 3, 2, 4, 0.2, False),          # one query token: a single round, then exact
    (2, 128, 128, 300, 5, 5, 16, 0.3, False),       # the largest T and B of this build
    (1, 32, 128, 1100, 1024, 0, 4, 0.2, False),     # the largest K
    (300, 16, 64, 500, 5, 5, 4, 0.2, False),        # many queries: several column groups, d=64
    (3, 40, 64, 400, 4, 3, 5, 0.5, True),           # int8 rounds with d=64 and B not dividing T
    (2, 100, 128, 300, 5, 5, 7, 1.0, True),         # int8 rounds, 7 tiles of query tokens
    (4, 32, 128, 6, 5, 5, 4, 0.2, True),            # N <= K + M: no round at all
    (2, 64, 128, 300, 5, 5, 1, 0.6, False),         # one token per round: the 64-round limit
    (3, 32, 96, 400, 5, 5, 4, 0.3, False),          # widths that only the gather kernels cover
    (2, 24, 32, 300, 3, 2, 4, 0.5, False),
])
def test_colbandit_corner_shapes(B, S, oracle_mod, nq, T, d, N, K, M, Bsz, alpha, coarse):
    rng = np.random.default_rng(N + T)
    w = _custom(S, rng.integers(1, 70, N).tolist(), nq, T, d, "bf16", 59)
    co = B.colbandit_quantize_i8(w.docs) if coarse else None
    if nq > 16:                                     # keep the oracle leg to a few queries
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, want_cells=True)
        res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, 0.01, M, 5, B=Bsz, trace=True)
        torch.cuda.synchronize()
        for q in (0, 17, nq - 1):
            Hq = full["cells"][q].cpu().numpy().astype(np.float64)
            pi = B.colbandit_permutation(5, q, T)
            div, orc = _compare_rounds(oracle_mod, res["trace"], q, Hq, K, M, Bsz, alpha, 0.01, pi)
            assert res["stats"][q]["rounds"] == orc.rounds
            got = res["topk_ids"][q]
            assert torch.equal(res["topk_scores"][q], full["scores"][q][got])
            sfin = full["scores"][q].cpu().numpy()[orc.final_ids].astype(np.float64)
            order = orc.final_ids[np.lexsort((orc.final_ids, -sfin))][:K]
            np.testing.assert_array_equal(got.cpu().numpy(), order)
        return
    _run_colbandit_case(B, oracle_mod, w, K, M, Bsz, alpha, seed=5, coarse=co)


def test_explicit_permutation_and_determinism(B, S):
    w = S.config(1, device="cuda", scale=0.02, nq=4)
    pi = torch.tensor(np.stack([B.colbandit_permutation(77, q, w.T) for q in range(w.nq)]),
                      dtype=torch.int32, device="cuda")
    r1 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 77, trace=True)
    r2 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 123456, pi=pi, trace=True)
    r3 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 77, trace=True)
    torch.cuda.synchronize()
    for other in (r2, r3):
        assert torch.equal(r1["topk_ids"], other["topk_ids"])
        assert torch.equal(r1["topk_scores"], other["topk_scores"])
        np.testing.assert_array_equal(r1["trace"].alive, other["trace"].alive)
    assert [s["survivors"] for s in r1["stats"]] == [s["survivors"] for s in r2["stats"]]


def test_async_call_without_stats(B, S):
    w = S.config(1, device="cuda", scale=0.02, nq=4)
    r1 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 1)
    r2 = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, 0.01, 5, 1, want_stats=False)
    torch.cuda.synchronize()
    assert r2["stats"] is None
    assert torch.equal(r1["topk_ids"], r2["topk_ids"]) and torch.equal(r1["topk_scores"], r2["topk_scores"])


def test_both_calls_can_be_captured_in_a_graph_and_replayed(B, S):
    """Without statistics both entry points only enqueue kernels on the caller's stream (no
    allocation, no memset, no read-back), so a caller may capture them in a HIP graph.  Every
    replay, with eager work of the same library in between, must reproduce the eager result."""
    w = S.config(1, device="cuda", scale=0.06, nq=8)            # N=3000
    K = 5
    ws = B.new_workspace(w.nq, w.T, w.d, w.N, w.total_tokens, "cuda")
    d8, ds = B.colbandit_quantize_i8(w.docs)
    outs = [{"topk_ids": torch.empty((w.nq, K), dtype=torch.int64, device="cuda"),
             "topk_scores": torch.empty((w.nq, K), dtype=torch.float32, device="cuda")} for _ in range(3)]
    scores = torch.empty((w.nq, w.N), dtype=torch.float32, device="cuda")

    def run():
        B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws,
                                out={**outs[0], "scores": scores})
        B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.2, 0.01, 5, 3, workspace=ws, out=outs[1],
                         want_stats=False)
        B.colbandit_topk(w.Q, w.docs, w.offsets, K, 0.2, 0.01, 5, 3, workspace=ws, out=outs[2],
                         want_stats=False, docs_i8=d8, docs_scale=ds)

    run()
    torch.cuda.synchronize()
    ref = [(o["topk_ids"].clone(), o["topk_scores"].clone()) for o in outs]
    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            run()
    torch.cuda.synchronize()
    for _ in range(3):
        for o in outs:
            o["topk_ids"].fill_(-7)
            o["topk_scores"].fill_(0.0)
        ws.fill_(0xAB)                                # the calls must not rely on workspace contents
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for o, (ids, sc) in zip(outs, ref):
            assert torch.equal(o["topk_ids"], ids) and torch.equal(o["topk_scores"], sc)
        other = B.colbandit_topk(w.Q, w.docs, w.offsets, 3, 0.5, 0.01, 2, 9, workspace=ws)   # eager, other knobs
        torch.cuda.synchronize()
        assert other["stats"][0]["rounds"] >= 1


def test_validate_offsets(B, S):
    w = S.config(0, device="cuda")
    assert B.colbandit_validate_offsets(w.offsets, w.total_tokens) == 0
    bad = w.offsets.clone(); bad[10] = bad[9]                   # an empty document
    assert B.colbandit_validate_offsets(bad, w.total_tokens) == -8
    assert B.colbandit_validate_offsets(w.offsets, w.total_tokens - 1) == -8
    # a bad table must not fault: rows are clamped, results are merely meaningless
    B.colbandit_full_maxsim(w.Q, w.docs, bad, K=0)
    torch.cuda.synchronize()


# ------------------------------------------------------------------ int8 coarse elimination pass
def _host_values(x):
    return x.float().cpu().numpy()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("rows,d,nseg,permille", [(3001, 128, 1, 999), (64, 128, 4, 999), (32 * 9, 64, 9, 999),
                                                   (1, 128, 1, 999), (500, 128, 1, 1000), (500, 128, 5, 500),
                                                   (1200, 128, 2, 999), (1026, 100, 2, 900), (1001, 100, 1, 999)])
def test_quantize_i8_codes_and_scales_match_oracle(B, oracle_mod, dtype, rows, d, nseg, permille):
    """Percentile clip and codes are integer results: exact equality with the oracle, which
    takes the deciding arithmetic in single precision as well."""
    g = torch.Generator(device="cpu"); g.manual_seed(rows * 7 + d + nseg)
    x = torch.randn((rows, d), generator=g) * 0.09
    x[0, 0] = 3.0                                   # an outlier far above the clip
    x = x.to(torch.bfloat16 if dtype == "bf16" else torch.float32).cuda()
    codes, scales = B.colbandit_quantize_i8(x, n_segments=nseg, permille=permille)
    torch.cuda.synchronize()
    xs = _host_values(x).reshape(nseg, -1)
    for sidx in range(nseg):
        clip = oracle_mod.abs_percentile(xs[sidx], permille)
        assert scales[sidx].item() == np.float32(clip) / np.float32(127.0)
        want = oracle_mod.quantize_i8(xs[sidx], clip)
        np.testing.assert_array_equal(codes.cpu().numpy().reshape(nseg, -1)[sidx], want)
    if permille == 999 and rows * d // nseg >= 2000:
        assert codes.abs().max().item() == 127       # the outlier saturates
    z = torch.zeros((4, d), dtype=x.dtype, device="cuda")
    cz, sz = B.colbandit_quantize_i8(z)
    assert int(cz.abs().max()) == 0 and float(sz[0]) == 0.0


@pytest.mark.parametrize("nq,T,d", [(1, 32, 128), (5, 32, 128), (20, 24, 128), (3, 40, 128), (2, 100, 128),
                                    (4, 32, 64), (70, 16, 64)])
def test_coarse_maxsim_cells_are_the_integer_maxima(B, S, oracle_mod, nq, T, d):
    """Cells from int8 codes: the integer dot products and their maxima are exact, so the
    decoded cell must equal float(int) * (sq * sd) bit for bit."""
    lengths = [1, 2, 15, 16, 17, 31, 33, 63, 64, 65, 100, 255, 257, 1030] + \
        np.random.default_rng(d + T).integers(1, 200, 150).tolist()
    w = _custom(S, lengths, nq, T, d, "bf16", 11 + nq)
    d8, ds = B.colbandit_quantize_i8(w.docs)
    cm = B.colbandit_coarse_maxsim(w.Q, d8, ds, w.offsets, want_cells=True)
    torch.cuda.synchronize()
    q8 = cm["q_codes"].cpu().numpy()
    qs = cm["q_scales"].cpu().numpy()
    Qh = w.host_queries()
    off = w.offsets.cpu().numpy()
    D8 = d8.cpu().numpy()
    sd = np.float32(ds.cpu().numpy()[0])
    cells = cm["cells"].cpu().numpy()
    for q in range(nq):
        # the call's own query codes follow the same scheme
        clip = oracle_mod.abs_percentile(Qh[q], 999)
        assert qs[q] == np.float32(clip) / np.float32(127.0)
        np.testing.assert_array_equal(q8[q], oracle_mod.quantize_i8(Qh[q], clip))
        if q < 6:
            _, Hint = oracle_mod.maxsim_cells_i8(q8[q], qs[q], D8, sd, off)
            want = Hint.astype(np.float32) * (np.float32(qs[q]) * sd)
            np.testing.assert_array_equal(cells[q], want)
    # row sums in the kernels' fixed order vs a plain sum
    np.testing.assert_allclose(cm["scores"].cpu().numpy(), cells.sum(axis=2), rtol=1e-5, atol=1e-5)


def test_every_position_of_a_document_end_inside_a_block(B, S, oracle_mod):
    """The wide dense kernels fold a block in which a document ends by code specialised for the
    row at which it ends; here every such row 1..15 occurs (a document of b tokens from a block
    start, then one of 32 - b tokens that ends with a block), and two and three ends in one
    block (which take the general fold).  Exhaustive cells (bf16, 20 queries: eight column tiles
    per wavefront), integer cells of the int8 codes, and the round-1 statistics of Col-Bandit
    over 72 queries (eight tiles per wavefront in the reveal pass) against the oracle."""
    lengths = []
    for b in range(1, 16):
        lengths += [b, 32 - b]
    lengths += [3, 4, 9, 5, 5, 6, 16, 1, 1, 1, 13] + list(range(1, 40))
    nq, T, d = 20, 32, 128
    w = _custom(S, lengths, nq, T, d, "bf16", 77)
    H, Sor = _oracle_scores(oracle_mod, w)
    r = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=3, want_cells=True)
    torch.cuda.synchronize()
    np.testing.assert_allclose(r["cells"].cpu().numpy(), H, rtol=TOL["bf16"], atol=1e-5)
    np.testing.assert_allclose(r["scores"].cpu().numpy(), Sor, rtol=TOL["bf16"], atol=1e-4)
    # int8 codes: exact integer maxima
    d8, ds = B.colbandit_quantize_i8(w.docs)
    cm = B.colbandit_coarse_maxsim(w.Q, d8, ds, w.offsets, want_cells=True)
    torch.cuda.synchronize()
    q8, qs = cm["q_codes"].cpu().numpy(), cm["q_scales"].cpu().numpy()
    off, D8 = w.offsets.cpu().numpy(), d8.cpu().numpy()
    sd = np.float32(ds.cpu().numpy()[0])
    for q in (0, 7, 19):
        _, Hint = oracle_mod.maxsim_cells_i8(q8[q], qs[q], D8, sd, off)
        np.testing.assert_array_equal(cm["cells"][q].cpu().numpy(),
                                      Hint.astype(np.float32) * (np.float32(qs[q]) * sd))
    # the reveal pass with eight tiles per wavefront: 72 queries x 4 revealed tokens
    w2 = _custom(S, lengths, 72, T, d, "bf16", 78)
    full = B.colbandit_full_maxsim(w2.Q, w2.docs, w2.offsets, K=0, want_cells=True)
    res = B.colbandit_topk(w2.Q, w2.docs, w2.offsets, 3, 1.0, 0.01, 2, 9, B=4, trace=True)
    e8, es = B.colbandit_quantize_i8(w2.docs)
    res8 = B.colbandit_topk(w2.Q, w2.docs, w2.offsets, 3, 1.0, 0.01, 2, 9, B=4, trace=True,
                            docs_i8=e8, docs_scale=es)
    cm2 = B.colbandit_coarse_maxsim(w2.Q, e8, es, w2.offsets, want_cells=True)
    torch.cuda.synchronize()
    for q in (0, 35, 71):
        Hq = full["cells"][q].cpu().numpy().astype(np.float64)
        Hc = cm2["cells"][q].cpu().numpy().astype(np.float64)
        pi = B.colbandit_permutation(9, q, T)
        div, orc = _compare_rounds(oracle_mod, res["trace"], q, Hq, 3, 2, 4, 1.0, 0.01, pi)
        assert res["stats"][q]["rounds"] == orc.rounds
        div, orc = _compare_rounds(oracle_mod, res8["trace"], q, Hc, 3, 2, 4, 1.0, 0.01, pi, Hexact=Hq)
        assert res8["stats"][q]["rounds"] == orc.rounds


@pytest.mark.parametrize("alpha,K,M,Bsz", [(0.2, 5, 5, 4), (1.0, 5, 5, 4), (0.5, 10, 5, 3), (0.2, 5, 0, 16)])
def test_colbandit_on_int8_codes_rounds_match_oracle(B, S, oracle_mod, alpha, K, M, Bsz):
    """Rounds decided on coarse cells, survivors rescored exactly (implementation appendix):
    every bound, threshold and survivor against the oracle's coarse-elimination mode, and the
    returned scores carry the exhaustive path's bits."""
    w = S.config(1, device="cuda", scale=0.04, nq=6)            # N=2000, planted docs
    d8, ds = B.colbandit_quantize_i8(w.docs)
    _run_colbandit_case(B, oracle_mod, w, K, M, Bsz, alpha, coarse=(d8, ds))
    w = S.config(3, device="cuda", scale=0.005, nq=4)           # 100 pages x 1030 tokens, T=24
    d8, ds = B.colbandit_quantize_i8(w.docs)
    _run_colbandit_case(B, oracle_mod, w, K, M, Bsz, alpha, coarse=(d8, ds))


def test_colbandit_on_int8_codes_all_reveal_paths_agree(B, S, oracle_mod):
    rng = np.random.default_rng(3)
    w = _custom(S, rng.integers(1, 120, 2500).tolist(), 5, 32, 128, "bf16", 23)
    d8, ds = B.colbandit_quantize_i8(w.docs)
    kw = dict(docs_i8=d8, docs_scale=ds, trace=True)
    base = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.5, 0.01, 5, 3, **kw)
    for extra in (dict(force_gather=True), dict(no_cell_cache=True), dict(later_rounds=1),
                  dict(later_rounds=2), dict(later_rounds=1, no_cell_cache=True)):
        other = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.5, 0.01, 5, 3, **kw, **extra)
        torch.cuda.synchronize()
        _same_run(base, other)
    # fp32 embeddings with int8 codes: the rounds use the codes, the rescore the fp32 gather
    w32 = _custom(S, rng.integers(1, 60, 600).tolist(), 2, 32, 128, "f32", 29)
    d8, ds = B.colbandit_quantize_i8(w32.docs)
    _run_colbandit_case(B, oracle_mod, w32, 5, 5, 4, 0.3, coarse=(d8, ds))


# ------------------------------------------------------------------ non-adaptive baselines
def _clustered_queries(w, S, n_dir, noise, seed):
    """Replaces the workload's queries by tokens scattered around n_dir directions with random
    norms, so that a sweep of the cosine threshold gives anything from one cluster to T."""
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    nq, T, d = w.Q.shape
    base = torch.randn((nq, n_dir, d), generator=g)
    base = base / base.norm(dim=2, keepdim=True)
    pick = torch.randint(0, n_dir, (nq, T), generator=g)
    Q = torch.gather(base, 1, pick[..., None].expand(nq, T, d)) + noise * torch.randn((nq, T, d), generator=g) / d ** 0.5
    Q = Q * (0.5 + 1.5 * torch.rand((nq, T, 1), generator=g))
    w.Q = Q.to(w.Q.dtype).cuda()
    return w


@pytest.mark.parametrize("dtype,nq,T,d,m", [("bf16", 3, 32, 128, 4), ("bf16", 20, 32, 128, 13),
                                            ("bf16", 2, 64, 128, 64), ("bf16", 5, 7, 64, 1),
                                            ("bf16", 4, 30, 128, 30), ("f32", 2, 32, 128, 8),
                                            ("f32", 3, 24, 64, 5), ("bf16", 3, 32, 96, 5),
                                            ("f32", 2, 24, 32, 7)])
def test_doc_uniform_masks_scores_and_topk_match_oracle(B, S, oracle_mod, dtype, nq, T, d, m):
    """Doc-Uniform (appendix "Compared Methods"): the per-document token subsets are the oracle's
    bit for bit (same counter-based generator, implemented on each side), the partial row sums
    agree within the score tolerance, the top-K follows them."""
    rng = np.random.default_rng(T * 100 + m)
    lengths = [1, 16, 17, 63, 65, 300, 1] + rng.integers(1, 120, 260).tolist()
    w = _custom(S, lengths, nq, T, d, dtype, 41)
    seed, K = 1234567, 6
    r = B.colbandit_doc_uniform(w.Q, w.docs, w.offsets, K, m, seed=seed, want_masks=True)
    torch.cuda.synchronize()
    H, _ = _oracle_scores(oracle_mod, w)
    masks = r["masks"].cpu().numpy().view(np.uint64)
    got = r["scores"].cpu().numpy()
    tol = TOL[dtype]
    for q in range(nq):
        mo, So, _, _ = oracle_mod.doc_uniform_from_H(H[q], m, seed, q, K)
        np.testing.assert_array_equal(masks[q], mo)
        np.testing.assert_allclose(got[q], So, rtol=tol, atol=tol)
        _check_topk(r["topk_ids"][q].cpu().numpy(), r["topk_scores"][q].cpu().numpy(), So, K, tol)
    if m == T:      # every cell revealed: the exhaustive scores (other summation order)
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=0)
        torch.cuda.synchronize()
        np.testing.assert_allclose(got, full["scores"].cpu().numpy(), rtol=1e-5, atol=1e-5)
    # top-K only (scores kept in the workspace) gives the same ranking
    r2 = B.colbandit_doc_uniform(w.Q, w.docs, w.offsets, K, m, seed=seed, want_scores=False)
    torch.cuda.synchronize()
    assert torch.equal(r2["topk_ids"], r["topk_ids"]) and torch.equal(r2["topk_scores"], r["topk_scores"])


@pytest.mark.parametrize("dtype,nq,T,d,tau", [("bf16", 3, 32, 128, 0.7), ("bf16", 40, 32, 128, 0.9),
                                              ("bf16", 6, 32, 128, 0.4), ("bf16", 2, 64, 128, 0.8),
                                              ("bf16", 5, 7, 64, 0.6), ("bf16", 4, 30, 128, 1.0),
                                              ("bf16", 1, 1, 128, 0.5), ("f32", 2, 32, 128, 0.7),
                                              ("f32", 3, 24, 64, 0.5), ("bf16", 3, 32, 96, 0.7),
                                              ("f32", 2, 24, 32, 0.6)])
def test_ball_carving_clusters_centroids_scores_match_oracle(B, S, oracle_mod, dtype, nq, T, d, tau):
    """Ball-carving (appendix "Compared Methods"): cluster labels and cluster counts are exact
    (the membership test is taken in the same double-precision form on both sides), the
    centroids are the oracle's bit for bit, scores and top-K agree within the score tolerance."""
    rng = np.random.default_rng(T * 10 + nq)
    lengths = [1, 16, 17, 63, 65, 300, 1] + rng.integers(1, 120, 260).tolist()
    w = _clustered_queries(_custom(S, lengths, nq, T, d, dtype, 43), S, 4, 0.6, 5)
    K = 6
    r = B.colbandit_ball_carving(w.Q, w.docs, w.offsets, K, tau)
    torch.cuda.synchronize()
    E, off = w.host_docs()
    Qh = w.host_queries()
    tol = TOL[dtype]
    ks = []
    for q in range(nq):
        k, labels, C, So, _, _ = oracle_mod.ball_carving(Qh[q], E, off, tau, K, round_bf16=(dtype == "bf16"))
        ks.append(k)
        assert int(r["n_clusters"][q]) == k
        np.testing.assert_array_equal(r["labels"][q].cpu().numpy(), labels)
        np.testing.assert_array_equal(r["centroids"][q].float().cpu().numpy(), C)
        scale = max(1.0, float(np.abs(So).max()))
        np.testing.assert_allclose(r["scores"][q].cpu().numpy(), So, rtol=tol, atol=tol * scale)
        _check_topk(r["topk_ids"][q].cpu().numpy(), r["topk_scores"][q].cpu().numpy(), So, K, tol)
    if tau == 1.0:
        assert ks == [T] * nq
        full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=0)
        torch.cuda.synchronize()
        np.testing.assert_allclose(r["scores"].cpu().numpy(), full["scores"].cpu().numpy(),
                                   rtol=1e-4, atol=1e-4)
    if T >= 24 and tau <= 0.7:
        assert min(ks) < T                               # the sweep point does compress


def test_ball_carving_identical_tokens_collapse_to_one_centroid(B, S, oracle_mod):
    w = _custom(S, np.random.default_rng(3).integers(1, 90, 150).tolist(), 2, 32, 128, "bf16", 47)
    w.Q = (w.Q[:, :1, :].float() * torch.tensor([1.0, 2.0, 0.5, 4.0] * 8, device="cuda")[None, :, None]) \
        .to(torch.bfloat16).contiguous()
    r = B.colbandit_ball_carving(w.Q, w.docs, w.offsets, 3, 1.0)
    torch.cuda.synchronize()
    assert r["n_clusters"].tolist() == [1, 1] and int(r["labels"].abs().sum()) == 0
    E, off = w.host_docs()
    for q in range(2):
        k, _, C, So, _, _ = oracle_mod.ball_carving(w.host_queries()[q], E, off, 1.0, 3, round_bf16=True)
        assert k == 1
        np.testing.assert_array_equal(r["centroids"][q].float().cpu().numpy(), C)
        np.testing.assert_allclose(r["scores"][q].cpu().numpy(), So, rtol=TOL["bf16"], atol=1e-3)


def _rounds_of_sampled_queries(B, oracle_mod, w, res, qs, K, alpha, scores_of, coarse=None):
    """Full-size protocol for a traced batch call `res` (trace_queries=qs): for each sampled
    query the GPU's own cells of that query (one exhaustive single-query call with the cell
    output) go through the oracle and every round is compared (_compare_rounds); then rounds,
    counters, final set and the returned top-K.  scores_of(q) -> the exhaustive path's scores of
    query q as a host array.  coarse = (docs_i8, docs_scale) when the rounds ran on int8 codes.
    Returns the number of queries that needed a re-entry at a band document."""
    tr, T = res["trace"], w.T
    diverged = 0
    for j, q in enumerate(qs):
        Qq = w.Q[q:q + 1].contiguous()
        one = B.colbandit_full_maxsim(Qq, w.docs, w.offsets, K=0, want_cells=True)
        torch.cuda.synchronize()
        Sq = scores_of(q)
        np.testing.assert_array_equal(one["scores"][0].cpu().numpy(), Sq)   # batch position does not matter
        Hq = one["cells"][0].cpu().numpy().astype(np.float64)
        del one
        Hc = None
        if coarse is not None:
            cm = B.colbandit_coarse_maxsim(Qq, coarse[0], coarse[1], w.offsets, want_cells=True)
            torch.cuda.synchronize()
            Hc = cm["cells"][0].cpu().numpy().astype(np.float64)
            del cm
        pi = B.colbandit_permutation(w.seed, q, T)
        np.testing.assert_array_equal(pi, oracle_mod.permutation(w.seed, q, T))
        if Hc is None:
            div, orc = _compare_rounds(oracle_mod, tr, j, Hq, K, w.M, w.B, alpha, w.delta, pi)
        else:
            div, orc = _compare_rounds(oracle_mod, tr, j, Hc, K, w.M, w.B, alpha, w.delta, pi, Hexact=Hq)
        st = res["stats"][q]
        assert st["survivors"] == [int(x) for x in tr.count[: st["rounds"] + 1, j]]
        assert st["rounds"] == orc.rounds and st["cells_rescore"] == orc.cells_rescore
        if div == 0:
            assert (st["cells_elim"], st["cells_unique"]) == (orc.cells_elim, orc.cells_unique)
        diverged += div > 0
        kk = min(K, len(orc.final_ids))
        order = orc.final_ids[np.lexsort((orc.final_ids, -Sq[orc.final_ids].astype(np.float64)))][:kk]
        np.testing.assert_array_equal(res["topk_ids"][q].cpu().numpy()[:kk], order)
        np.testing.assert_array_equal(res["topk_scores"][q].cpu().numpy()[:kk], Sq[order])
        # the rescore is the exact row sum: fp32 fixed-order sum vs the double sum of the same cells
        np.testing.assert_allclose(Sq[order], Hq[order].sum(axis=1), rtol=1e-5)
        print(f"  query {q}: {orc.rounds} rounds, survivors {st['survivors']}, re-entries {div}", flush=True)
    return diverged


# ------------------------------------------------------------------ full size, bench launch configuration
@pytest.fixture(scope="module")
def big(B, S):
    """The benchmark's workload and call pattern: N=500,000 documents, 128 queries, preallocated
    workspace and outputs, K=5, alpha_ef=0.2."""
    print("generating the full-size corpus ...", flush=True)
    w = S.config(2, device="cuda")
    ws = B.new_workspace(w.nq, w.T, w.d, w.N, w.total_tokens, "cuda")
    K = 5
    out = {"topk_ids": torch.empty((w.nq, K), dtype=torch.int64, device="cuda"),
           "topk_scores": torch.empty((w.nq, K), dtype=torch.float32, device="cuda"),
           "scores": torch.empty((w.nq, w.N), dtype=torch.float32, device="cuda")}
    print("full-size Full-MaxSim ...", flush=True)
    full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws, out=out)
    torch.cuda.synchronize()
    return w, ws, full, K


def test_full_size_scores_on_sampled_documents(B, oracle_mod, big):
    w, ws, full, K = big
    assert (w.N, w.nq, w.T, w.d, w.dtype) == (500000, 128, 32, 128, "bf16")
    rng = np.random.default_rng(2026)
    qs = [0, 31, 77, 127]
    Qh = w.host_queries(qs)
    ids_gpu = full["topk_ids"].cpu().numpy()
    for j, q in enumerate(qs):
        # random documents, the first and last of the corpus, and the GPU's winners
        docs = np.unique(np.concatenate([rng.integers(0, w.N, 40), [0, w.N - 1], ids_gpu[q]]))
        E, off = w.host_docs(docs.tolist())
        H = oracle_mod.maxsim_cells(Qh[j], E, off)
        want = H.sum(axis=1)
        got = full["scores"][q][torch.as_tensor(docs, device="cuda")].cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=TOL["bf16"], atol=0)
    # the top-K is the ordered head of the GPU's own score rows
    for q in qs + [5, 64]:
        sc = full["scores"][q].cpu().numpy()
        order = np.lexsort((np.arange(w.N), -sc))[:K]
        np.testing.assert_array_equal(ids_gpu[q], order)
        np.testing.assert_array_equal(full["topk_scores"][q].cpu().numpy(), sc[order])


def test_full_size_colbandit_rounds_and_survivor_scores(B, oracle_mod, big):
    w, ws, full, K = big
    qs = [3, 90]
    alpha, delta, M, Bsz = 0.2, w.delta, w.M, w.B
    out = {"topk_ids": torch.empty((w.nq, K), dtype=torch.int64, device="cuda"),
           "topk_scores": torch.empty((w.nq, K), dtype=torch.float32, device="cuda")}
    print("full-size Col-Bandit with trace ...", flush=True)
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, delta, M, w.seed, workspace=ws, out=out,
                           trace=True, trace_queries=qs)
    plain = B.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, delta, M, w.seed, workspace=ws,
                             want_stats=False)
    torch.cuda.synchronize()
    # tracing changes nothing
    assert torch.equal(res["topk_ids"], plain["topk_ids"])
    assert torch.equal(res["topk_scores"], plain["topk_scores"])
    # every query: survivor scores are the exhaustive path's bits; accounting identities
    ids = res["topk_ids"]
    assert bool((ids >= 0).all())
    assert torch.equal(res["topk_scores"], torch.gather(full["scores"], 1, ids))
    T = w.T
    for q, st in enumerate(res["stats"]):
        surv = st["survivors"]
        assert surv[0] == w.N and all(surv[r + 1] <= surv[r] for r in range(st["rounds"]))
        cells = sum((min((r + 1) * Bsz, T) - r * Bsz) * surv[r] for r in range(st["rounds"]))
        assert st["cells_elim"] == cells and st["cells_rescore"] == T * surv[st["rounds"]]
    # two queries: every round against the oracle, fed the GPU's own cells of these queries
    print("full-size cells of two queries ...", flush=True)
    scores_of = lambda q: full["scores"][q].cpu().numpy()
    _rounds_of_sampled_queries(B, oracle_mod, w, res, qs, K, alpha, scores_of)


def test_full_size_colbandit_rounds_at_k10_and_on_int8_codes(B, oracle_mod, big):
    """The large text configuration's second setting (K = 10) and its int8 coarse pass, in the
    benchmark's launch configuration: every round of sampled queries against the oracle."""
    w, ws, full, _ = big
    scores_of = lambda q: full["scores"][q].cpu().numpy()
    qs = [17, 101]
    print("full-size Col-Bandit, K = 10, with trace ...", flush=True)
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, 10, 0.2, w.delta, w.M, w.seed, workspace=ws,
                           trace=True, trace_queries=qs)
    torch.cuda.synchronize()
    assert torch.equal(res["topk_scores"], torch.gather(full["scores"], 1, res["topk_ids"]))
    _rounds_of_sampled_queries(B, oracle_mod, w, res, qs, 10, 0.2, scores_of)
    del res
    print("full-size Col-Bandit on int8 codes, K = 5, with trace ...", flush=True)
    d8, ds = B.colbandit_quantize_i8(w.docs)
    qs = [64]
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, 5, 0.2, w.delta, w.M, w.seed, workspace=ws,
                           trace=True, trace_queries=qs, docs_i8=d8, docs_scale=ds)
    torch.cuda.synchronize()
    assert torch.equal(res["topk_scores"], torch.gather(full["scores"], 1, res["topk_ids"]))
    _rounds_of_sampled_queries(B, oracle_mod, w, res, qs, 5, 0.2, scores_of, coarse=(d8, ds))


def test_full_size_baselines_on_sampled_documents(B, oracle_mod, big):
    """Doc-Uniform and Ball-carving at the benchmark's size: subsets, clusters and centroids exact
    for sampled queries; scores of sampled documents against the oracle."""
    w, ws, full, K = big
    rng = np.random.default_rng(77)
    qs = [0, 64, 127]
    docs = np.unique(np.concatenate([rng.integers(0, w.N, 30), [0, w.N - 1]]))
    E, off = w.host_docs(docs.tolist())
    Qh = w.host_queries(qs)
    dsel = torch.as_tensor(docs, device="cuda")
    print("full-size Doc-Uniform ...", flush=True)
    m, seed = 8, 99
    ru = B.colbandit_doc_uniform(w.Q, w.docs, w.offsets, K, m, seed=seed, want_masks=True)
    torch.cuda.synchronize()
    for j, q in enumerate(qs):
        H = oracle_mod.maxsim_cells(Qh[j], E, off)
        masks = ru["masks"][q][dsel].cpu().numpy().view(np.uint64)
        for n, i in enumerate(docs.tolist()):
            R = oracle_mod.uniform_subset(seed, q, i, w.T, m)
            assert int(masks[n]) == R
            want = sum(H[n, t] for t in range(w.T) if (R >> t) & 1)
            assert float(ru["scores"][q, i]) == pytest.approx(want, rel=TOL["bf16"], abs=1e-4)
        sc = ru["scores"][q].cpu().numpy()
        np.testing.assert_array_equal(ru["topk_ids"][q].cpu().numpy(), np.lexsort((np.arange(w.N), -sc))[:K])
    del ru
    print("full-size Ball-carving ...", flush=True)
    tau = 0.7
    rb = B.colbandit_ball_carving(w.Q, w.docs, w.offsets, K, tau)
    torch.cuda.synchronize()
    for j, q in enumerate(qs):
        k, labels, C, So, _, _ = oracle_mod.ball_carving(Qh[j], E, off, tau, 1, round_bf16=True)
        assert int(rb["n_clusters"][q]) == k
        np.testing.assert_array_equal(rb["labels"][q].cpu().numpy(), labels)
        np.testing.assert_array_equal(rb["centroids"][q].float().cpu().numpy(), C)
        got = rb["scores"][q][dsel].cpu().numpy()
        np.testing.assert_allclose(got, So, rtol=TOL["bf16"], atol=1e-3)
        sc = rb["scores"][q].cpu().numpy()
        np.testing.assert_array_equal(rb["topk_ids"][q].cpu().numpy(), np.lexsort((np.arange(w.N), -sc))[:K])


@pytest.mark.parametrize("idx,shape", [(1, (50000, 64, 32)), (3, (20000, 64, 24)), (4, (100000, 256, 32))])
def test_other_configurations_at_full_size(B, S, oracle_mod, idx, shape):
    """The mid-text, page-like and knob-sweep configurations at their full sizes: exhaustive
    scores of sampled documents against the oracle, then properties that hold at any size -
    the top-K is the ordered head of the score rows, Col-Bandit (bf16 reveals and int8 reveals)
    returns distinct valid documents with the exhaustive path's score bits, the cell accounting
    adds up, and the planted documents of the mid-text corpus are found.  Then every round of
    sampled queries against the oracle (the knob-sweep configuration: at its grid corners)."""
    print(f"generating configuration {idx} at full size ...", flush=True)
    w = S.config(idx, device="cuda")
    assert (w.N, w.nq, w.T) == shape and w.dtype == "bf16"
    K, T = w.K, w.T
    ws = B.new_workspace(w.nq, T, w.d, w.N, w.total_tokens, "cuda")
    full = B.colbandit_full_maxsim(w.Q, w.docs, w.offsets, K=K, workspace=ws)
    res = B.colbandit_topk(w.Q, w.docs, w.offsets, K, w.alpha_ef, w.delta, w.M, w.seed, workspace=ws)
    d8, ds = B.colbandit_quantize_i8(w.docs)
    res8 = B.colbandit_topk(w.Q, w.docs, w.offsets, K, w.alpha_ef, w.delta, w.M, w.seed, workspace=ws,
                            docs_i8=d8, docs_scale=ds)
    torch.cuda.synchronize()
    rng = np.random.default_rng(idx)
    qs = [0, w.nq // 2, w.nq - 1]
    Qh = w.host_queries(qs)
    ids_full = full["topk_ids"].cpu().numpy()
    for j, q in enumerate(qs):
        docs = np.unique(np.concatenate([rng.integers(0, w.N, 12), [0, w.N - 1], ids_full[q]]))
        E, off = w.host_docs(docs.tolist())
        want = oracle_mod.maxsim_cells(Qh[j], E, off).sum(axis=1)
        got = full["scores"][q][torch.as_tensor(docs, device="cuda")].cpu().numpy()
        np.testing.assert_allclose(got, want, rtol=TOL["bf16"], atol=0)
        sc = full["scores"][q].cpu().numpy()
        order = np.lexsort((np.arange(w.N), -sc))[:K]
        np.testing.assert_array_equal(ids_full[q], order)
        np.testing.assert_array_equal(full["topk_scores"][q].cpu().numpy(), sc[order])
    for r in (res, res8):
        ids = r["topk_ids"]
        assert bool((ids >= 0).all()) and bool((ids < w.N).all())
        assert all(len(set(row)) == K for row in ids.tolist())
        assert torch.equal(r["topk_scores"], torch.gather(full["scores"], 1, ids))
        for st in r["stats"]:
            surv = st["survivors"]
            assert surv[0] == w.N and all(surv[k + 1] <= surv[k] for k in range(st["rounds"]))
            assert surv[st["rounds"]] >= K
            cells = sum((min((k + 1) * w.B, T) - k * w.B) * surv[k] for k in range(st["rounds"]))
            assert st["cells_elim"] == cells and st["cells_rescore"] == T * surv[st["rounds"]]
            assert st["cells_unique"] <= w.N * T
    if idx == 1:      # the five strongest planted documents of each query win the exhaustive top-5
        for q in range(w.nq):
            assert set(ids_full[q].tolist()) <= set(w.planted[q])
    overlap = np.mean([len(set(ids_full[q]) & set(res["topk_ids"][q].tolist())) / K for q in range(w.nq)])
    print(f"configuration {idx}: Overlap@{K} {overlap:.3f}, "
          f"coverage {sum(s['cells_unique'] for s in res['stats']) / (w.nq * w.N * T):.3f}", flush=True)
    assert overlap >= 0.5
    # Algorithm 1 round by round against the oracle at this size, in the same batched launch
    # configuration: sampled queries at the configuration's own knobs (bf16 reveals and int8
    # reveals), and for the knob-sweep configuration the corners of its (alpha_ef, K) grid
    scores_of = lambda q: full["scores"][q].cpu().numpy()
    settings = [(w.alpha_ef, K, None, [qs[1]]), (w.alpha_ef, K, (d8, ds), [qs[2]])]
    if idx == 4:
        settings += [(1.0, 1, None, [5]), (1.0, 50, None, [200]), (0.05, 1, None, [77]),
                     (0.05, 50, None, [130]), (0.5, 10, None, [31])]
    for alpha, KK, co, tq in settings:
        print(f"configuration {idx}: traced run alpha_ef={alpha} K={KK} int8={co is not None} queries {tq}",
              flush=True)
        ckw = {} if co is None else {"docs_i8": co[0], "docs_scale": co[1]}
        rt = B.colbandit_topk(w.Q, w.docs, w.offsets, KK, alpha, w.delta, w.M, w.seed, workspace=ws,
                              trace=True, trace_queries=tq, **ckw)
        torch.cuda.synchronize()
        ok = rt["topk_ids"] >= 0
        assert torch.equal(rt["topk_scores"][ok], torch.gather(full["scores"], 1, rt["topk_ids"].clamp(min=0))[ok])
        if (alpha, KK) == (w.alpha_ef, K):                          # tracing changes nothing
            base = res8 if co is not None else res
            assert torch.equal(rt["topk_ids"], base["topk_ids"])
        _rounds_of_sampled_queries(B, oracle_mod, w, rt, tq, KK, alpha, scores_of, coarse=co)
        del rt


# ------------------------------------------------------------------ the C-ABI without Python
def test_c_abi_from_a_plain_host_program(B):
    """tests/native/abi_check.cpp drives the library with hipMalloc'ed buffers and its own
    stream (no torch anywhere in the process) and checks scores against the definition."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(os.path.abspath(__file__)), "native", "abi_check.bin")
    if not os.path.exists(exe):
        pytest.skip("tests/native/abi_check.bin is not built (__graft_entry__.build() builds it)")
    r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "abi_check ok" in r.stdout
