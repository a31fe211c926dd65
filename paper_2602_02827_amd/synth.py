"""Seeded synthetic corpora and query batches shaped like the paper's workloads.

This module holds input generation only: Gaussian / mixture sampling,
L2-normalisation and rounding to the storage dtype.  None of the method's
arithmetic (MaxSim, bounds, elimination) lives here, so the CPU oracle's tests
and the HIP path can both be fed from it.

The shapes follow the paper's experimental setup (Appendix "Datasets and
Models": T=32 query tokens and d=128 for the text encoders, hundreds of patch
tokens per page for the vision encoder) and the five configurations this
repository is measured on.  The real suites are not available; these stand in
for them.

Conventions
-----------
* "noise sigma" means an isotropic Gaussian vector with E||noise||^2 = sigma^2
  (per-coordinate standard deviation sigma/sqrt(d)), added to a unit vector and
  renormalised, so the cosine to the clean vector is about 1/sqrt(1+sigma^2).
* Document lengths are always drawn on the CPU generator so that the ragged
  structure does not depend on the device that fills in the token values.
* Values are rounded once (round-to-nearest-even) to the storage dtype; every
  consumer reads the rounded values.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch


@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" or "bf16" (storage of Q and docs)
    Q: torch.Tensor                 # [nq, T, d]
    docs: torch.Tensor              # [total_tokens, d]
    offsets: torch.Tensor           # int64 [N+1], on the same device as docs
    K: int = 5
    alpha_ef: float = 0.2
    delta: float = 0.01
    M: int = 5
    B: int = 4
    seed: int = 0
    planted: list = field(default_factory=list)   # per query: list of doc ids
    recipe: str = ""

    @property
    def N(self) -> int:
        return int(self.offsets.shape[0] - 1)

    @property
    def nq(self) -> int:
        return int(self.Q.shape[0])

    @property
    def T(self) -> int:
        return int(self.Q.shape[1])

    @property
    def d(self) -> int:
        return int(self.Q.shape[2])

    @property
    def total_tokens(self) -> int:
        return int(self.docs.shape[0])

    def host_queries(self, qs=None) -> np.ndarray:
        Q = self.Q if qs is None else self.Q[qs]
        return Q.float().cpu().numpy()

    def host_docs(self, doc_ids=None):
        """(E float32 [tokens,d], offsets int64) for all docs or a subset, on the host."""
        off = self.offsets.cpu()
        if doc_ids is None:
            return self.docs.float().cpu().numpy(), off.numpy()
        ids = torch.as_tensor(doc_ids, dtype=torch.int64)
        lens = off[ids + 1] - off[ids]
        new_off = torch.zeros(len(ids) + 1, dtype=torch.int64)
        new_off[1:] = torch.cumsum(lens, 0)
        rows = torch.cat([torch.arange(int(off[i]), int(off[i + 1])) for i in ids.tolist()]) \
            if len(ids) else torch.zeros(0, dtype=torch.int64)
        E = self.docs[rows.to(self.docs.device)].float().cpu().numpy()
        return E, new_off.numpy()


def _gens(seed: int, device):
    gc = torch.Generator(device="cpu")
    gc.manual_seed(seed)
    gd = torch.Generator(device=device)
    gd.manual_seed(seed + 0x5EED)
    return gc, gd


def _unit(x: torch.Tensor) -> torch.Tensor:
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-20)


def _noise(shape, d, sigma, gen, device):
    return torch.randn(shape, generator=gen, device=device) * (sigma / np.sqrt(d))


def _store(x: torch.Tensor, dtype: str) -> torch.Tensor:
    return x.to(torch.bfloat16) if dtype == "bf16" else x.to(torch.float32)


def _lengths(N, Lmin, Lmax, gc):
    L = torch.randint(Lmin, Lmax + 1, (N,), generator=gc, dtype=torch.int64)
    off = torch.zeros(N + 1, dtype=torch.int64)
    off[1:] = torch.cumsum(L, 0)
    return L, off


def _distinct(N, n, k, gc):
    """[N,k] int64: k distinct values of range(n) per row (uniform without replacement)."""
    chosen = torch.zeros((N, 0), dtype=torch.int64)
    for j in range(k):
        r = torch.randint(0, n - j, (N,), generator=gc, dtype=torch.int64)
        srt = torch.sort(chosen, dim=1).values
        for c in range(j):
            r = r + (r >= srt[:, c]).to(torch.int64)
        chosen = torch.cat([chosen, r.unsqueeze(1)], 1)
    return chosen


def _fill_chunks(N, L, off, d, dtype, device, token_fn, chunk_tokens=2_000_000):
    """Allocate docs and fill it doc-chunk by doc-chunk with token_fn(doc_lo, doc_hi, tok_doc)."""
    total = int(off[-1])
    docs = torch.empty((total, d), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32,
                       device=device)
    lo = 0
    while lo < N:
        hi = int(torch.searchsorted(off, off[lo] + chunk_tokens, right=False))
        hi = max(lo + 1, min(N, hi))
        tok_doc = torch.repeat_interleave(torch.arange(lo, hi), L[lo:hi]).to(device)
        x = token_fn(lo, hi, tok_doc)
        docs[int(off[lo]):int(off[hi])] = _store(_unit(x), dtype)
        lo = hi
    return docs


def _plant(docs, off, L, Qf, doc_ids, sigmas, frac, d, dtype, gc, gd, device):
    """Overwrite a fraction of each listed doc's tokens with noisy copies of query tokens."""
    T = Qf.shape[0]
    for i, sg in zip(doc_ids, sigmas):
        Li = int(L[i])
        m = max(1, int(round(frac * Li)))
        pos = torch.randperm(Li, generator=gc)[:m] + int(off[i])
        t = torch.randint(0, T, (m,), generator=gc)
        x = Qf[t.to(device)] + _noise((m, d), d, sg, gd, device)
        docs[pos.to(device)] = _store(_unit(x), dtype)


def text_iid(name, N, Lmin, Lmax, nq, T, d, dtype, n_planted, sigmas, seed, device="cpu",
             frac=0.6, **knobs) -> Workload:
    """i.i.d. Gaussian unit tokens with planted relevant documents per query."""
    gc, gd = _gens(seed, device)
    L, off = _lengths(N, Lmin, Lmax, gc)
    docs = _fill_chunks(N, L, off, d, dtype, device,
                        lambda lo, hi, td: torch.randn((td.shape[0], d), generator=gd,
                                                       device=device))
    Qf = _unit(torch.randn((nq, T, d), generator=gd, device=device))
    Q = _store(Qf, dtype)
    ids = torch.randperm(N, generator=gc)[: nq * n_planted].view(nq, n_planted)
    planted = []
    for q in range(nq):
        sg = [sigmas[k % len(sigmas)] for k in range(n_planted)]
        _plant(docs, off, L, Q[q].float(), ids[q].tolist(), sg, frac, d, dtype, gc, gd, device)
        planted.append(sorted(ids[q].tolist()))
    recipe = (f"N={N}, L~U[{Lmin},{Lmax}], d={d}, iid Gaussian unit tokens, {nq} queries x T={T}, "
              f"{n_planted} planted docs/query ({int(frac*100)}% of tokens = query token + noise "
              f"sigma in {list(sigmas)}), {dtype}")
    return Workload(name, dtype, Q, docs, off.to(device), seed=seed, planted=planted,
                    recipe=recipe, **knobs)


def text_topics(name, N, Lmin, Lmax, nq, T, d, dtype, n_topics, seed, device="cpu",
                topics_per_doc=3, topics_per_query=2, sigma=0.5, **knobs) -> Workload:
    """Gaussian-mixture topic corpus: each doc picks topics, tokens = centroid + noise."""
    gc, gd = _gens(seed, device)
    L, off = _lengths(N, Lmin, Lmax, gc)
    C = _unit(torch.randn((n_topics, d), generator=gd, device=device))
    doc_topics = _distinct(N, n_topics, topics_per_doc, gc)
    doc_topics_d = doc_topics.to(device)

    def token_fn(lo, hi, tok_doc):
        n = tok_doc.shape[0]
        pick = torch.randint(0, topics_per_doc, (n,), generator=gd, device=device)
        top = doc_topics_d[tok_doc, pick]
        return C[top] + _noise((n, d), d, sigma, gd, device)

    docs = _fill_chunks(N, L, off, d, dtype, device, token_fn)
    q_topics = torch.stack([torch.randperm(n_topics, generator=gc)[:topics_per_query]
                            for _ in range(nq)]).to(device)
    pick = torch.randint(0, topics_per_query, (nq, T), generator=gd, device=device)
    Qf = _unit(C[torch.gather(q_topics, 1, pick)] + _noise((nq, T, d), d, sigma, gd, device))
    recipe = (f"N={N}, L~U[{Lmin},{Lmax}], d={d}, {n_topics}-topic Gaussian mixture "
              f"({topics_per_doc} topics/doc, token = centroid + noise sigma={sigma}), "
              f"{nq} queries x T={T} from {topics_per_query} topics each, {dtype}")
    return Workload(name, dtype, _store(Qf, dtype), docs, off.to(device), seed=seed,
                    recipe=recipe, **knobs)


def pages(name, N, L_page, nq, T, d, dtype, n_centroids, seed, device="cpu",
          centroids_per_page=8, centroids_per_query=3, background_frac=0.10,
          background_sigma=0.1, query_sigma=0.5, **knobs) -> Workload:
    """Multimodal page-like corpus: fixed-length docs of patch tokens, heavy-tailed norms
    before normalisation (log-normal multiplier on the centroid part, unit-scale noise)
    and a near-duplicate background patch cluster."""
    gc, gd = _gens(seed, device)
    L = torch.full((N,), L_page, dtype=torch.int64)
    off = torch.arange(N + 1, dtype=torch.int64) * L_page
    C = _unit(torch.randn((n_centroids, d), generator=gd, device=device))
    bg = _unit(torch.randn((d,), generator=gd, device=device))
    page_c = torch.randint(0, n_centroids, (N, centroids_per_page), generator=gc).to(device)

    def token_fn(lo, hi, tok_doc):
        n = tok_doc.shape[0]
        pick = torch.randint(0, centroids_per_page, (n,), generator=gd, device=device)
        cen = C[page_c[tok_doc, pick]]
        mult = torch.exp(torch.randn((n, 1), generator=gd, device=device))
        x = mult * cen + _noise((n, d), d, 1.0, gd, device)
        is_bg = torch.rand((n,), generator=gd, device=device) < background_frac
        xb = bg.unsqueeze(0) + _noise((n, d), d, background_sigma, gd, device)
        return torch.where(is_bg.unsqueeze(1), xb, x)

    docs = _fill_chunks(N, L, off, d, dtype, device, token_fn)
    q_c = torch.stack([torch.randperm(n_centroids, generator=gc)[:centroids_per_query]
                       for _ in range(nq)]).to(device)
    pick = torch.randint(0, centroids_per_query, (nq, T), generator=gd, device=device)
    Qf = _unit(C[torch.gather(q_c, 1, pick)] + _noise((nq, T, d), d, query_sigma, gd, device))
    recipe = (f"N={N} pages x {L_page} patch tokens, d={d}, {n_centroids}-centroid mixture "
              f"({centroids_per_page} centroids/page), log-normal(0,1) norm multiplier + unit "
              f"noise before normalisation, {int(background_frac*100)}% background patches "
              f"(sigma={background_sigma}), {nq} queries x T={T} from {centroids_per_query} "
              f"centroids, {dtype}")
    return Workload(name, dtype, _store(Qf, dtype), docs, off.to(device), seed=seed,
                    recipe=recipe, **knobs)


# The five measured configurations.  `scale` shrinks N (and nothing else) so that the
# same recipe can serve quick tests.
def config(idx: int, device="cpu", scale: float = 1.0, nq: int | None = None,
           seed: int | None = None, d: int = 128) -> Workload:
    """The five synthetic configurations; `d` other than 128 gives the same recipe at another
    embedding width (64: the shape of the paper's Matryoshka-projection experiment)."""
    def n(x):
        return max(64, int(round(x * scale)))

    if idx == 0:   # tiny text rerank, fp32
        return text_iid("C1-tiny-text-f32", n(1000), 32, 64, nq or 1, 32, d, "f32", 5, (0.3,),
                        0 if seed is None else seed, device)
    if idx == 1:   # mid text rerank, bf16
        return text_iid("C2-mid-text-bf16", n(50_000), 32, 180, nq or 64, 32, d, "bf16", 20,
                        (0.2, 0.4, 0.6), 1 if seed is None else seed, device)
    if idx == 2:   # large text corpus, bf16
        return text_topics("C3-large-text-bf16", n(500_000), 32, 180, nq or 128, 32, d, "bf16",
                           1024, 2 if seed is None else seed, device)
    if idx == 3:   # multimodal page-like corpus, bf16
        return pages("C4-pages-bf16", n(20_000), 1030, nq or 64, 24, d, "bf16", 256,
                     3 if seed is None else seed, device)
    if idx == 4:   # knob sweep corpus, bf16
        return text_topics("C5-sweep-bf16", n(100_000), 32, 180, nq or 256, 32, d, "bf16", 512,
                           4 if seed is None else seed, device)
    raise ValueError("config index must be 0..4")
