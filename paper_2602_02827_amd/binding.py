"""ctypes binding of libcolbandit.so: argument marshalling only.

Every step of the scoring path runs in the library's HIP kernels; torch is used here for
device memory (inputs, outputs, workspace) and for the current stream handle.  There is no
fallback: if the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcolbandit.so")

F32, BF16 = 0, 1
MAX_ROUNDS = 64
STATIC_SCRATCH_BYTES = 64 << 20

EXPORTS = [
    "colbandit_full_maxsim", "colbandit_topk", "colbandit_workspace_bytes",
    "colbandit_trace_bytes", "colbandit_permutation", "colbandit_radius_prefactor",
    "colbandit_validate_offsets", "colbandit_strerror", "colbandit_sizeof_opts",
    "colbandit_sizeof_stats", "colbandit_quantize_i8", "colbandit_quantize_workspace_bytes",
    "colbandit_coarse_maxsim", "colbandit_doc_uniform", "colbandit_doc_uniform_workspace_bytes",
    "colbandit_ball_carving", "colbandit_ball_carving_workspace_bytes", "colbandit_cells_per_doc",
    "colbandit_topk_static",
]


class ColbanditOpts(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int), ("a", ctypes.c_float), ("b", ctypes.c_float),
                ("pi", ctypes.c_void_p), ("trace", ctypes.c_void_p),
                ("trace_bytes", ctypes.c_size_t), ("force_gather", ctypes.c_int),
                ("no_cell_cache", ctypes.c_int), ("docs_i8", ctypes.c_void_p),
                ("docs_scale", ctypes.c_void_p), ("coarse_permille", ctypes.c_int),
                ("later_rounds", ctypes.c_int)]


class ColbanditStats(ctypes.Structure):
    _fields_ = [("rounds", ctypes.c_int32), ("survivors", ctypes.c_int32 * (MAX_ROUNDS + 2)),
                ("cells_elim", ctypes.c_int64), ("cells_rescore", ctypes.c_int64),
                ("cells_unique", ctypes.c_int64), ("ms_total", ctypes.c_float),
                ("ms_first_reveal", ctypes.c_float), ("ms_later_reveals", ctypes.c_float),
                ("ms_select_prune", ctypes.c_float), ("ms_rescore_topk", ctypes.c_float),
                ("ms_reveal_round2", ctypes.c_float), ("corpus_pass_rounds", ctypes.c_uint64),
                ("cells_computed", ctypes.c_int64), ("pairs_round2", ctypes.c_uint64),
                ("tokens_round2", ctypes.c_uint64)]


class ColbanditError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: {strerror(code)} ({code})")


_lib = None


def lib():
    """Loads the built library; raises if it is missing (build it with build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} not built: run `python -m paper_2602_02827_amd.build` "
                "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, i64, sz, f = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_float
        L.colbandit_full_maxsim.restype = i
        L.colbandit_full_maxsim.argtypes = [vp, i, i, i, i, vp, vp, i64, i64, i, vp, vp, vp, vp,
                                            ctypes.POINTER(ctypes.c_float), vp, sz, vp]
        L.colbandit_topk.restype = i
        L.colbandit_topk.argtypes = [vp, i, i, i, i, vp, vp, i64, i64, i, f, f, i, ctypes.c_uint64,
                                     ctypes.POINTER(ColbanditOpts), vp, vp,
                                     ctypes.POINTER(ColbanditStats), vp, sz, vp]
        L.colbandit_topk_static.restype = i
        L.colbandit_topk_static.argtypes = [vp, i, i, i, i, vp, vp, i64, i64, i, f, f, i, ctypes.c_uint64,
                                            ctypes.POINTER(ColbanditOpts), vp, vp, vp]
        L.colbandit_workspace_bytes.restype = sz
        L.colbandit_workspace_bytes.argtypes = [i, i, i, i64, i64, i, i]
        L.colbandit_trace_bytes.restype = sz
        L.colbandit_trace_bytes.argtypes = [i, i, i, i64]
        L.colbandit_permutation.restype = i
        L.colbandit_permutation.argtypes = [ctypes.c_uint64, i64, i, vp]
        L.colbandit_radius_prefactor.restype = ctypes.c_double
        L.colbandit_radius_prefactor.argtypes = [f, f, i, i64, i]
        L.colbandit_validate_offsets.restype = i
        L.colbandit_validate_offsets.argtypes = [vp, i64, i64, vp, sz, vp]
        L.colbandit_quantize_workspace_bytes.restype = sz
        L.colbandit_quantize_workspace_bytes.argtypes = [i64]
        L.colbandit_quantize_i8.restype = i
        L.colbandit_quantize_i8.argtypes = [vp, i, i64, i64, i, i, vp, vp, vp, sz, vp]
        L.colbandit_coarse_maxsim.restype = i
        L.colbandit_coarse_maxsim.argtypes = [vp, i, i, i, i, vp, vp, vp, i64, i64, i, vp, vp, vp, vp,
                                              vp, sz, vp]
        L.colbandit_doc_uniform_workspace_bytes.restype = sz
        L.colbandit_doc_uniform_workspace_bytes.argtypes = [i, i, i, i64, i64]
        L.colbandit_doc_uniform.restype = i
        L.colbandit_doc_uniform.argtypes = [vp, i, i, i, i, vp, vp, i64, i64, i, i, ctypes.c_uint64,
                                            vp, vp, vp, vp, vp, sz, vp]
        L.colbandit_ball_carving_workspace_bytes.restype = sz
        L.colbandit_ball_carving_workspace_bytes.argtypes = [i, i, i, i, i64, i64]
        L.colbandit_ball_carving.restype = i
        L.colbandit_ball_carving.argtypes = [vp, i, i, i, i, vp, vp, i64, i64, i, f, vp, vp, vp, vp,
                                             vp, vp, vp, sz, vp]
        L.colbandit_cells_per_doc.restype = i
        L.colbandit_cells_per_doc.argtypes = [ctypes.c_double, i]
        L.colbandit_sizeof_opts.restype = sz
        L.colbandit_sizeof_opts.argtypes = []
        L.colbandit_sizeof_stats.restype = sz
        L.colbandit_sizeof_stats.argtypes = []
        if (L.colbandit_sizeof_opts() != ctypes.sizeof(ColbanditOpts)
                or L.colbandit_sizeof_stats() != ctypes.sizeof(ColbanditStats)):
            raise ImportError("libcolbandit.so was built from a different colbandit.h: rebuild it")
        L.colbandit_strerror.restype = ctypes.c_char_p
        L.colbandit_strerror.argtypes = [i]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().colbandit_strerror(int(code)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise TypeError("Q / doc_tokens must be float32 or bfloat16")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _shapes(Q, docs, offsets):
    if Q.dim() == 2:
        Q = Q.unsqueeze(0)
    assert Q.is_contiguous() and docs.is_contiguous() and offsets.is_contiguous()
    assert offsets.dtype == torch.int64 and Q.shape[2] == docs.shape[1]
    assert Q.dtype == docs.dtype or docs.dtype == torch.int8
    nq, T, d = Q.shape
    return Q, nq, T, d, int(offsets.shape[0] - 1), int(docs.shape[0])


def colbandit_workspace_bytes(nq, T, d, N, total_tokens, K=0, M=0) -> int:
    return int(lib().colbandit_workspace_bytes(nq, T, d, N, total_tokens, K, M))


def colbandit_trace_bytes(nq, T, B, N) -> int:
    return int(lib().colbandit_trace_bytes(nq, T, B, N))


def colbandit_permutation(seed: int, query_index: int, T: int) -> np.ndarray:
    pi = np.empty(T, dtype=np.int32)
    rc = lib().colbandit_permutation(ctypes.c_uint64(seed & (2**64 - 1)), query_index, T,
                                     pi.ctypes.data_as(ctypes.c_void_p))
    if rc:
        raise ColbanditError(rc, "colbandit_permutation")
    return pi


def colbandit_radius_prefactor(alpha_ef, delta, T, N, n) -> float:
    return float(lib().colbandit_radius_prefactor(alpha_ef, delta, T, N, n))


def new_workspace(nq, T, d, N, total_tokens, device="cuda") -> torch.Tensor:
    return torch.empty(colbandit_workspace_bytes(nq, T, d, N, total_tokens), dtype=torch.uint8,
                       device=device)


def colbandit_validate_offsets(offsets: torch.Tensor, total_tokens: int, workspace=None) -> int:
    ws = workspace if workspace is not None else torch.empty(256, dtype=torch.uint8,
                                                             device=offsets.device)
    return int(lib().colbandit_validate_offsets(_ptr(offsets), offsets.shape[0] - 1, total_tokens,
                                                _ptr(ws), ws.numel(), _stream()))


def colbandit_full_maxsim(Q, docs, offsets, K=0, want_scores=True, want_cells=False,
                          workspace=None, out=None, want_phase_ms=False):
    """Exhaustive scoring.  Returns dict(scores [nq,N] | None, topk_ids, topk_scores, cells,
    phase_ms).  `want_phase_ms` makes the call synchronous and returns (scoring kernel ms,
    top-K ms) measured by the library with events on the launch stream."""
    Q, nq, T, d, N, total = _shapes(Q, docs, offsets)
    dev = docs.device
    ws = workspace if workspace is not None else new_workspace(nq, T, d, N, total, dev)
    o = out or {}
    scores = o.get("scores")
    if scores is None and (want_scores or K == 0):
        scores = torch.empty((nq, N), dtype=torch.float32, device=dev)
    ids = sc = None
    if K > 0:
        ids = o.get("topk_ids") if o.get("topk_ids") is not None else \
            torch.empty((nq, K), dtype=torch.int64, device=dev)
        sc = o.get("topk_scores") if o.get("topk_scores") is not None else \
            torch.empty((nq, K), dtype=torch.float32, device=dev)
    cells = torch.empty((nq, N, T), dtype=torch.float32, device=dev) if want_cells else None
    phase = (ctypes.c_float * 2)() if want_phase_ms else None
    rc = lib().colbandit_full_maxsim(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs), _ptr(offsets), N, total,
                                     K, _ptr(scores), _ptr(ids), _ptr(sc), _ptr(cells), phase,
                                     _ptr(ws), ws.numel(), _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_full_maxsim")
    return {"scores": scores, "topk_ids": ids, "topk_scores": sc, "cells": cells,
            "phase_ms": (phase[0], phase[1]) if want_phase_ms else None}


def colbandit_quantize_i8(x, n_segments=1, permille=999):
    """int8 codes of x ([rows, d], rows = n_segments * rows_per_segment).  Returns
    (codes int8 like x, scales float32 [n_segments])."""
    assert x.is_contiguous() and x.dim() >= 2
    d = x.shape[-1]
    rows = x.numel() // d
    assert rows % n_segments == 0
    codes = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    scales = torch.empty((n_segments,), dtype=torch.float32, device=x.device)
    nb = lib().colbandit_quantize_workspace_bytes(n_segments)
    ws = torch.empty((nb,), dtype=torch.uint8, device=x.device)
    rc = lib().colbandit_quantize_i8(_ptr(x), _dt(x), n_segments, rows // n_segments, d, int(permille),
                                     _ptr(codes), _ptr(scales), _ptr(ws), nb, _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_quantize_i8")
    return codes, scales


def colbandit_coarse_maxsim(Q, docs_i8, docs_scale, offsets, permille=999, want_cells=False,
                            workspace=None):
    """Exhaustive MaxSim on int8 codes.  Returns dict(scores, cells, q_codes, q_scales)."""
    Q, nq, T, d, N, total = _shapes(Q, docs_i8, offsets)
    dev = docs_i8.device
    ws = workspace if workspace is not None else new_workspace(nq, T, d, N, total, dev)
    scores = torch.empty((nq, N), dtype=torch.float32, device=dev)
    cells = torch.empty((nq, N, T), dtype=torch.float32, device=dev) if want_cells else None
    qc = torch.empty((nq, T, d), dtype=torch.int8, device=dev)
    qs = torch.empty((nq,), dtype=torch.float32, device=dev)
    rc = lib().colbandit_coarse_maxsim(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs_i8), _ptr(docs_scale),
                                       _ptr(offsets), N, total, int(permille), _ptr(scores), _ptr(cells),
                                       _ptr(qc), _ptr(qs), _ptr(ws), ws.numel(), _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_coarse_maxsim")
    return {"scores": scores, "cells": cells, "q_codes": qc, "q_scales": qs}


def colbandit_cells_per_doc(gamma: float, T: int) -> int:
    """Cells per document of Doc-Uniform at coverage gamma (computed by the library)."""
    m = int(lib().colbandit_cells_per_doc(ctypes.c_double(gamma), int(T)))
    if m < 0:
        raise ColbanditError(m, "colbandit_cells_per_doc")
    return m


def colbandit_doc_uniform(Q, docs, offsets, K, m, seed=0, want_scores=True, want_masks=False,
                          workspace=None):
    """Doc-Uniform baseline with m cells per document.  Returns dict(scores, masks (int64 view
    of the uint64 bit masks), topk_ids, topk_scores)."""
    Q, nq, T, d, N, total = _shapes(Q, docs, offsets)
    dev = docs.device
    nb = int(lib().colbandit_doc_uniform_workspace_bytes(nq, T, d, N, total))
    ws = workspace if workspace is not None else torch.empty(nb, dtype=torch.uint8, device=dev)
    scores = torch.empty((nq, N), dtype=torch.float32, device=dev) if (want_scores or K == 0) else None
    masks = torch.empty((nq, N), dtype=torch.int64, device=dev) if want_masks else None
    ids = torch.empty((nq, K), dtype=torch.int64, device=dev) if K > 0 else None
    sc = torch.empty((nq, K), dtype=torch.float32, device=dev) if K > 0 else None
    rc = lib().colbandit_doc_uniform(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs), _ptr(offsets), N, total,
                                     int(K), int(m), ctypes.c_uint64(seed & (2**64 - 1)),
                                     _ptr(scores), _ptr(masks), _ptr(ids), _ptr(sc), _ptr(ws),
                                     ws.numel(), _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_doc_uniform")
    return {"scores": scores, "masks": masks, "topk_ids": ids, "topk_scores": sc}


def colbandit_ball_carving(Q, docs, offsets, K, tau, want_scores=True, workspace=None):
    """Ball-carving baseline at cosine threshold tau.  Returns dict(n_clusters [nq] int32,
    labels [nq,T] int32, centroids [nq,T,d] (storage dtype), scores, topk_ids, topk_scores)."""
    Q, nq, T, d, N, total = _shapes(Q, docs, offsets)
    dev = docs.device
    nb = int(lib().colbandit_ball_carving_workspace_bytes(nq, T, d, _dt(Q), N, total))
    ws = workspace if workspace is not None else torch.empty(nb, dtype=torch.uint8, device=dev)
    kq = torch.empty((nq,), dtype=torch.int32, device=dev)
    labels = torch.empty((nq, T), dtype=torch.int32, device=dev)
    cent = torch.empty((nq, T, d), dtype=Q.dtype, device=dev)
    scores = torch.empty((nq, N), dtype=torch.float32, device=dev) if (want_scores or K == 0) else None
    ids = torch.empty((nq, K), dtype=torch.int64, device=dev) if K > 0 else None
    sc = torch.empty((nq, K), dtype=torch.float32, device=dev) if K > 0 else None
    rc = lib().colbandit_ball_carving(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs), _ptr(offsets), N, total,
                                      int(K), ctypes.c_float(tau), _ptr(kq), _ptr(labels), _ptr(cent),
                                      _ptr(scores), _ptr(ids), _ptr(sc), _ptr(ws), ws.numel(),
                                      _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_ball_carving")
    return {"n_clusters": kq, "labels": labels, "centroids": cent, "scores": scores,
            "topk_ids": ids, "topk_scores": sc}


@dataclass
class Trace:
    count: np.ndarray    # [R+1, nq]
    tau: np.ndarray      # [R, nq]
    lcb: np.ndarray      # [R, nq, N]
    ucb: np.ndarray
    alive: np.ndarray    # bool


def _parse_trace(buf: torch.Tensor, nq, T, B, N, queries=None) -> Trace:
    """Splits the device trace buffer; `queries` keeps only those query columns (in that order)."""
    R = (T + B - 1) // B
    al = lambda x: (x + 255) // 256 * 256
    qs = list(range(nq)) if queries is None else list(queries)
    qi = torch.as_tensor(qs, dtype=torch.int64, device=buf.device)

    def part(o, nbytes, dtype, shape):
        t = buf[o:o + nbytes].view(dtype).view(shape)
        return t.index_select(1, qi).cpu().numpy()

    o = 0
    count = part(o, 4 * (R + 1) * nq, torch.int32, (R + 1, nq)); o += al(4 * (R + 1) * nq)
    tau = part(o, 4 * R * nq, torch.float32, (R, nq)); o += al(4 * R * nq)
    lcb = part(o, 4 * R * nq * N, torch.float32, (R, nq, N)); o += al(4 * R * nq * N)
    ucb = part(o, 4 * R * nq * N, torch.float32, (R, nq, N)); o += al(4 * R * nq * N)
    alive = part(o, R * nq * N, torch.uint8, (R, nq, N)).astype(bool)
    return Trace(count, tau, lcb, ucb, alive)


def colbandit_topk(Q, docs, offsets, K, alpha_ef=0.2, delta=0.01, M=5, seed=0, B=0, a=0.0, b=0.0,
                   pi=None, trace=False, force_gather=False, want_stats=True, workspace=None,
                   out=None, no_cell_cache=False, trace_queries=None, later_rounds=0,
                   docs_i8=None, docs_scale=None, coarse_permille=0):
    """Col-Bandit top-K.  Returns dict(topk_ids, topk_scores, stats (list of dict) | None,
    trace (Trace) | None).  `pi`: optional int32 device tensor [nq,T]; `trace_queries`: keep
    only these queries' columns of the trace (the device buffer still covers all of them);
    `later_rounds`: 0 auto, 1 corpus-streaming pass in every round >= 2, 2 always gather;
    `docs_i8`/`docs_scale` (from colbandit_quantize_i8): run the elimination rounds on int8
    codes, rescore exactly."""
    Q, nq, T, d, N, total = _shapes(Q, docs, offsets)
    dev = docs.device
    ws = workspace if workspace is not None else new_workspace(nq, T, d, N, total, dev)
    o = out or {}
    ids = o.get("topk_ids") if o.get("topk_ids") is not None else \
        torch.empty((nq, K), dtype=torch.int64, device=dev)
    sc = o.get("topk_scores") if o.get("topk_scores") is not None else \
        torch.empty((nq, K), dtype=torch.float32, device=dev)
    opts = ColbanditOpts(B=B, a=a, b=b, pi=None, trace=None, trace_bytes=0,
                         force_gather=1 if force_gather else 0,
                         no_cell_cache=1 if no_cell_cache else 0, later_rounds=int(later_rounds),
                         docs_i8=None if docs_i8 is None else docs_i8.data_ptr(),
                         docs_scale=None if docs_scale is None else docs_scale.data_ptr(),
                         coarse_permille=int(coarse_permille))
    tbuf = None
    Beff = B if B > 0 else 4
    if pi is not None:
        assert pi.dtype == torch.int32 and pi.is_contiguous() and tuple(pi.shape) == (nq, T)
        opts.pi = pi.data_ptr()
    if trace:
        tbuf = torch.empty(colbandit_trace_bytes(nq, T, Beff, N), dtype=torch.uint8, device=dev)
        opts.trace = tbuf.data_ptr()
        opts.trace_bytes = tbuf.numel()
    stats = (ColbanditStats * nq)() if want_stats else None
    rc = lib().colbandit_topk(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs), _ptr(offsets), N, total, K,
                              alpha_ef, delta, M, ctypes.c_uint64(seed & (2**64 - 1)),
                              ctypes.byref(opts), _ptr(ids), _ptr(sc), stats, _ptr(ws), ws.numel(),
                              _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_topk")
    st = None
    if stats is not None:
        st = [{"rounds": s.rounds, "survivors": list(s.survivors[: s.rounds + 1]),
               "cells_elim": s.cells_elim, "cells_rescore": s.cells_rescore,
               "cells_unique": s.cells_unique, "ms_total": s.ms_total,
               "ms_first_reveal": s.ms_first_reveal, "ms_later_reveals": s.ms_later_reveals,
               "ms_select_prune": s.ms_select_prune, "ms_rescore_topk": s.ms_rescore_topk,
               "ms_reveal_round2": s.ms_reveal_round2, "cells_computed": s.cells_computed,
               "pairs_round2": s.pairs_round2, "tokens_round2": s.tokens_round2,
               "corpus_pass_rounds": [r + 1 for r in range(64) if (s.corpus_pass_rounds >> r) & 1]}
              for s in stats]
    tr = None
    if trace:
        torch.cuda.synchronize()
        tr = _parse_trace(tbuf, nq, T, Beff, N, trace_queries)
    return {"topk_ids": ids, "topk_scores": sc, "stats": st, "trace": tr}


def colbandit_topk_static(Q, docs, offsets, K, alpha_ef=0.2, delta=0.01, M=5, seed=0, B=0, out=None,
                          docs_i8=None, docs_scale=None):
    """colbandit_topk on the library's built-in scratch buffer: no workspace, no statistics,
    nothing allocated by the call (`out` supplies the two output tensors; they are created
    here only when it is omitted).  Returns dict(topk_ids, topk_scores)."""
    Q, nq, T, d, N, total = _shapes(Q, docs, offsets)
    dev = docs.device
    o = out or {}
    ids = o.get("topk_ids") if o.get("topk_ids") is not None else \
        torch.empty((nq, K), dtype=torch.int64, device=dev)
    sc = o.get("topk_scores") if o.get("topk_scores") is not None else \
        torch.empty((nq, K), dtype=torch.float32, device=dev)
    opts = ColbanditOpts(B=B, a=0.0, b=0.0, pi=None, trace=None, trace_bytes=0, force_gather=0,
                         no_cell_cache=0, later_rounds=0,
                         docs_i8=None if docs_i8 is None else docs_i8.data_ptr(),
                         docs_scale=None if docs_scale is None else docs_scale.data_ptr(),
                         coarse_permille=0)
    rc = lib().colbandit_topk_static(_ptr(Q), nq, T, d, _dt(Q), _ptr(docs), _ptr(offsets), N, total, K,
                                     alpha_ef, delta, M, ctypes.c_uint64(seed & (2**64 - 1)),
                                     ctypes.byref(opts), _ptr(ids), _ptr(sc), _stream())
    if rc:
        raise ColbanditError(rc, "colbandit_topk_static")
    return {"topk_ids": ids, "topk_scores": sc}
