"""CPU oracle for the Col-Bandit scoring path (ctypes front of colbandit_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  The product package never imports this module
and this module never imports the product package.

All arithmetic lives in the C file; this module only marshals numpy arrays.
Citations (paper): MaxSim cell / score Eq. (1)-(2), (4)-(5); top-K Eq. (3);
bounds Eq. (7)-(8) and Appendix A; Algorithm 1 and its detailed listing; the Doc-Uniform and
Ball-carving baselines of the appendix "Compared Methods".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "colbandit_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


_SELFTEST_SRC = os.path.join(_HERE, "selftest.c")
_SELFTEST = os.path.join(_HERE, "selftest.bin")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP across queries, no intrinsics)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_selftest(sanitize: bool = True, out: str | None = None) -> str:
    """Compile the oracle together with its driver selftest.c into an executable, by default
    under AddressSanitizer + UndefinedBehaviorSanitizer (host code only)."""
    out = out or _SELFTEST
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-fno-omit-frame-pointer"]
    if sanitize:
        cmd += ["-fsanitize=address,undefined", "-fno-sanitize-recover=all"]
    cmd += [_SRC, _SELFTEST_SRC, "-lm", "-o", out]
    subprocess.run(cmd, check=True)
    return out


_lib = None


def _L():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.oracle_cell.restype = ctypes.c_double
        _lib.oracle_rho.restype = ctypes.c_double
        _lib.oracle_rho.argtypes = [ctypes.c_int, ctypes.c_int]
        _lib.oracle_radius.restype = ctypes.c_double
        _lib.oracle_radius.argtypes = [ctypes.c_double, ctypes.c_int, ctypes.c_double,
                                       ctypes.c_int64, ctypes.c_double, ctypes.c_int]
        _lib.oracle_splitmix64_next.restype = ctypes.c_uint64
        _lib.oracle_uniform_subset.restype = ctypes.c_uint64
        _lib.oracle_uniform_subset.argtypes = [ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64,
                                               ctypes.c_int, ctypes.c_int]
        _lib.oracle_round_bf16.restype = ctypes.c_float
        _lib.oracle_round_bf16.argtypes = [ctypes.c_float]
    return _lib


def _p(a, ct):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ct))


def _f32(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.float32))


def _i64(x):
    return np.ascontiguousarray(np.asarray(x, dtype=np.int64))


def _check(rc, what):
    if rc < 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")
    return rc


def maxsim_cells(Q, E, offsets):
    """H[N,T] in float64: Eq. (4)."""
    Q, E, offsets = _f32(Q), _f32(E), _i64(offsets)
    T, d = Q.shape
    N = offsets.shape[0] - 1
    H = np.empty((N, T), dtype=np.float64)
    _check(_L().oracle_maxsim_cells(_p(Q, ctypes.c_float), T, d, _p(E, ctypes.c_float),
                                    _p(offsets, ctypes.c_int64), ctypes.c_int64(N),
                                    _p(H, ctypes.c_double)), "maxsim_cells")
    return H


def row_sums(H):
    """S[N]: Eq. (5)."""
    H = np.ascontiguousarray(H, dtype=np.float64)
    N, T = H.shape
    S = np.empty(N, dtype=np.float64)
    _check(_L().oracle_row_sums(_p(H, ctypes.c_double), ctypes.c_int64(N), T,
                                _p(S, ctypes.c_double)), "row_sums")
    return S


def topk(S, K, ids=None):
    """First K of the (score desc, id asc) order: Eq. (3)."""
    S = np.ascontiguousarray(S, dtype=np.float64)
    n = S.shape[0]
    ids_a = None if ids is None else _i64(ids)
    m = min(K, n)
    out_ids = np.empty(m, dtype=np.int64)
    out_s = np.empty(m, dtype=np.float64)
    _check(_L().oracle_topk(_p(S, ctypes.c_double), _p(ids_a, ctypes.c_int64),
                            ctypes.c_int64(n), K, _p(out_ids, ctypes.c_int64),
                            _p(out_s, ctypes.c_double)), "topk")
    return out_ids, out_s


def rho(n, T):
    return _L().oracle_rho(int(n), int(T))


def radius(alpha, T, sigma, N, delta, n):
    return _L().oracle_radius(float(alpha), int(T), float(sigma), int(N), float(delta), int(n))


def bounds(vals, T, a, b, alpha, delta, N):
    """dict(lcb, ucb, mean, sigma, radius, lb_hard, ub_hard) from revealed values."""
    vals = np.ascontiguousarray(vals, dtype=np.float64)
    out = np.empty(7, dtype=np.float64)
    _check(_L().oracle_bounds(_p(vals, ctypes.c_double), int(vals.shape[0]), int(T),
                              ctypes.c_double(a), ctypes.c_double(b), ctypes.c_double(alpha),
                              ctypes.c_double(delta), ctypes.c_int64(N),
                              _p(out, ctypes.c_double)), "bounds")
    keys = ("lcb", "ucb", "mean", "sigma", "radius", "lb_hard", "ub_hard")
    return dict(zip(keys, out.tolist()))


def splitmix64_stream(state, count):
    st = ctypes.c_uint64(state)
    return [int(_L().oracle_splitmix64_next(ctypes.byref(st))) for _ in range(count)]


def permutation(seed, query_index, T):
    pi = np.empty(T, dtype=np.int32)
    _check(_L().oracle_permutation(ctypes.c_uint64(seed & (2**64 - 1)),
                                   ctypes.c_int64(query_index), int(T),
                                   _p(pi, ctypes.c_int32)), "permutation")
    return pi


@dataclass
class ColBanditResult:
    topk_ids: np.ndarray
    topk_scores: np.ndarray
    final_ids: np.ndarray
    rounds: int
    counts: np.ndarray            # |A_r| entering each round, then after the last one
    tau: np.ndarray               # [rounds]
    cells_elim: int
    cells_rescore: int
    cells_unique: int
    lcb: np.ndarray | None = None     # [rounds, N], NaN where inactive
    ucb: np.ndarray | None = None
    alive: np.ndarray | None = None   # [rounds, N] membership of A_{r+1}
    extra: dict = field(default_factory=dict)


def colbandit_from_H(H, K, M, B, alpha, delta, pi, a=-1.0, b=1.0, trace=True):
    """Algorithm 1 over a given MaxSim matrix."""
    H = np.ascontiguousarray(H, dtype=np.float64)
    N, T = H.shape
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    Rmax = (T + B - 1) // B
    out_ids = np.full(K, -1, dtype=np.int64)
    out_s = np.full(K, np.nan, dtype=np.float64)
    final_ids = np.empty(N, dtype=np.int64)
    n_final = ctypes.c_int64(0)
    counts = np.full(Rmax + 1, -1, dtype=np.int64)
    tau = np.full(Rmax, np.nan, dtype=np.float64)
    cells = np.zeros(3, dtype=np.int64)
    lcb = np.empty((Rmax, N), dtype=np.float64) if trace else None
    ucb = np.empty((Rmax, N), dtype=np.float64) if trace else None
    alive = np.empty((Rmax, N), dtype=np.uint8) if trace else None
    rc = _check(_L().oracle_colbandit_from_H(
        _p(H, ctypes.c_double), ctypes.c_int64(N), T, K, M, B,
        ctypes.c_double(alpha), ctypes.c_double(delta), ctypes.c_double(a), ctypes.c_double(b),
        _p(pi, ctypes.c_int32), _p(out_ids, ctypes.c_int64), _p(out_s, ctypes.c_double),
        _p(final_ids, ctypes.c_int64), ctypes.byref(n_final), _p(counts, ctypes.c_int64),
        _p(tau, ctypes.c_double), _p(lcb, ctypes.c_double), _p(ucb, ctypes.c_double),
        _p(alive, ctypes.c_uint8), _p(cells, ctypes.c_int64)), "colbandit_from_H")
    return ColBanditResult(out_ids, out_s, final_ids[: n_final.value].copy(), rc,
                           counts[: rc + 1].copy(), tau[:rc].copy(),
                           int(cells[0]), int(cells[1]), int(cells[2]),
                           None if lcb is None else lcb[:rc],
                           None if ucb is None else ucb[:rc],
                           None if alive is None else alive[:rc].astype(bool))


def colbandit_coarse(H_coarse, H_exact, K, M, B, alpha, delta, pi, a=-1.0, b=1.0, trace=True):
    """Algorithm 1 deciding on coarse cells and rescoring the survivors from exact ones
    (implementation appendix, cache-separated quantized layout)."""
    Hc = np.ascontiguousarray(H_coarse, dtype=np.float64)
    He = np.ascontiguousarray(H_exact, dtype=np.float64)
    assert Hc.shape == He.shape
    N, T = Hc.shape
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    Rmax = (T + B - 1) // B
    out_ids = np.full(K, -1, dtype=np.int64)
    out_s = np.full(K, np.nan, dtype=np.float64)
    final_ids = np.empty(N, dtype=np.int64)
    n_final = ctypes.c_int64(0)
    counts = np.full(Rmax + 1, -1, dtype=np.int64)
    tau = np.full(Rmax, np.nan, dtype=np.float64)
    cells = np.zeros(3, dtype=np.int64)
    lcb = np.empty((Rmax, N), dtype=np.float64) if trace else None
    ucb = np.empty((Rmax, N), dtype=np.float64) if trace else None
    alive = np.empty((Rmax, N), dtype=np.uint8) if trace else None
    rc = _check(_L().oracle_colbandit_coarse(
        _p(Hc, ctypes.c_double), _p(He, ctypes.c_double), ctypes.c_int64(N), T, K, M, B,
        ctypes.c_double(alpha), ctypes.c_double(delta), ctypes.c_double(a), ctypes.c_double(b),
        _p(pi, ctypes.c_int32), _p(out_ids, ctypes.c_int64), _p(out_s, ctypes.c_double),
        _p(final_ids, ctypes.c_int64), ctypes.byref(n_final), _p(counts, ctypes.c_int64),
        _p(tau, ctypes.c_double), _p(lcb, ctypes.c_double), _p(ucb, ctypes.c_double),
        _p(alive, ctypes.c_uint8), _p(cells, ctypes.c_int64)), "colbandit_coarse")
    return ColBanditResult(out_ids, out_s, final_ids[: n_final.value].copy(), rc,
                           counts[: rc + 1].copy(), tau[:rc].copy(),
                           int(cells[0]), int(cells[1]), int(cells[2]),
                           None if lcb is None else lcb[:rc],
                           None if ucb is None else ucb[:rc],
                           None if alive is None else alive[:rc].astype(bool))


def colbandit_resume(H, K, M, B, alpha, delta, pi, active_ids, r0, a=-1.0, b=1.0, H_exact=None):
    """Algorithm 1 entered at round r0 (1-based) with the active set `active_ids` (ascending
    document indices) whose first (r0-1)*B cells of the shared order count as revealed.  The
    result's per-round arrays are indexed by absolute round: entries below r0-1 are the
    initial fill (NaN / -1 / False); `rounds` is the index of the last executed round;
    cells_elim counts the resumed rounds only.  H_exact: exact cells for the rescore when H
    holds coarse ones."""
    H = np.ascontiguousarray(H, dtype=np.float64)
    He = None if H_exact is None else np.ascontiguousarray(H_exact, dtype=np.float64)
    N, T = H.shape
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    A0 = _i64(active_ids)
    Rmax = (T + B - 1) // B
    out_ids = np.full(K, -1, dtype=np.int64)
    out_s = np.full(K, np.nan, dtype=np.float64)
    final_ids = np.empty(N, dtype=np.int64)
    n_final = ctypes.c_int64(0)
    counts = np.full(Rmax + 1, -1, dtype=np.int64)
    tau = np.full(Rmax, np.nan, dtype=np.float64)
    cells = np.zeros(3, dtype=np.int64)
    lcb = np.empty((Rmax, N), dtype=np.float64)
    ucb = np.empty((Rmax, N), dtype=np.float64)
    alive = np.empty((Rmax, N), dtype=np.uint8)
    rc = _check(_L().oracle_colbandit_resume(
        _p(H, ctypes.c_double), _p(He, ctypes.c_double), ctypes.c_int64(N), T, K, M, B,
        ctypes.c_double(alpha), ctypes.c_double(delta), ctypes.c_double(a), ctypes.c_double(b),
        _p(pi, ctypes.c_int32), _p(A0, ctypes.c_int64), ctypes.c_int64(A0.shape[0]), int(r0),
        _p(out_ids, ctypes.c_int64), _p(out_s, ctypes.c_double),
        _p(final_ids, ctypes.c_int64), ctypes.byref(n_final), _p(counts, ctypes.c_int64),
        _p(tau, ctypes.c_double), _p(lcb, ctypes.c_double), _p(ucb, ctypes.c_double),
        _p(alive, ctypes.c_uint8), _p(cells, ctypes.c_int64)), "colbandit_resume")
    return ColBanditResult(out_ids, out_s, final_ids[: n_final.value].copy(), rc,
                           counts[: rc + 1].copy(), tau[:rc].copy(),
                           int(cells[0]), int(cells[1]), int(cells[2]),
                           lcb[:rc], ucb[:rc], alive[:rc].astype(bool))


def abs_percentile(x, permille=999) -> float:
    """Nearest-rank percentile (permille/1000) of |x| over all entries of x."""
    x = np.ascontiguousarray(x, dtype=np.float32).reshape(-1)
    out = ctypes.c_float(0.0)
    _check(_L().oracle_abs_percentile(_p(x, ctypes.c_float), ctypes.c_int64(x.size), int(permille),
                                      ctypes.byref(out)), "abs_percentile")
    return float(out.value)


def quantize_i8(x, clip) -> np.ndarray:
    """int8 codes of x after clipping at +-clip (same shape as x)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty(x.shape, dtype=np.int8)
    _check(_L().oracle_quantize_i8(_p(x, ctypes.c_float), ctypes.c_int64(x.size), ctypes.c_float(clip),
                                   _p(out, ctypes.c_int8)), "quantize_i8")
    return out


def maxsim_cells_i8(Q8, sq, D8, sd, offsets):
    """(H [N,T] float64 decoded coarse cells, Hint [N,T] int32 integer maxima)."""
    Q8 = np.ascontiguousarray(Q8, dtype=np.int8)
    D8 = np.ascontiguousarray(D8, dtype=np.int8)
    offsets = _i64(offsets)
    T, d = Q8.shape
    N = offsets.shape[0] - 1
    H = np.empty((N, T), dtype=np.float64)
    Hint = np.empty((N, T), dtype=np.int32)
    _check(_L().oracle_maxsim_cells_i8(_p(Q8, ctypes.c_int8), ctypes.c_float(sq), T, d,
                                       _p(D8, ctypes.c_int8), ctypes.c_float(sd),
                                       _p(offsets, ctypes.c_int64), ctypes.c_int64(N),
                                       _p(H, ctypes.c_double), _p(Hint, ctypes.c_int32)),
           "maxsim_cells_i8")
    return H, Hint


def cells_per_doc(gamma, T) -> int:
    """ceil(gamma * T) of Doc-Uniform's algorithm box (decimal gamma, see the C source)."""
    _L().oracle_cells_per_doc.argtypes = [ctypes.c_double, ctypes.c_int]
    return _check(_L().oracle_cells_per_doc(float(gamma), int(T)), "cells_per_doc")


def uniform_subset(seed, q, i, T, m) -> int:
    """Bit mask of the m query tokens Doc-Uniform reveals for (query q, document i)."""
    return int(_L().oracle_uniform_subset(ctypes.c_uint64(seed & (2**64 - 1)), int(q), int(i),
                                          int(T), int(m)))


def doc_uniform_from_H(H, m, seed, query_index, K):
    """Doc-Uniform over a MaxSim matrix H [N,T] (appendix "Compared Methods"): returns
    (masks [N] uint64, S [N] float64 partial sums, top-K ids, top-K scores)."""
    H = np.ascontiguousarray(H, dtype=np.float64)
    N, T = H.shape
    masks = np.empty(N, dtype=np.uint64)
    S = np.empty(N, dtype=np.float64)
    ids = np.empty(K, dtype=np.int64)
    sc = np.empty(K, dtype=np.float64)
    _check(_L().oracle_doc_uniform_from_H(_p(H, ctypes.c_double), ctypes.c_int64(N), T, int(m),
                                          ctypes.c_uint64(seed & (2**64 - 1)),
                                          ctypes.c_int64(query_index), int(K),
                                          _p(masks, ctypes.c_uint64), _p(S, ctypes.c_double),
                                          _p(ids, ctypes.c_int64), _p(sc, ctypes.c_double)),
           "doc_uniform_from_H")
    return masks, S, ids, sc


def round_bf16(x: float) -> float:
    return float(_L().oracle_round_bf16(ctypes.c_float(x)))


def ball_carving_clusters(Q, tau, round_bf16=False):
    """Greedy query clustering of Ball-carving: (k, labels [T] int32, C [T,d] float32 whose
    first k rows are the centroids)."""
    Q = _f32(Q)
    T, d = Q.shape
    labels = np.empty(T, dtype=np.int32)
    C = np.empty((T, d), dtype=np.float32)
    k = _check(_L().oracle_ball_carving_clusters(_p(Q, ctypes.c_float), T, d, ctypes.c_float(tau),
                                                 int(bool(round_bf16)), _p(labels, ctypes.c_int32),
                                                 _p(C, ctypes.c_float)), "ball_carving_clusters")
    return k, labels, C


def ball_carving(Q, E, offsets, tau, K, round_bf16=False):
    """Ball-carving of one query: (k, labels, C, S [N] float64, top-K ids, top-K scores)."""
    Q, E, offsets = _f32(Q), _f32(E), _i64(offsets)
    T, d = Q.shape
    N = offsets.shape[0] - 1
    labels = np.empty(T, dtype=np.int32)
    C = np.empty((T, d), dtype=np.float32)
    S = np.empty(N, dtype=np.float64)
    ids = np.empty(K, dtype=np.int64)
    sc = np.empty(K, dtype=np.float64)
    k = _check(_L().oracle_ball_carving(_p(Q, ctypes.c_float), T, d, ctypes.c_float(tau),
                                        int(bool(round_bf16)), _p(E, ctypes.c_float),
                                        _p(offsets, ctypes.c_int64), ctypes.c_int64(N), int(K),
                                        _p(labels, ctypes.c_int32), _p(C, ctypes.c_float),
                                        _p(S, ctypes.c_double), _p(ids, ctypes.c_int64),
                                        _p(sc, ctypes.c_double)), "ball_carving")
    return k, labels, C, S, ids, sc


def colbandit_lazy(Q, E, offsets, K, M, B, alpha, delta, pi, a=-1.0, b=1.0):
    """Algorithm 1 computing each revealed cell from the embeddings."""
    Q, E, offsets = _f32(Q), _f32(E), _i64(offsets)
    T, d = Q.shape
    N = offsets.shape[0] - 1
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    Rmax = (T + B - 1) // B
    out_ids = np.full(K, -1, dtype=np.int64)
    out_s = np.full(K, np.nan, dtype=np.float64)
    final_ids = np.empty(N, dtype=np.int64)
    n_final = ctypes.c_int64(0)
    counts = np.full(Rmax + 1, -1, dtype=np.int64)
    tau = np.full(Rmax, np.nan, dtype=np.float64)
    cells = np.zeros(3, dtype=np.int64)
    rc = _check(_L().oracle_colbandit_lazy(
        _p(Q, ctypes.c_float), T, d, _p(E, ctypes.c_float), _p(offsets, ctypes.c_int64),
        ctypes.c_int64(N), K, M, B, ctypes.c_double(alpha), ctypes.c_double(delta),
        ctypes.c_double(a), ctypes.c_double(b), _p(pi, ctypes.c_int32),
        _p(out_ids, ctypes.c_int64), _p(out_s, ctypes.c_double),
        _p(final_ids, ctypes.c_int64), ctypes.byref(n_final), _p(counts, ctypes.c_int64),
        _p(tau, ctypes.c_double), _p(cells, ctypes.c_int64)), "colbandit_lazy")
    return ColBanditResult(out_ids, out_s, final_ids[: n_final.value].copy(), rc,
                           counts[: rc + 1].copy(), tau[:rc].copy(),
                           int(cells[0]), int(cells[1]), int(cells[2]))


def num_threads():
    return int(_L().oracle_num_threads())


def full_batch(Q, E, offsets, K, want_scores=False):
    """Exhaustive scoring of a query batch Q[nq,T,d], one thread per query."""
    Q, E, offsets = _f32(Q), _f32(E), _i64(offsets)
    nq, T, d = Q.shape
    N = offsets.shape[0] - 1
    S = np.empty((nq, N), dtype=np.float64) if want_scores else None
    out_ids = np.empty((nq, K), dtype=np.int64)
    out_s = np.empty((nq, K), dtype=np.float64)
    _check(_L().oracle_full_batch(_p(Q, ctypes.c_float), nq, T, d, _p(E, ctypes.c_float),
                                  _p(offsets, ctypes.c_int64), ctypes.c_int64(N), K,
                                  _p(S, ctypes.c_double), _p(out_ids, ctypes.c_int64),
                                  _p(out_s, ctypes.c_double)), "full_batch")
    return out_ids, out_s, S


def colbandit_batch(Q, E, offsets, K, M, B, alpha, delta, pi, a=-1.0, b=1.0):
    """Col-Bandit (lazy reveals) for a query batch, one thread per query."""
    Q, E, offsets = _f32(Q), _f32(E), _i64(offsets)
    nq, T, d = Q.shape
    N = offsets.shape[0] - 1
    pi = np.ascontiguousarray(pi, dtype=np.int32).reshape(nq, T)
    out_ids = np.empty((nq, K), dtype=np.int64)
    out_s = np.empty((nq, K), dtype=np.float64)
    cells = np.zeros((nq, 3), dtype=np.int64)
    rounds = np.zeros(nq, dtype=np.int32)
    _check(_L().oracle_colbandit_batch(
        _p(Q, ctypes.c_float), nq, T, d, _p(E, ctypes.c_float), _p(offsets, ctypes.c_int64),
        ctypes.c_int64(N), K, M, B, ctypes.c_double(alpha), ctypes.c_double(delta),
        ctypes.c_double(a), ctypes.c_double(b), _p(pi, ctypes.c_int32),
        _p(out_ids, ctypes.c_int64), _p(out_s, ctypes.c_double), _p(cells, ctypes.c_int64),
        _p(rounds, ctypes.c_int32)), "colbandit_batch")
    return out_ids, out_s, cells, rounds
