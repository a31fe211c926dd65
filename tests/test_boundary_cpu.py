"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
the header declares, rejects bad arguments before touching the device, and its host
helpers (reveal permutation, radius pre-factor) agree with the oracle's."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2602_02827_amd import binding, build
    build.build_library()
    binding.lib()
    return binding


def test_library_exports_every_declared_symbol(B):
    hdr = open(os.path.join(ROOT, "include", "colbandit.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(colbandit_[a-z_0-9]+)\s*\(", hdr))
    assert {"colbandit_full_maxsim", "colbandit_topk"} <= declared
    assert declared == set(B.EXPORTS)
    L = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(L, name) is not None


def test_struct_layouts_match_the_header(B):
    # survivors[MAX_ROUNDS + 2] and the limits the binding mirrors
    hdr = open(os.path.join(ROOT, "include", "colbandit.h")).read()
    assert int(re.search(r"#define COLBANDIT_MAX_ROUNDS (\d+)", hdr).group(1)) == B.MAX_ROUNDS
    assert ctypes.sizeof(B.ColbanditStats) == B.lib().colbandit_sizeof_stats()
    assert ctypes.sizeof(B.ColbanditOpts) == B.lib().colbandit_sizeof_opts()


def test_strerror_is_defined_for_every_code(B):
    msgs = {B.strerror(c) for c in range(0, -10, -1)}
    assert len(msgs) == 10 and "unknown error code" not in msgs
    assert B.strerror(-99) == "unknown error code"


def _call_full(B, **kw):
    a = dict(Q=0x1000, nq=1, T=32, d=128, dt=1, docs=0x2000, off=0x3000, N=10, total=400, K=0,
             scores=0x4000, ids=None, sc=None, cells=None, ws=0x10000, wsb=1 << 40, stream=None)
    a.update(kw)
    return B.lib().colbandit_full_maxsim(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["docs"],
                                         a["off"], a["N"], a["total"], a["K"], a["scores"],
                                         a["ids"], a["sc"], a["cells"], None, a["ws"], a["wsb"],
                                         a["stream"])


def test_full_maxsim_argument_errors(B):
    # every case fails validation, so nothing is ever launched (no GPU needed)
    assert _call_full(B, Q=None) == -1
    assert _call_full(B, docs=None) == -1
    assert _call_full(B, off=None) == -1
    assert _call_full(B, scores=None) == -1                 # K == 0 needs scores
    assert _call_full(B, K=3) == -1                         # K > 0 needs the top-K outputs
    assert _call_full(B, nq=0) == -2
    assert _call_full(B, T=0) == -2
    assert _call_full(B, N=0) == -2
    assert _call_full(B, total=5) == -2                     # fewer tokens than documents
    assert _call_full(B, K=11, ids=0x5000, sc=0x6000) == -2  # K > N
    assert _call_full(B, dt=7) == -2
    assert _call_full(B, d=100) == -4
    assert _call_full(B, T=129) == -4
    assert _call_full(B, dt=0, T=65) == -4
    assert _call_full(B, Q=0x1004) == -6
    assert _call_full(B, ws=None) == -1
    assert _call_full(B, ws=0x10010) == -6
    assert _call_full(B, wsb=1024) == -5


def _call_topk(B, opts=None, **kw):
    a = dict(Q=0x1000, nq=2, T=32, d=128, dt=1, docs=0x2000, off=0x3000, N=100, total=4000, K=5,
             alpha=0.2, delta=0.01, M=5, seed=0, ids=0x5000, sc=0x6000, stats=None, ws=0x10000,
             wsb=1 << 40, stream=None)
    a.update(kw)
    o = ctypes.byref(opts) if opts is not None else None
    return B.lib().colbandit_topk(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["docs"], a["off"],
                                  a["N"], a["total"], a["K"], a["alpha"], a["delta"], a["M"],
                                  ctypes.c_uint64(a["seed"]), o, a["ids"], a["sc"], a["stats"],
                                  a["ws"], a["wsb"], a["stream"])


def test_topk_argument_errors(B):
    assert _call_topk(B, ids=None) == -1
    assert _call_topk(B, K=0) == -2
    assert _call_topk(B, K=101) == -2
    assert _call_topk(B, N=5000, total=500000, K=2000) == -4
    for alpha in (0.0, -0.1, 1.5, float("nan")):
        assert _call_topk(B, alpha=alpha) == -3
    for delta in (0.0, 1.0, -1.0, float("nan")):
        assert _call_topk(B, delta=delta) == -3
    assert _call_topk(B, M=-1) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(B=-2)) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(B=17)) == -4
    assert _call_topk(B, T=66, opts=B.ColbanditOpts(B=1)) == -4      # 66 rounds > the 64-round limit
    assert _call_topk(B, T=128, opts=B.ColbanditOpts(B=1)) == -4       # more than 64 rounds
    assert _call_topk(B, opts=B.ColbanditOpts(a=1.0, b=-1.0)) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(a=0.5, b=0.5)) == -3
    assert _call_topk(B, wsb=4096) == -5
    o = B.ColbanditOpts(trace=0x20000, trace_bytes=16)
    assert _call_topk(B, opts=o) == -5


def test_coarse_pass_argument_errors(B):
    # opts of colbandit_topk
    assert _call_topk(B, opts=B.ColbanditOpts(later_rounds=3)) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(later_rounds=-1)) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(docs_i8=0x7000)) == -1            # codes without their scale
    assert _call_topk(B, opts=B.ColbanditOpts(docs_i8=0x7004, docs_scale=0x8000)) == -6
    assert _call_topk(B, opts=B.ColbanditOpts(docs_i8=0x7000, docs_scale=0x8002)) == -6
    assert _call_topk(B, opts=B.ColbanditOpts(docs_i8=0x7000, docs_scale=0x8000, coarse_permille=1001)) == -3
    assert _call_topk(B, opts=B.ColbanditOpts(docs_i8=0x7000, docs_scale=0x8000, coarse_permille=-1)) == -3
    # int8 codes need a width the int8 matrix instruction covers (multiples of 64)
    assert _call_topk(B, d=96, opts=B.ColbanditOpts(docs_i8=0x7000, docs_scale=0x8000)) == -4
    assert _call_topk(B, d=32, opts=B.ColbanditOpts(docs_i8=0x7000, docs_scale=0x8000)) == -4
    assert _call_topk(B, d=48) == -4 and _call_topk(B, d=256) == -4

    # colbandit_quantize_i8
    L = B.lib()
    def quant(x=0x1000, dt=1, nseg=1, rows=10, d=128, pm=999, codes=0x2000, scales=0x3000,
              ws=0x10000, wsb=1 << 30):
        return L.colbandit_quantize_i8(x, dt, nseg, rows, d, pm, codes, scales, ws, wsb, None)
    assert quant(x=None) == -1 and quant(codes=None) == -1 and quant(scales=None) == -1
    assert quant(nseg=0) == -2 and quant(rows=0) == -2 and quant(d=0) == -2 and quant(dt=5) == -2
    assert quant(nseg=70000) == -2
    assert quant(pm=0) == -3 and quant(pm=1001) == -3
    assert quant(x=0x1008) == -6 and quant(scales=0x3001) == -6
    assert quant(ws=None) == -1 and quant(ws=0x10001) == -6 and quant(wsb=16) == -5
    assert L.colbandit_quantize_workspace_bytes(0) == 0
    w1, w4 = L.colbandit_quantize_workspace_bytes(1), L.colbandit_quantize_workspace_bytes(4)
    assert 0 < w1 < w4 and w1 % 256 == 0

    # colbandit_coarse_maxsim
    def coarse(**kw):
        a = dict(Q=0x1000, nq=1, T=32, d=128, dt=1, d8=0x2000, ds=0x2100, off=0x3000, N=10, total=400,
                 pm=999, scores=0x4000, cells=None, qc=None, qs=None, ws=0x10000, wsb=1 << 40)
        a.update(kw)
        return L.colbandit_coarse_maxsim(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["d8"], a["ds"],
                                         a["off"], a["N"], a["total"], a["pm"], a["scores"], a["cells"],
                                         a["qc"], a["qs"], a["ws"], a["wsb"], None)
    assert coarse(Q=None) == -1 and coarse(d8=None) == -1 and coarse(ds=None) == -1
    assert coarse(scores=None) == -1
    assert coarse(pm=0) == -3
    assert coarse(N=0) == -2 and coarse(d=96) == -4
    assert coarse(wsb=1024) == -5


def test_baseline_argument_errors(B):
    """colbandit_doc_uniform / colbandit_ball_carving reject bad arguments before any launch."""
    L = B.lib()

    def uni(**kw):
        a = dict(Q=0x1000, nq=1, T=32, d=128, dt=1, docs=0x2000, off=0x3000, N=10, total=400, K=0,
                 m=4, seed=0, scores=0x4000, masks=None, ids=None, sc=None, ws=0x10000, wsb=1 << 40)
        a.update(kw)
        return L.colbandit_doc_uniform(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["docs"], a["off"],
                                       a["N"], a["total"], a["K"], a["m"], a["seed"], a["scores"],
                                       a["masks"], a["ids"], a["sc"], a["ws"], a["wsb"], None)
    assert uni(Q=None) == -1 and uni(docs=None) == -1 and uni(off=None) == -1
    assert uni(scores=None) == -1                       # K == 0 needs the scores
    assert uni(K=3) == -1                               # K > 0 needs the top-K outputs
    assert uni(K=11) == -2 and uni(N=0) == -2 and uni(dt=7) == -2
    assert uni(m=0) == -3 and uni(m=33) == -3
    assert uni(T=65, m=4) == -4 and uni(d=48) == -4 and uni(d=160) == -4
    assert uni(masks=0x5004) == -6 and uni(Q=0x1008) == -6
    assert uni(ws=None) == -1 and uni(wsb=1024) == -5
    assert L.colbandit_doc_uniform_workspace_bytes(0, 32, 128, 10, 400) == 0
    base = B.colbandit_workspace_bytes(2, 32, 128, 1000, 48000)
    wu = L.colbandit_doc_uniform_workspace_bytes(2, 32, 128, 1000, 48000)
    assert wu >= base + 4 * 2 * 1000 * 32 and wu % 256 == 0

    def ball(**kw):
        a = dict(Q=0x1000, nq=1, T=32, d=128, dt=1, docs=0x2000, off=0x3000, N=10, total=400, K=0,
                 tau=0.7, kq=None, labels=None, cent=None, scores=0x4000, ids=None, sc=None,
                 ws=0x10000, wsb=1 << 40)
        a.update(kw)
        return L.colbandit_ball_carving(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["docs"], a["off"],
                                        a["N"], a["total"], a["K"], a["tau"], a["kq"], a["labels"],
                                        a["cent"], a["scores"], a["ids"], a["sc"], a["ws"], a["wsb"],
                                        None)
    assert ball(Q=None) == -1 and ball(docs=None) == -1 and ball(scores=None) == -1 and ball(K=2) == -1
    assert ball(K=11) == -2 and ball(nq=0) == -2
    assert ball(tau=0.0) == -3 and ball(tau=-0.5) == -3 and ball(tau=1.5) == -3
    assert ball(tau=float("nan")) == -3
    assert ball(T=65) == -4
    assert ball(kq=0x5002) == -6 and ball(labels=0x5001) == -6 and ball(cent=0x5008) == -6
    assert ball(ws=None) == -1 and ball(wsb=1024) == -5
    wb16 = L.colbandit_ball_carving_workspace_bytes(2, 32, 128, 1, 1000, 48000)
    wb32 = L.colbandit_ball_carving_workspace_bytes(2, 32, 128, 0, 1000, 48000)
    assert wb16 >= base + 8 * 2 * 8 * 1000 and wb32 >= base + 4 * 2 * 32 * 128
    assert L.colbandit_ball_carving_workspace_bytes(2, 32, 128, 5, 1000, 48000) == 0


def test_cells_per_doc_of_doc_uniform(B, oracle_mod):
    """colbandit_cells_per_doc against exact rational arithmetic on the paper's gamma sweep and
    against the oracle's separately written counterpart; error codes."""
    from test_oracle_pins import GAMMA_SWEEP, exact_cells_per_doc
    for g in GAMMA_SWEEP + ["0.001", "0.125", "0.3333", "0.99"]:
        for T in range(1, 129):
            m = B.colbandit_cells_per_doc(float(g), T)
            assert m == exact_cells_per_doc(g, T) == oracle_mod.cells_per_doc(float(g), T), (g, T)
    assert B.colbandit_cells_per_doc(0.1, 30) == 3 and B.colbandit_cells_per_doc(0.05, 32) == 2
    assert B.colbandit_cells_per_doc(1.0, 32) == 32 and B.colbandit_cells_per_doc(0.001, 32) == 1
    L = B.lib()
    assert L.colbandit_cells_per_doc(0.0, 32) == -3 and L.colbandit_cells_per_doc(1.01, 32) == -3
    assert L.colbandit_cells_per_doc(float("nan"), 32) == -3 and L.colbandit_cells_per_doc(0.5, 0) == -2


def test_topk_static_argument_errors_need_no_device(B):
    """colbandit_topk_static validates like colbandit_topk and rejects sizes beyond its built-in
    buffer before it asks the runtime for anything (so all of this runs without a GPU)."""
    def call(**kw):
        a = dict(Q=0x1000, nq=2, T=32, d=128, dt=1, docs=0x2000, off=0x3000, N=100, total=4000, K=5,
                 alpha=0.2, delta=0.01, M=5, ids=0x5000, sc=0x6000, opts=None)
        a.update(kw)
        o = ctypes.byref(a["opts"]) if a["opts"] is not None else None
        return B.lib().colbandit_topk_static(a["Q"], a["nq"], a["T"], a["d"], a["dt"], a["docs"], a["off"],
                                             a["N"], a["total"], a["K"], a["alpha"], a["delta"], a["M"],
                                             ctypes.c_uint64(0), o, a["ids"], a["sc"], None)
    assert call(Q=None) == -1 and call(ids=None) == -1
    assert call(K=0) == -2 and call(K=101) == -2 and call(nq=0) == -2
    assert call(alpha=0.0) == -3 and call(delta=1.0) == -3 and call(M=-1) == -3
    assert call(d=100) == -4 and call(opts=B.ColbanditOpts(B=17)) == -4
    assert call(Q=0x1004) == -6
    # the benchmark's sizes need 2.3 GB of scratch: far beyond the built-in 64 MiB
    assert call(nq=128, N=500000, total=53040331) == -9
    assert "COLBANDIT_STATIC_SCRATCH_BYTES" in B.strerror(-9)
    hdr = open(os.path.join(ROOT, "include", "colbandit.h")).read()
    assert "#define COLBANDIT_STATIC_SCRATCH_BYTES (64u << 20)" in hdr and B.STATIC_SCRATCH_BYTES == 64 << 20
    # the largest sizes that fit are accepted by the size check of the workspace query
    assert B.colbandit_workspace_bytes(8, 32, 128, 6000, 640000) <= B.STATIC_SCRATCH_BYTES


def test_workspace_and_trace_sizes(B):
    assert B.colbandit_workspace_bytes(0, 32, 128, 10, 100) == 0
    assert B.colbandit_workspace_bytes(1, 32, 128, 10, 5) == 0
    w1 = B.colbandit_workspace_bytes(1, 32, 128, 1000, 48000)
    w2 = B.colbandit_workspace_bytes(2, 32, 128, 1000, 48000)
    w3 = B.colbandit_workspace_bytes(2, 32, 128, 2000, 96000)
    assert 0 < w1 < w2 < w3 and w1 % 256 == 0
    # the big configuration fits comfortably in one GPU's memory
    assert B.colbandit_workspace_bytes(128, 32, 128, 500_000, 53_000_000) < 4 << 30
    R, nq, N = 8, 3, 1000
    t = B.colbandit_trace_bytes(nq, 32, 4, N)
    assert t >= 4 * (R + 1) * nq + 4 * R * nq + 9 * R * nq * N


def test_permutation_matches_the_oracle_spec(B, oracle_mod):
    for seed, q, T in [(0, 0, 32), (7, 5, 24), (2**63 + 11, 127, 64), (1, 0, 1), (3, 2, 2)]:
        np.testing.assert_array_equal(B.colbandit_permutation(seed, q, T),
                                      oracle_mod.permutation(seed, q, T))


def test_radius_prefactor_matches_the_oracle(B, oracle_mod):
    for N, T in [(1000, 32), (500_000, 32), (20_000, 24)]:
        for n in (2, 4, 12, T // 2, T // 2 + 1, T - 1, T):
            a32, d32 = float(np.float32(0.2)), float(np.float32(0.01))
            want = oracle_mod.radius(a32, T, 1.0, N, d32, n)
            assert B.colbandit_radius_prefactor(0.2, 0.01, T, N, n) == pytest.approx(want, rel=1e-12,
                                                                                     abs=1e-300)
    assert B.colbandit_radius_prefactor(0.2, 0.01, 32, 1000, 1) == float("inf")


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2602_02827_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in src and "from oracle" not in src, f
                assert "oracle/" not in src, f


def test_header_is_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 and as C++ without any HIP or
    torch type in sight, and every declaration must be usable from C."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include <string.h>\n'
        '#include "colbandit.h"\n'
        "int main(void) {\n"
        "    colbandit_opts o;\n"
        "    colbandit_stats s;\n"
        "    memset(&o, 0, sizeof o);\n"
        "    memset(&s, 0, sizeof s);\n"
        "    return (int)(colbandit_sizeof_opts() == sizeof(colbandit_opts)) - 1 +\n"
        "           (int)(colbandit_sizeof_stats() == sizeof(colbandit_stats)) - 1;\n"
        "}\n")
    inc = os.path.join(ROOT, "include")
    for cc, std in (("gcc", "-std=c99"), ("g++", "-std=c++11")):
        r = subprocess.run([cc, std, "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", "-x",
                            "c" if cc == "gcc" else "c++", "-I", inc, str(src)],
                           capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
