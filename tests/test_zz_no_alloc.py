"""colbandit_topk_static: the entry point for callers that cannot allocate (its scratch is a
buffer inside the library's device image).  Its results must be those of colbandit_topk, bit for
bit, also when a call follows a larger one on the same GPU (the buffer keeps the last call's
contents)."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    assert torch.cuda.is_available(), "these tests need the GPU"
    from paper_2602_02827_amd import binding
    binding.lib()
    return binding


def _pair(lib, w, K, alpha, seed, **kw):
    ref = lib.colbandit_topk(w.Q, w.docs, w.offsets, K, alpha, w.delta, w.M, seed, want_stats=False, **kw)
    got = lib.colbandit_topk_static(w.Q, w.docs, w.offsets, K, alpha, w.delta, w.M, seed, **kw)
    torch.cuda.synchronize()
    assert torch.equal(got["topk_ids"], ref["topk_ids"])
    assert torch.equal(got["topk_scores"].view(torch.int32), ref["topk_scores"].view(torch.int32))
    assert bool((got["topk_ids"] >= 0).all())
    return got


def test_static_scratch_entry_point_matches_the_workspace_one_on_consecutive_calls(B):
    from paper_2602_02827_amd import synth
    big = synth.config(1, device="cuda", scale=0.12, nq=8)         # N = 6,000, 8 queries
    small = synth.config(1, device="cuda", scale=0.03, nq=3)       # N = 1,500, 3 queries
    assert B.colbandit_workspace_bytes(big.nq, big.T, big.d, big.N, big.total_tokens) <= B.STATIC_SCRATCH_BYTES
    r1 = _pair(B, big, 5, 0.2, 3)
    r2 = _pair(B, small, 5, 0.2, 3)                                # right after, smaller input
    r3 = _pair(B, big, 10, 1.0, 11)                                # conservative radius: long lists, corpus passes
    r4 = _pair(B, small, 3, 0.5, 7, B=3)
    # the same again must give the same (nothing depends on what the buffer held)
    again = B.colbandit_topk_static(big.Q, big.docs, big.offsets, 5, 0.2, big.delta, big.M, 3)
    torch.cuda.synchronize()
    assert torch.equal(again["topk_ids"], r1["topk_ids"]) and torch.equal(again["topk_scores"], r1["topk_scores"])
    # int8 elimination rounds through the same entry point
    d8, ds = B.colbandit_quantize_i8(small.docs)
    _pair(B, small, 5, 0.2, 3, docs_i8=d8, docs_scale=ds)
    # exhaustive scores are what the survivors carry
    full = B.colbandit_full_maxsim(small.Q, small.docs, small.offsets, K=0)
    torch.cuda.synchronize()
    assert torch.equal(r2["topk_scores"], torch.gather(full["scores"], 1, r2["topk_ids"]))


def test_static_scratch_entry_point_rejects_sizes_beyond_its_buffer(B):
    from paper_2602_02827_amd import synth
    w = synth.config(1, device="cuda", scale=0.12, nq=8)
    many = w.Q.repeat(40, 1, 1).contiguous()                         # 320 queries x 6,000 documents
    assert B.colbandit_workspace_bytes(320, w.T, w.d, w.N, w.total_tokens) > B.STATIC_SCRATCH_BYTES
    out = {"topk_ids": torch.full((320, 5), -7, dtype=torch.int64, device="cuda"),
           "topk_scores": torch.zeros((320, 5), dtype=torch.float32, device="cuda")}
    with pytest.raises(B.ColbanditError) as e:
        B.colbandit_topk_static(many, w.docs, w.offsets, 5, 0.2, w.delta, w.M, 0, out=out)
    assert e.value.code == -9
    torch.cuda.synchronize()
    assert bool((out["topk_ids"] == -7).all())                       # nothing was written
