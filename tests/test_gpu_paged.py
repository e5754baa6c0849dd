"""The paged KV cache (DBL_FLAG_PAGED_KV) against the contiguous one: the arithmetic is the same,
only the addresses differ, so every logit must be bit-identical -- with sequences of diverging
lengths whose pages interleave in the pool, across page boundaries, after rollbacks and resets
that return pages, and for the seeded cache fill.  One step is also checked against the oracle."""
import numpy as np
import pytest
import torch

from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref
from tests.test_gpu_parity import SMALL_BF16, SMALL_QWEN, TINY, TOL

pytestmark = pytest.mark.gpu

K = 8


@pytest.mark.parametrize("shape", [TINY, SMALL_BF16, SMALL_QWEN], ids=["tiny_f32", "small_bf16_hd64", "small_qwen_hd128"])
def test_paged_cache_is_bit_identical_to_the_contiguous_one(shape):
    V = shape["vocab"]
    kw = dict(seed=5, max_batch=3, max_ctx=1024, max_window=K, max_hist=2048)
    flat, paged = Gpu(shape, **kw), Gpu(shape, kv_pages=0, **kw)
    r = Ref(shape, seed=5, max_batch=3, max_ctx=1024, max_hist=2048)
    prompts = [synth.zipf_history(60 + b, 241, V) for b in range(3)]       # 240 cached tokens: just below a page
    for g in (flat, paged):
        g.prefill(prompts, 8)
    r.prefill(prompts, 8)
    rng = np.random.default_rng(2)
    # sequence 0 grows by 8 a step, sequence 1 sits out, sequence 2 grows by 3: the lengths diverge
    # (560 / 240 / 360 after 40 steps) and the pages of 0 and 2 interleave in the pool
    lens, keep = [8, 0, 3], [8, 0, 3]
    for step in range(40):
        w = rng.integers(0, V, (3, K)).astype(np.int32)
        a = flat.verify(w, win_len=lens)
        b = paged.verify(w, win_len=lens)
        for s in (0, 2):
            assert np.array_equal(a[s][:lens[s]], b[s][:lens[s]]), (step, s)
        if step in (3, 20):     # across the first page boundary (step 3: 264 > 256) and later
            for s in (0, 2):
                ref = r.seqs[s].verify_block(w[s][:lens[s]])
                assert np.abs(b[s][:lens[s]] - ref).max() <= TOL[shape["dtype"]], (step, s)
        for g in (flat, paged):
            g.accept(B.DBL_GREEDY)
            g.commit(keep)
        for s in (0, 2):
            if step not in (3, 20):
                r.seqs[s].verify_block(w[s][:lens[s]])
            r.seqs[s].commit(keep[s], [])
    assert list(flat.kv_len()) == list(paged.kv_len()) == [240 + 320, 240, 240 + 120]
    # rollback of sequence 0 to 300 tokens (its third page goes back to the pool), then new rows
    for g in (flat, paged):
        B.dbl_truncate(g.ctx, 0, kv_len=300)
    w = rng.integers(0, V, (3, K)).astype(np.int32)
    a, b = flat.verify(w), paged.verify(w)
    assert np.array_equal(a, b)
    flat.close(); paged.close()


def test_pool_exhaustion_is_an_error_and_pages_come_back():
    shape = SMALL_BF16
    V = shape["vocab"]
    g = Gpu(shape, seed=9, max_batch=2, max_ctx=1024, max_window=K, max_hist=2048, kv_pages=4)
    fresh = Gpu(shape, seed=9, max_batch=2, max_ctx=1024, max_window=K, max_hist=2048)
    prompts = [synth.zipf_history(80 + b, 481, V) for b in range(2)]      # 480 tokens: two pages each
    g.prefill(prompts, 8)
    fresh.prefill(prompts, 8)
    rng = np.random.default_rng(4)
    # 4 more steps of 8 reach 512 = the end of the second page; the fifth needs a third page for both
    for _ in range(4):
        w = rng.integers(0, V, (2, K)).astype(np.int32)
        assert np.array_equal(g.verify(w), fresh.verify(w))
        for x in (g, fresh):
            x.accept(B.DBL_GREEDY); x.commit([K, K])
    w = rng.integers(0, V, (2, K)).astype(np.int32)
    with pytest.raises(RuntimeError, match="pool exhausted"):
        g.verify(w)
    # sequence 1 gives everything back; sequence 0 can go on, alone
    B.dbl_reset(g.ctx, 1)
    B.dbl_reset(fresh.ctx, 1)
    a, b = g.verify(w[:1]), fresh.verify(w[:1])
    assert np.array_equal(a, b)
    for x in (g, fresh):
        x.accept(B.DBL_GREEDY); x.commit([K])
    assert g.kv_len()[0] == 520
    # and sequence 1 starts over in whatever page is left
    B.dbl_history_set(g.ctx, 1, np.ascontiguousarray(prompts[1][:9], dtype=np.int32))
    B.dbl_history_set(fresh.ctx, 1, np.ascontiguousarray(prompts[1][:9], dtype=np.int32))
    w2 = np.stack([w[0], prompts[1][:8]]).astype(np.int32)
    assert np.array_equal(g.verify(w2), fresh.verify(w2))
    g.close(); fresh.close()


def test_seeded_fill_has_the_same_content_in_both_forms():
    shape = SMALL_QWEN
    V = shape["vocab"]
    kw = dict(seed=3, max_batch=2, max_ctx=1024, max_window=K, max_hist=2048)
    flat, paged = Gpu(shape, **kw), Gpu(shape, kv_pages=7, **kw)
    for g in (flat, paged):
        B.dbl_kv_fill(g.ctx, 1, 700, 123)        # sequence 1 first: its pages come before sequence 0's
        B.dbl_kv_fill(g.ctx, 0, 300, 456)
    w = np.random.default_rng(1).integers(0, V, (2, K)).astype(np.int32)
    a, b = flat.verify(w), paged.verify(w)
    assert np.isfinite(a).all() and np.array_equal(a, b)
    flat.close(); paged.close()
