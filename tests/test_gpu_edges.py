"""Edge cases of the GPU path against the oracle: one-row and maximum windows, empty and
one-token histories, rollback, dead rows behind a commit, resetting one sequence of a batch."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref

pytestmark = pytest.mark.gpu

TINY = synth.CONFIGS["tiny"]
SMALL_BF16 = dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1408, vocab=4096,
                  qk_norm=0, dtype=1, rms_eps=1e-5, rope_base=1e4)


def pair(shape, seed, **kw):
    return Gpu(shape, seed=seed, **kw), Ref(shape, seed=seed, **{k: v for k, v in kw.items() if k != "max_window"})


def test_one_row_and_maximum_windows():
    g, r = pair(TINY, 3, max_ctx=256, max_window=32)
    V = TINY["vocab"]
    prompt = synth.uniform_history(9, length=50, vocab=V, span=8, every=16, tail=2)
    g.prefill([prompt], 32)
    r.prefill([prompt], 32)
    rng = np.random.default_rng(0)
    for k in (1, 32, 1, 17):
        w = np.concatenate([[prompt[-1]], rng.integers(0, V, k - 1)]).astype(np.int32)
        got = g.verify([w])[0]
        ref = r.verify([w])[0]
        assert np.abs(got - ref).max() <= 1e-4, k
        n, emit, _ = g.accept(B.DBL_GREEDY)
        n_ref, e_ref, _, m = O.accept_greedy(ref, w)
        if m[:n_ref + 1].min() > 1e-3:
            assert n[0] == n_ref and list(emit[0][:n_ref + 1]) == list(e_ref[:n_ref + 1])
    g.close()


def test_empty_and_one_token_histories():
    g = Gpu(dict(TINY, n_layers=0), seed=1, max_batch=2, max_ctx=64, max_window=4, max_hist=64)
    B.dbl_reset(g.ctx, -1)
    cont, cl, mn, mp = g.retrieve(2, 3, 1, 4)                      # both histories empty
    assert cl.tolist() == [0, 0] and mn.tolist() == [0, 0] and mp.tolist() == [-1, -1] and (cont == -1).all()
    B.dbl_history_set(g.ctx, 1, np.array([7], np.int32))          # one token: nothing to match against
    cont, cl, mn, mp = g.retrieve(2, 3, 1, 4)
    assert cl.tolist() == [0, 0] and O.retrieve(np.array([7], np.int32), 3, 1, 4)[1] == 0
    window = g.i32(2, 4, fill=-5)
    cd, cld = g.i32(2, 4, fill=-1), g.i32(2)
    B.dbl_build_window(g.ctx, 2, 4, 4, cd, cld, 9, window)
    torch.cuda.synchronize()
    assert window.cpu().numpy().tolist() == [[9, 9, 9, 9], [7, 9, 9, 9]]   # empty history: pad in row 0 too
    g.close()


def test_rollback_then_new_tokens_equals_a_fresh_run():
    g, r = pair(SMALL_BF16, 5, max_ctx=256, max_window=8)
    V = SMALL_BF16["vocab"]
    prompt = synth.zipf_history(2, 41, V)
    g.prefill([prompt], 8)
    r.prefill([prompt], 8)
    rng = np.random.default_rng(1)
    w1 = np.concatenate([[prompt[-1]], rng.integers(0, V, 7)]).astype(np.int32)
    g.verify([w1], want_logits=False)
    g.commit([8])                                                  # keep all 8 rows: kv_len = 48
    assert g.kv_len()[0] == 48
    B.dbl_truncate(g.ctx, 0, kv_len=43)                            # roll 5 of them back
    assert g.kv_len()[0] == 43
    w2 = np.concatenate([w1[3:4], rng.integers(0, V, 5)]).astype(np.int32)   # continue after w1[0..2]
    got = g.verify([w2])[0]
    s = r.seqs[0]
    s.verify_block(w1); s.commit(8, []); s.truncate(kv_len=43)
    ref = s.verify_block(w2)
    assert np.abs(got - ref).max() <= 2e-2
    fresh = Gpu(SMALL_BF16, seed=5, max_ctx=256, max_window=8)     # never saw the rolled-back rows
    fresh.prefill([list(prompt) + [int(t) for t in w1[1:4]]], 8)
    assert np.array_equal(fresh.verify([w2])[0], got)
    fresh.close(); g.close()


def test_rows_behind_a_commit_are_dead():
    g = Gpu(SMALL_BF16, seed=6, max_ctx=256, max_window=8)
    V = SMALL_BF16["vocab"]
    prompt = synth.zipf_history(4, 30, V)
    g.prefill([prompt], 8)
    rng = np.random.default_rng(2)
    junk = np.concatenate([[prompt[-1]], rng.integers(0, V, 7)]).astype(np.int32)
    w = np.concatenate([[prompt[-1]], rng.integers(0, V, 3)]).astype(np.int32)
    clean = g.verify([w])[0]
    g.verify([junk], want_logits=False)        # writes 8 K/V rows behind kv_len, nothing is committed
    assert np.array_equal(g.verify([w])[0], clean)
    g.close()


def test_reset_of_one_sequence_leaves_the_others():
    g = Gpu(SMALL_BF16, seed=7, max_batch=2, max_ctx=256, max_window=8)
    V = SMALL_BF16["vocab"]
    prompts = [synth.zipf_history(5 + b, 25, V) for b in range(2)]
    g.prefill(prompts, 8)
    rng = np.random.default_rng(3)
    ws = [np.concatenate([[p[-1]], rng.integers(0, V, 3)]).astype(np.int32) for p in prompts]
    before = g.verify(ws)
    B.dbl_reset(g.ctx, 0)
    assert g.kv_len().tolist() == [0, 24] and g.hist_len().tolist() == [0, 25]
    after = g.verify(ws)
    assert np.array_equal(after[1], before[1])
    assert not np.array_equal(after[0], before[0])    # sequence 0 now starts from an empty context
    g.close()
