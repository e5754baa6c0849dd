"""Pins for the oracle's KV commit / truncate (Alg. 1 "rollback", Alg. 2 truncate + update)."""
import numpy as np

import oracle as O
from tests.torch_decoder import forward_full

CFG = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=97,
           max_ctx=64, rms_eps=1e-5, rope_base=1e4)


def test_commit_truncates_and_stale_tail_is_dead():
    m = O.Model(**CFG, dtype=0, seed=31)
    rng = np.random.default_rng(1)
    toks = rng.integers(0, 97, 30).astype(np.int32)
    s = O.Seq(m)
    s.hist_set(toks[:10])
    s.verify_block(toks[:9]); s.commit(9, [])
    assert (s.kv_len, s.hist_len) == (9, 10)
    # a window of 6 rows of which only the first 3 are kept
    junk = rng.integers(0, 97, 3).astype(np.int32)
    s.verify_block(np.concatenate([toks[9:12], junk]))
    s.commit(3, toks[10:13])
    assert (s.kv_len, s.hist_len) == (12, 13)
    assert list(s.history()) == list(toks[:13])
    # the three dropped rows' KV is dead: poison it, results must not change
    s.kcache()[:, :, 12:] = np.nan
    s.vcache()[:, :, 12:] = np.nan
    lg = s.verify_block(toks[12:16])
    assert np.isfinite(lg).all()
    # the incremental cache equals a from-scratch recompute of the committed sequence
    ref = forward_full(m, toks[:16])[12:16]
    np.testing.assert_allclose(lg, ref, rtol=0, atol=2e-6)
    # committing nothing keeps the state; over-committing is refused
    s.commit(0, [])
    assert (s.kv_len, s.hist_len) == (12, 13)
    try:
        s.commit(60, [])
        assert False
    except ValueError:
        pass


def test_reset_flushes_session():
    m = O.Model(**CFG, dtype=1, seed=32)
    s = O.Seq(m)
    a = s.verify_block([1, 2, 3]); s.commit(3, [1, 2, 3])
    s.reset()
    assert (s.kv_len, s.hist_len) == (0, 0)
    assert np.array_equal(s.verify_block([1, 2, 3]), a)
