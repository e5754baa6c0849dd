"""The projection kernel on awkward shapes, through the shortest path that reaches it: models
without layers (embedding -> final RMSNorm -> LM head), so logits = W_lm . norm(E[token]) and the
oracle is a handful of dot products.  Vocabulary sizes that leave the last tile, the last unit of
tile rows and the last workgroup round partly empty; widths of a single k-block chunk and of a
chunk whose last waves have nothing to do; 1 .. 128 rows (1, 2, 4 row groups, two passes)."""
import numpy as np
import pytest

from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref

pytestmark = pytest.mark.gpu


def lm_only(d_model, vocab, dtype):
    return dict(n_layers=0, d_model=d_model, n_q_heads=2, n_kv_heads=1, head_dim=64, d_ffn=64, vocab=vocab,
                qk_norm=0, dtype=dtype, rms_eps=1e-5, rope_base=1e4)


@pytest.mark.parametrize("d_model,vocab,dtype", [(128, 1000, 1), (320, 1016, 1), (1024, 4104, 1), (2048, 777, 1),
                                                 (96, 530, 0), (384, 2049, 0)])
def test_lm_head_only_models_on_awkward_shapes(d_model, vocab, dtype):
    shape = lm_only(d_model, vocab, dtype)
    g = Gpu(shape, seed=17, max_batch=4, max_ctx=128, max_window=32, max_hist=256)
    r = Ref(shape, seed=17, max_batch=4, max_ctx=128, max_hist=256)
    rng = np.random.default_rng(d_model + vocab)
    gains = (1.0 + 0.25 * rng.standard_normal(d_model)).astype(np.float32)
    g.set_tensor("gf", 0, gains); r.set_tensor("gf", 0, gains)
    tol = 2e-2 if dtype == 1 else 1e-4
    for Bn, k in ((1, 1), (1, 8), (1, 13), (2, 16), (3, 20), (4, 16), (4, 32)):
        ws = rng.integers(0, vocab, (Bn, k)).astype(np.int32)
        got = g.verify(ws)
        ref = r.verify(ws)
        assert np.isfinite(got).all()
        assert np.abs(got - ref).max() <= tol, (Bn, k, np.abs(got - ref).max())
        n, emit, guide = g.accept(B.DBL_GREEDY)
        # the fused row statistics against the returned logits (lowest id on ties)
        for b in range(Bn):
            assert np.array_equal(guide[b], got[b].argmax(axis=1)), (Bn, k, b)
    g.close()
