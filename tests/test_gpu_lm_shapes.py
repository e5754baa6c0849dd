"""The projection kernel on awkward shapes, through the shortest path that reaches it: models
without layers (embedding -> final RMSNorm -> LM head), so logits = W_lm . norm(E[token]) and the
oracle is a handful of dot products.  Vocabulary sizes that leave the last tile, the last unit of
tile rows and the last workgroup round partly empty; widths of a single k-block chunk and of a
chunk whose last waves have nothing to do; 1 .. 128 rows (1, 2, 4 row groups in the row-group kernel, two passes; 4 and 8 in the LDS-shared LM-head kernel, one pass)."""
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


@pytest.mark.parametrize("wide", [1, 0], ids=["lds_shared_lm_head", "row_group_lm_head"])
@pytest.mark.parametrize("d_model,vocab", [(1024, 4104), (256, 1000)])
def test_sampling_statistics_of_many_row_windows(monkeypatch, d_model, vocab, wide):
    """Acceptance under T > 0 from the fused row statistics for windows of 32 .. 128 rows: the LDS-shared LM-head
    kernel (from 33 rows on, one pass) and, with it switched off,
    the row-group kernel's 64-row passes (80 rows = a full pass and a ragged one that must leave the same number
    of statistics entries per row).  Accepted length, emitted tokens and the target's own draws against the
    oracle's acceptance on the oracle's logits, wherever its margins exceed the measured logit error."""
    import oracle as O
    from tests import gpu_util
    from tests.test_gpu_parity import guide_rows, sample_margin_ok
    monkeypatch.setattr(gpu_util, "TUNING", dict(wide_lm_head=wide))
    shape = lm_only(d_model, vocab, 1)
    g = Gpu(shape, seed=23, max_batch=4, max_ctx=128, max_window=32, max_hist=256)
    r = Ref(shape, seed=23, max_batch=4, max_ctx=128, max_hist=256)
    rng = np.random.default_rng(vocab + wide)
    # a final-norm gain of about 4 and T = 0.2 make the distributions sharp enough for accepted lengths to vary
    gains = (4.0 + 0.5 * rng.standard_normal(d_model)).astype(np.float32)
    g.set_tensor("gf", 0, gains); r.set_tensor("gf", 0, gains)
    T, seed = 0.2, 0xC0FFEE11
    compared = total = 0
    lengths = set()
    for step, (Bn, k) in enumerate(((4, 8), (3, 20), (4, 16), (4, 20), (4, 32), (3, 32), (4, 25))):
        plan = B.dbl_projection_plan(g.ctx, 4, Bn * k)
        assert plan[0] == (4 if (wide and Bn * k > 32) else 1), plan
        # a layer-less model's row depends on its own token only: drafts = the oracle's most likely token after
        # the row before, for a prefix of every window, random afterwards
        ws = rng.integers(0, vocab, (Bn, k)).astype(np.int32)
        for b in range(Bn):
            for j in range(1, 2 + (3 * b + step) % (k - 1)):
                ws[b, j] = int(r.verify([ws[b, j - 1:j]])[0][0].argmax())
        ref = r.verify(ws)
        got = g.verify(ws, temperature=T, seed=seed, step=40 + step)
        err = np.abs(got - ref).max()
        assert err <= 2e-2, (Bn, k, err)
        n, emit, guide = g.accept(B.DBL_SAMPLE)
        for b in range(Bn):
            n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(ref[b], ws[b], None, T, seed, 40 + step, b, guide_gaps=True)
            total += 1
            if sample_margin_ok(ref[b], ws[b], None, T, am, gap, n_ref, err):
                assert n[b] == n_ref, (Bn, k, b)
                assert np.array_equal(emit[b], e_ref), (Bn, k, b)
                rows = guide_rows(gg, n_ref, T, err)
                assert np.array_equal(guide[b][rows], gd_ref[rows]) and (guide[b][n_ref + 1:] == -1).all(), (Bn, k, b)
                compared += 1
                lengths.add(int(n_ref))
    print("compared %d of %d windows, accepted lengths %s, last logit error %.3g" % (compared, total, sorted(lengths), err))
    assert compared >= total // 2 and len(lengths) >= 3
    # windows of different lengths, one of them absent, in a 128-row call: rows beyond a sequence's length carry random
    # tokens that must not reach its statistics
    lens = [32, 17, 1, 0]
    ws = rng.integers(0, vocab, (4, 32)).astype(np.int32)
    for b, L in enumerate(lens):
        for j in range(1, min(L, 6 + b)):
            ws[b, j] = int(r.verify([ws[b, j - 1:j]])[0][0].argmax())
    g.verify(ws, temperature=T, seed=seed, step=90, win_len=lens, want_logits=False)
    n, emit, guide = g.accept(B.DBL_SAMPLE)
    ragged = 0
    for b, L in enumerate(lens):
        if L == 0:
            assert n[b] == -1 and (emit[b] == -1).all() and (guide[b] == -1).all()
            continue
        ref = r.verify([ws[b, :L]])[0]
        n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(ref, ws[b, :L], None, T, seed, 90, b, guide_gaps=True)
        if sample_margin_ok(ref, ws[b, :L], None, T, am, gap, n_ref, err):
            assert n[b] == n_ref and np.array_equal(emit[b][:n_ref + 1], e_ref[:n_ref + 1]), (b, L)
            assert (emit[b][n_ref + 1:] == -1).all() and (guide[b][n_ref + 1:] == -1).all(), (b, L)
            rows = guide_rows(gg, n_ref, T, err)
            assert np.array_equal(guide[b][rows], gd_ref[rows]), (b, L)
            ragged += 1
    assert ragged >= 2
    g.close()
