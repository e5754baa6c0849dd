"""Pins for the oracle's decoder forward (the verify step of Sec. 2.1 / App. D.2)."""
import os

import numpy as np
import pytest

import oracle as O
from paper_2601_05524_amd import synth
from tests.torch_decoder import forward_full, np_round_bf16

GOLD = os.path.join(os.path.dirname(__file__), "golden")

SMALL = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=97,
             max_ctx=64, rms_eps=1e-5, rope_base=1e4)


def jitter_gains(model, seed=5):
    """Non-trivial norm gains, so a dropped or misplaced gain cannot hide."""
    rng = np.random.default_rng(seed)
    c = model.cfg
    model.tensor(O.T_GF)[:] = 1.0 + 0.3 * rng.standard_normal(c.d_model).astype(np.float32)
    for l in range(c.n_layers):
        for tid in (O.T_G1, O.T_G2, O.T_GQ, O.T_GK):
            t = model.tensor(tid, l)
            t[:] = 1.0 + 0.3 * rng.standard_normal(t.size).astype(np.float32)


def scale_weights(model, f):
    """Larger projections => attention and SwiGLU far from their linear regime."""
    c = model.cfg
    for l in range(c.n_layers):
        for tid in (O.T_WQ, O.T_WK, O.T_WV, O.T_WO, O.T_WG, O.T_WU, O.T_WD):
            model.tensor(tid, l)[:] *= f
    model.tensor(O.T_EMB)[:] *= f


def run_chunks(model, tokens, chunks):
    """Feed `tokens` through verify_block + commit in the given chunk sizes."""
    s = O.Seq(model)
    out = []
    i = 0
    for k in chunks:
        lg = s.verify_block(tokens[i:i + k])
        out.append(lg)
        s.commit(k, tokens[i:i + k])
        i += k
    assert i == len(tokens)
    return np.concatenate(out), s


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("qk_norm", [0, 1])
def test_matches_library_decoder(dtype, qk_norm):
    m = O.Model(**SMALL, qk_norm=qk_norm, dtype=dtype, seed=11)
    scale_weights(m, 6.0)
    jitter_gains(m)
    if dtype == 1:   # keep the bf16 model's weights bf16 after scaling
        for l in range(2):
            for tid in range(O.T_G1, O.T_WD + 1):
                t = m.tensor(tid, l)
                t[:] = np_round_bf16(t.astype(np.float64)).astype(np.float32)
        for tid in (O.T_EMB, O.T_GF):
            t = m.tensor(tid)
            t[:] = np_round_bf16(t.astype(np.float64)).astype(np.float32)
    rng = np.random.default_rng(1)
    toks = rng.integers(0, 97, 23).astype(np.int32)
    got, _ = run_chunks(m, toks, [5, 1, 8, 4, 2, 3])
    ref = forward_full(m, toks)
    # sanity only: the comparison below is not between two near-zero tensors.  The largest reference logit of
    # the four cases is 0.501, 0.499 (fp32 with q/k-norm), 0.527, 0.526 -- hence 0.45 and not 0.5
    assert np.abs(ref).max() > 0.45
    if dtype == 0:
        # only difference: the oracle's cos/sin go through an fp32 table
        np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6)
    else:
        # identical rounding points => equal up to the rare rounding flipped by the
        # 1e-8 table difference (one bf16 ulp of one activation)
        err = np.abs(got - ref)
        assert np.median(err) < 1e-7
        assert err.max() < 2e-3
    # and the bf16 model is close to, but not the same as, its unrounded twin
    if dtype == 1:
        m0 = O.Model(**SMALL, qk_norm=qk_norm, dtype=0, seed=11)
        for tid in (O.T_EMB, O.T_LM, O.T_GF):
            m0.tensor(tid)[:] = m.tensor(tid)
        for l in range(2):
            for tid in range(O.T_G1, O.T_WD + 1):
                m0.tensor(tid, l)[:] = m.tensor(tid, l)
        got0, _ = run_chunks(m0, toks, [23])
        dev = np.abs(got0 - got).max()
        assert 1e-5 < dev < 0.2


def test_window_equals_single_row_steps_bitwise():
    m = O.Model(**SMALL, qk_norm=1, dtype=1, seed=2)
    jitter_gains(m)
    toks = np.random.default_rng(0).integers(0, 97, 20).astype(np.int32)
    a, sa = run_chunks(m, toks, [7, 6, 7])
    b, sb = run_chunks(m, toks, [1] * 20)
    assert np.array_equal(a, b)
    assert np.array_equal(sa.kcache()[:, :, :20], sb.kcache()[:, :, :20])
    assert np.array_equal(sa.vcache()[:, :, :20], sb.vcache()[:, :, :20])
    # the cache holds bf16 values
    kc = sa.kcache()[:, :, :20]
    assert np.array_equal(kc, np_round_bf16(kc))


def test_zero_layers_closed_form():
    m = O.Model(**{**SMALL, "n_layers": 0}, dtype=0, seed=4)
    jitter_gains(m)
    d, V = 64, 97
    emb = m.tensor(O.T_EMB).reshape(V, d).astype(np.float64)
    lm = m.tensor(O.T_LM).reshape(V, d).astype(np.float64)
    gf = m.tensor(O.T_GF).astype(np.float64)
    lg = O.Seq(m).verify_block([3, 50])
    for j, t in enumerate([3, 50]):
        x = emb[t]
        a = x / np.sqrt((x * x).mean() + 1e-5) * gf
        np.testing.assert_allclose(lg[j], lm @ a, rtol=1e-12, atol=1e-14)


def test_zero_output_projections_make_layers_identity():
    m = O.Model(**SMALL, dtype=1, seed=6)
    for l in range(2):
        m.tensor(O.T_WO, l)[:] = 0
        m.tensor(O.T_WD, l)[:] = 0
    m0 = O.Model(**{**SMALL, "n_layers": 0}, dtype=1, seed=6)
    toks = [5, 9, 33, 2]
    assert np.array_equal(O.Seq(m).verify_block(toks), O.Seq(m0).verify_block(toks))


def test_uniform_attention_is_running_mean_of_v():
    # Wq = 0 -> all scores equal -> attention output = mean of v over slots 0..t.
    # With Wo = identity, Wd = 0 and one layer: hidden_t = emb_t + mean_{s<=t} v_s.
    cfg = dict(n_layers=1, d_model=32, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=16, vocab=50,
               max_ctx=32, rms_eps=1e-5, rope_base=1e4)
    m = O.Model(**cfg, dtype=0, seed=8)
    m.tensor(O.T_WQ, 0)[:] = 0
    m.tensor(O.T_WD, 0)[:] = 0
    m.tensor(O.T_WO, 0)[:] = np.eye(32, dtype=np.float32).ravel()
    toks = [4, 7, 7, 19, 0, 23]
    _, hid = O.Seq(m).verify_block(toks, want_hidden=True)
    emb = m.tensor(O.T_EMB).reshape(50, 32).astype(np.float64)
    wv = m.tensor(O.T_WV, 0).reshape(16, 32).astype(np.float64)
    x = emb[toks]
    a = x / np.sqrt((x * x).mean(axis=1, keepdims=True) + 1e-5)
    v = a @ wv.T                                          # [T][Hkv*hd]
    run = np.cumsum(v, axis=0) / np.arange(1, 7)[:, None]
    # query head h reads kv head h // 2
    exp = x + np.concatenate([run[:, 0:8], run[:, 0:8], run[:, 8:16], run[:, 8:16]], axis=1)
    np.testing.assert_allclose(hid, exp, rtol=1e-10, atol=1e-12)


def test_gqa_equals_mha_with_duplicated_kv_heads():
    a = O.Model(**SMALL, dtype=0, seed=9)
    b = O.Model(**{**SMALL, "n_kv_heads": 4}, dtype=0, seed=9)
    for tid in (O.T_EMB, O.T_LM):
        b.tensor(tid)[:] = a.tensor(tid)
    for l in range(2):
        for tid in (O.T_WQ, O.T_WO, O.T_WG, O.T_WU, O.T_WD):
            b.tensor(tid, l)[:] = a.tensor(tid, l)
        for tid in (O.T_WK, O.T_WV):
            w = a.tensor(tid, l).reshape(2, 16, 64)
            b.tensor(tid, l)[:] = np.repeat(w, 2, axis=0).ravel()
    toks = [1, 2, 3, 4, 5, 6, 7]
    np.testing.assert_allclose(O.Seq(a).verify_block(toks), O.Seq(b).verify_block(toks), rtol=0, atol=1e-13)


def test_rope_properties():
    base = 1e4
    # hd = 2: a plane rotation by pos * base^0 = pos radians
    for pos in (0, 1, 5, 77):
        out = O.rope([1.0, 0.0], pos, base)
        np.testing.assert_allclose(out, [np.cos(pos), np.sin(pos)], atol=1e-7)
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal(64), rng.standard_normal(64)
    # position 0 is the identity; norms are kept
    assert np.array_equal(O.rope(q, 0, base), q)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, 1234, base)), np.linalg.norm(q), rtol=1e-6)
    # scores depend on the position difference only
    ref = O.rope(q, 9, base) @ O.rope(k, 4, base)
    for shift in (1, 100, 2000):
        np.testing.assert_allclose(O.rope(q, 9 + shift, base) @ O.rope(k, 4 + shift, base), ref, atol=1e-4)
    # pairing is (i, i + hd/2) with frequency base^(-2i/hd): rotating the unit vector of dim 3
    e = np.zeros(64); e[3] = 1.0
    out = O.rope(e, 10, base)
    ang = 10 * base ** (-6.0 / 64)
    np.testing.assert_allclose([out[3], out[35]], [np.cos(ang), np.sin(ang)], atol=1e-7)
    assert np.count_nonzero(out) == 2


def test_rmsnorm_matches_library():
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(4)
    x = rng.standard_normal(300) * 3
    g = (1 + 0.2 * rng.standard_normal(300)).astype(np.float32)
    ref = F.rms_norm(torch.from_numpy(x), (300,), torch.from_numpy(g.astype(np.float64)), 1e-6).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-6), ref, rtol=1e-13)


def test_shapes_follow_paper_table():
    rows = {}
    for line in open(os.path.join(GOLD, "model_shapes.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, L, d, f, v = line.split()
        rows[name] = (int(L), int(d), int(f), int(v))
    for name, (L, d, f, v) in rows.items():
        c = synth.CONFIGS[name]
        assert (c["n_layers"], c["d_model"], c["d_ffn"], c["vocab"]) == (L, d, f, v)


def test_rejects_bad_windows():
    m = O.Model(**SMALL, dtype=0, seed=1)
    s = O.Seq(m)
    with pytest.raises(ValueError):
        s.verify_block([97])
    with pytest.raises(ValueError):
        s.verify_block(list(range(65)))
