"""GPU parity: libdbl (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: retrieval results, accepted lengths and emitted ids bit-exact, except rows whose
deciding margin in the oracle is below the tolerance (those are counted, and must stay
rare); logits within 2e-2 max-abs for bf16 models and 1e-4 for fp32 models.
"""
import numpy as np
import pytest

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref

pytestmark = pytest.mark.gpu

TOL = {0: 1e-4, 1: 2e-2}     # logits max-abs, by model dtype

TINY = synth.CONFIGS["tiny"]
SMALL_BF16 = dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1408, vocab=4096,
                  qk_norm=0, dtype=1, rms_eps=1e-5, rope_base=1e4)
SMALL_QWEN = dict(n_layers=2, d_model=1024, n_q_heads=16, n_kv_heads=2, head_dim=128, d_ffn=2080, vocab=3000,
                  qk_norm=1, dtype=1, rms_eps=1e-6, rope_base=1e6)
SMALL_F32_128 = dict(n_layers=1, d_model=384, n_q_heads=6, n_kv_heads=3, head_dim=128, d_ffn=1024, vocab=1000,
                     qk_norm=1, dtype=0, rms_eps=1e-5, rope_base=1e4)


def pair(shape, seed, **kw):
    return Gpu(shape, seed=seed, **kw), Ref(shape, seed=seed, **{k: v for k, v in kw.items() if k != "max_window"})


def jitter_gains(g, r, shape, seed=3):
    rng = np.random.default_rng(seed)
    names = [("gf", 0)] + [(n, l) for l in range(shape["n_layers"]) for n in ("g1", "g2", "gq", "gk")]
    for name, l in names:
        n = shape["head_dim"] if name in ("gq", "gk") else shape["d_model"]
        v = (1.0 + 0.25 * rng.standard_normal(n)).astype(np.float32)
        g.set_tensor(name, l, v)
        r.set_tensor(name, l, v)


# ------------------------------------------------------------------ weights

@pytest.mark.parametrize("shape", [TINY, SMALL_BF16, SMALL_QWEN], ids=["tiny_f32", "small_bf16", "small_qwen"])
def test_seeded_weights_are_bit_identical(shape):
    g, r = pair(shape, 77)
    for name in ("emb", "lm", "gf"):
        assert np.array_equal(g.get_tensor(name), r.get_tensor(name)), name
    for l in range(shape["n_layers"]):
        for name in ("g1", "wq", "wk", "wv", "gq", "gk", "wo", "g2", "wg", "wu", "wd"):
            assert np.array_equal(g.get_tensor(name, l), r.get_tensor(name, l)), (name, l)
    g.close()


def test_set_get_weights_round_trip():
    g = Gpu(SMALL_BF16, seed=1)
    rng = np.random.default_rng(0)
    for name, l in (("wq", 1), ("wk", 0), ("wv", 1), ("wo", 0), ("wg", 1), ("wu", 1), ("wd", 0), ("lm", 0), ("emb", 0)):
        before = {n: g.get_tensor(n, l) for n in ("wq", "wk", "wv", "wg", "wu")}
        n = g._numel(name)
        v = (rng.integers(-64, 64, n) / 128.0).astype(np.float32)     # bf16-exact values
        g.set_tensor(name, l, v)
        assert np.array_equal(g.get_tensor(name, l), v), name
        for other, old in before.items():                             # neighbours in the same container untouched
            if other != name:
                assert np.array_equal(g.get_tensor(other, l), old), (name, other)
    g.close()


# ------------------------------------------------------------------ forward

def check_logits(got, ref, dtype):
    err = np.abs(got.astype(np.float64) - ref).max()
    assert np.isfinite(got).all()
    assert err <= TOL[dtype], "logits max-abs error %.3g" % err
    return err


@pytest.mark.parametrize("shape,seed", [(TINY, 5), (SMALL_BF16, 6), (SMALL_QWEN, 7), (SMALL_F32_128, 8)],
                         ids=["tiny_f32", "small_bf16", "small_qwen", "f32_hd128"])
def test_forward_parity_windows_and_prefill(shape, seed):
    g, r = pair(shape, seed, max_ctx=256, max_window=16)
    jitter_gains(g, r, shape)
    V = shape["vocab"]
    rng = np.random.default_rng(seed)
    toks = rng.integers(0, V, 150).astype(np.int32)
    # ragged chunk sizes: 1-row steps, a full window, odd sizes, spans over several attention steps
    chunks = [16, 1, 7, 16, 16, 3, 16, 16, 2, 5, 16, 9, 1, 16]
    i = 0
    for k in chunks:
        w = toks[i:i + k]
        got = g.verify([w])[0]
        ref = r.verify([w])[0]
        check_logits(got, ref, shape["dtype"])
        # keep only part of some windows: the dropped rows must not leak into later steps
        keep = k if k != 7 else 4
        g.commit([keep])
        r.seqs[0].commit(keep, [])
        i += keep
    assert g.kv_len()[0] == r.seqs[0].kv_len == i
    g.close()


def test_forward_parity_batched_sequences():
    shape = SMALL_BF16
    g, r = pair(shape, 9, max_batch=3, max_ctx=256, max_window=8)
    rng = np.random.default_rng(2)
    # sequences of different committed lengths
    # per-sequence n_keep drives the three sequences to different committed lengths
    for step in range(4):
        ws = [rng.integers(0, shape["vocab"], 8).astype(np.int32) for _ in range(3)]
        got = g.verify(ws)
        ref = r.verify(ws)
        check_logits(got, ref, 1)
        keep = [(3, 8, 1), (8, 2, 5), (1, 1, 8), (4, 4, 4)][step]
        g.commit(list(keep))
        for b in range(3):
            r.seqs[b].commit(keep[b], [])
    assert list(g.kv_len()) == [s.kv_len for s in r.seqs]
    g.close()


def test_long_context_many_splits():
    shape = dict(SMALL_BF16, n_layers=1)
    g, r = pair(shape, 10, max_ctx=2048, max_window=16, max_hist=4096)
    prompt = synth.zipf_history(5, 1500, shape["vocab"])
    g.prefill([prompt], 16)
    r.prefill([prompt], 16)
    assert g.kv_len()[0] == 1499
    w = np.concatenate([prompt[-1:], prompt[3:10]]).astype(np.int32)
    check_logits(g.verify([w])[0], r.verify([w])[0], 1)
    g.close()


# ------------------------------------------------------------------- accept

def sharpen(g, r, factor):
    """Scale the LM head by a power of two on both sides: livelier logits, so that
    accepted lengths vary and top-2 margins are mostly far above the tolerance."""
    lm = r.get_tensor("lm") * np.float32(factor)
    g.set_tensor("lm", 0, lm)
    r.set_tensor("lm", 0, lm)


@pytest.mark.parametrize("shape,seed", [(TINY, 11), (SMALL_BF16, 12)], ids=["tiny_f32", "small_bf16"])
def test_greedy_accept_and_commit_parity(shape, seed):
    g, r = pair(shape, seed, max_ctx=512, max_window=8, max_hist=1024)
    sharpen(g, r, 8.0)
    V = shape["vocab"]
    tol = 8.0 * TOL[shape["dtype"]]           # logits are 8x larger, so is their error bound
    prompt = synth.uniform_history(seed, length=96, vocab=V, span=8, every=24, tail=4)
    g.prefill([prompt], 8)
    r.prefill([prompt], 8)
    s = r.seqs[0]
    compared, exempt, n_seen = 0, 0, set()
    for step in range(24):
        # drafts: the oracle's own greedy continuation, corrupted at a random place
        pending = int(s.history()[-1])
        cont, tmpw = [], [pending]
        for _ in range(7):
            lg = s.verify_block(tmpw)
            cont.append(int(lg[-1].argmax()))
            tmpw.append(cont[-1])
        drafts = synth.corrupt_drafts(1000 + step, np.array(cont, np.int32), V, alpha=0.7)
        w = np.concatenate([[pending], drafts]).astype(np.int32)
        lg_ref = s.verify_block(w)
        n_ref, emit_ref, guide_ref, margin = O.accept_greedy(lg_ref, w)
        lg = g.verify([w])[0]
        err = np.abs(lg - lg_ref).max()
        assert err <= tol
        n, emit, guide = g.accept(B.DBL_GREEDY)
        ex = margin < max(4 * err, 1e-5)      # rows whose top-2 gap the measured error could flip
        assert np.array_equal(guide[0][~ex], guide_ref[~ex])
        if not ex[:n_ref + 1].any():
            assert n[0] == n_ref and np.array_equal(emit[0], emit_ref)
            compared += 1
        else:
            exempt += 1
        n_seen.add(n_ref)
        # teacher forcing: both sides continue from the oracle's decision
        g.commit([n_ref + 1])
        s.commit(n_ref + 1, emit_ref[:n_ref + 1])
        B.dbl_history_set(g.ctx, 0, s.history())
    assert compared >= 16 and exempt <= 8, (compared, exempt)
    assert len(n_seen) >= 3, sorted(n_seen)
    assert g.kv_len()[0] == s.kv_len
    g.close()


def test_free_running_tiny_model_64_tokens():
    """The tiny workload end to end: retrieval-extended drafts, k = 4, greedy, 64 tokens;
    every device-side step chained without host decisions, then compared with the oracle
    run the same way and with plain autoregressive decoding (losslessness)."""
    shape = TINY
    # weight seed chosen so that no row of the oracle's run is under the exemption margin
    g, r = pair(shape, synth.BASE_SEED + 5, max_ctx=512, max_window=4, max_hist=1024)
    prompt = synth.uniform_history(synth.BASE_SEED, length=256, vocab=2048, span=8, every=32, tail=4)
    g.prefill([prompt], 4)
    r.prefill([prompt], 4)
    s = r.seqs[0]
    k, max_cont = 4, 8
    cont, cl, mn, mp = g.i32(1, max_cont), g.i32(1), g.i32(1), g.i32(1)
    window, n_acc, emit, guide = g.i32(1, k), g.i32(1), g.i32(1, k), g.i32(1, k)
    ref_out, accs, margins = [], [], []
    while len(ref_out) < 64:
        c, c_len, _, _ = s.retrieve(3, 1, max_cont)
        w = [int(s.history()[-1])] + [int(t) for t in c[:k - 1]] + [0] * max(0, k - 1 - c_len)
        lg = s.verify_block(w)
        n, e, _, m = O.accept_greedy(lg, w)
        s.commit(n + 1, e[:n + 1])
        ref_out += [int(t) for t in e[:n + 1]]
        accs.append(n)
        margins.append(m[:n + 1].min())
    steps = len(accs)
    for _ in range(steps):
        B.dbl_retrieve(g.ctx, 1, 3, 1, max_cont, cont, cl, mn, mp)
        B.dbl_build_window(g.ctx, 1, k, max_cont, cont, cl, 0, window)
        B.dbl_verify_block(g.ctx, window, 1, k)
        B.dbl_accept(g.ctx, B.DBL_GREEDY, None, n_acc, emit, guide)
        B.dbl_kv_commit(g.ctx, None)
    assert min(margins) > 2 * TOL[0], "oracle run has a near-tie; pick another seed"
    assert g.hist_len()[0] == 256 + len(ref_out)
    assert g.kv_len()[0] == s.kv_len
    assert list(g.history()) == list(prompt) + ref_out        # committed ids, token for token
    assert sum(accs) > 0, "retrieval never helped: workload recipe broken"
    # plain AR decoding of the oracle gives the same tokens (lossless)
    ar = O.Seq(r.model, max_hist=1024)
    ar.hist_set(prompt); ar.verify_block(prompt[:-1]); ar.commit(255, [])
    pend = int(prompt[-1]); ar_out = []
    for _ in range(len(ref_out)):
        lg = ar.verify_block([pend]); pend = int(lg[0].argmax()); ar.commit(1, [pend]); ar_out.append(pend)
    assert ar_out == ref_out
    # the GPU's final retrieval sees the same history: same result as the oracle's
    c_ref, cl_ref, mn_ref, mp_ref = s.retrieve(3, 1, max_cont)
    c_g, cl_g, mn_g, mp_g = g.retrieve(1, 3, 1, max_cont)
    assert (cl_g[0], mn_g[0], mp_g[0]) == (cl_ref, mn_ref, mp_ref)
    assert list(c_g[0][:cl_ref]) == list(c_ref)
    B.dbl_retrieve(g.ctx, 1, 3, 1, max_cont, cont, cl, mn, mp)
    B.dbl_build_window(g.ctx, 1, k, max_cont, cont, cl, 0, window)
    wlast = window.cpu().numpy()[0]
    assert int(wlast[0]) == ref_out[-1]
    assert list(wlast[1:1 + min(cl_ref, k - 1)]) == list(c_ref[:k - 1])
    g.close()


def sample_margin_ok(lg_ref, w, q, T, u_margin, gap, n, err):
    """Compare a sequence's decisions only if the oracle's margins exceed what the measured
    logit error can move: p(x) by a factor exp(+-2 err/T), Gumbel scores by 2 err/T."""
    k = len(w)
    rel = 2.0 * err / T
    for j in range(min(n + 1, k - 1)):
        z = lg_ref[j] / T
        p = np.exp(z - z.max()); p /= p.sum()
        px = p[w[j + 1]]
        if u_margin[j] <= 1.5 * rel * px + 1e-9:
            return False
    return gap > 1.5 * rel + 1e-6


def guide_rows(guide_gap, n, T, err):
    """Rows j <= n whose own draw (the guidance Eq. 6 consumes) is decided by more than the logit
    error can move: the same rule as for the emitted token's draw."""
    return [j for j in range(n + 1) if guide_gap[j] > 1.5 * (2.0 * err / T) + 1e-6]


@pytest.mark.parametrize("dense", [False, True], ids=["one_hot_q", "dense_q"])
def test_sampling_accept_parity(dense):
    shape = SMALL_BF16
    g, r = pair(shape, 14, max_batch=2, max_ctx=512, max_window=8)
    sharpen(g, r, 8.0)
    V = shape["vocab"]
    T = 0.7
    rng = np.random.default_rng(4)
    prompts = [synth.zipf_history(20 + b, 40, V) for b in range(2)]
    g.prefill(prompts, 8)
    r.prefill(prompts, 8)
    compared, exempt, n_hist, guides = 0, 0, [], 0
    for step in range(30):
        ws, qs, refs = [], [], []
        for b in range(2):
            s = r.seqs[b]
            pending = int(s.history()[-1])
            # drafts: mostly the oracle's own top-1, so that several survive at T = 0.7
            tmpw, cont = [pending], []
            for _ in range(7):
                lg = s.verify_block(tmpw)
                cont.append(int(lg[-1].argmax()) if rng.random() < 0.85 else int(rng.integers(0, V)))
                tmpw.append(cont[-1])
            w = np.array([pending] + cont, np.int32)
            lg_ref = s.verify_block(w)
            q = synth.dense_q(900 + 2 * step + b, 7, V, T, mix_logits=lg_ref[:7] * 1.5) if dense else None
            ws.append(w); qs.append(q); refs.append(lg_ref)
        lg = g.verify(ws, temperature=T, seed=0xABCDEF0123, step=1000 + step)
        qd = np.stack(qs) if dense else None
        n, emit, guide = g.accept(B.DBL_SAMPLE, qd)
        commits = g.ncommit   # the Philox step word is step + commits run so far
        for b in range(2):
            err = np.abs(lg[b] - refs[b]).max()
            assert err <= 8.0 * TOL[1]
            n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(refs[b], ws[b], qs[b], T, 0xABCDEF0123,
                                                                1000 + step + commits, b, guide_gaps=True)
            if sample_margin_ok(refs[b], ws[b], qs[b], T, am, gap, n_ref, err):
                assert n[b] == n_ref, (step, b)
                assert np.array_equal(emit[b], e_ref), (step, b)
                assert np.array_equal(guide[b][n_ref + 1:], gd_ref[n_ref + 1:])
                # the target's own draws up to the first rejection: what forward guidance consumes
                rows = guide_rows(gg, n_ref, T, err)
                assert np.array_equal(guide[b][rows], gd_ref[rows]), (step, b, rows)
                guides += len(rows)
                compared += 1
            else:
                exempt += 1
            n_hist.append(n_ref)
            r.seqs[b].commit(n_ref + 1, e_ref[:n_ref + 1])
        g.commit([n + 1 for n in n_hist[-2:]])
        for b in range(2):
            B.dbl_history_set(g.ctx, b, r.seqs[b].history())
    assert compared >= 36, (compared, exempt)
    assert guides >= compared, (guides, compared)
    assert len(set(n_hist)) >= 3, "accepted lengths should vary: %s" % sorted(set(n_hist))
    g.close()


def test_stress_shape_batch4_ragged_contexts_windows_4_to_32():
    """The long-context stress workload's structure at a width the oracle can follow: batch 4
    with different context lengths, verify windows k = 4, 8, 16, 32 (16, 32, 64, 128 rows: one
    pass over the weights with 1, 2, 4, 8 row groups), speculative sampling at temperature 1.0."""
    shape = SMALL_BF16
    Bn, T, seed = 4, 1.0, 0x5EED5EED
    g, r = pair(shape, 15, max_batch=Bn, max_ctx=1280, max_window=32, max_hist=2048)
    sharpen(g, r, 8.0)
    V = shape["vocab"]
    rng = np.random.default_rng(6)
    lens = [97, 333, 650, 1021]
    prompts = [synth.zipf_history(40 + b, lens[b] + 1, V) for b in range(Bn)]
    # ragged prefill: 16-row chunks; a sequence that is done keeps 0 rows of its (dummy) chunk
    B.dbl_reset(g.ctx, -1)
    done = [0] * Bn
    for b in range(Bn):
        B.dbl_history_set(g.ctx, b, np.ascontiguousarray(prompts[b], dtype=np.int32))
    while any(done[b] < lens[b] for b in range(Bn)):
        ws, keep = [], []
        for b in range(Bn):
            n = min(16, lens[b] - done[b])
            w = np.zeros(16, np.int32)
            w[:n] = prompts[b][done[b]:done[b] + n]
            ws.append(w); keep.append(n); done[b] += n
        g.verify(ws, want_logits=False)
        g.commit(keep)
    assert g.kv_len().tolist() == lens
    r.prefill(prompts, 16)
    compared, exempt, n_hist = 0, 0, []
    for step, k in enumerate((4, 8, 16, 32, 8)):
        ws, refs = [], []
        for b in range(Bn):
            s = r.seqs[b]
            tmpw = [int(s.history()[-1])]
            for _ in range(k - 1):     # drafts: mostly the oracle's own top-1
                lg = s.verify_block(tmpw)
                tmpw.append(int(lg[-1].argmax()) if rng.random() < 0.9 else int(rng.integers(0, V)))
            w = np.array(tmpw, np.int32)
            ws.append(w); refs.append(s.verify_block(w))
        lg = g.verify(ws, temperature=T, seed=seed, step=50 + step)
        n, emit, guide = g.accept(B.DBL_SAMPLE, None)
        commits = g.ncommit
        keep = []
        for b in range(Bn):
            err = np.abs(lg[b] - refs[b]).max()
            assert err <= 8.0 * TOL[1], (k, b, err)     # sharpened LM head: 8 x the logit scale
            n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(refs[b], ws[b], None, T, seed, 50 + step + commits, b,
                                                                guide_gaps=True)
            if sample_margin_ok(refs[b], ws[b], None, T, am, gap, n_ref, err):
                assert n[b] == n_ref, (k, b)
                assert np.array_equal(emit[b], e_ref), (k, b)
                rows = guide_rows(gg, n_ref, T, err)
                assert np.array_equal(guide[b][rows], gd_ref[rows]) and (guide[b][n_ref + 1:] == -1).all(), (k, b, rows)
                compared += 1
            else:
                exempt += 1
            n_hist.append(n_ref)
            keep.append(n_ref + 1)
            r.seqs[b].commit(n_ref + 1, e_ref[:n_ref + 1])
        g.commit(keep)
        for b in range(Bn):
            B.dbl_history_set(g.ctx, b, r.seqs[b].history())
        assert g.kv_len().tolist() == [len(r.seqs[b].history()) - 1 for b in range(Bn)]
    assert compared >= 14, (compared, exempt)
    assert len(set(n_hist)) >= 3, "accepted lengths should vary: %s" % sorted(set(n_hist))
    g.close()


# ----------------------------------------------------------------- retrieve

def test_retrieval_parity():
    shape = dict(TINY, n_layers=0)
    g = Gpu(shape, seed=1, max_batch=4, max_ctx=64, max_window=4, max_hist=40000)
    cases = []
    for seed in range(6):
        cases.append(synth.zipf_history(300 + seed, 32768 if seed < 2 else 4096, 50000, repeat_frac=0.3,
                                        span_lo=8, span_hi=64))
    cases.append(synth.uniform_history(9, length=256, vocab=2048))
    cases += [np.array(x, np.int32) for x in ([1, 2] * 40, [5], [], [4, 4], [9, 3, 3, 3, 3], list(range(100)),
                                               [7] * 1500, [1, 2, 3, 10, 11, 12, 0, 0, 1, 2, 3, 20, 1, 2, 3])]
    params = [(3, 1, 8), (3, 3, 8), (1, 1, 1), (5, 2, 10), (32, 1, 64), (8, 8, 3)]
    for i in range(0, len(cases), 4):
        batch = cases[i:i + 4]
        B.dbl_reset(g.ctx, -1)
        for b, h in enumerate(batch):
            B.dbl_history_set(g.ctx, b, np.ascontiguousarray(h, np.int32))
        for (n_max, n_min, mc) in params:
            c, cl, mn, mp = g.retrieve(len(batch), n_max, n_min, mc)
            for b, h in enumerate(batch):
                for cut in ([len(h)] if len(h) < 1000 else [len(h)]):
                    rc, rcl, rmn, rmp = O.retrieve(h[:cut], n_max, n_min, mc)
                    assert (cl[b], mn[b], mp[b]) == (rcl, rmn, rmp), (i + b, n_max, n_min, mc)
                    assert list(c[b][:rcl]) == list(rc) and (c[b][rcl:] == -1).all()
    g.close()
