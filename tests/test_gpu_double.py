"""The full Double round on the GPU against the oracle.

(1) The device-side pieces one by one, through the C ABI: dbl_merge (Eq. 6) on hand-written cases with the expected
    outputs written out, and on random cases against the oracle's merge; dbl_build_guided_window against the oracle's
    retrieval over x + U; dbl_history_splice / dbl_catchup_window / dbl_history_tail against plain list arithmetic.
(2) Whole runs (two contexts on two streams, paper_2601_05524_amd/double_round.py enqueues, one wait per round)
    against the reference orchestration on the oracle: same tokens, same per-round records (mode, drafts under test,
    accepted length, draft chain length, drafts kept) -- greedy, where both must also equal plain greedy decoding of
    the target, and sampling at T > 0 with the same Philox seeds and step words."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import double_round as REF
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import double_round as DR
from paper_2601_05524_amd import synth
from tests.gpu_util import DEV, TENSORS, Gpu

pytestmark = pytest.mark.gpu

TINY = dict(synth.CONFIGS["tiny"])
T_SEED = synth.BASE_SEED + 5
SHAPE0 = dict(TINY, n_layers=0)


def dev(a):
    return torch.as_tensor(np.asarray(a, dtype=np.int32), device=DEV)


# ------------------------------------------------------------------ dbl_merge

def gpu_merge(g, cases, k, max_chain, max_u, base_len=None):
    """cases: list of (U, E, Xq).  Returns per case (U', text, splice_pos, record)."""
    Bn = len(cases)
    n_u, n_acc = dev([len(c[0]) for c in cases]), dev([len(c[1]) - 1 for c in cases])
    emit = np.full((Bn, k), -1, np.int32)
    chain = np.full((Bn, max_chain), -1, np.int32)
    for b, (U, E, X) in enumerate(cases):
        emit[b, :len(E)] = E
        chain[b, :len(X)] = X
    n_chain = dev([len(c[2]) for c in cases])
    base = None if base_len is None else dev(base_len)
    u_out, n_u_out = g.i32(Bn, max_u, fill=-9), g.i32(Bn, fill=-9)
    text, n_text, pos, rec = g.i32(Bn, k + max_u, fill=-9), g.i32(Bn, fill=-9), g.i32(Bn, fill=-9), g.i32(Bn, 8, fill=-9)
    B.dbl_merge(g.ctx, Bn, k, n_u, n_acc, dev(emit), dev(chain), n_chain, max_chain, max_u, base, u_out, n_u_out, text, n_text,
                pos, rec)
    torch.cuda.synchronize()
    u_out, n_u_out, text, n_text, pos, rec = (t.cpu().numpy() for t in (u_out, n_u_out, text, n_text, pos, rec))
    out = []
    for b in range(Bn):
        assert (u_out[b, n_u_out[b]:] == -1).all()
        out.append((list(u_out[b, :n_u_out[b]]), list(text[b, :n_text[b]]), int(pos[b]), list(rec[b])))
    return out


def test_merge_hand_written_cases():
    """Expected outputs written by hand from Eq. 6: U' and the record {|U|, n_acc, |E|, |X_q|, |U'|, agreeing tokens,
    valid length of the draft's old text}."""
    g = Gpu(SHAPE0, seed=1, max_batch=8, max_ctx=64, max_window=8, max_hist=64)
    cases = [
        ([], [7], [7, 8, 9]),                         # pre-verify, chain starts with the target's token and goes on
        ([], [7], [5, 8, 9]),                         # ... starts differently
        ([], [7, 8], [7, 8]),                         # ... agrees but ends inside G
        ([1, 2], [1, 2, 5, 6, 4], [5, 6, 4, 3, 3]),   # all of U accepted, guidance accepted, chain agrees and goes on
        ([1, 2], [1, 2, 5, 6, 4], [5, 9, 4, 3]),      # chain diverges inside G
        ([1, 2, 3], [1, 9], [4, 4, 4]),               # a token in the middle of U rejected
        ([1, 2, 3], [9], [4, 4, 4]),                  # the first token of U rejected
        ([], [7], [7, 1, 2, 3, 4, 5]),                # more left over than the next window can carry (max_u = 4)
    ]
    want = [
        ([8, 9], [7, 8, 9], [0, 0, 1, 3, 2, 1, 3, 0]),
        ([], [7], [0, 0, 1, 3, 0, 0, 0, 0]),
        ([], [7, 8], [0, 1, 2, 2, 0, 2, 2, 0]),
        ([3, 3], [1, 2, 5, 6, 4, 3, 3], [2, 4, 5, 5, 2, 3, 7, 0]),
        ([], [1, 2, 5, 6, 4], [2, 4, 5, 4, 0, 1, 3, 0]),
        ([], [1, 9], [3, 1, 2, 3, 0, 0, 1, 0]),
        ([], [9], [3, 0, 1, 3, 0, 0, 0, 0]),
        ([1, 2, 3, 4], [7, 1, 2, 3, 4], [0, 0, 1, 6, 4, 1, 5, 0]),
    ]
    base = [100 + len(c[0]) for c in cases]           # the draft's text held x (100 tokens) + U when the chain began
    got = gpu_merge(g, cases, 8, 6, 4, base)
    for c, (u, text, pos, rec), (wu, wtext, wrec) in zip(cases, got, want):
        assert (u, text, rec) == (wu, wtext, wrec), c
        assert pos == 100
    g.close()


def test_merge_random_cases_against_the_oracle():
    g = Gpu(SHAPE0, seed=1, max_batch=8, max_ctx=64, max_window=8, max_hist=64)
    rng = np.random.default_rng(17)
    k, max_chain, max_u = 8, 12, 7
    kinds = set()
    for it in range(60):
        cases = []
        for b in range(8):
            nu = int(rng.integers(0, k))
            U = [int(t) for t in rng.integers(0, 3, nu)]
            if rng.random() < 0.35 and nu > 0:        # reject inside U
                na = int(rng.integers(0, nu))
                E = U[:na] + [3]
            else:
                g_len = int(rng.integers(1, k - nu + 1))
                E = U + [int(t) for t in rng.integers(0, 3, g_len)]
            G = E[len(U):] if len(E) > len(U) else []
            nc = int(rng.integers(0, max_chain + 1))
            X = [int(t) for t in rng.integers(0, 3, nc)]
            if rng.random() < 0.6:                    # a chain that follows G for a while
                m = int(rng.integers(0, len(G) + 1))
                X[:m] = G[:m][:nc]
                if rng.random() < 0.6:
                    X = (G + X)[:max_chain]
            cases.append((U, E, X))
        got = gpu_merge(g, cases, k, max_chain, max_u)
        for (U, E, X), (u, text, pos, rec) in zip(cases, got):
            wu, agree, valid = REF.merge(U, E, X, max_u)
            assert u == wu and text == E + wu
            assert rec == [len(U), len(E) - 1, len(E), len(X), len(wu), agree, valid, 0]
            kinds.add(("reject" if len(E) - 1 < len(U) else "kept" if wu else "agree_short" if agree == len(E) - len(U) else "diverge"))
    assert kinds == {"reject", "kept", "agree_short", "diverge"}
    g.close()


# ------------------------------------------------------------------ guided window, splice, catch-up, tail

def test_guided_window_against_the_oracle_retrieval_over_text_plus_drafts():
    Bn, k = 4, 8
    g = Gpu(SHAPE0, seed=1, max_batch=Bn, max_ctx=64, max_window=k, max_hist=40000)
    rng = np.random.default_rng(23)
    for case in range(30):
        big = case % 6 == 5
        V = int(rng.integers(2, 6)) if not big else 300
        hists, aheads = [], []
        for b in range(Bn):
            L = int(rng.integers(1, 60)) if not big else int(rng.integers(8000, 32768))
            h = rng.integers(0, V, L).astype(np.int32)
            if big:
                for _ in range(30):
                    n = int(rng.integers(8, 40)); s = int(rng.integers(0, L - n)); t = int(rng.integers(0, L - n))
                    h[t:t + n] = h[s:s + n]
            nu = int(rng.integers(0, k))                 # 0 .. k-1 unverified drafts
            u = rng.integers(0, V, nu).astype(np.int32)
            if big and nu >= 3:                          # drafts that continue a span of the text: the key straddles x | U
                s = int(rng.integers(0, L - 40)); h[L - 2:] = h[s:s + 2]; u[:] = h[s + 2:s + 2 + nu]
            B.dbl_history_set(g.ctx, b, h)
            hists.append(h); aheads.append(u)
        n_max, n_min, d = int(rng.integers(1, 5)), 1, int(rng.integers(1, 11))
        ah = np.full((Bn, k - 1), -5, np.int32)
        for b, u in enumerate(aheads):
            ah[b, :len(u)] = u
        window, n_draft = g.i32(Bn, k, fill=-9), g.i32(Bn, fill=-9)
        B.dbl_build_guided_window(g.ctx, Bn, k, dev(ah), dev([len(u) for u in aheads]), k - 1, n_max, n_min, d, 0, window, n_draft)
        torch.cuda.synchronize()
        window, n_draft = window.cpu().numpy(), n_draft.cpu().numpy()
        for b in range(Bn):
            x, u = [int(t) for t in hists[b]], [int(t) for t in aheads[b]]
            room = k - 1 - len(u)
            Y = []
            if room > 0:
                cont, cl, _, _ = O.retrieve(np.asarray(x + u, np.int32), n_max, n_min, min(d, room))
                Y = [int(t) for t in cont[:cl]]
            want = REF.padded_window(x[-1], u + Y, k)
            assert list(window[b]) == want, (case, b)
            assert n_draft[b] == len(u) + len(Y)
        # without drafts the window is dbl_retrieve + dbl_build_window
        w2, nd2 = g.i32(Bn, k, fill=-9), g.i32(Bn, fill=-9)
        B.dbl_build_guided_window(g.ctx, Bn, k, None, None, 0, n_max, n_min, d, 0, w2, nd2)
        torch.cuda.synchronize()
        w2 = w2.cpu().numpy()
        for b in range(Bn):
            cont, cl, _, _ = O.retrieve(hists[b], n_max, n_min, min(d, k - 1))
            assert list(w2[b]) == REF.padded_window(hists[b][-1], list(cont[:cl]), k)
    g.close()


def test_splice_catchup_and_tail():
    """A two-layer model so that KV rows exist: after a splice the kept rows are the common prefix, the catch-up
    window holds exactly the tokens between the cache and the last token, and after the catch-up forward the context
    gives the logits of a context that was loaded with the new text from scratch."""
    g = Gpu(TINY, seed=T_SEED, max_batch=2, max_ctx=256, max_window=8, max_hist=256)
    fresh = Gpu(TINY, seed=T_SEED, max_batch=2, max_ctx=256, max_window=8, max_hist=256)
    rng = np.random.default_rng(3)
    V = TINY["vocab"]
    texts = [rng.integers(0, V, 41).astype(np.int32), rng.integers(0, V, 41).astype(np.int32)]
    g.prefill(texts, 8)
    assert list(g.kv_len()[:2]) == [40, 40]
    # tail: tokens from position 30 / 38 on
    out, n_out = g.i32(2, 6, fill=-9), g.i32(2, fill=-9)
    B.dbl_history_tail(g.ctx, 2, dev([30, 38]), 6, out, n_out)
    torch.cuda.synchronize()
    assert list(n_out.cpu().numpy()) == [6, 3]
    assert list(out.cpu().numpy()[0]) == list(texts[0][30:36]) and list(out.cpu().numpy()[1][:3]) == list(texts[1][38:41])
    assert (out.cpu().numpy()[1][3:] == -1).all()
    # splice: sequence 0 keeps 35 tokens, of the 5 new ones the first two equal the old text; sequence 1 only grows
    new0 = np.concatenate([texts[0][35:37], (texts[0][37:40] + 1) % V]).astype(np.int32)
    new1 = rng.integers(0, V, 4).astype(np.int32)
    toks = np.zeros((2, 8), np.int32); toks[0, :5] = new0; toks[1, :4] = new1
    missing = g.i32(2, fill=-9)
    B.dbl_history_splice(g.ctx, 2, dev([35, 41]), dev(toks), dev([5, 4]), 8, missing)
    torch.cuda.synchronize()
    want0 = np.concatenate([texts[0][:35], new0]); want1 = np.concatenate([texts[1], new1])
    assert np.array_equal(g.history(0), want0) and np.array_equal(g.history(1), want1)
    assert list(g.kv_len()[:2]) == [37, 40]                      # common prefix of old and new text / unchanged
    assert list(missing.cpu().numpy()) == [39 - 37, 44 - 40]
    window, win_len = g.i32(2, 8, fill=-9), g.i32(2, fill=-9)
    B.dbl_catchup_window(g.ctx, 2, 8, 0, window, win_len)
    torch.cuda.synchronize()
    assert list(win_len.cpu().numpy()) == [2, 4]
    assert list(window.cpu().numpy()[0][:2]) == list(want0[37:39]) and list(window.cpu().numpy()[1][:4]) == list(want1[40:44])
    B.dbl_verify_block_ragged(g.ctx, window, win_len, 2, 8)
    B.dbl_kv_commit(g.ctx, win_len)
    torch.cuda.synchronize()
    assert list(g.kv_len()[:2]) == [39, 44]
    # against a context that never saw the old text (same length both, so prefill one at a time)
    for b, w in ((0, want0), (1, want1)):
        fresh.prefill([w, w], 8)
        probe = np.stack([[w[-1], 5, 6], [w[-1], 5, 6]]).astype(np.int32)
        ref = fresh.verify(probe)[0]
        both = np.stack([[want0[-1], 5, 6], [want1[-1], 5, 6]]).astype(np.int32)
        got = g.verify(both)[b]
        assert np.abs(got - ref).max() <= 1e-5
    g.close(); fresh.close()


# ------------------------------------------------------------------ whole runs

def prompt():
    return synth.uniform_history(synth.BASE_SEED, length=256, vocab=2048, span=8, every=32, tail=4)


def make_pair(kind):
    """(oracle draft model, GPU draft lane) of one kind, same weights on both sides."""
    kw = dict(max_ctx=640, max_window=8, max_hist=1024)
    if kind == "same":
        return O.Model(**TINY, max_ctx=640, seed=T_SEED), DR.Lane(TINY, T_SEED, **kw)
    if kind == "unrelated":
        return O.Model(**TINY, max_ctx=640, seed=999), DR.Lane(TINY, 999, **kw)
    # the target's weights with the second layer's MLP switched off
    m, e = O.Model(**TINY, max_ctx=640, seed=T_SEED), DR.Lane(TINY, T_SEED, **kw)
    z = np.zeros(TINY["d_model"] * TINY["d_ffn"], np.float32)
    m.tensor(TENSORS["wd"][1], 1)[:] = z
    B.dbl_set_weights(e.ctx, TENSORS["wd"][0], 1, z)
    return m, e


@pytest.mark.parametrize("kind", ["same", "unrelated", "weakened"])
@pytest.mark.parametrize("gamma,k_p,k_q", [(2, 8, 4), (3, 6, 3)])
def test_greedy_rounds_match_the_reference_and_are_lossless(kind, gamma, k_p, k_q):
    torch.cuda.set_device(0)
    p = prompt()
    tm = O.Model(**TINY, max_ctx=640, seed=T_SEED)
    dm, d_lane = make_pair(kind)
    ref_out, ref_rounds = REF.double_decode(O.Seq(tm, max_hist=1024), O.Seq(dm, max_hist=1024), p, 64, gamma, k_p, k_q)
    ar = REF.autoregressive(O.Seq(tm, max_hist=1024), p, len(ref_out))
    assert ref_out == ar

    t_lane = DR.Lane(TINY, T_SEED, max_ctx=640, max_window=8, max_hist=1024)
    dec = DR.DoubleDecoder(t_lane, d_lane, gamma=gamma, k_p=k_p, k_q=k_q)
    out, rounds = dec.decode(p, 64)
    assert out == ref_out
    assert rounds == ref_rounds
    kv = np.zeros(1, np.int32)
    B.dbl_kv_len(t_lane.ctx, kv)
    assert kv[0] == len(p) + len(out) - 1
    # the same kernels, one token per forward
    assert DR.autoregressive(t_lane, p, len(out)) == out
    print(kind, gamma, k_p, k_q, "rounds", len(rounds), "tokens", len(out),
          "post-verify", sum(r["mode"] == "post" for r in rounds), "catch-up rounds seen:", sum(r["kept"] == 0 for r in rounds))
    t_lane.close(); d_lane.close()


@pytest.mark.parametrize("kind,T", [("same", 0.3), ("weakened", 0.3), ("same", 1.0)])
def test_sampling_rounds_match_the_reference(kind, T):
    """T > 0: the target's acceptance of round r draws with Philox step r, the draft's j-th Retrieval Forward with
    step r * gamma + j, on both sides.  fp32 models, so the two sides' logits differ by ~1e-6 and a decision flips
    only if it is closer than that (the seeds below have no such decision)."""
    torch.cuda.set_device(0)
    p = prompt()
    gamma, k_p, k_q = 2, 8, 4
    tm = O.Model(**TINY, max_ctx=640, seed=T_SEED)
    dm, d_lane = make_pair(kind)
    # livelier logits, so that drafts survive at these temperatures
    for m in {id(tm): tm, id(dm): dm}.values():
        m.tensor(O.T_LM)[:] *= np.float32(16.0)
    t_lane = DR.Lane(TINY, T_SEED, max_ctx=640, max_window=8, max_hist=1024)
    for lane, m in ((t_lane, tm), (d_lane, dm)):
        B.dbl_set_weights(lane.ctx, B.T_LM, 0, np.ascontiguousarray(m.tensor(O.T_LM)))
    st, sq = 0x5EED0001, 0x5EED0002
    ref_out, ref_rounds = REF.double_decode(O.Seq(tm, max_hist=1024), O.Seq(dm, max_hist=1024), p, 48, gamma, k_p, k_q,
                                            temperature=T, seed_target=st, seed_draft=sq)
    dec = DR.DoubleDecoder(t_lane, d_lane, gamma=gamma, k_p=k_p, k_q=k_q, temperature=T, seed_target=st, seed_draft=sq)
    out, rounds = dec.decode(p, 48)
    print(kind, T, "rounds", len(rounds), "tokens", len(out), "post-verify", sum(r["mode"] == "post" for r in rounds),
          "mean accepted", np.mean([r["n_acc"] for r in rounds]))
    assert out == ref_out
    assert rounds == ref_rounds
    assert any(r["mode"] == "post" for r in rounds) or kind != "same"
    t_lane.close(); d_lane.close()
