"""The reference Double round (oracle/double_round.py) against what the paper fixes for it:
greedy output token-identical to plain autoregressive decoding of the target (Sec. 4.2
"maintaining the original distribution under greedy sampling"; App. D.2), whatever the draft
model proposes; Eq. 6's merge on hand-made chains; the mode machine's bookkeeping."""
import numpy as np
import pytest

import oracle as O
from oracle import double_round as DR
from paper_2601_05524_amd import synth

TINY = dict(synth.CONFIGS["tiny"], max_ctx=640)
T_ALL = (O.T_EMB, O.T_LM, O.T_GF)
T_LAYER = (O.T_G1, O.T_WQ, O.T_WK, O.T_WV, O.T_WO, O.T_G2, O.T_WG, O.T_WU, O.T_WD)


def tiny_prompt():
    return synth.uniform_history(synth.BASE_SEED, length=256, vocab=2048, span=8, every=32, tail=4)


def weakened_copy(target, seed):
    """A draft that mostly agrees with the target: the target's weights with the second
    layer's MLP switched off."""
    m = O.Model(**TINY, seed=seed)
    for t in T_ALL:
        m.tensor(t, 0)[:] = target.tensor(t, 0)
    for l in range(TINY["n_layers"]):
        for t in T_LAYER:
            m.tensor(t, l)[:] = target.tensor(t, l)
    m.tensor(O.T_WD, 1)[:] = 0.0
    return m


@pytest.fixture(scope="module")
def target_model():
    return O.Model(**TINY, seed=synth.BASE_SEED + 5)


@pytest.fixture(scope="module")
def ar_tokens(target_model):
    return DR.autoregressive(O.Seq(target_model, max_hist=1024), tiny_prompt(), 72)


@pytest.mark.parametrize("draft_kind", ["same", "unrelated", "weakened"])
@pytest.mark.parametrize("gamma,k_p,k_q", [(2, 8, 4), (3, 6, 3), (1, 4, 2)])
def test_double_round_is_lossless(target_model, ar_tokens, draft_kind, gamma, k_p, k_q):
    if draft_kind == "same":
        dm = target_model
    elif draft_kind == "unrelated":
        dm = O.Model(**TINY, seed=999)
    else:
        dm = weakened_copy(target_model, 7)
    out, rounds = DR.double_decode(O.Seq(target_model, max_hist=1024), O.Seq(dm, max_hist=1024), tiny_prompt(),
                                   64, gamma, k_p, k_q)
    assert len(out) >= 64
    assert out[:64] == ar_tokens[:64]
    assert out == ar_tokens[:len(out)]
    assert sum(r["emitted"] for r in rounds) == len(out)
    for r in rounds:
        assert 1 <= r["emitted"] <= k_p and r["n_u"] <= k_p - 1 and r["kept"] <= k_p - 1
        assert (r["mode"] == "post") == (r["n_u"] > 0)
    per_round = len(out) / len(rounds)
    if draft_kind == "same":
        # a draft identical to the target is never wrong: once drafts are in flight every
        # round verifies them all, and far fewer target forwards than tokens are needed
        assert all(r["n_acc"] >= r["n_u"] for r in rounds)
        if gamma >= 2:    # (one draft forward per round cannot get ahead of the target)
            assert sum(r["mode"] == "post" for r in rounds) >= len(rounds) - 2
            assert per_round > 1.5
    if draft_kind == "unrelated":
        assert per_round >= 1.0
    print(draft_kind, gamma, k_p, k_q, "tokens per target forward %.2f" % per_round,
          "post-verify rounds %d of %d" % (sum(r["mode"] == "post" for r in rounds), len(rounds)))


def test_more_draft_iterations_never_change_the_text(target_model, ar_tokens):
    dm = weakened_copy(target_model, 7)
    outs = []
    for gamma in (1, 2, 4):
        out, _ = DR.double_decode(O.Seq(target_model, max_hist=1024), O.Seq(dm, max_hist=1024), tiny_prompt(),
                                  40, gamma, 8, 4)
        outs.append(out[:40])
    assert outs[0] == outs[1] == outs[2] == ar_tokens[:40]


def test_sync_to_reuses_the_valid_cache_prefix(target_model):
    s = O.Seq(target_model, max_hist=1024)
    p = [int(t) for t in tiny_prompt()[:40]]
    DR.sync_to(s, p)
    assert s.kv_len == 39 and list(s.history()) == p
    k_before = s.kcache()[:, :, :39].copy()
    q = p[:30] + [5, 6, 7]
    DR.sync_to(s, q)                       # rows 0..29 kept, 30 and 31 recomputed
    assert s.kv_len == 32 and list(s.history()) == q
    assert np.array_equal(s.kcache()[:, :, :30], k_before[:, :, :30])
    fresh = O.Seq(target_model, max_hist=1024)
    DR.sync_to(fresh, q)
    assert np.array_equal(fresh.kcache()[:, :, :32], s.kcache()[:, :, :32])
    assert np.array_equal(fresh.verify_block([q[-1], 1, 2]), s.verify_block([q[-1], 1, 2]))


def test_truncate_refuses_to_grow():
    m = O.Model(**dict(TINY, n_layers=0), seed=1)
    s = O.Seq(m, max_hist=16)
    s.hist_set([1, 2, 3])
    with pytest.raises(ValueError):
        s.truncate(hist_len=4)
    s.truncate(hist_len=2)
    assert list(s.history()) == [1, 2]


# ------------------------------------------------------------------ Eq. 6 on hand-made chains

def test_merge_hand_cases():
    """U = drafts under test, E = accepted window tokens + the target's own token, Xq = the draft's new chain."""
    m = DR.merge
    # pre-verify (no U): the target emitted one token, the draft's chain starts with it and goes on
    assert m([], [7], [7, 8, 9], 4) == ([8, 9], 1, 3)
    # ... goes on further than the next window can carry
    assert m([], [7], [7, 8, 9, 10, 11, 12], 3) == ([8, 9, 10], 1, 4)
    # ... starts differently: the target's token stands, nothing of the chain survives
    assert m([], [7], [5, 8, 9], 4) == ([], 0, 0)
    # ... agrees but does not reach past the target's tokens
    assert m([], [7, 8], [7, 8], 4) == ([], 2, 2)
    assert m([], [7, 8], [7], 4) == ([], 1, 1)
    # post-verify: all of U accepted, guidance tokens 5 6 accepted too, target's own token 4; chain agrees and goes on
    assert m([1, 2], [1, 2, 5, 6, 4], [5, 6, 4, 3, 3], 7) == ([3, 3], 3, 7)
    # ... chain diverges inside G (second token)
    assert m([1, 2], [1, 2, 5, 6, 4], [5, 9, 4, 3], 7) == ([], 1, 3)
    # a token in the middle of U rejected: E = accepted part of U + the replacement; the chain built on U is void
    assert m([1, 2, 3], [1, 9], [4, 4, 4], 7) == ([], 0, 1)
    assert m([1, 2, 3], [9], [4, 4, 4], 7) == ([], 0, 0)
    # all of U accepted and nothing else: G is the target's single token
    assert m([1, 2], [1, 2, 8], [8, 6], 7) == ([6], 1, 4)


# ------------------------------------------------------------------ sampling rounds

SMALLV = dict(n_layers=1, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ffn=48, vocab=5, qk_norm=0, dtype=0,
              max_ctx=128, rms_eps=1e-5, rope_base=1e4)


def small_pair():
    tm = O.Model(**SMALLV, seed=101)
    tm.tensor(O.T_LM)[:] *= 24.0           # livelier logits: next-token probabilities between ~1 % and ~70 %
    dm = O.Model(**SMALLV, seed=101)       # a draft that mostly agrees: the same weights, LM head slightly off
    dm.tensor(O.T_LM)[:] = tm.tensor(O.T_LM) * np.float32(1.25)
    return tm, dm


def exact_joint(tm, prompt, T, depth):
    """p(t1..t_depth | prompt) of the target by enumeration with plain one-token forwards."""
    V = SMALLV["vocab"]
    out = {}

    def walk(prefix, p):
        if len(prefix) == depth:
            out[tuple(prefix)] = p
            return
        s = O.Seq(tm, max_hist=128)
        DR.sync_to(s, list(prompt) + prefix)
        z = s.verify_block([(list(prompt) + prefix)[-1]])[0] / T
        q = np.exp(z - z.max()); q /= q.sum()
        for v in range(V):
            walk(prefix + [v], p * q[v])

    walk([], 1.0)
    return out


def test_sampling_round_emits_the_targets_distribution():
    """Lossless under T > 0 (App. D.2 "Stochastic Sampling"): over many seeds the first three tokens a Double run
    emits follow the target's own joint distribution, computed exactly by enumeration -- with drafts in flight (U not
    empty), accepted guidance, rejected drafts and rollbacks all occurring on the way."""
    from scipy import stats
    tm, dm = small_pair()
    T, depth, N = 1.0, 3, 4000
    prompt = [1, 2, 3, 1, 2, 4, 0, 1, 2, 3, 3, 1, 2]
    exact = exact_joint(tm, prompt, T, depth)
    assert abs(sum(exact.values()) - 1.0) < 1e-9
    counts = dict.fromkeys(exact, 0)
    seen = dict(post=0, kept=0, mid_u_reject=0, guidance=0)
    for s in range(N):
        out, rounds = DR.double_decode(O.Seq(tm, max_hist=128), O.Seq(dm, max_hist=128), prompt, depth, 2, 4, 3,
                                       temperature=T, seed_target=s, seed_draft=10 ** 6 + s)
        counts[tuple(out[:depth])] += 1
        for r in rounds:
            seen["post"] += r["mode"] == "post"
            seen["kept"] += r["kept"] > 0
            seen["mid_u_reject"] += r["n_acc"] < r["n_u"]
            seen["guidance"] += r["n_acc"] > r["n_u"]
    print(seen)
    assert min(seen.values()) > N // 50, seen
    cells = sorted(exact, key=exact.get)
    obs, exp, o_acc, e_acc = [], [], 0, 0.0
    for c in cells:                      # pool the rare cells until each expects at least 8 draws
        o_acc += counts[c]; e_acc += exact[c] * N
        if e_acc >= 8:
            obs.append(o_acc); exp.append(e_acc); o_acc, e_acc = 0, 0.0
    obs[-1] += o_acc; exp[-1] += e_acc
    assert len(obs) >= 20
    assert stats.chisquare(obs, exp).pvalue > 1e-3


def test_sampling_round_at_vanishing_temperature_is_the_greedy_round(target_model, ar_tokens):
    dm = weakened_copy(target_model, 7)
    out, rounds = DR.double_decode(O.Seq(target_model, max_hist=1024), O.Seq(dm, max_hist=1024), tiny_prompt(),
                                   40, 2, 8, 4, temperature=1e-4, seed_target=5, seed_draft=6)
    ref, ref_rounds = DR.double_decode(O.Seq(target_model, max_hist=1024), O.Seq(dm, max_hist=1024), tiny_prompt(),
                                       40, 2, 8, 4)
    assert out == ref == ar_tokens[:len(out)]
    assert rounds == ref_rounds
