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
