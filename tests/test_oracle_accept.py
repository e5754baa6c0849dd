"""Pins for the oracle's acceptance rules (Sec. 2.1; App. D.2) and the lossless invariant."""
import os

import numpy as np
import pytest
from scipy import stats

import oracle as O
from paper_2601_05524_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")
TINY = dict(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, head_dim=16, d_ffn=96, vocab=61,
            max_ctx=256, rms_eps=1e-5, rope_base=1e4)


# ------------------------------------------------------------------ greedy

def test_greedy_hand_cases():
    V = 5
    z = np.full((4, V), -1.0)
    top = [2, 4, 0, 3]
    for j, t in enumerate(top):
        z[j, t] = 1.0
    # drafts 2,4,0 all match -> 3 accepted + bonus = argmax of the last row
    n, emit, guide, margin = O.accept_greedy(z, [9 % V, 2, 4, 0])
    assert (n, list(emit), list(guide)) == (3, [2, 4, 0, 3], top)
    assert np.allclose(margin, 2.0)
    # first draft wrong -> nothing accepted, correction = argmax of row 0
    n, emit, _, _ = O.accept_greedy(z, [0, 1, 4, 0])
    assert (n, list(emit)) == (0, [2, -1, -1, -1])
    # mismatch in the middle: later matching drafts do not count
    n, emit, _, _ = O.accept_greedy(z, [0, 2, 1, 0])
    assert (n, list(emit)) == (1, [2, 4, -1, -1])
    # window of one row (plain autoregressive step)
    n, emit, _, _ = O.accept_greedy(z[:1], [3])
    assert (n, list(emit)) == (0, [2])
    # exact tie -> lowest id
    z2 = np.zeros((1, V)); z2[0, 1] = z2[0, 3] = 7.0
    n, emit, guide, margin = O.accept_greedy(z2, [0])
    assert guide[0] == 1 and margin[0] == 0.0


def ar_decode(model, prompt, n_new):
    s = O.Seq(model)
    s.hist_set(prompt)
    if len(prompt) > 1:
        s.verify_block(prompt[:-1]); s.commit(len(prompt) - 1, [])
    pending = int(prompt[-1])
    out = []
    for _ in range(n_new):
        lg = s.verify_block([pending])
        _, emit, _, _ = O.accept_greedy(lg, [pending])
        s.commit(1, emit[:1])
        pending = int(emit[0]); out.append(pending)
    return out


def spec_decode(model, prompt, n_new, k, draft_fn):
    s = O.Seq(model)
    s.hist_set(prompt)
    if len(prompt) > 1:
        s.verify_block(prompt[:-1]); s.commit(len(prompt) - 1, [])
    pending = int(prompt[-1])
    out, accs = [], []
    while len(out) < n_new:
        drafts = draft_fn(s, len(out), k - 1)
        window = [pending] + [int(t) for t in drafts]
        lg = s.verify_block(window)
        n, emit, _, _ = O.accept_greedy(lg, window)
        s.commit(n + 1, emit[:n + 1])
        out += [int(t) for t in emit[:n + 1]]
        accs.append((len(out) - n - 1, window, n))
        pending = out[-1]
    return out, accs, s


@pytest.mark.parametrize("kind", ["random", "retrieved", "oracle_then_wrong", "all_right"])
def test_lossless_greedy_equals_autoregressive(kind):
    """App. D.2: under greedy acceptance the speculative output is token-identical
    to plain autoregressive decoding, whatever the draft source."""
    m = O.Model(**TINY, dtype=0, seed=21)
    for l in range(2):            # livelier logits
        for tid in (O.T_WQ, O.T_WK, O.T_WV, O.T_WO, O.T_WG, O.T_WU, O.T_WD):
            m.tensor(tid, l)[:] *= 5
    prompt = synth.uniform_history(3, length=48, vocab=61, span=6, every=12, tail=3)
    n_new = 40
    ref = ar_decode(m, prompt, n_new + 8)
    rng = np.random.default_rng(5)

    def draft_fn(seq, pos, n):
        if kind == "random":
            return rng.integers(0, 61, n)
        if kind == "retrieved":
            cont, cl, _, _ = seq.retrieve(3, 1, n)
            return list(cont) + [0] * (n - cl)
        d = list(ref[pos:pos + n])
        if kind == "oracle_then_wrong":
            w = int(rng.integers(0, n + 1))
            if w < n:
                d[w] = (d[w] + 1) % 61
        return d

    out, accs, seq = spec_decode(m, prompt, n_new, 5, draft_fn)
    assert out[:n_new] == ref[:n_new]
    # accepted length = length of the common prefix of the drafts with the AR continuation
    for pos, window, n in accs:
        drafts = window[1:]
        cp = 0
        while cp < len(drafts) and drafts[cp] == ref[pos + cp]:
            cp += 1
        assert n == cp
    if kind == "all_right":
        assert all(n == 4 for _, _, n in accs)
    assert list(seq.history()) == list(prompt) + out
    assert seq.kv_len == len(prompt) + len(out) - 1


# ---------------------------------------------------------------- sampling

def logits_of(p):
    return np.log(np.asarray(p, dtype=np.float64))


def test_theorem1_expected_length():
    """Eq. 1: with a constant per-token acceptance rate alpha and gamma drafts the
    expected number of emitted tokens is (1 - alpha^(gamma+1)) / (1 - alpha)."""
    for line in open(os.path.join(GOLD, "theorem1.txt")):
        if line.startswith("#") or not line.strip():
            continue
        alpha, gamma, expect = line.split()
        alpha, gamma, expect = float(alpha), int(gamma), float(expect)
        V = 4
        # every draft is token 1 and every row gives it probability alpha (deterministic
        # proposal => accepted with probability p(x) = alpha)
        p = np.array([(1 - alpha) * 0.5, alpha, (1 - alpha) * 0.3, (1 - alpha) * 0.2])
        z = np.tile(logits_of(p), (gamma + 1, 1))
        window = [0] + [1] * gamma
        N = 40000
        tot = 0
        for s in range(N):
            n, _, _, _, _ = O.accept_sample(z, window, None, 1.0, 99, s)
            tot += n + 1
        se = np.sqrt(gamma + 1) / np.sqrt(N)
        assert abs(tot / N - expect) < 4 * se, (alpha, gamma, tot / N, expect)


def test_sampling_accept_length_and_marginal_dense_q():
    """Drafts drawn from q, verified against p: P(n_acc = j) = prod_{i<j} beta_i (1 - beta_j),
    beta_i = sum_v min(p_i, q_i); and the first emitted token is distributed as p_0."""
    rng = np.random.default_rng(12)
    V, k = 6, 4
    P = rng.dirichlet(np.ones(V) * 0.8, size=k)
    Q = rng.dirichlet(np.ones(V) * 0.8, size=k - 1)
    T = 0.7
    z = logits_of(P) * T + rng.standard_normal((k, 1))       # softmax(z/T) == P
    beta = np.minimum(P[:k - 1], Q).sum(axis=1)
    N = 60000
    hist_n = np.zeros(k, int)
    first = np.zeros(V, int)
    for s in range(N):
        drafts = [int(rng.choice(V, p=Q[j])) for j in range(k - 1)]
        n, emit, _, _, _ = O.accept_sample(z, [0] + drafts, Q.astype(np.float32), T, 7, s)
        hist_n[n] += 1
        first[emit[0]] += 1
        assert list(emit[:n]) == drafts[:n] and emit[n] >= 0 and all(emit[n + 1:] == -1)
    expect_n = np.array([np.prod(beta[:j]) * (1 - beta[j] if j < k - 1 else 1.0) for j in range(k)])
    assert stats.chisquare(hist_n, expect_n * N).pvalue > 1e-4
    assert stats.chisquare(first, P[0] * N).pvalue > 1e-4
    e_len = sum(np.prod(beta[:j]) for j in range(k))          # sum_j prod_{i<j} beta_i
    assert abs((hist_n * np.arange(1, k + 1)).sum() / N - e_len) < 0.03


def test_sampling_one_hot_proposals():
    """q = NULL: the draft x was proposed deterministically; it survives with probability
    p(x), and the replacement is p with x removed (never x itself)."""
    V = 5
    p = np.array([0.1, 0.35, 0.05, 0.3, 0.2])
    z = np.tile(logits_of(p), (2, 1)) * 0.5      # T = 0.5 restores p
    N = 50000
    acc = 0
    repl = np.zeros(V, int)
    bonus = np.zeros(V, int)
    for s in range(N):
        n, emit, guide, am, _ = O.accept_sample(z, [2, 3], None, 0.5, 1234, s, b=2)
        if n == 1:
            acc += 1
            bonus[emit[1]] += 1
            assert emit[0] == 3 and guide[1] == emit[1]
        else:
            repl[emit[0]] += 1
            assert guide[1] == -1        # guidance after a rejection is discarded
    assert abs(acc / N - 0.3) < 4 * np.sqrt(0.21 / N)
    assert repl[3] == 0
    res = p.copy(); res[3] = 0; res /= res.sum()
    keep = res > 0
    assert stats.chisquare(repl[keep], res[keep] * repl.sum()).pvalue > 1e-4
    assert stats.chisquare(bonus, p * bonus.sum()).pvalue > 1e-4


def test_sampling_overall_output_is_target_distribution():
    """Losslessness at T > 0: whatever q is, the token emitted at the first position
    follows p_0 -- also for a q that puts zero mass where p has mass."""
    rng = np.random.default_rng(3)
    V = 4
    p = np.array([0.5, 0.25, 0.125, 0.125])
    q = np.array([0.0, 0.7, 0.3, 0.0])
    z = np.tile(logits_of(p), (2, 1))
    N = 50000
    first = np.zeros(V, int)
    for s in range(N):
        x = int(rng.choice(V, p=q))
        _, emit, _, _, _ = O.accept_sample(z, [1, x], q[None].astype(np.float32), 1.0, 5, s)
        first[emit[0]] += 1
    assert stats.chisquare(first, p * N).pvalue > 1e-4


def test_sampling_identical_p_q_never_rejects():
    p = np.array([0.2, 0.3, 0.5])
    z = np.tile(logits_of(p), (3, 1))
    q = np.tile(p, (2, 1)).astype(np.float64)
    # use the fp32-rounded q as the target too, so that p == q exactly
    z = np.tile(logits_of(q[0].astype(np.float32).astype(np.float64)), (3, 1))
    for s in range(300):
        n, _, _, _, _ = O.accept_sample(z, [0, s % 3, (s // 3) % 3], q.astype(np.float32), 1.0, 8, s)
        assert n == 2


def test_sampling_low_temperature_reproduces_greedy():
    rng = np.random.default_rng(10)
    for s in range(50):
        z = rng.standard_normal((4, 9)) * 3
        top = z.argmax(axis=1)
        window = [0] + [int(t) for t in top[:3]]
        if s % 2:
            window[2] = (window[2] + 1) % 9
        ng, eg, _, _ = O.accept_greedy(z, window)
        n, e, _, _, _ = O.accept_sample(z, window, None, 1e-3, 17, s)
        assert n == ng and list(e) == list(eg)


def test_sampling_streams_are_keyed():
    z = np.zeros((3, 64))
    w = [0, 1, 2]
    base = O.accept_sample(z, w, None, 1.0, 1, 0, b=0)
    same = O.accept_sample(z, w, None, 1.0, 1, 0, b=0)
    assert base[0] == same[0] and list(base[1]) == list(same[1])
    diff = sum(list(O.accept_sample(z, w, None, 1.0, 1, s, b=0)[1]) != list(base[1]) for s in range(1, 20))
    diff_b = sum(list(O.accept_sample(z, w, None, 1.0, 1, 0, b=b)[1]) != list(base[1]) for b in range(1, 20))
    diff_seed = sum(list(O.accept_sample(z, w, None, 1.0, sd, 0)[1]) != list(base[1]) for sd in range(2, 21))
    assert min(diff, diff_b, diff_seed) >= 15


def test_guide_draws_and_their_gaps_match_an_independent_recomputation():
    """guide[j] is row j's own Gumbel-max draw from p_j and guide_gap[j] the winner's score minus
    the runner-up's: recomputed here from the python-integer Philox of tests/test_oracle_rng.py
    (counter {step, b, j, 1 + v/4}, word v%4, u = ((x >> 9) + 0.5) / 2^23), for every row up to
    the first rejection; rows behind it report -1.  The first guide of many seeds follows p_0."""
    from tests.test_oracle_rng import py_philox
    rng = np.random.default_rng(3)
    V, k, T, seed, b = 11, 4, 0.8, 0xC0FFEE1234, 3
    counts = np.zeros(V, int)
    z0 = rng.normal(0, 1.5, size=V)
    for step in range(400):
        z = rng.normal(0, 1.5, size=(k, V))
        z[0] = z0
        w = [int(t) for t in rng.integers(0, V, size=k)]
        n, emit, guide, am, gap, gg = O.accept_sample(z, w, None, T, seed, step, b=b, guide_gaps=True)
        for j in range(k):
            if j > n:
                assert guide[j] == -1 and gg[j] == -1.0
                continue
            sc = np.empty(V)
            for v in range(V):
                x = py_philox([step, b, j, 1 + v // 4], [seed & 0xffffffff, seed >> 32])[v % 4]
                u = ((int(x) >> 9) + 0.5) / 8388608.0
                sc[v] = z[j, v] / T - np.log(-np.log(u))       # log p_v + Gumbel_v up to the row's constant
            order = np.argsort(-sc)
            assert guide[j] == order[0]
            assert abs(gg[j] - (sc[order[0]] - sc[order[1]])) < 1e-9
        counts[guide[0]] += 1
    p0 = np.exp(z0 / T - (z0 / T).max()); p0 /= p0.sum()
    assert stats.chisquare(counts, p0 * counts.sum()).pvalue > 1e-4
