"""Pins for the oracle's n-gram suffix retrieval (Alg. 3's descending-n search of the
sequence in itself; Eq. 2's "retrieve up to d tokens")."""
import numpy as np

import oracle as O
from paper_2601_05524_amd import synth


def R(h, n_max=3, n_min=1, max_cont=4):
    cont, cl, mn, mp = O.retrieve(h, n_max, n_min, max_cont)
    return list(cont), cl, mn, mp


def test_hand_built_histories():
    # planted span: "7 8 9" occurred before, followed by 1 2 3 4 5
    h = [7, 8, 9, 1, 2, 3, 4, 5, 6, 6, 7, 8, 9]
    assert R(h) == ([1, 2, 3, 4], 4, 3, 0)
    assert R(h, max_cont=2) == ([1, 2], 2, 3, 0)
    # no token of the suffix occurred before: miss
    assert R([1, 2, 3, 4, 5]) == ([], 0, 0, -1)
    # only a shorter suffix matches: n falls from 3 to 1
    assert R([5, 1, 2, 9, 9, 4, 3, 2]) == ([9, 9, 4, 3], 4, 1, 2)
    # with n_min = 3 the same history misses
    assert R([5, 1, 2, 9, 9, 4, 3, 2], n_min=3) == ([], 0, 0, -1)
    # history shorter than n: n is clipped to len - 1
    assert R([4, 4]) == ([4], 1, 1, 0)
    assert R([4]) == ([], 0, 0, -1)
    assert R([]) == ([], 0, 0, -1)
    # periodic text: every period matches; the longest continuation wins, then the latest start
    h = [1, 2] * 6                     # len 12, suffix (2,1,2)
    cont, cl, mn, mp = R(h, max_cont=4)
    assert (cont, cl, mn) == ([1, 2, 1, 2], 4, 3)
    assert mp == 5                     # starts 1,3,5 give 4 tokens; 7 gives 2; latest full one is 5
    # match only at the last legal position (overlapping the suffix), continuation cut by the end
    assert R([9, 3, 3, 3, 3], n_max=3) == ([3], 1, 3, 1)
    # two candidates with equal continuation length: the later start wins
    h = [1, 2, 3, 10, 11, 0, 1, 2, 3, 20, 21, 0, 1, 2, 3]
    assert R(h, max_cont=2) == ([20, 21], 2, 3, 6)
    # the longer continuation beats the later start
    h = [1, 2, 3, 10, 11, 12, 0, 0, 1, 2, 3, 20, 1, 2, 3]
    assert R(h, max_cont=3) == ([20, 1, 2], 3, 3, 8)     # both give 3 tokens: later start
    assert R(h, max_cont=4) == ([20, 1, 2, 3], 4, 3, 8)
    assert R(h, max_cont=5) == ([10, 11, 12, 0, 0], 5, 3, 0)  # start 8 is cut to 4 by the end
    # longest n beats everything: a 3-gram match with a short continuation wins over 1-gram ones
    h = [3, 50, 51, 52, 53, 1, 2, 3, 60, 1, 2, 3]
    assert R(h, max_cont=4)[2:] == (3, 5)


def brute(h, n_max, n_min, max_cont):
    """Independent formulation: enumerate (n, cont_len, start) keys and take the maximum."""
    h = list(h)
    L = len(h)
    keys = []
    for n in range(max(n_min, 1), min(n_max, L - 1) + 1):
        suf = tuple(h[L - n:])
        for s in range(0, L - n):
            if tuple(h[s:s + n]) == suf:
                keys.append((n, min(max_cont, L - s - n), s))
    if not keys:
        return [], 0, 0, -1
    n, c, s = max(keys)
    return h[s + n:s + n + c], c, n, s


def test_matches_brute_force_on_random_small_histories():
    rng = np.random.default_rng(0)
    for it in range(1500):
        L = int(rng.integers(0, 40))
        vocab = int(rng.integers(1, 5))
        h = rng.integers(0, vocab, L)
        n_max = int(rng.integers(1, 6)); n_min = int(rng.integers(1, n_max + 1))
        mc = int(rng.integers(1, 9))
        assert R(h, n_max, n_min, mc) == brute(h, n_max, n_min, mc), (list(h), n_max, n_min, mc)


def test_returned_span_is_real_and_maximal():
    for seed in range(5):
        h = synth.zipf_history(100 + seed, 2048, 5000, repeat_frac=0.2)
        for cut in (2048, 1500, 777):
            hh = h[:cut]
            cont, cl, mn, mp = R(hh, 3, 1, 10)
            if mn == 0:
                continue
            assert list(hh[mp:mp + mn]) == list(hh[cut - mn:])
            assert list(hh[mp + mn:mp + mn + cl]) == cont and 1 <= cl <= 10
            assert mp + mn <= cut - 1
            # no longer n matches anywhere
            for n in range(mn + 1, 4):
                suf = list(hh[cut - n:])
                assert not any(list(hh[s:s + n]) == suf for s in range(cut - n))


def test_synthetic_history_recipe_hits():
    # the tiny workload's history ends inside a copied span, so the first retrieval hits
    h = synth.uniform_history(synth.BASE_SEED, length=256, vocab=2048, span=8, every=32, tail=4)
    cont, cl, mn, mp = R(h, 3, 1, 8)
    assert mn == 3 and cl >= 1
    z = synth.zipf_history(synth.BASE_SEED + 1, 1024, 128256, repeat_frac=0.15)
    assert z.min() >= 0 and z.max() < 128256
    top = np.bincount(z).max()
    assert top > 20          # Zipf head
