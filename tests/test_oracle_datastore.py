"""Pins for the oracle's hierarchical datastore (Alg. 3, Sec. 4.3): brute force on tiny inputs,
hand-made priority cases, reduction to the plain search, the rejected tier's update rule."""
import numpy as np
import pytest

import oracle as O


def brute(prior, hist, prompt_len, rej, n_max, n_min, max_cont):
    """Alg. 3 written as directly as possible: for n from long to short, tiers in the order
    prior, dynamic, rejected; inside a tier every occurrence is listed and the best picked."""
    prior, hist, rej = list(prior), list(hist), list(rej)
    L = len(hist)

    def occurrences(buf, lo, hi_end, key):
        n, out = len(key), []
        for s in range(lo, hi_end - n + 1):
            if buf[s:s + n] == key:
                c = 0
                while c < max_cont and s + n + c < len(buf) and buf[s + n + c] >= 0:
                    c += 1
                if c >= 1:
                    out.append((c, s))
        return out

    for n in range(min(n_max, L), max(n_min, 1) - 1, -1):
        key = hist[L - n:]
        for tier, (buf, lo, hi_end) in enumerate(((prior, 0, len(prior)), (hist, prompt_len, L - 1), (rej, 0, len(rej)))):
            occ = occurrences(buf, lo, hi_end, key)
            if occ:
                c, s = max(occ)
                return buf[s + n:s + n + c], n, s, tier
    for n in range(min(n_max, L - 1), max(n_min, 1) - 1, -1):
        occ = occurrences(hist, 0, L - 1, hist[L - n:])
        if occ:
            c, s = max(occ)
            return hist[s + n:s + n + c], n, s, 3
    return [], 0, -1, -1


def test_against_brute_force_on_small_alphabets():
    rng = np.random.default_rng(0)
    tiers_hit = set()
    for case in range(600):
        V = int(rng.integers(2, 6))
        prior = rng.integers(0, V, rng.integers(0, 30))
        if prior.size > 6:
            prior[rng.integers(0, prior.size, 2)] = -1
        L = int(rng.integers(1, 40))
        hist = rng.integers(0, V, L)
        prompt_len = int(rng.integers(0, L + 1))
        rej = rng.integers(0, V, rng.integers(0, 20))
        if rej.size > 4:
            rej[rng.integers(0, rej.size, 2)] = -1
        n_max, n_min, mc = int(rng.integers(1, 6)), 1, int(rng.integers(1, 6))
        cont, cl, mn, mp, mt = O.retrieve_tiered(prior, hist, prompt_len, rej, n_max, n_min, mc)
        b_cont, b_n, b_s, b_t = brute(prior, hist, prompt_len, rej, n_max, n_min, mc)
        assert (list(cont), cl, mn, mp, mt) == (b_cont, len(b_cont), b_n, b_s, b_t), case
        tiers_hit.add(mt)
    assert tiers_hit == {-1, 0, 1, 2, 3}


def test_reduces_to_the_plain_search_without_tiers():
    rng = np.random.default_rng(1)
    for _ in range(200):
        hist = rng.integers(0, 4, rng.integers(2, 50))
        a = O.retrieve_tiered([], hist, hist.size, [], 3, 1, 5)
        cont, cl, mn, mp = O.retrieve(hist, 3, 1, 5)
        assert (list(a[0]), a[1], a[2], a[3]) == (list(cont), cl, mn, mp)
        assert a[4] == (3 if mn > 0 else -1)


def test_priority_order_of_alg3():
    hist = [9, 9, 9, 1, 2, 3, 50, 51, 1, 2, 3]          # prompt = first 3 tokens
    # the same 3-gram in all tiers: the prior wins
    assert O.retrieve_tiered([1, 2, 3, 70], hist, 3, [1, 2, 3, 80], 3, 1, 4)[-1] == 0
    assert list(O.retrieve_tiered([1, 2, 3, 70], hist, 3, [1, 2, 3, 80], 3, 1, 4)[0]) == [70]
    # no prior: generated text before rejected chains
    r = O.retrieve_tiered([], hist, 3, [1, 2, 3, 80], 3, 1, 4)
    assert r[-1] == 1 and list(r[0]) == [50, 51, 1, 2]
    # a longer n-gram in a lower tier beats a shorter one in a higher tier
    r = O.retrieve_tiered([2, 3, 70], hist, 3, [1, 2, 3, 80], 3, 1, 4)
    assert r[-1] == 1 and r[2] == 3
    r = O.retrieve_tiered([2, 3, 70], [9, 9, 9, 1, 2, 3], 3, [1, 2, 3, 80], 3, 1, 4)
    assert r[-1] == 2 and r[2] == 3 and list(r[0]) == [80]
    # the sequence itself is searched only after every length failed in every tier: a 1-gram of
    # generated text beats a 3-gram that only the prompt holds
    h2 = [1, 2, 3, 60, 7, 3, 8, 1, 2, 3]                  # prompt = first 5 tokens
    r = O.retrieve_tiered([], h2, 5, [], 3, 1, 4)
    assert r[-1] == 1 and r[2] == 1 and list(r[0]) == [8, 1, 2, 3]
    assert O.retrieve(h2, 3, 1, 4)[2] == 3                # what the plain search would have taken


def test_segments_do_not_leak():
    # the key must not straddle a separator and a continuation stops in front of one
    r = O.retrieve_tiered([1, 2, -1, 3, 4, 5, -1, 6], [7, 2, 3], 3, [], 3, 1, 5)
    assert r[-1] == 0 and r[2] == 1 and list(r[0]) == [4, 5]      # "3" -> 4 5 | stop
    r = O.retrieve_tiered([1, 2, 3, -1], [7, 2, 3], 3, [], 3, 1, 5)
    assert r[-1] == -1                                            # nothing follows "2 3" in its segment


def test_rejected_update_rule():
    hist = [11, 12, 13, 14, 15]
    w = [15, 20, 21, 22, 23]
    assert list(O.rejected_append([], 64, hist, w, 1, 4)) == [13, 14, 15, 20, 21, 22, 23, -1]
    assert list(O.rejected_append([], 64, hist, w, 0, 2)) == [12, 13, 14, 15, 20, 21, -1]
    assert list(O.rejected_append([], 64, hist, w, 4, 4)) == []            # nothing rejected
    assert list(O.rejected_append([], 64, [15], w, 0, 1, ctx_tokens=4)) == [15, 20, -1]   # short text
    assert list(O.rejected_append([1, -1], 9, hist, w, 1, 4)) == [1, -1]   # does not fit: unchanged
    two = O.rejected_append(O.rejected_append([], 64, hist, w, 1, 4), 64, hist + [20, 30], [30, 40, 41], 0, 2)
    assert list(two) == [13, 14, 15, 20, 21, 22, 23, -1, 14, 15, 20, 30, 40, 41, -1]
    # a rejected chain is found again when its context recurs
    r = O.retrieve_tiered([], [1, 2, 13, 14, 15], 5, two, 3, 1, 4)
    assert r[-1] == 2 and r[3] == 0 and list(r[0]) == [20, 21, 22, 23]
    # equal n and equal continuation length: the later chain
    r = O.retrieve_tiered([], [1, 2, 14, 15, 20], 5, two, 3, 1, 3)
    assert r[-1] == 2 and r[3] == 8 and list(r[0]) == [30, 40, 41]
