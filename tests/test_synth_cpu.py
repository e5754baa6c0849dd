"""The seeded input generators both sides share (paper_2601_05524_amd/synth.py): that they produce the workload
structure the design states -- Zipf(1.1) token streams with a given share of positions inside spans copied from
earlier text, uniform histories whose last tokens start a copied span (so the first retrieval hits and its
continuation is known), drafts that go wrong at a geometric position, draft distributions that are distributions --
and the same arrays for the same seed.  They hold none of the method's arithmetic; the oracle's brute-force
retrieval is used below only to show that the copied spans are what an n-gram search finds."""
import numpy as np

import oracle as O
from paper_2601_05524_amd import synth


def test_same_seed_same_arrays():
    assert np.array_equal(synth.zipf_history(7, 4096, 128256, 1.1, 0.2, 16, 16), synth.zipf_history(7, 4096, 128256, 1.1, 0.2, 16, 16))
    assert np.array_equal(synth.uniform_history(7, 256, 2048), synth.uniform_history(7, 256, 2048))
    assert not np.array_equal(synth.zipf_history(7, 4096, 128256), synth.zipf_history(8, 4096, 128256))
    assert np.array_equal(synth.dense_q(3, 2, 1000, 0.7), synth.dense_q(3, 2, 1000, 0.7))


def test_splitmix64_known_values():
    # the published reference outputs of splitmix64 seeded with 1234567 (first three)
    got = synth.splitmix64(1234567, 3)
    assert [int(v) for v in got] == [6457827717110365317, 3203168211198807973, 9817491932198370423]


def copied_share(h, span_lo):
    """Share of positions that lie in a window of span_lo tokens occurring earlier in the history as well."""
    n = len(h)
    seen, inside = {}, np.zeros(n, bool)
    for i in range(n - span_lo + 1):
        key = h[i:i + span_lo].tobytes()
        if key in seen:
            inside[i:i + span_lo] = True
        else:
            seen[key] = i
    return inside.mean()


def test_zipf_history_has_the_stated_repeated_share_and_skew():
    for frac, lo, hi, length in ((0.15, 16, 16, 1024), (0.20, 16, 16, 2049), (0.30, 8, 64, 32768)):
        h = synth.zipf_history(11, length, 128256, 1.1, frac, lo, hi)
        assert h.dtype == np.int32 and h.min() >= 0 and h.max() < 128256 and len(h) == length
        share = copied_share(h, lo)
        # copied spans cover the target share (a little more where random text repeats a window by itself, a little
        # less where one span's source was later overwritten by another copy)
        assert frac - 0.04 <= share <= frac + 0.06, (frac, share)
    # skew: under Zipf(1.1) over 128 256 ids the most frequent id takes about 1 / H(V, 1.1) = 13.8 % of the draws and the
    # ten most frequent about 34 %
    h = synth.zipf_history(5, 200000, 128256, 1.1, 0.0)
    counts = np.sort(np.bincount(h, minlength=128256))[::-1]
    w = np.arange(1, 128257, dtype=np.float64) ** -1.1
    assert abs(counts[0] / len(h) - w[0] / w.sum()) < 0.01
    assert abs(counts[:10].sum() / len(h) - w[:10].sum() / w.sum()) < 0.01


def test_uniform_history_ends_inside_a_copied_span_that_retrieval_finds():
    for seed in range(5):
        h = synth.uniform_history(100 + seed, length=256, vocab=2048, span=8, every=32, tail=4)
        assert len(h) == 256 and h.max() < 2048
        # the last `tail` tokens were copied from the first half: a 3-gram suffix search hits there and proposes what follows
        cont, cont_len, match_n, match_pos = O.retrieve(h, 3, 1, 8)
        assert match_n == 3 and cont_len >= 1
        assert np.array_equal(h[match_pos:match_pos + 3], h[-3:])                       # (match_pos = where the n-gram starts)
        assert np.array_equal(cont, h[match_pos + 3:match_pos + 3 + cont_len])


def test_corrupt_drafts_changes_one_position_geometrically():
    cont = np.arange(100, 108, dtype=np.int32)
    first_wrong = []
    for seed in range(4000):
        d = synth.corrupt_drafts(seed, cont, 2048, alpha=0.8)
        wrong = np.nonzero(d != cont)[0]
        assert len(wrong) <= 1 and d.min() >= 0 and d.max() < 2048
        first_wrong.append(int(wrong[0]) if len(wrong) else 8)
    first_wrong = np.array(first_wrong)
    # P(first wrong position = j) = 0.2 * 0.8^j; P(no position wrong among 8) = 0.8^8
    for j in range(4):
        assert abs((first_wrong == j).mean() - 0.2 * 0.8 ** j) < 0.02
    assert abs((first_wrong == 8).mean() - 0.8 ** 8) < 0.02


def test_dense_q_rows_are_distributions_that_overlap_the_given_logits():
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((3, 5000)) * 3.0
    q = synth.dense_q(9, 3, 5000, 0.7, mix_logits=lg)
    assert q.dtype == np.float32 and q.shape == (3, 5000) and (q >= 0).all()
    assert np.allclose(q.sum(axis=1), 1.0, atol=1e-5)
    # mixing in the logits moves mass toward their arg-max
    q0 = synth.dense_q(9, 3, 5000, 0.7)
    for r in range(3):
        assert q[r, lg[r].argmax()] > q0[r, lg[r].argmax()]
