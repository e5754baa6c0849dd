"""dbl_retrieve_tiered_static -- the tiered retrieval whose scratch is a fixed device array of the
library instead of allocated memory -- against dbl_retrieve_tiered (and the oracle), bit for bit,
on two calls in a row, the second with a smaller input: fewer sequences, shorter histories, a
shorter prior.  The static array keeps the first call's contents in between; stale keys of the
larger call must not leak into the smaller one."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu

pytestmark = pytest.mark.gpu

SHAPE0 = dict(synth.CONFIGS["tiny"], n_layers=0)


def call(g, fn, Bn, n_max, n_min, mc):
    cont = g.i32(Bn, mc, fill=-7)
    cl, mn, mp, mt = (g.i32(Bn, fill=-7) for _ in range(4))
    fn(g.ctx, Bn, n_max, n_min, mc, cont, cl, mn, mp, mt)
    torch.cuda.synchronize()
    return [t.cpu().numpy() for t in (cont, cl, mn, mp, mt)]


def load(g, rng, Bn, V, prior_len, hist_lo, hist_hi):
    prior = rng.integers(0, V, prior_len).astype(np.int32)
    if prior.size > 8:
        prior[rng.integers(0, prior.size, max(2, prior.size // 50))] = -1
    B.dbl_prior_set(g.ctx, prior)
    hists, plens = [], []
    for b in range(Bn):
        L = int(rng.integers(hist_lo, hist_hi))
        h = rng.integers(0, V, L).astype(np.int32)
        for _ in range(max(1, L // 200)):                       # repeated spans
            n = int(rng.integers(4, 17)); s = int(rng.integers(0, L - n)); d = int(rng.integers(0, L - n))
            h[d:d + n] = h[s:s + n]
        pl = int(rng.integers(0, L + 1))
        B.dbl_history_set(g.ctx, b, h)
        B.dbl_session_mark(g.ctx, b, pl)
        hists.append(h); plens.append(pl)
    return prior, hists, plens


def check(g, prior, hists, plens, Bn, n_max, n_min, mc):
    ref = call(g, B.dbl_retrieve_tiered, Bn, n_max, n_min, mc)
    got = call(g, B.dbl_retrieve_tiered_static, Bn, n_max, n_min, mc)
    for a, b in zip(got, ref):
        assert np.array_equal(a, b)
    cont, cl, mn, mp, mt = got
    tiers = set()
    for b in range(Bn):
        r = O.retrieve_tiered(prior, hists[b], plens[b], [], n_max, n_min, mc)
        assert (cl[b], mn[b], mp[b], mt[b]) == (r[1], r[2], r[3], r[4]), b
        assert list(cont[b][:r[1]]) == list(r[0]) and (cont[b][r[1]:] == -1).all()
        tiers.add(int(mt[b]))
    return tiers


def test_static_scratch_retrieval_matches_on_two_calls_the_second_smaller():
    g = Gpu(SHAPE0, seed=1, max_batch=8, max_ctx=64, max_window=4, max_hist=40000)
    rng = np.random.default_rng(12)
    # call 1: 8 sequences, long histories, a prior of three scan chunks
    prior, hists, plens = load(g, rng, 8, 300, 40000, 20000, 32768)
    t1 = check(g, prior, hists, plens, 8, 4, 1, 10)
    # call 2, directly after: 3 sequences, short histories over a small alphabet, a short prior
    B.dbl_reset(g.ctx, -1)
    prior, hists, plens = load(g, rng, 3, 5, 40, 2, 60)
    t2 = check(g, prior, hists, plens, 3, 3, 1, 5)
    # and once more with no prior and no generated text (everything is prompt): the plain fallback search, one sequence
    B.dbl_prior_set(g.ctx, np.zeros(0, np.int32))
    B.dbl_session_mark(g.ctx, 0, len(hists[0]))
    t3 = check(g, np.zeros(0, np.int32), hists[:1], [len(hists[0])], 1, 3, 1, 8)
    print("tiers hit:", sorted(t1), sorted(t2), sorted(t3))
    assert len(t1 | t2 | t3) >= 3
    g.close()


def test_static_scratch_rejects_what_it_cannot_hold():
    g = Gpu(SHAPE0, seed=1, max_batch=2, max_ctx=64, max_window=4, max_hist=64)
    out = [g.i32(2, 4), g.i32(2), g.i32(2), g.i32(2), g.i32(2)]
    with pytest.raises(B.DblError) as e:
        B.dbl_retrieve_tiered_static(g.ctx, 3, 3, 1, 4, *out)      # more sequences than the context has
    assert e.value.code == B.DBL_EINVAL
    with pytest.raises(B.DblError) as e:
        B.dbl_retrieve_tiered_static(g.ctx, 2, 3, 1, 65, *out)
    assert e.value.code == B.DBL_EINVAL
    g.close()
