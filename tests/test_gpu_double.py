"""The full Double round on the GPU (two libdbl contexts on two streams, host orchestration in
paper_2601_05524_amd/double_round.py) against the reference orchestration on the oracle: same
emitted tokens, same per-round records (mode, verified drafts, accepted length, draft chain
length, drafts kept), and both identical to plain greedy decoding of the target."""
import numpy as np
import pytest
import torch

import oracle as O
from oracle import double_round as REF
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import double_round as DR
from paper_2601_05524_amd import synth
from tests.gpu_util import TENSORS

pytestmark = pytest.mark.gpu

TINY = dict(synth.CONFIGS["tiny"])
T_SEED = synth.BASE_SEED + 5


def prompt():
    return synth.uniform_history(synth.BASE_SEED, length=256, vocab=2048, span=8, every=32, tail=4)


def make_pair(kind):
    """(oracle draft model, GPU draft engine) of one kind, same weights on both sides."""
    kw = dict(max_ctx=640, max_window=8, max_hist=1024)
    if kind == "same":
        return O.Model(**TINY, max_ctx=640, seed=T_SEED), DR.Engine(TINY, T_SEED, **kw)
    if kind == "unrelated":
        return O.Model(**TINY, max_ctx=640, seed=999), DR.Engine(TINY, 999, **kw)
    # the target's weights with the second layer's MLP switched off
    m, e = O.Model(**TINY, max_ctx=640, seed=T_SEED), DR.Engine(TINY, T_SEED, **kw)
    z = np.zeros(TINY["d_model"] * TINY["d_ffn"], np.float32)
    m.tensor(TENSORS["wd"][1], 1)[:] = z
    B.dbl_set_weights(e.ctx, TENSORS["wd"][0], 1, z)
    return m, e


@pytest.mark.parametrize("kind", ["same", "unrelated", "weakened"])
@pytest.mark.parametrize("gamma,k_p,k_q", [(2, 8, 4), (3, 6, 3)])
def test_double_round_matches_the_reference_and_is_lossless(kind, gamma, k_p, k_q):
    torch.cuda.set_device(0)
    p = prompt()
    tm = O.Model(**TINY, max_ctx=640, seed=T_SEED)
    dm, d_eng = make_pair(kind)
    ref_out, ref_rounds = REF.double_decode(O.Seq(tm, max_hist=1024), O.Seq(dm, max_hist=1024), p, 64, gamma, k_p, k_q)
    ar = REF.autoregressive(O.Seq(tm, max_hist=1024), p, len(ref_out))
    assert ref_out == ar

    t_eng = DR.Engine(TINY, T_SEED, max_ctx=640, max_window=8, max_hist=1024)
    out, rounds = DR.double_decode(t_eng, d_eng, p, 64, gamma, k_p, k_q)
    assert out == ref_out
    assert rounds == ref_rounds
    # the same kernels, one token per forward
    assert DR.autoregressive(t_eng, p, len(out)) == out
    assert t_eng.hist == [int(t) for t in p] + out
    kv = np.zeros(1, np.int32)
    B.dbl_kv_len(t_eng.ctx, kv)
    assert kv[0] == len(p) + len(out) - 1
    print(kind, gamma, k_p, k_q, "rounds", len(rounds), "tokens", len(out),
          "post-verify", sum(r["mode"] == "post" for r in rounds))
    t_eng.close(); d_eng.close()
