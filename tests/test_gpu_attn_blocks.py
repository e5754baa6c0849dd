"""GPU parity of the attention kernel's forms for many query rows: two query blocks per wave (one set
of K/V fragments in registers for 32 query rows, two sets of fragments in flight), and the shared
form (see the fixture below).

The library takes that form by itself only for many query rows over long ranges of cached tokens
(8 or more query blocks per kv head and at least 1024 tokens per split); the tuning attn_blocks = 3
makes it the form wherever a kv head has at least two query blocks, so that small models
reach it: odd numbers of blocks (the last wave's second block is padding), windows of more than 16
rows, batches with different context lengths, ranges that end inside a 32-token step, the paged
cache.  Bars as in the other parity tests."""
import numpy as np
import pytest

from paper_2601_05524_amd import synth
from tests import gpu_util
from tests.gpu_util import Gpu, Ref
from tests.test_gpu_parity import SMALL_BF16, SMALL_QWEN, TOL, jitter_gains

pytestmark = pytest.mark.gpu


# The shared form (the waves of a workgroup walk one token range together, K/V staged through LDS) is
# taken by itself from 2 query blocks per kv head and 384 cached tokens per split on (where the chip has fewer CUs
# than the step has attention workgroups); the tuning attn_shared = 2
# (two blocks per wave) / 3 (one) makes it the form wherever a kv head has two query blocks and the
# cache is not empty, with 2, 4 or 8 waves per workgroup depending on the window.
@pytest.fixture(params=[dict(attn_blocks=3), dict(attn_shared=2), dict(attn_shared=3)],
                ids=["two_blocks_per_wave", "shared_two_blocks", "shared_one_block"])
def forced(monkeypatch, request):
    monkeypatch.setattr(gpu_util, "TUNING", request.param)


def max_err(got, ref):
    assert np.isfinite(got).all()
    return float(np.abs(got.astype(np.float64) - ref).max())


@pytest.mark.parametrize("shape,seed", [(SMALL_BF16, 61), (SMALL_QWEN, 62)], ids=["hd64_g4", "hd128_g8_qknorm"])
def test_two_blocks_per_wave_windows_and_growing_context(forced, shape, seed):
    g, r = Gpu(shape, seed=seed, max_ctx=512, max_window=32), Ref(shape, seed=seed, max_ctx=512)
    jitter_gains(g, r, shape)
    rng = np.random.default_rng(seed)
    toks = rng.integers(0, shape["vocab"], 400).astype(np.int32)
    i = 0
    # g = 4: 5 rows -> 2 blocks, 9 -> 3 (odd), 32 -> 8; g = 8: 3 rows -> 2 blocks, 5 -> 3 (odd), 32 -> 16
    for k in [32, 5, 9, 16, 3, 32, 7, 12, 32, 10, 32, 6, 32, 11]:
        w = toks[i:i + k]
        err = max_err(g.verify([w])[0], r.verify([w])[0])
        assert err <= TOL[1], (i, k, err)
        keep = k if k != 9 else 4
        g.commit([keep])
        r.seqs[0].commit(keep, [])
        i += keep
    assert g.kv_len()[0] == r.seqs[0].kv_len == i
    g.close()


def test_two_blocks_per_wave_batch_with_ragged_contexts(forced):
    shape = SMALL_QWEN
    g, r = Gpu(shape, seed=63, max_batch=3, max_ctx=512, max_window=8), Ref(shape, seed=63, max_batch=3, max_ctx=512)
    rng = np.random.default_rng(63)
    for step in range(12):
        ws = [rng.integers(0, shape["vocab"], 8).astype(np.int32) for _ in range(3)]
        err = max_err(g.verify(ws), r.verify(ws))
        assert err <= TOL[1], (step, err)
        keep = [8, 1 + step % 3, 5]          # contexts 96 / about 24 / 60 after 12 steps
        g.commit(keep)
        for b in range(3):
            r.seqs[b].commit(keep[b], [])
    assert list(g.kv_len()) == [s.kv_len for s in r.seqs]
    g.close()


def test_two_blocks_per_wave_paged_equals_contiguous(forced):
    shape = SMALL_QWEN
    kw = dict(seed=64, max_batch=2, max_ctx=1024, max_window=16, max_hist=2048)
    flat, paged = Gpu(shape, **kw), Gpu(shape, kv_pages=0, **kw)
    prompts = [synth.zipf_history(70 + b, 250, shape["vocab"]) for b in range(2)]
    for g in (flat, paged):
        g.prefill(prompts, 16)
    rng = np.random.default_rng(64)
    for step in range(6):               # crosses the first page boundary (256) in step 0
        w = rng.integers(0, shape["vocab"], (2, 16)).astype(np.int32)
        a, b = flat.verify(w), paged.verify(w)
        assert np.array_equal(a, b), step
        for g in (flat, paged):
            g.commit([16, 3])
    flat.close(); paged.close()
