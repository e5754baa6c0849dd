"""GPU self-consistency of the attention's forms at the full 70B width over a long KV cache.

The library takes the shared form of the attention (one token range per workgroup, K/V staged
through LDS) by itself only where a step has more attention workgroups than the chip has CUs and
at least 384 cached tokens per split: 4 sequences x 8 kv heads over 16 384 cached tokens do that
for every window of the long-context workloads (k = 4: 2 query blocks per kv head, 2 waves per
workgroup; k = 16: 8 blocks, two per wave, 4 waves; k = 32: 16 blocks, 8 waves).  The oracle
cannot prefill such a cache in a test's time, so the cache is the library's seeded fill and the
reference is the library itself with that form switched off (tuning attn_shared = 0): the register forms,
which the other parity tests pin to the oracle.  The two differ in the order of their sums only;
over two full-width layers that rounding noise compounds (any two forms, also two register forms
with different splits, end up 0.03-0.04 apart at a logit rms of 1.8), so the bars are the ones
tests/test_gpu_wide.py derives for two-layer composites.  Sequence lengths are ragged and one
ends inside a 32-token step.
"""
import numpy as np
import pytest

from paper_2601_05524_amd import binding as B
from tests import gpu_util
from tests.gpu_util import Gpu
from tests.test_gpu_wide import COMPOSITE_MAX, COMPOSITE_REL, slice_of

pytestmark = pytest.mark.gpu

CTX = [16384, 16001, 9000, 16384]


def run(monkeypatch, mode, k, windows):
    monkeypatch.setattr(gpu_util, "TUNING", dict(attn_shared=mode))
    g = Gpu(slice_of("llama70b"), seed=71, max_batch=4, max_ctx=16384 + 64, max_window=32)
    for b, n in enumerate(CTX):
        B.dbl_kv_fill(g.ctx, b, n, 900 + b)
    assert list(g.kv_len()) == CTX
    out = g.verify(windows)
    g.close()
    return out


@pytest.mark.parametrize("k", [4, 16, 32])
def test_shared_form_agrees_with_register_forms_over_long_cache(monkeypatch, k):
    V = slice_of("llama70b")["vocab"]
    rng = np.random.default_rng(100 + k)
    windows = rng.integers(0, V, (4, k)).astype(np.int32)
    ref = run(monkeypatch, 0, k, windows)
    got = run(monkeypatch, 1, k, windows)
    assert np.isfinite(got).all() and np.isfinite(ref).all()
    d = np.abs(got.astype(np.float64) - ref)
    rel = np.sqrt((d ** 2).mean()) / np.sqrt((ref.astype(np.float64) ** 2).mean())
    print("k=%d: max-abs %.3g, rms difference / rms logits %.3g" % (k, d.max(), rel))
    assert d.max() > 0.0, "both runs took the same form"
    assert rel <= COMPOSITE_REL and d.max() <= COMPOSITE_MAX
