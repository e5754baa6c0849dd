"""Where the full-width parity bars of tests/test_gpu_wide.py come from: measured on the CPU.

The bf16 contract rounds at four points per layer.  Two implementations that follow it exactly --
same weights, same rounding points, same grid -- still differ wherever a value lies within their
arithmetic difference of a rounding boundary: it then lands on the neighbouring bf16 value, an error
of 2^-9 relative in that activation, which the next layers carry on.  How large that gets in the
logits is a property of the contract and of the model's width and weight scale, not of a kernel.  It
is measured here between the oracle (fp64 accumulation, row at a time) and the independent PyTorch
decoder of tests/torch_decoder.py run the way a device computes (fp32 values in front of every
rounding point, the library's blocked fp32 sums), on the shapes the GPU tests use:

  two layers at the 70B width (d_model 8192, FFN 28 672, full vocabulary 128 256), 8 rows;
  all 16 layers of the 1B shape, 8 rows.

Measured (seeded, deterministic): two 70B-width layers rms 0.33-0.40 % of the logit rms, max-abs
0.039-0.040 over 8 x 128 256 logits (one layer: 0.09-0.19 %, 0.020-0.021; two layers at the 32B width:
0.40 %, 0.028); 1B shape at full depth 0.80-0.84 %, 0.040.
So the 2e-2 bar, which every kernel meets where the noise has not compounded, cannot hold for any
exact-contract implementation after two full-width layers, and the bars of the composite GPU tests
are set as multiples of this floor: they must stay within 2.1 x (max-abs) and 2.2 x (rms) of what
two CPU implementations differ by.
"""
import numpy as np
import torch

import oracle as O
from paper_2601_05524_amd import synth
from tests import torch_decoder as TD
from tests.test_gpu_wide import COMPOSITE_MAX, COMPOSITE_REL, FULL_DEPTH_REL, TOL_BF16


def floor_of(name, n_layers, seed):
    shape = dict(synth.CONFIGS[name])
    shape["n_layers"] = n_layers
    m = O.Model(**shape, max_ctx=64, seed=seed)
    s = O.Seq(m, max_hist=64)
    w = np.random.default_rng(seed).integers(0, shape["vocab"], 8).astype(np.int32)
    ref = s.verify_block(w)
    got = TD.forward_full(m, w, acc="f32")
    s.close()
    d = got.astype(np.float64) - ref
    rms = np.sqrt((ref ** 2).mean())
    out = float(np.sqrt((d ** 2).mean()) / rms), float(np.abs(d).max()), float(rms)
    del ref, got, d
    m.close()
    return out


def test_two_exact_contract_implementations_at_70b_width_two_layers():
    torch.set_num_threads(8)
    rel, mx, rms = floor_of("llama70b", 2, 31)
    print("70B width, two layers: logit rms %.3f; fp32 against fp64 implementation: rms %.3g of it, max-abs %.3g" % (rms, rel, mx))
    assert 1.5 < rms < 2.1
    assert mx > TOL_BF16, "the noise floor of the contract itself lies above the single-kernel bar"
    assert 2e-3 < rel < 5e-3 and mx < 6e-2           # the figures quoted above
    assert COMPOSITE_MAX <= 2.1 * mx, "composite max-abs bar is more than 2.1 x the CPU-measured floor"
    assert COMPOSITE_REL <= 2.2 * rel, "composite rms bar is more than 2.2 x the CPU-measured floor"


def test_two_exact_contract_implementations_at_1b_full_depth():
    torch.set_num_threads(8)
    rel, mx, rms = floor_of("llama1b", 16, 47)
    print("1B shape, 16 layers: logit rms %.3f; fp32 against fp64 implementation: rms %.3g of it, max-abs %.3g" % (rms, rel, mx))
    assert 5e-3 < rel < 1.2e-2
    assert FULL_DEPTH_REL <= 2.2 * rel, "full-depth rms bar is more than 2.2 x the CPU-measured floor"
