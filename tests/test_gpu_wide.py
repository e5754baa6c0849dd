"""GPU parity at full layer width: two-layer slices of the 70B-shaped and the 32B-shaped
models.  Every projection, the attention and the LM head run with the tile plans, grids
and workgroup sizes of the full-depth model; only the depth is cut so that the oracle
finishes in about a minute.  Logits are compared element by element over the whole
vocabulary.

Two bars.  A bf16 pipeline rounds at four points per layer; two implementations whose
pre-rounding values differ by a few fp32 ulps round a small fraction of elements to
neighbouring bf16 values, and each later rounding point amplifies that until the
difference sits at the bf16 quantisation-noise level (about 2^-9 relative per stage).
With N(0, 0.02) weights at d_model = 8192 the logits have rms 1.8 and maxima near 9, and
the maximum over a million logits of that noise exceeds 2e-2 after one full layer.
So (1) every kernel is held to the 2e-2 bar on paths where the noise has not yet
compounded: the LM head alone, the attention half of a layer alone, the MLP half alone;
(2) the composite two-layer run is held to COMPOSITE_REL of the logit rms (rms error) and
COMPOSITE_MAX (max-abs).  Those two bars are not chosen: tests/test_noise_floor_full_width.py
measures, on the CPU, what two implementations that both follow the rounding contract
exactly differ by at these shapes (the oracle against an fp32-accumulating PyTorch
decoder: 0.40 % rms, 0.040 max-abs after two 70B-width layers) and asserts that the bars
here stay within 2.1-2.2 x of that floor.
"""
import numpy as np
import pytest

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref

pytestmark = pytest.mark.gpu

TOL_BF16 = 2e-2
COMPOSITE_REL = 7e-3     # rms error / rms logits, two full layers: 2.1 x what two exact-contract CPU implementations differ by
COMPOSITE_MAX = 8e-2     # max-abs over all logits, two full layers: 2.05 x that CPU-measured floor (tests/test_noise_floor_full_width.py)


def slice_of(name):
    s = dict(synth.CONFIGS[name])
    s["n_layers"] = 2
    return s


_REF = {}


def reference(name, seed):
    """The oracle model of a slice is built once (its weights take longest); the tests
    zero some of its tensors and restore them afterwards."""
    key = (name, seed)
    if key not in _REF:
        _REF.clear()                # one wide model at a time: they are several GB each
        r = Ref(slice_of(name), seed=seed, max_batch=4, max_ctx=512)
        saved = {(t, l): r.get_tensor(t, l) for t in ("wo", "wd") for l in (0, 1)}
        _REF[key] = (r, saved)
    return _REF[key]


def run_slice(name, seed, zero, ctx_tokens, k, chunk):
    """zero: set of (tensor, layer) replaced by zeros on both sides.  Returns per-window
    (gpu logits, oracle logits)."""
    shape = slice_of(name)
    r, saved = reference(name, seed)
    g = Gpu(shape, seed=seed, max_ctx=512, max_window=max(k, chunk))
    for (t, l), v in saved.items():
        if (t, l) in zero:
            z = np.zeros_like(v)
            r.set_tensor(t, l, z)
            g.set_tensor(t, l, z)
        else:
            r.set_tensor(t, l, v)
    V = shape["vocab"]
    prompt = synth.zipf_history(seed, ctx_tokens + 1, V)
    g.prefill([prompt], chunk)
    r.prefill([prompt], chunk)
    rng = np.random.default_rng(seed)
    out = []
    for it in range(2):
        first = [prompt[-1]] if it == 0 else rng.integers(0, V, 1)
        w = np.concatenate([first, rng.integers(0, V, k - 1)]).astype(np.int32)
        got = g.verify([w])[0]
        ref = r.verify([w])[0]
        assert np.isfinite(got).all()
        assert np.abs(ref).max() > 0.3          # the comparison is not between two zero tensors
        out.append((got, ref))
        g.commit([3])
        r.seqs[0].commit(3, [])
    assert g.kv_len()[0] == ctx_tokens + 6
    g.close()
    return out


def max_err(got, ref):
    return float(np.abs(got.astype(np.float64) - ref).max())


LAYER1_OFF = {("wo", 1), ("wd", 1)}
PATHS = {
    "lm_head": LAYER1_OFF | {("wo", 0), ("wd", 0)},      # embedding -> final norm -> LM head
    "attention": LAYER1_OFF | {("wd", 0)},               # + norm, q/k/v, RoPE, attention, output projection
    "mlp": LAYER1_OFF | {("wo", 0)},                     # + norm, gate/up + SwiGLU, down projection
}


def one_path(name, k, chunk, path):
    out = run_slice(name, 31, PATHS[path], ctx_tokens=24 if chunk == 8 else 37, k=k, chunk=chunk)
    errs = [max_err(g, r) for g, r in out]
    print("%s %s: logits max-abs errors %s" % (name, path, errs))
    assert max(errs) <= TOL_BF16


# the tests of one model stay together: its oracle weights are generated once
@pytest.mark.parametrize("path", list(PATHS))
def test_llama70b_width_one_path_at_a_time(path):
    one_path("llama70b", 8, 8, path)


def test_llama70b_width_lm_head_sampling_statistics():
    """The fused LM-head statistics over the full vocabulary (8016 tiles, 256 workgroups x 4 waves) in
    sampling mode: accepted lengths and emitted tokens against the oracle's acceptance on the
    oracle's own logits, for windows whose decisions lie outside the measured logit error."""
    from tests.test_gpu_parity import guide_rows, sample_margin_ok
    shape = slice_of("llama70b")
    r, saved = reference("llama70b", 31)
    g = Gpu(shape, seed=31, max_ctx=512, max_window=8)
    for (t, l), v in saved.items():        # embedding -> final norm -> LM head on both sides
        z = np.zeros_like(v)
        r.set_tensor(t, l, z); g.set_tensor(t, l, z)
    V, T, seed = shape["vocab"], 0.25, 0x70B5A3
    prompt = synth.zipf_history(31, 17, V)
    g.prefill([prompt], 8)
    r.prefill([prompt], 8)
    rng = np.random.default_rng(5)
    compared, lengths = 0, []
    for step in range(6):
        s = r.seqs[0]
        pending = int(s.history()[-1]) if step == 0 else int(rng.integers(0, V))
        # drafts: the oracle's own most likely continuation for the first rows, random afterwards
        w = [pending]
        for j in range(7):
            lg = s.verify_block(w)
            w.append(int(lg[-1].argmax()) if j < 2 + step % 4 else int(rng.integers(0, V)))
        w = np.array(w, np.int32)
        ref = s.verify_block(w)
        got = g.verify([w], temperature=T, seed=seed, step=100 + step)[0]
        err = np.abs(got - ref).max()
        assert err <= TOL_BF16
        n, emit, guide = g.accept(B.DBL_SAMPLE)
        n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(ref, w, None, T, seed, 100 + step + g.ncommit, 0, guide_gaps=True)
        if sample_margin_ok(ref, w, None, T, am, gap, n_ref, err):
            assert n[0] == n_ref, step
            assert np.array_equal(emit[0], e_ref), step
            rows = guide_rows(gg, n_ref, T, err)          # the target's own draws up to the rejection
            assert np.array_equal(guide[0][rows], gd_ref[rows]) and (guide[0][n_ref + 1:] == -1).all(), (step, rows)
            compared += 1
        lengths.append(n_ref)
        g.commit([1]); s.commit(1, [])
    print("compared %d of 6 windows, accepted lengths %s" % (compared, lengths))
    assert compared >= 3
    for (t, l), v in saved.items():
        r.set_tensor(t, l, v)
    g.close()


@pytest.mark.parametrize("name,k,T", [("llama70b", 8, 1.0), ("qwen32b", 16, 0.7)])
def test_full_vocabulary_dense_q_acceptance_and_residual_draw(name, k, T):
    """Speculative sampling with dense draft distributions at the full vocabulary (128 256 and 151 936
    entries), the case the 32B-shaped and the long-context workloads name: the acceptance test
    u q(x) < p(x) with q read from the caller's rows, and at the first rejection the draw from
    max(0, p - q), one pass of the acceptance kernel over a full row of logits and a full row of q.
    Layer-less models of the full width (embedding -> final norm -> LM head), so the oracle is cheap.
    The leading drafts are the oracle's most likely tokens (they survive), then comes a draft that q
    favours heavily and p does not (a rejection at a known row), so the residual draw happens at rows
    0 .. 3.  Windows whose decisions lie inside the measured logit error are not compared."""
    from tests.test_gpu_parity import guide_rows, sample_margin_ok
    shape = dict(synth.CONFIGS[name], n_layers=0)
    _REF.clear()
    r = Ref(shape, seed=33, max_batch=1, max_ctx=64)
    g = Gpu(shape, seed=33, max_ctx=64, max_window=k)
    V, seed = shape["vocab"], 0xD15EA5E + k
    rng = np.random.default_rng(k)
    s = r.seqs[0]
    compared, rejected_at = 0, []
    for step in range(6):
        n_good = step % 4                       # drafts that should survive
        w = [int(rng.integers(0, V))]
        for j in range(k - 1):                  # (no layers: a row's logits depend on its own token only)
            w.append(int(s.verify_block([w[-1]])[0].argmax()) if j < n_good else int(rng.integers(0, V)))
        w = np.array(w, np.int32)
        ref = s.verify_block(w)
        q = synth.dense_q(7000 + step, k - 1, V, T, mix_logits=ref[:k - 1] * 1.5)
        x = w[n_good + 1]                       # the first random draft: q puts half of its mass there
        q[n_good] *= np.float32(0.5)
        q[n_good, x] += np.float32(0.5)
        got = g.verify([w], temperature=T, seed=seed, step=300 + step)[0]
        err = np.abs(got - ref).max()
        assert err <= TOL_BF16
        n, emit, guide = g.accept(B.DBL_SAMPLE, q[None])
        n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(ref, w, q, T, seed, 300 + step + g.ncommit, 0, guide_gaps=True)
        rejected_at.append(n_ref)
        if sample_margin_ok(ref, w, q, T, am, gap, n_ref, err):
            assert n[0] == n_ref, step
            assert np.array_equal(emit[0], e_ref), step
            if n_ref < k - 1:                    # a token drawn from the residual has p > q
                assert q[n_ref, e_ref[n_ref]] < np.exp(ref[n_ref, e_ref[n_ref]] / T - np.log(np.exp(ref[n_ref] / T).sum()))
            rows = guide_rows(gg, n_ref, T, err)
            assert np.array_equal(guide[0][rows], gd_ref[rows]) and (guide[0][n_ref + 1:] == -1).all(), (step, rows)
            compared += 1
    print("%s vocabulary %d: compared %d of 6 windows, first rejections at rows %s, max logit error %.3g"
          % (name, V, compared, rejected_at, err))
    assert compared >= 4 and len(set(rejected_at)) >= 3
    g.close()


def composite(name, k, chunk, ctx_tokens):
    out = run_slice(name, 31, set(), ctx_tokens=ctx_tokens, k=k, chunk=chunk)
    for got, ref in out:
        d = got.astype(np.float64) - ref
        rel = np.sqrt((d ** 2).mean()) / np.sqrt((ref ** 2).mean())
        print("%s width, two layers: rms error / rms logits %.3g, max-abs %.3g" % (name, rel, np.abs(d).max()))
        assert rel <= COMPOSITE_REL
        assert np.abs(d).max() <= COMPOSITE_MAX


def test_llama70b_width_two_layers():
    composite("llama70b", 8, 8, 40)


def test_llama70b_width_two_layers_16_row_chunks():
    """Windows of 9..16 rows: one row group of the row-group projection kernel for every projection."""
    composite("llama70b", 12, 16, 35)


@pytest.mark.parametrize("nseq", [1, 2, 4], ids=["32_rows", "64_rows", "128_rows"])
def test_llama70b_width_two_layers_many_row_window(nseq):
    """One / two / four sequences with 32-row windows: 32 / 64 / 128 rows go through the projection
    kernels with two / four / eight row groups per weight fragment at the full 70B width (the
    gate/up projection through the kernel that shares its activations through LDS)."""
    shape = slice_of("llama70b")
    r, saved = reference("llama70b", 31)
    for (t, l), v in saved.items():
        r.set_tensor(t, l, v)
    g = Gpu(shape, seed=31, max_batch=nseq, max_ctx=512, max_window=32)
    V = shape["vocab"]
    prompts = [synth.zipf_history(31 + b, 33, V) for b in range(nseq)]
    g.prefill(prompts, 32)
    r.prefill(prompts, 16)
    rng = np.random.default_rng(9)
    ws = [np.concatenate([[p[-1]], rng.integers(0, V, 31)]).astype(np.int32) for p in prompts]
    got = g.verify(ws)
    refs = r.verify(ws)
    for b in range(nseq):
        ref = refs[b]
        d = got[b].astype(np.float64) - ref
        rel = np.sqrt((d ** 2).mean()) / np.sqrt((ref ** 2).mean())
        print("%d-row window, sequence %d: rms error / rms logits %.3g, max-abs %.3g" % (32 * nseq, b, rel, np.abs(d).max()))
        assert np.isfinite(got[b]).all()
        assert rel <= COMPOSITE_REL
        assert np.abs(d).max() <= COMPOSITE_MAX
    g.close()


@pytest.mark.parametrize("path", list(PATHS))
def test_qwen32b_width_one_path_at_a_time(path):
    one_path("qwen32b", 6, 16, path)


def test_qwen32b_width_two_layers():
    composite("qwen32b", 6, 16, 37)


# ---- the 1B-shaped draft model: its projections take the 8-row streaming kernels ----------
@pytest.mark.parametrize("path", list(PATHS))
def test_llama1b_width_one_path_at_a_time(path):
    one_path("llama1b", 8, 8, path)


def test_llama1b_width_two_layers():
    composite("llama1b", 8, 8, 40)


FULL_DEPTH_REL = 1.7e-2    # rms error / rms logits after 16 layers: 2.1 x the CPU-measured floor of the contract at this shape


def test_llama1b_full_depth_greedy_steps():
    """All 16 layers of the 1B-shaped model: greedy steps (verify, accept, commit), teacher-forced
    from the oracle's decisions.  Logits are held to the compounded-noise bar; the target's top-1
    per row, the accepted length and the emitted tokens must be equal wherever the oracle's top-2
    margins exceed the measured error."""
    shape = dict(synth.CONFIGS["llama1b"])
    _REF.clear()
    r = Ref(shape, seed=47, max_batch=1, max_ctx=512)
    g = Gpu(shape, seed=47, max_ctx=512, max_window=8)
    V, k = shape["vocab"], 8
    prompt = synth.zipf_history(47, 121, V, 1.1, 0.15, 16, 16)
    g.prefill([prompt], 8)
    r.prefill([prompt], 8)
    rng = np.random.default_rng(47)
    compared, rows_decided = 0, 0
    for step in range(6):
        s = r.seqs[0]
        pending = int(s.history()[-1])
        # drafts: the oracle's own greedy continuation for the first rows, random afterwards
        w = [pending]
        for j in range(k - 1):
            lg = s.verify_block(w)
            w.append(int(lg[-1].argmax()) if j < 1 + step % 4 else int(rng.integers(0, V)))
        w = np.array(w, np.int32)
        ref = s.verify_block(w)
        got = g.verify([w])[0]
        d = got.astype(np.float64) - ref
        rel = np.sqrt((d ** 2).mean()) / np.sqrt((ref ** 2).mean())
        err = np.abs(d).max()
        print("step %d: rms error / rms logits %.3g, max-abs %.3g" % (step, rel, err))
        assert np.isfinite(got).all() and rel <= FULL_DEPTH_REL
        n, emit, guide = g.accept(B.DBL_GREEDY)
        n_ref, e_ref, gd_ref, margin = O.accept_greedy(ref, w)
        err_row = np.abs(d).max(axis=1)
        ex = margin < 2 * err_row           # rows whose top-2 gap the row's measured error could flip
        assert np.array_equal(guide[0][~ex], gd_ref[~ex])
        rows_decided += int((~ex).sum())
        for j in np.nonzero(ex)[0]:         # there, any token within the error of the maximum is a valid top-1
            assert ref[j, guide[0, j]] >= ref[j].max() - 2 * err_row[j], (step, j)
        if not ex[:n_ref + 1].any():
            assert n[0] == n_ref and np.array_equal(emit[0], e_ref), step
            compared += 1
        # teacher forcing: both sides continue from the oracle's decision
        g.commit([n_ref + 1])
        s.commit(n_ref + 1, e_ref[:n_ref + 1])
        B.dbl_history_set(g.ctx, 0, s.history())
    print("compared %d of 6 steps, %d of 48 rows decided" % (compared, rows_decided))
    assert compared >= 1 and rows_decided >= 24
    g.close()
