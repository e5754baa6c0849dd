"""Properties of the hot path at the full benchmark size: the LLaMA-3.3-70B-shaped model
(80 layers, 141 GB of weights resident), a 2048-token KV cache built by real prefill,
window k = 8, batch 1 -- the launch configuration bench.py times.

The oracle cannot run 80 full-width layers, and at this depth bf16 rounding noise decorrelates
any two implementations anyway (the two-layer full-width slices in test_gpu_wide.py are the
element-wise check).  What is checked here holds at any size:
  * the logits are finite and not degenerate;
  * sampled logits, one by one, against the oracle: from the residual stream the GPU's 80th layer left, the
    oracle's own final RMSNorm, rounding and dot product with its own (seeded, bit-identical) LM-head rows give
    the logit of 80 sampled (row, token) pairs per step -- the arg-max of every row among them -- within the
    single-path bar of 2e-2; that is the part of this size the oracle can reach without running 80 layers;
  * the acceptance results agree, bit for bit, with the oracle's greedy acceptance run on the logits the same
    call returned, and with the greedy rule re-evaluated in numpy (the fused LM-head statistics over 256
    workgroups x 4 waves and the acceptance kernel against a plain arg-max over 128 256 logits per row);
  * the device counters move by exactly the accepted length + 1;
  * a second run from a reset context reproduces every logit bit for bit (every sum over
    waves, workgroups and attention splits is taken in a fixed order), and so does a third run
    with the paged KV cache.
"""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu

pytestmark = pytest.mark.gpu

CTX, K, STEPS = 2048, 8, 3


def greedy_rule(logits, window):
    """Paper Sec. 2.1 / App. D.2 at T = 0: draft j+1 survives iff it equals the arg-max of row j
    (lowest id on ties); the emitted tokens are the surviving drafts plus the arg-max of the
    first row that disagrees (or of the last row)."""
    best = logits.argmax(axis=1)          # numpy returns the first (lowest) index of the maximum
    k = len(window)
    n = 0
    while n < k - 1 and window[n + 1] == best[n]:
        n += 1
    return n, list(window[1:n + 1]) + [int(best[n])], best


def oracle_logits_of(g, shape, seed, rows, pairs):
    """The oracle's final RMSNorm (gain 1, as the oracle's model has it) -> rounding r1 -> LM-head dot product for
    the given (row, token) pairs, from the residual stream the last dbl_verify_block left on the GPU."""
    d = shape["d_model"]
    n = g.cfg.max_batch * g.cfg.max_window
    buf = np.empty((n, 16384), np.float32)
    ld = B.dbl_debug_buffer(g.ctx, 0, buf)
    h = buf.ravel()[:n * ld].reshape(n, ld)[:rows, :d].astype(np.float64)
    gf = g.get_tensor("gf")
    assert (gf == 1.0).all()
    xn = [np.array([O.round_bf16(v) for v in O.rmsnorm(h[m], gf, shape["rms_eps"])]) for m in range(rows)]
    out = []
    for m, v in pairs:
        w = O.weight_fill(seed, O.T_LM, 0, int(v) * d, d, shape["dtype"]).astype(np.float64)
        out.append(float(np.dot(w, xn[m])))
    return np.array(out)


def test_llama70b_full_depth_properties():
    free, total = torch.cuda.mem_get_info(0)
    if total < 250e9:
        pytest.skip("not the target device: the 141 GB model needs an MI355X-class memory (288 GB)")
    # on the target device the test runs or fails: it never turns into a silent skip
    assert free >= 170e9, "only %.0f GB of device memory free: something else holds the rest" % (free / 1e9)
    shape = dict(synth.CONFIGS["llama70b"])
    V = shape["vocab"]
    seed = synth.BASE_SEED + 2
    g = Gpu(shape, seed=seed, max_ctx=CTX + 128, max_window=16, max_hist=CTX + 256)
    prompt = synth.zipf_history(seed, CTX + 1, V, 1.1, 0.20, 16, 16)
    rng = np.random.default_rng(5)
    first = [np.concatenate([[prompt[-1]], rng.integers(0, V, K - 1)]).astype(np.int32)]

    # run 1: window i+1 starts with the token step i emitted last
    windows, res = list(first), []
    g.prefill([prompt], 16)
    assert g.kv_len()[0] == CTX
    for i in range(STEPS):
        w = windows[i]
        if i == 1:
            # make the first two drafts right: verify without committing, copy the model's own
            # continuation into the window, twice (row j only sees rows <= j, so row 0's
            # arg-max is unchanged by the drafts behind it)
            for d in (1, 2):
                best = g.verify([w])[0].argmax(axis=1)
                w = w.copy()
                w[d] = best[d - 1]
            windows[i] = w
        logits = g.verify([w])[0]
        n_acc, emit, guide = g.accept(B.DBL_GREEDY)
        before = g.kv_len()[0]
        g.commit()
        after = g.kv_len()[0]
        assert np.isfinite(logits).all()
        assert logits.std() > 0.1
        n_ref, emit_ref, best = greedy_rule(logits, w)
        assert int(n_acc[0]) == n_ref, (i, int(n_acc[0]), n_ref)
        assert emit[0][:n_ref + 1].tolist() == emit_ref, i
        assert after - before == n_ref + 1
        # the oracle's acceptance on the same logits, and its own LM head on sampled (row, token) pairs
        n_orc, e_orc, g_orc, _ = O.accept_greedy(logits.astype(np.float64), w)
        assert int(n_acc[0]) == n_orc and emit[0][:n_orc + 1].tolist() == list(e_orc[:n_orc + 1]), i
        assert guide[0].tolist() == list(g_orc), i
        pairs = [(m, int(best[m])) for m in range(K)] + [(int(rng.integers(0, K)), int(rng.integers(0, V))) for _ in range(72)]
        ref = oracle_logits_of(g, shape, seed, K, pairs)
        got = np.array([logits[m, v] for m, v in pairs], np.float64)
        print("step %d: %d sampled logits against the oracle's LM head: max-abs %.3g" % (i, len(pairs), np.abs(got - ref).max()))
        assert np.abs(got - ref).max() <= 2e-2
        res.append(logits)
        # next window: pending = last emitted token; drafts = what this step's rows predicted
        # after it (a correct guess for the first draft whenever the model repeats itself)
        nxt = np.concatenate([[emit_ref[-1]], best[n_ref:n_ref + 1], rng.integers(0, V, K - 2)]).astype(np.int32)
        windows.append(nxt)
    accepted = [greedy_rule(l, w)[0] for l, w in zip(res, windows)]
    print("accepted lengths:", accepted)
    assert accepted[1] >= 2

    # the first row of a k-row window sees exactly what a one-row window sees (same token, same
    # cache); the two differ only in how the attention splits the context, i.e. in summation order
    w8 = windows[-1]
    row0_k8 = g.verify([w8])[0][0]
    row0_k1 = g.verify([w8[:1]])[0][0]
    d = np.abs(row0_k8.astype(np.float64) - row0_k1)
    print("row 0 of a k=8 window vs a k=1 window: max-abs %.3g, rms %.3g (logit rms %.3g)" % (
        d.max(), np.sqrt((d ** 2).mean()), row0_k8.std()))
    assert np.sqrt((d ** 2).mean()) <= 0.05 * row0_k8.std()

    # run 2 from a reset context: identical bits
    g.prefill([prompt], 16)            # resets the context first
    for i in range(STEPS):
        logits = g.verify([windows[i]])[0]
        g.accept(B.DBL_GREEDY)
        g.commit()
        assert np.array_equal(logits, res[i]), "step %d differs between two runs" % i
    g.close()

    # run 3 with the KV cache as a pool of pages: other addresses, the same arithmetic, identical bits
    g = Gpu(shape, seed=seed, max_ctx=CTX + 256, max_window=16, max_hist=CTX + 256, kv_pages=0)
    g.prefill([prompt], 16)
    for i in range(STEPS):
        logits = g.verify([windows[i]])[0]
        g.accept(B.DBL_GREEDY)
        g.commit()
        assert np.array_equal(logits, res[i]), "step %d differs between the paged and the contiguous cache" % i
    g.close()


@pytest.mark.parametrize("name,Bn,k,ctx,T", [("qwen32b", 1, 16, 8192, 0.7), ("llama70b", 4, 32, 32768, 0.7)],
                         ids=["qwen32b_ctx8192_k16_b1_sample", "llama70b_ctx32768_k32_b4_sample"])
def test_other_benchmark_configurations_at_full_depth(name, Bn, k, ctx, T):
    """The two other full-size configurations bench.py knows (the 32B-shaped model at 8192 tokens with 16-row
    windows, the 70B-shaped one at 4 x 32 768 tokens with 32-row windows), at full depth and vocabulary, sampling:
    the KV cache is the library's seeded fill (as in the benchmark's long-context runs); per step, sampled logits
    recomputed one by one by the oracle's final norm and LM head from the GPU's residual stream, the oracle's
    speculative-sampling acceptance (same Philox draws) run on the logits the call returned against the fused
    statistics' decisions wherever its margins exceed fp32 evaluation noise, finite non-degenerate logits, and the
    same bits when the step is run again."""
    from tests.test_gpu_parity import guide_rows, sample_margin_ok
    free, total = torch.cuda.mem_get_info(0)
    if total < 250e9:
        pytest.skip("not the target device")
    assert free >= 170e9, "only %.0f GB of device memory free" % (free / 1e9)
    shape = dict(synth.CONFIGS[name])
    V, seed, sseed = shape["vocab"], synth.BASE_SEED + 9, 0xFACADE
    g = Gpu(shape, seed=seed, max_batch=Bn, max_ctx=ctx + 64, max_window=k, max_hist=256)
    rng = np.random.default_rng(k)
    lens = [ctx - 37 * b for b in range(Bn)]
    for b in range(Bn):
        B.dbl_kv_fill(g.ctx, b, lens[b], 300 + b)
        B.dbl_history_set(g.ctx, b, rng.integers(0, V, 64).astype(np.int32))
    assert list(g.kv_len()[:Bn]) == lens
    compared = 0
    for step in range(2):
        ws = rng.integers(0, V, (Bn, k)).astype(np.int32)
        if step == 1:      # make a few drafts the model's own most likely tokens, so that some are accepted
            best = g.verify(ws, temperature=T, seed=sseed, step=step)[:, :, :].argmax(axis=2)
            for b in range(Bn):
                ws[b, 1] = best[b, 0]
            best = g.verify(ws, temperature=T, seed=sseed, step=step).argmax(axis=2)
            for b in range(Bn):
                ws[b, 2] = best[b, 1]
        logits = g.verify(ws, temperature=T, seed=sseed, step=step)
        assert np.isfinite(logits).all() and logits.std() > 0.1
        n, emit, guide = g.accept(B.DBL_SAMPLE)
        rows = min(Bn * k, 16)
        pairs = [(m, int(logits.reshape(Bn * k, V)[m].argmax())) for m in range(rows)] + \
                [(int(rng.integers(0, rows)), int(rng.integers(0, V))) for _ in range(48)]
        ref = oracle_logits_of(g, shape, seed, rows, pairs)
        got = np.array([logits.reshape(Bn * k, V)[m, v] for m, v in pairs], np.float64)
        print("%s step %d: %d sampled logits against the oracle's LM head: max-abs %.3g" % (name, step, len(pairs), np.abs(got - ref).max()))
        assert np.abs(got - ref).max() <= 2e-2
        for b in range(Bn):
            lg = logits[b].astype(np.float64)
            n_ref, e_ref, gd_ref, am, gap, gg = O.accept_sample(lg, ws[b], None, T, sseed, step + g.ncommit, b, guide_gaps=True)
            if sample_margin_ok(lg, ws[b], None, T, am, gap, n_ref, 2e-4):
                assert n[b] == n_ref and np.array_equal(emit[b][:n_ref + 1], e_ref[:n_ref + 1]), (step, b)
                rws = guide_rows(gg, n_ref, T, 2e-4)
                assert np.array_equal(guide[b][rws], gd_ref[rws]) and (guide[b][n_ref + 1:] == -1).all(), (step, b)
                compared += 1
        again = g.verify(ws, temperature=T, seed=sseed, step=step)
        assert np.array_equal(again, logits), "step %d differs between two runs" % step
    print("%s: acceptance compared on %d of %d windows" % (name, compared, 2 * Bn))
    assert compared >= Bn
    g.close()
