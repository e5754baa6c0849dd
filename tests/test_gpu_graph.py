"""The step's calls only enqueue kernels (and one device-to-device copy) on the context's
stream and keep every counter on the device, so a whole step -- retrieve, window, verify,
accept, commit -- can be captured into a HIP graph once and replayed.  Checked here: replays
interleaved with eager work and synchronisations reproduce the eager run's committed tokens
exactly, under greedy acceptance and under sampling (the Philox step word advances with the
device-side commit counter, so every replay draws fresh numbers)."""
import numpy as np
import pytest
import torch

from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu

pytestmark = pytest.mark.gpu

SMALL_BF16 = dict(n_layers=2, d_model=512, n_q_heads=8, n_kv_heads=2, head_dim=64, d_ffn=1408, vocab=4096,
                  qk_norm=0, dtype=1, rms_eps=1e-5, rope_base=1e4)


def make(stream, shape, seed):
    with torch.cuda.stream(stream):
        g = Gpu(shape, seed=seed, max_ctx=1024, max_window=8, max_hist=2048)
    return g


class Step:
    def __init__(self, g, k, mode, T):
        self.g, self.k, self.mode, self.T = g, k, mode, T
        self.mc = 8
        self.cont, self.cl, self.mn, self.mp = g.i32(1, self.mc), g.i32(1), g.i32(1), g.i32(1)
        self.window, self.n_acc = g.i32(1, k), g.i32(1)
        self.emit, self.guide = g.i32(1, k), g.i32(1, k)

    def __call__(self):
        c = self.g.ctx
        B.dbl_retrieve(c, 1, 3, 1, self.mc, self.cont, self.cl, self.mn, self.mp)
        B.dbl_build_window(c, 1, self.k, self.mc, self.cont, self.cl, 0, self.window)
        B.dbl_verify_block(c, self.window, 1, self.k, self.T, 0xFEED, 7)
        B.dbl_accept(c, self.mode, None, self.n_acc, self.emit, self.guide)
        B.dbl_kv_commit(c, None)


@pytest.mark.parametrize("mode,T", [(B.DBL_GREEDY, 0.0), (B.DBL_SAMPLE, 0.7)], ids=["greedy", "sample"])
def test_captured_step_replays_like_the_eager_step(mode, T):
    torch.cuda.set_device(0)
    stream = torch.cuda.Stream()
    prompt = synth.zipf_history(3, 200, SMALL_BF16["vocab"], 1.1, 0.3, 8, 8)
    n_steps = 12

    # eager reference
    g = make(stream, SMALL_BF16, 21)
    with torch.cuda.stream(stream):
        g.prefill([prompt], 8)
        step = Step(g, 8, mode, T)
        for _ in range(n_steps):
            step()
        stream.synchronize()
        ref = list(g.history())
    g.close()
    assert len(ref) >= len(prompt) + n_steps

    # captured: one step in a graph, replayed n_steps times with eager work in between
    g = make(stream, SMALL_BF16, 21)
    with torch.cuda.stream(stream):
        g.prefill([prompt], 8)
        step = Step(g, 8, mode, T)
        step()                                  # warm-up outside the capture (first-use set-up)
        stream.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        step()
    # the capture enqueued nothing; it only advanced the library's host-side bounds by one step
    got = [list(g.history())]
    scratch = torch.zeros(1 << 20, device="cuda:0")
    for i in range(n_steps - 1):
        graph.replay()
        if i % 3 == 1:                          # the program's own eager work and synchronisations
            scratch.add_(1.0)
            torch.cuda.synchronize()
        if i % 4 == 2:
            got.append(list(g.history()))       # synchronises, reads the counters back
    torch.cuda.synchronize()
    final = list(g.history())
    assert final == ref, "graph replays diverge from the eager run at token %d" % next(
        i for i, (a, b) in enumerate(zip(final + [None], ref + [None])) if a != b)
    for h in got:
        assert h == ref[:len(h)]
    kv = g.kv_len()[0]
    assert kv == len(ref) - 1
    g.close()


def test_drafter_chain_in_one_graph_on_the_1b_shape_against_the_oracle():
    """The iterative retrieval drafter (Eq. 5): gamma chained Retrieval Forwards of the 1B-shaped draft model at its
    full 16 layers, captured into ONE graph with no host decision in between, replayed twice (eager work and a new
    session in between) and compared with the ORACLE, forward by forward: the oracle follows the text the device
    produced, so every forward is judged on the same state -- same retrieved window (bit-exact), logits within the
    full-depth bar, and the same accepted length and emitted tokens wherever the oracle's top-2 margins exceed the
    measured logit error (an undecidable row cannot cascade into later forwards)."""
    import oracle as O
    from tests.gpu_util import Ref
    from tests.test_gpu_wide import FULL_DEPTH_REL
    torch.cuda.set_device(0)
    shape = dict(synth.CONFIGS["llama1b"])
    V, k, gamma, mc = shape["vocab"], 8, 3, 7
    stream = torch.cuda.Stream()
    prompt = synth.zipf_history(47, 57, V, 1.1, 0.3, 8, 8)
    g = make(stream, shape, 47)
    r = Ref(shape, seed=47, max_batch=1, max_ctx=256, max_hist=512)

    bufs = []
    with torch.cuda.stream(stream):
        for j in range(gamma):
            bufs.append(dict(cont=g.i32(1, mc), cl=g.i32(1), mn=g.i32(1), mp=g.i32(1), window=g.i32(1, k), n_acc=g.i32(1),
                             emit=g.i32(1, k), guide=g.i32(1, k),
                             logits=torch.empty((1, k, V), dtype=torch.float32, device="cuda:0")))

    def chain():
        for b in bufs:
            B.dbl_retrieve(g.ctx, 1, 3, 1, mc, b["cont"], b["cl"], b["mn"], b["mp"])
            B.dbl_build_window(g.ctx, 1, k, mc, b["cont"], b["cl"], 0, b["window"])
            B.dbl_verify_block(g.ctx, b["window"], 1, k, 0.0, 0, 0, b["logits"])
            B.dbl_accept(g.ctx, B.DBL_GREEDY, None, b["n_acc"], b["emit"], b["guide"])
            B.dbl_kv_commit(g.ctx, None)

    with torch.cuda.stream(stream):
        g.prefill([prompt], 8)
        chain()                                 # warm-up outside the capture
        stream.synchronize()
        g.prefill([prompt], 8)                  # a fresh session for the capture's bounds
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):
        chain()

    def replay_and_read():
        graph.replay()
        torch.cuda.synchronize()
        return [{n: b[n].cpu().numpy().copy() for n in ("window", "n_acc", "emit", "logits")} for b in bufs], list(g.history())

    first, hist1 = replay_and_read()
    scratch = torch.zeros(1 << 20, device="cuda:0"); scratch.add_(1.0); torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        g.prefill([prompt], 8)                  # new session (resets the counters), eager
        stream.synchronize()
    second, hist2 = replay_and_read()
    assert hist1 == hist2 and len(hist1) >= len(prompt) + gamma
    for a, b in zip(first, second):
        for n in a:
            assert np.array_equal(a[n], b[n]), n

    # the oracle, forward by forward, on the device's text
    r.prefill([prompt], 8)
    s = r.seqs[0]
    decided = 0
    for j, out in enumerate(first):
        cont, cl, _, _ = s.retrieve(3, 1, mc)
        w = np.array([int(s.history()[-1])] + [int(t) for t in cont[:cl]] + [0] * (k - 1 - cl), np.int32)
        assert np.array_equal(out["window"][0], w), j
        ref = s.verify_block(w)
        d = out["logits"][0].astype(np.float64) - ref
        rel = np.sqrt((d ** 2).mean()) / np.sqrt((ref ** 2).mean())
        print("forward %d: rms error / rms logits %.3g, max-abs %.3g, accepted %d" % (j, rel, np.abs(d).max(), out["n_acc"][0]))
        assert rel <= FULL_DEPTH_REL
        n_ref, e_ref, gd_ref, margin = O.accept_greedy(ref, w)
        n = int(out["n_acc"][0])
        if not (margin[:max(n, n_ref) + 1] < 2 * np.abs(d).max(axis=1)[:max(n, n_ref) + 1]).any():
            assert n == n_ref and np.array_equal(out["emit"][0], e_ref), j
            decided += 1
        s.commit(n + 1, out["emit"][0][:n + 1])          # follow the device
    assert list(s.history()) == hist1
    assert decided >= 1
    g.close()
