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
