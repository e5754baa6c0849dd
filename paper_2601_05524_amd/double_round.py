"""A full Double round on one GPU: draft model and target model as two libdbl contexts on two
HIP streams, orchestrated from the host (paper Sec. 4.1 "Iterative Retrieval Drafter" and
"Synchronous Parallel Execution", Sec. 4.2 "Target-Guided Verification" with Eq. 6, Alg. 1 / 2).
Greedy decoding.

Every forward, acceptance, retrieval and commit runs in the library's kernels; the host only
moves a handful of token ids per round and takes the mode decision, as the paper's own
implementation does (App. D.3).  Per round:

  (a) target stream: one Retrieval Forward over  pending token + U + Y_p  (U = draft tokens
      not verified yet, Y_p = target-side retrieval continuing x + U), greedy acceptance, commit;
  (b) draft stream, at the same time and from x + U: gamma chained Retrieval Forwards
      (retrieve -> window -> forward -> accept -> commit, chained on the device);
  (c) host: x <- x + E (the target's accepted tokens + its own next token).  If all of U held,
      the draft's new chain is checked against the part of E that lies beyond U; when it agrees
      with all of it and goes further, the remainder becomes the new U, otherwise the target's
      tokens win (Eq. 6) and the draft context is rolled back and caught up.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


def common_prefix(a, b) -> int:
    n = 0
    while n < len(a) and n < len(b) and int(a[n]) == int(b[n]):
        n += 1
    return n


class Engine:
    """One model: a libdbl context on its own stream, the device buffers its calls need, and
    a host mirror of what the context holds (history tokens, number of valid KV rows)."""

    def __init__(self, shape: dict, weight_seed: int, *, max_ctx: int, max_window: int, max_hist: int,
                 stream: torch.cuda.Stream | None = None, device: str = "cuda:0", max_cont: int = 16):
        self.dev = device
        self.stream = stream if stream is not None else torch.cuda.Stream(device=device)
        self.k_max, self.max_cont = max_window, max_cont
        cfg = B.make_cfg(**shape, max_batch=1, max_ctx=max_ctx, max_window=max_window, max_hist=max_hist)
        self.max_ctx, self.max_hist = max_ctx, max_hist
        self.ctx = B.dbl_create(cfg, weight_seed, self.stream.cuda_stream)
        with torch.cuda.stream(self.stream):
            i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=device)
            self.cont, self.cl, self.mn, self.mp = i32(1, max_cont), i32(1), i32(1), i32(1)
            self.window = i32(1, max_window)
            self.n_acc, self.emit, self.guide = i32(1), i32(1, max_window), i32(1, max_window)
            self.keep = i32(1)
        self.hist: list[int] = []
        self.kv = 0
        self._k_last = 0

    def close(self):
        if self.ctx is not None:
            B.dbl_destroy(self.ctx)
            self.ctx = None

    # ---- state ------------------------------------------------------------
    def sync_to(self, tokens):
        """Hold `tokens` as history with the KV of all but the last one: keep the valid prefix
        of the cache, roll the rest back, run the model over what is missing."""
        tokens = [int(t) for t in tokens]
        assert 1 <= len(tokens) <= self.max_hist and len(tokens) - 1 <= self.max_ctx
        keep = min(common_prefix(self.hist, tokens), self.kv, len(tokens) - 1)
        with torch.cuda.stream(self.stream):
            B.dbl_truncate(self.ctx, 0, kv_len=keep)
            B.dbl_history_set(self.ctx, 0, np.ascontiguousarray(tokens, dtype=np.int32))
            pos = keep
            while pos < len(tokens) - 1:
                n = min(self.k_max, len(tokens) - 1 - pos)
                w = torch.as_tensor(np.asarray([tokens[pos:pos + n]], dtype=np.int32), device=self.dev)
                self.keep.fill_(n)
                B.dbl_verify_block(self.ctx, w, 1, n)
                B.dbl_kv_commit(self.ctx, self.keep)
                pos += n
        self.hist, self.kv = tokens, len(tokens) - 1

    # ---- draft side -------------------------------------------------------
    def retrieval_forwards(self, gamma: int, k: int, n_max: int, n_min: int, d: int):
        """Enqueue gamma chained Retrieval Forwards (Eq. 5); nothing is read back."""
        assert 1 <= k <= self.k_max
        assert len(self.hist) + gamma * k <= self.max_hist and self.kv + gamma * k <= self.max_ctx
        mc = max(1, min(d, k - 1, self.max_cont))
        with torch.cuda.stream(self.stream):
            for _ in range(gamma):
                B.dbl_retrieve(self.ctx, 1, n_max, n_min, mc, self.cont, self.cl, self.mn, self.mp)
                B.dbl_build_window(self.ctx, 1, k, mc, self.cont, self.cl, 0, self.window)
                B.dbl_verify_block(self.ctx, self.window, 1, k)
                B.dbl_accept(self.ctx, B.DBL_GREEDY, None, self.n_acc, self.emit, self.guide)
                B.dbl_kv_commit(self.ctx, None)

    def collect_history(self):
        """Wait for the stream; return the tokens appended since the mirror was last updated."""
        buf = np.zeros(self.max_hist, np.int32)
        n = B.dbl_history_get(self.ctx, 0, buf)
        new = [int(t) for t in buf[len(self.hist):n]]
        self.hist = [int(t) for t in buf[:n]]
        self.kv = n - 1
        return new

    # ---- target side ------------------------------------------------------
    def guided_verify(self, x, U, k: int, n_max: int, n_min: int, d: int):
        """Enqueue the target's Retrieval Forward over pending + U + retrieved guidance (padded
        to k rows), acceptance and commit.  The context must hold x.  Returns the window."""
        assert self.hist == x and len(U) <= k - 1 <= self.k_max - 1
        room = k - 1 - len(U)
        Y = []
        with torch.cuda.stream(self.stream):
            if room > 0:
                mc = max(1, min(d, room, self.max_cont))
                if U:   # the retrieval key is the end of x + U
                    B.dbl_history_set(self.ctx, 0, np.ascontiguousarray(x + U, dtype=np.int32))
                B.dbl_retrieve(self.ctx, 1, n_max, n_min, mc, self.cont, self.cl, self.mn, self.mp)
                cl = int(self.cl.cpu()[0])
                Y = [int(t) for t in self.cont.cpu()[0, :min(cl, room)]]
                if U:
                    B.dbl_truncate(self.ctx, 0, hist_len=len(x))
            W = [x[-1]] + list(U) + Y
            W = W + [0] * (k - len(W))
            self.window[0, :k] = torch.as_tensor(np.asarray(W, dtype=np.int32), device=self.dev)
            B.dbl_verify_block(self.ctx, self.window, 1, k)
            B.dbl_accept(self.ctx, B.DBL_GREEDY, None, self.n_acc, self.emit, self.guide)
            B.dbl_kv_commit(self.ctx, None)
        self._k_last = k
        return W

    def collect_accept(self):
        """Wait for the stream; return (n_acc, emitted tokens) of the last guided_verify."""
        self.stream.synchronize()
        n = int(self.n_acc.cpu()[0])
        E = [int(t) for t in self.emit.cpu()[0, :n + 1]]
        self.hist = self.hist + E
        self.kv += n + 1
        return n, E


def double_decode(target: Engine, draft: Engine, prompt, max_new: int, gamma: int, k_p: int, k_q: int,
                  n_max: int = 3, n_min: int = 1, d: int = 10):
    """Greedy decoding of the target model with the draft model running ahead on its own stream.
    Returns (new tokens, per-round records)."""
    x, U, rounds = [int(t) for t in prompt], [], []
    target.sync_to(x)
    draft.sync_to(x)
    while len(x) - len(prompt) < max_new:
        target.guided_verify(x, U, k_p, n_max, n_min, d)          # (a), asynchronous
        draft.retrieval_forwards(gamma, k_q, n_max, n_min, d)     # (b), asynchronous, other stream
        n, E = target.collect_accept()
        Xq = draft.collect_history()
        U_new = []
        if n >= len(U):
            G = E[len(U):]
            if common_prefix(Xq, G) == len(G) and len(Xq) > len(G):
                U_new = Xq[len(G):][:k_p - 1]
        rounds.append({"mode": "post" if U else "pre", "n_u": len(U), "n_acc": n, "emitted": len(E),
                       "drafted": len(Xq), "kept": len(U_new)})
        x = x + E
        U = U_new
        draft.sync_to(x + U)
    return x[len(prompt):], rounds


def autoregressive(engine: Engine, prompt, n_new: int):
    """Plain greedy decoding on the same kernels, one token per forward, chained on the device."""
    engine.sync_to([int(t) for t in prompt])
    with torch.cuda.stream(engine.stream):
        engine.cl.zero_()
        for _ in range(n_new):
            B.dbl_build_window(engine.ctx, 1, 1, engine.max_cont, engine.cont, engine.cl, 0, engine.window)
            B.dbl_verify_block(engine.ctx, engine.window, 1, 1)
            B.dbl_accept(engine.ctx, B.DBL_GREEDY, None, engine.n_acc, engine.emit, engine.guide)
            B.dbl_kv_commit(engine.ctx, None)
    return engine.collect_history()
