"""Double rounds on one GPU (paper Sec. 4.1 "Iterative Retrieval Drafter" / "Synchronous Parallel
Execution", Sec. 4.2 "Target-Guided Verification", Eq. 6, Alg. 1 / Alg. 2): a draft model and a target
model as two libdbl contexts on two HIP streams.

Nothing of the method is computed here.  Every token of a round stays on the device: the target's window
is assembled by dbl_build_guided_window from the unverified drafts U and the target's own retrieval, the
draft's chain is read off its history by dbl_history_tail, Eq. 6 is dbl_merge, and the draft model is
re-aligned with the verified text by dbl_history_splice.  This module only enqueues those calls on the two
streams, waits once per round, and reads back nine integers (the round's record) to know how far the text
has grown and whether the draft needs a catch-up forward.

One round, with x the text the target has verified and U the drafts behind it:

  target stream   guided window (pending + U + Y_p) -> verify -> accept -> commit            x += E
  draft stream    [catch-up forward] -> gamma Retrieval Forwards from x + U -> chain X_q
                  -> wait for the target's event -> merge -> splice                          U <- U'
  host            synchronise the draft stream, read the record

Random numbers (T > 0): an acceptance draws from Philox with a step word.  The library adds the number of
commits a context has run to the `step` argument; a Lane counts its own commits and passes the difference,
so that the target's acceptance of round r draws with step r and the draft's j-th Retrieval Forward of
round r with step r * gamma + j, whatever prefill and catch-up forwards came before.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_U64 = (1 << 64) - 1


class Lane:
    """One model on its own stream: a libdbl context and the device buffers its calls write."""

    def __init__(self, shape: dict, weight_seed: int, *, max_ctx: int, max_window: int, max_hist: int,
                 stream: torch.cuda.Stream | None = None, device: str = "cuda:0", max_cont: int = 16):
        self.dev = device
        self.stream = stream if stream is not None else torch.cuda.Stream(device=device)
        self.k_max, self.max_cont, self.max_ctx, self.max_hist = max_window, max_cont, max_ctx, max_hist
        cfg = B.make_cfg(**shape, max_batch=1, max_ctx=max_ctx, max_window=max_window, max_hist=max_hist)
        self.ctx = B.dbl_create(cfg, weight_seed, self.stream.cuda_stream)
        with torch.cuda.stream(self.stream):
            i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=device)
            self.cont, self.cl, self.mn, self.mp = i32(1, max_cont), i32(1), i32(1), i32(1)
            self.window, self.win_len = i32(1, max_window), i32(1)
            self.n_acc, self.emit, self.guide = i32(1), i32(1, max_window), i32(1, max_window)
            self.n_draft, self.keep = i32(1), i32(1)
        self.commits = 0          # dbl_kv_commit calls so far on this context
        self.prompt_len = 0

    def close(self):
        if self.ctx is not None:
            B.dbl_destroy(self.ctx)
            self.ctx = None

    def step_arg(self, want: int) -> int:
        """`step` argument that makes the library's step word (argument + commits run) equal `want`."""
        return (want - self.commits) & _U64

    def commit(self, n_keep=None):
        B.dbl_kv_commit(self.ctx, n_keep)
        self.commits += 1

    def load(self, prompt):
        """Start a session: the prompt becomes the history, its tokens but the last go through the model."""
        p = np.ascontiguousarray(prompt, dtype=np.int32)
        assert 1 <= p.size <= self.max_hist and p.size - 1 <= self.max_ctx
        with torch.cuda.stream(self.stream):
            B.dbl_reset(self.ctx, 0)
            B.dbl_history_set(self.ctx, 0, p)
            for i in range(0, p.size - 1, self.k_max):
                n = min(self.k_max, p.size - 1 - i)
                w = torch.as_tensor(p[None, i:i + n], device=self.dev)
                self.keep.fill_(n)
                B.dbl_verify_block(self.ctx, w, 1, n)
                self.commit(self.keep)
        self.prompt_len = int(p.size)

    def retrieval_forward(self, k, n_max, n_min, d, temperature=0.0, seed=0, want_step=0):
        """Enqueue one Retrieval Forward (Eq. 2) of this model on its own text; call inside its stream."""
        sample = temperature > 0.0
        # retrieval and window in one launch (no unverified drafts in front of this model's own text)
        B.dbl_build_guided_window(self.ctx, 1, k, None, None, 0, n_max, n_min, max(1, min(d, 64)), 0, self.window, self.n_draft)
        B.dbl_verify_block(self.ctx, self.window, 1, k, temperature if sample else 0.0, seed, self.step_arg(want_step))
        B.dbl_accept(self.ctx, B.DBL_SAMPLE if sample else B.DBL_GREEDY, None, self.n_acc, self.emit, self.guide)
        self.commit()

    def chain(self, n_forwards, k, n_max=3, n_min=1, d=10):
        """Enqueue n chained greedy Retrieval Forwards (the iterative retrieval drafter, Eq. 5); nothing is read back."""
        with torch.cuda.stream(self.stream):
            for _ in range(n_forwards):
                self.retrieval_forward(k, n_max, n_min, d)

    def tighten(self):
        """Refresh the library's host-side length bounds from the device counters (the stream must be idle)."""
        kv = np.zeros(1, np.int32)
        B.dbl_kv_len(self.ctx, kv)
        return int(kv[0])

    def generated(self):
        """Synchronise and return the tokens behind the prompt."""
        buf = np.zeros(self.max_hist, np.int32)
        n = B.dbl_history_get(self.ctx, 0, buf)
        return [int(t) for t in buf[self.prompt_len:n]]


class DoubleDecoder:
    """Target lane + draft lane + the device buffers of the resolve step."""

    def __init__(self, target: Lane, draft: Lane, *, gamma: int, k_p: int, k_q: int, n_max: int = 3, n_min: int = 1,
                 d: int = 10, temperature: float = 0.0, seed_target: int = 0, seed_draft: int = 0):
        assert 1 <= k_p <= target.k_max and 1 <= k_q <= draft.k_max and gamma >= 1
        assert max(1, k_p - 1) <= draft.k_max, "the draft's catch-up forward carries up to k_p - 1 rows"
        self.t, self.q = target, draft
        self.gamma, self.k_p, self.k_q, self.n_max, self.n_min, self.d = gamma, k_p, k_q, n_max, n_min, d
        self.T, self.seed_t, self.seed_q = float(temperature), seed_target, seed_draft
        self.max_u, self.max_chain = max(1, k_p - 1), gamma * k_q
        dev = target.dev
        i32 = lambda *s: torch.zeros(s, dtype=torch.int32, device=dev)
        with torch.cuda.stream(draft.stream):
            self.U, self.n_u = [i32(1, self.max_u), i32(1, self.max_u)], [i32(1), i32(1)]
            self.chain_buf, self.n_chain, self.mark = i32(1, self.max_chain), i32(1), i32(1)
            self.text, self.n_text, self.splice_pos = i32(1, k_p + self.max_u), i32(1), i32(1)
            self.rec = i32(9)                       # dbl_merge's record (8) + dbl_history_splice's missing (1)
        self.rec_host = torch.zeros(9, dtype=torch.int32, pin_memory=True)
        self.ev_target = torch.cuda.Event()
        self.cur, self.missing, self.rounds, self.emitted = 0, 0, [], 0

    def start(self, prompt):
        self.t.load(prompt)
        self.q.load(prompt)
        with torch.cuda.stream(self.q.stream):
            self.n_u[0].zero_(); self.n_u[1].zero_()
        torch.cuda.synchronize()
        self.cur, self.missing, self.rounds, self.emitted = 0, 0, [], 0

    def round(self):
        t, q, r = self.t, self.q, len(self.rounds)
        sample = self.T > 0.0
        U, n_u, U_next, n_u_next = self.U[self.cur], self.n_u[self.cur], self.U[1 - self.cur], self.n_u[1 - self.cur]
        with torch.cuda.stream(t.stream):
            B.dbl_build_guided_window(t.ctx, 1, self.k_p, U, n_u, self.max_u, self.n_max, self.n_min, self.d, 0,
                                      t.window, t.n_draft)
            B.dbl_verify_block(t.ctx, t.window, 1, self.k_p, self.T if sample else 0.0, self.seed_t, t.step_arg(r))
            B.dbl_accept(t.ctx, B.DBL_SAMPLE if sample else B.DBL_GREEDY, None, t.n_acc, t.emit, t.guide)
            t.commit()
            self.ev_target.record(t.stream)
        with torch.cuda.stream(q.stream):
            if self.missing > 0:                    # bring the draft's cache up to x + U
                m = self.missing
                B.dbl_catchup_window(q.ctx, 1, m, 0, q.window, q.win_len)
                B.dbl_verify_block_ragged(q.ctx, q.window, q.win_len, 1, m)
                q.commit(q.win_len)
            B.dbl_lengths_dev(q.ctx, 1, None, self.mark)
            for j in range(self.gamma):
                q.retrieval_forward(self.k_q, self.n_max, self.n_min, self.d, self.T, self.seed_q, r * self.gamma + j)
            B.dbl_history_tail(q.ctx, 1, self.mark, self.max_chain, self.chain_buf, self.n_chain)
            q.stream.wait_event(self.ev_target)
            B.dbl_merge(q.ctx, 1, self.k_p, n_u, t.n_acc, t.emit, self.chain_buf, self.n_chain, self.max_chain, self.max_u,
                        self.mark, U_next, n_u_next, self.text, self.n_text, self.splice_pos, self.rec[0:8])
            B.dbl_history_splice(q.ctx, 1, self.splice_pos, self.text, self.n_text, self.k_p + self.max_u, self.rec[8:9])
            self.rec_host.copy_(self.rec, non_blocking=True)
        q.stream.synchronize()                      # the round's one wait (the target's work precedes the merge)
        nu, na, ne, nc, kept, agree, valid, _, missing = (int(v) for v in self.rec_host.tolist())
        self.rounds.append({"mode": "post" if nu else "pre", "n_u": nu, "n_acc": na, "emitted": ne, "drafted": nc,
                            "kept": kept})
        self.emitted += ne
        self.missing = missing
        self.cur = 1 - self.cur
        t.tighten(); q.tighten()
        return self.rounds[-1]

    def decode(self, prompt, max_new: int):
        """Run rounds until at least max_new tokens are verified.  Returns (new tokens, per-round records)."""
        self.start(prompt)
        while self.emitted < max_new:
            self.round()
        return self.t.generated(), self.rounds


def autoregressive_steps(lane: Lane, n_new: int):
    """Enqueue n_new plain greedy decoding steps (one token per forward, chained on the device) on a loaded lane."""
    with torch.cuda.stream(lane.stream):
        lane.cl.zero_()
        for _ in range(n_new):
            B.dbl_build_window(lane.ctx, 1, 1, lane.max_cont, lane.cont, lane.cl, 0, lane.window)
            B.dbl_verify_block(lane.ctx, lane.window, 1, 1)
            B.dbl_accept(lane.ctx, B.DBL_GREEDY, None, lane.n_acc, lane.emit, lane.guide)
            lane.commit()


def autoregressive(lane: Lane, prompt, n_new: int):
    """Plain greedy decoding on the same kernels: load the prompt, n_new steps, return the new tokens."""
    lane.load(prompt)
    autoregressive_steps(lane, n_new)
    return lane.generated()
