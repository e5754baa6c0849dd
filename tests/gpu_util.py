"""Helpers for the GPU parity tests: one object driving libdbl through the C ABI, one
driving the oracle, fed with the same seeded inputs."""
import numpy as np
import torch

import oracle as O
from paper_2601_05524_amd import binding as B

DEV = "cuda:0"

# dbl_tuning fields every Gpu context of a test gets (tests that force a kernel form set this through monkeypatch)
TUNING = {}


def f32_to_bf16_bits(a):
    """Exact for arrays that already hold bf16 values."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    assert not np.any(u & 0xFFFF), "not a bf16 value"
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(a):
    return (np.ascontiguousarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


TENSORS = {"emb": (B.T_EMB, O.T_EMB), "lm": (B.T_LM, O.T_LM), "gf": (B.T_GF, O.T_GF),
           "g1": (B.T_G1, O.T_G1), "wq": (B.T_WQ, O.T_WQ), "wk": (B.T_WK, O.T_WK), "wv": (B.T_WV, O.T_WV),
           "gq": (B.T_GQ, O.T_GQ), "gk": (B.T_GK, O.T_GK), "wo": (B.T_WO, O.T_WO), "g2": (B.T_G2, O.T_G2),
           "wg": (B.T_WG, O.T_WG), "wu": (B.T_WU, O.T_WU), "wd": (B.T_WD, O.T_WD)}
GAINS = ("gf", "g1", "g2", "gq", "gk")


class Gpu:
    """libdbl context + the device buffers a caller needs."""

    def __init__(self, shape, *, seed, max_batch=1, max_ctx=512, max_window=8, max_hist=1024, kv_pages=None):
        """kv_pages: None = one contiguous cache region per sequence; n >= 0 = paged cache with a
        pool of n pages (0: the default pool size)."""
        self.shape = dict(shape)
        flags = 0 if kv_pages is None else (B.DBL_FLAG_PAGED_KV | (kv_pages << 8))
        self.cfg = B.make_cfg(**shape, max_batch=max_batch, max_ctx=max_ctx, max_window=max_window,
                              max_hist=max_hist, flags=flags)
        torch.cuda.set_device(0)
        self.stream = torch.cuda.current_stream()
        self.ctx = B.dbl_create(self.cfg, seed, self.stream.cuda_stream)
        if TUNING:
            B.dbl_set_tuning(self.ctx, **TUNING)
        self.V = shape["vocab"]
        self.bf16 = shape["dtype"] == B.DBL_BF16
        self.ncommit = 0     # dbl_kv_commit calls so far (they offset the Philox step word)

    def close(self):
        if self.ctx is not None:
            B.dbl_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def i32(self, *shape, fill=0):
        return torch.full(shape, fill, dtype=torch.int32, device=DEV)

    def get_tensor(self, name, layer=0):
        tid = TENSORS[name][0]
        n = self._numel(name)
        if name in GAINS or not self.bf16:
            a = np.empty(n, np.float32)
            B.dbl_get_weights(self.ctx, tid, layer, a)
            return a
        a = np.empty(n, np.uint16)
        B.dbl_get_weights(self.ctx, tid, layer, a)
        return bf16_bits_to_f32(a)

    def set_tensor(self, name, layer, values):
        tid = TENSORS[name][0]
        v = np.ascontiguousarray(values, dtype=np.float32).ravel()
        assert v.size == self._numel(name)
        if name in GAINS or not self.bf16:
            B.dbl_set_weights(self.ctx, tid, layer, v)
        else:
            B.dbl_set_weights(self.ctx, tid, layer, f32_to_bf16_bits(v))

    def _numel(self, name):
        s = self.shape
        d, hd, H, Hkv, F, V = s["d_model"], s["head_dim"], s["n_q_heads"], s["n_kv_heads"], s["d_ffn"], s["vocab"]
        return {"emb": V * d, "lm": V * d, "gf": d, "g1": d, "g2": d, "gq": hd, "gk": hd, "wq": H * hd * d,
                "wk": Hkv * hd * d, "wv": Hkv * hd * d, "wo": d * H * hd, "wg": F * d, "wu": F * d, "wd": d * F}[name]

    # -- one call each, returning host arrays (synchronising) -------------
    def verify(self, windows, temperature=0.0, seed=0, step=0, want_logits=True, win_len=None):
        w = torch.as_tensor(np.asarray(windows, dtype=np.int32), device=DEV)
        Bn, k = w.shape
        lg = torch.empty((Bn, k, self.V), dtype=torch.float32, device=DEV) if want_logits else None
        if win_len is None:
            B.dbl_verify_block(self.ctx, w, Bn, k, temperature, seed, step, lg)
        else:
            wl = torch.as_tensor(np.asarray(win_len, dtype=np.int32), device=DEV)
            B.dbl_verify_block_ragged(self.ctx, w, wl, Bn, k, temperature, seed, step, lg)
        self._bk = (Bn, k)
        torch.cuda.synchronize()
        return lg.cpu().numpy() if want_logits else None

    def accept(self, mode, q=None):
        Bn, k = self._bk
        n_acc, emit, guide = self.i32(Bn, fill=-7), self.i32(Bn, k, fill=-7), self.i32(Bn, k, fill=-7)
        qd = None if q is None else torch.as_tensor(np.asarray(q, dtype=np.float32), device=DEV).contiguous()
        B.dbl_accept(self.ctx, mode, qd, n_acc, emit, guide)
        torch.cuda.synchronize()
        return n_acc.cpu().numpy(), emit.cpu().numpy(), guide.cpu().numpy()

    def commit(self, n_keep=None):
        nk = None if n_keep is None else torch.as_tensor(np.asarray(n_keep, dtype=np.int32), device=DEV)
        B.dbl_kv_commit(self.ctx, nk)
        self.ncommit += 1
        torch.cuda.synchronize()

    def kv_len(self):
        out = np.zeros(self.cfg.max_batch, np.int32)
        B.dbl_kv_len(self.ctx, out)
        return out

    def hist_len(self):
        out = np.zeros(self.cfg.max_batch, np.int32)
        B.dbl_hist_len(self.ctx, out)
        return out

    def history(self, seq=0):
        out = np.zeros(self.cfg.max_hist, np.int32)
        n = B.dbl_history_get(self.ctx, seq, out)
        return out[:n]

    def retrieve(self, Bn, n_max, n_min, max_cont):
        cont = self.i32(Bn, max_cont, fill=-7)
        cl, mn, mp = self.i32(Bn, fill=-7), self.i32(Bn, fill=-7), self.i32(Bn, fill=-7)
        B.dbl_retrieve(self.ctx, Bn, n_max, n_min, max_cont, cont, cl, mn, mp)
        torch.cuda.synchronize()
        return cont.cpu().numpy(), cl.cpu().numpy(), mn.cpu().numpy(), mp.cpu().numpy()

    def prefill(self, prompts, chunk):
        """history = prompt; KV of prompt[:-1] through verify_block + commit(n_keep)."""
        Bn = len(prompts)
        P = len(prompts[0]) - 1
        assert all(len(p) == P + 1 for p in prompts)
        B.dbl_reset(self.ctx, -1)
        for b, p in enumerate(prompts):
            B.dbl_history_set(self.ctx, b, np.ascontiguousarray(p, dtype=np.int32))
        i = 0
        while i < P:
            k = min(chunk, P - i)
            self.verify([p[i:i + k] for p in prompts], want_logits=False)
            self.commit([k] * Bn)
            i += k


def oracle_shape(shape, max_ctx):
    s = dict(shape)
    s["max_ctx"] = max_ctx
    return s


class Ref:
    """The oracle side: one model, B sequences."""

    def __init__(self, shape, *, seed, max_batch=1, max_ctx=512, max_hist=1024):
        self.model = O.Model(**oracle_shape(shape, max_ctx), seed=seed)
        self.seqs = [O.Seq(self.model, max_hist=max_hist) for _ in range(max_batch)]

    def set_tensor(self, name, layer, values):
        self.model.tensor(TENSORS[name][1], layer)[:] = np.asarray(values, dtype=np.float32).ravel()

    def get_tensor(self, name, layer=0):
        return self.model.tensor(TENSORS[name][1], layer).copy()

    def verify(self, windows):
        return np.stack([self.seqs[b].verify_block(w) for b, w in enumerate(windows)])

    def prefill(self, prompts, chunk):
        for b, p in enumerate(prompts):
            s = self.seqs[b]
            s.reset()
            s.hist_set(p)
            i, P = 0, len(p) - 1
            while i < P:
                k = min(chunk, P - i)
                s.verify_block(p[i:i + k])
                s.commit(k, [])
                i += k
