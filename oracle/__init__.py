"""ctypes access to the CPU oracle (oracle/dbl_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dbl_oracle.c")
_LIB = os.path.join(_HERE, "libdbl_oracle.so")

T_EMB, T_LM, T_GF = 0, 1, 2
T_G1, T_WQ, T_WK, T_WV, T_GQ, T_GK, T_WO, T_G2, T_WG, T_WU, T_WD = range(10, 21)


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, no fast-math, no FP contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
             "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab",
                 "qk_norm", "dtype", "max_ctx")] + [("rms_eps", C.c_double), ("rope_base", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, f32p, f64p, u32p = (C.POINTER(C.c_int32), C.POINTER(C.c_float),
                                  C.POINTER(C.c_double), C.POINTER(C.c_uint32))
        L.orc_round_bf16.restype = C.c_double
        L.orc_round_bf16.argtypes = [C.c_double]
        L.orc_philox4x32_10.argtypes = [u32p, u32p, u32p]
        L.orc_weight_value.restype = C.c_float
        L.orc_weight_value.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_uint64, C.c_int]
        L.orc_weight_fill.argtypes = [C.c_uint64, C.c_int, C.c_int, C.c_uint64, C.c_uint64, C.c_int, f32p]
        L.orc_model_new.restype = C.c_void_p
        L.orc_model_new.argtypes = [C.POINTER(Cfg), C.c_uint64]
        L.orc_model_free.argtypes = [C.c_void_p]
        L.orc_model_tensor.restype = f32p
        L.orc_model_tensor.argtypes = [C.c_void_p, C.c_int, C.c_int, C.POINTER(C.c_int64)]
        L.orc_seq_new.restype = C.c_void_p
        L.orc_seq_new.argtypes = [C.c_void_p, C.c_int]
        L.orc_seq_free.argtypes = [C.c_void_p]
        L.orc_seq_kv_len.restype = C.c_int32
        L.orc_seq_kv_len.argtypes = [C.c_void_p]
        L.orc_seq_hist_len.restype = C.c_int32
        L.orc_seq_hist_len.argtypes = [C.c_void_p]
        L.orc_seq_hist.restype = i32p
        L.orc_seq_hist.argtypes = [C.c_void_p]
        L.orc_seq_kcache.restype = f64p
        L.orc_seq_kcache.argtypes = [C.c_void_p]
        L.orc_seq_vcache.restype = f64p
        L.orc_seq_vcache.argtypes = [C.c_void_p]
        L.orc_seq_reset.argtypes = [C.c_void_p]
        L.orc_seq_hist_set.argtypes = [C.c_void_p, i32p, C.c_int]
        L.orc_seq_truncate.argtypes = [C.c_void_p, C.c_int, C.c_int]
        L.orc_rmsnorm.argtypes = [f64p, f32p, C.c_int, C.c_double, f64p]
        L.orc_rope.argtypes = [f64p, C.c_int, C.c_int, C.c_double]
        L.orc_verify_block.argtypes = [C.c_void_p, C.c_void_p, i32p, C.c_int, f64p, f64p]
        L.orc_accept_greedy.argtypes = [f64p, C.c_int, C.c_int, i32p, i32p, i32p, i32p, f64p]
        L.orc_accept_sample.argtypes = [f64p, C.c_int, C.c_int, i32p, f32p, C.c_double, C.c_uint64,
                                        C.c_uint64, C.c_int, i32p, i32p, i32p, f64p, f64p, f64p]
        L.orc_retrieve.argtypes = [i32p, C.c_int, C.c_int, C.c_int, C.c_int, i32p, i32p, i32p, i32p]
        L.orc_retrieve_tiered.argtypes = [i32p, C.c_int, i32p, C.c_int, C.c_int, i32p, C.c_int, C.c_int, C.c_int,
                                          C.c_int, i32p, i32p, i32p, i32p, i32p]
        L.orc_rejected_append.argtypes = [i32p, C.c_int, C.c_int, i32p, C.c_int, i32p, C.c_int, C.c_int, C.c_int]
        L.orc_rejected_append.restype = C.c_int
        L.orc_commit.argtypes = [C.c_void_p, C.c_int, i32p, C.c_int]
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def round_bf16(x: float) -> float:
    return lib().orc_round_bf16(float(x))


def philox(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    o = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(_p(c, C.c_uint32), _p(k, C.c_uint32), _p(o, C.c_uint32))
    return o


def weight_fill(seed, tensor_id, layer, first, n, dtype):
    out = np.empty(n, dtype=np.float32)
    lib().orc_weight_fill(seed, tensor_id, layer, first, n, dtype, _p(out, C.c_float))
    return out


def rmsnorm(x, g, eps):
    x = np.ascontiguousarray(x, dtype=np.float64)
    g = np.ascontiguousarray(g, dtype=np.float32)
    out = np.empty_like(x)
    lib().orc_rmsnorm(_p(x, C.c_double), _p(g, C.c_float), x.size, float(eps), _p(out, C.c_double))
    return out


def rope(v, pos, base):
    v = np.array(v, dtype=np.float64)
    lib().orc_rope(_p(v, C.c_double), v.size, int(pos), float(base))
    return v


class Model:
    """Seeded synthetic decoder weights (row-major [out][in] float32 arrays)."""

    def __init__(self, *, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                 qk_norm=0, dtype=1, max_ctx=4096, rms_eps=1e-5, rope_base=1e4, seed=0):
        self.cfg = Cfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab,
                       qk_norm, dtype, max_ctx, rms_eps, rope_base)
        self.seed = seed
        self.h = lib().orc_model_new(C.byref(self.cfg), seed)
        if not self.h:
            raise MemoryError("orc_model_new")

    def tensor(self, tensor_id, layer=0) -> np.ndarray:
        """Writable flat view of one tensor's storage."""
        n = C.c_int64(0)
        p = lib().orc_model_tensor(self.h, tensor_id, layer, C.byref(n))
        if not p or n.value == 0:
            raise KeyError((tensor_id, layer))
        return np.ctypeslib.as_array(p, shape=(n.value,))

    def close(self):
        if self.h:
            lib().orc_model_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Seq:
    """One sequence: KV cache, committed length, token history."""

    def __init__(self, model: Model, max_hist=4096):
        self.model = model
        self.h = lib().orc_seq_new(model.h, max_hist)
        if not self.h:
            raise MemoryError("orc_seq_new")

    @property
    def kv_len(self):
        return lib().orc_seq_kv_len(self.h)

    @property
    def hist_len(self):
        return lib().orc_seq_hist_len(self.h)

    def history(self) -> np.ndarray:
        n = self.hist_len
        return np.ctypeslib.as_array(lib().orc_seq_hist(self.h), shape=(max(n, 1),))[:n].copy()

    def _cache(self, fn):
        c = self.model.cfg
        shape = (max(c.n_layers, 1), c.n_kv_heads, c.max_ctx, c.head_dim)
        return np.ctypeslib.as_array(fn(self.h), shape=shape)

    def kcache(self):
        return self._cache(lib().orc_seq_kcache)

    def vcache(self):
        return self._cache(lib().orc_seq_vcache)

    def reset(self):
        lib().orc_seq_reset(self.h)

    def truncate(self, kv_len=-1, hist_len=-1):
        if lib().orc_seq_truncate(self.h, int(kv_len), int(hist_len)) != 0:
            raise ValueError("truncate beyond the current lengths")

    def hist_set(self, tokens):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        if lib().orc_seq_hist_set(self.h, _p(t, C.c_int32), t.size) != 0:
            raise ValueError("history too long")

    def verify_block(self, window, want_hidden=False):
        w = np.ascontiguousarray(window, dtype=np.int32)
        k = w.size
        c = self.model.cfg
        logits = np.empty((k, c.vocab), dtype=np.float64)
        hid = np.empty((k, c.d_model), dtype=np.float64) if want_hidden else None
        rc = lib().orc_verify_block(self.model.h, self.h, _p(w, C.c_int32), k, _p(logits, C.c_double),
                                    _p(hid, C.c_double) if want_hidden else None)
        if rc != 0:
            raise ValueError("orc_verify_block rc=%d" % rc)
        return (logits, hid) if want_hidden else logits

    def commit(self, n_keep, emit):
        e = np.ascontiguousarray(emit, dtype=np.int32)
        rc = lib().orc_commit(self.h, int(n_keep), _p(e, C.c_int32), e.size)
        if rc != 0:
            raise ValueError("orc_commit rc=%d" % rc)

    def retrieve(self, n_max, n_min, max_cont):
        return retrieve(self.history(), n_max, n_min, max_cont)

    def close(self):
        if self.h:
            lib().orc_seq_free(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def accept_greedy(logits, window):
    z = np.ascontiguousarray(logits, dtype=np.float64)
    w = np.ascontiguousarray(window, dtype=np.int32)
    k, V = z.shape
    n = C.c_int32(0)
    emit = np.empty(k, np.int32)
    guide = np.empty(k, np.int32)
    margin = np.empty(k, np.float64)
    lib().orc_accept_greedy(_p(z, C.c_double), k, V, _p(w, C.c_int32), C.byref(n),
                            _p(emit, C.c_int32), _p(guide, C.c_int32), _p(margin, C.c_double))
    return n.value, emit, guide, margin


def accept_sample(logits, window, q, T, seed, step, b=0, guide_gaps=False):
    """(n_acc, emit, guide, acceptance margins, gap of the emitted token's draw); with
    guide_gaps=True a sixth item: the score gap of every row's own draw guide[j]."""
    z = np.ascontiguousarray(logits, dtype=np.float64)
    w = np.ascontiguousarray(window, dtype=np.int32)
    k, V = z.shape
    qa = None if q is None else np.ascontiguousarray(q, dtype=np.float32)
    if qa is not None:
        assert qa.shape == (k - 1, V)
    n = C.c_int32(0)
    emit = np.empty(k, np.int32)
    guide = np.empty(k, np.int32)
    am = np.empty(k, np.float64)
    gap = C.c_double(0.0)
    gg = np.empty(k, np.float64)
    lib().orc_accept_sample(_p(z, C.c_double), k, V, _p(w, C.c_int32),
                            None if qa is None else _p(qa, C.c_float), float(T), seed, step, b,
                            C.byref(n), _p(emit, C.c_int32), _p(guide, C.c_int32),
                            _p(am, C.c_double), C.byref(gap), _p(gg, C.c_double))
    if guide_gaps:
        return n.value, emit, guide, am, gap.value, gg
    return n.value, emit, guide, am, gap.value


def retrieve(hist, n_max, n_min, max_cont):
    h = np.ascontiguousarray(hist, dtype=np.int32)
    cont = np.full(max(max_cont, 1), -1, np.int32)
    cl, mn, mp = C.c_int32(0), C.c_int32(0), C.c_int32(0)
    lib().orc_retrieve(_p(h, C.c_int32), h.size, n_max, n_min, max_cont, _p(cont, C.c_int32),
                       C.byref(cl), C.byref(mn), C.byref(mp))
    return cont[:cl.value].copy(), cl.value, mn.value, mp.value


def retrieve_tiered(prior, hist, prompt_len, rejected, n_max, n_min, max_cont):
    """Alg. 3's priority search.  Returns (continuation, cont_len, match_n, match_pos, tier);
    tier 0 prior, 1 dynamic, 2 rejected, 3 the sequence itself, -1 miss."""
    pr = np.ascontiguousarray(prior, dtype=np.int32)
    h = np.ascontiguousarray(hist, dtype=np.int32)
    rj = np.ascontiguousarray(rejected, dtype=np.int32)
    cont = np.full(max(max_cont, 1), -1, np.int32)
    cl, mn, mp, mt = C.c_int32(0), C.c_int32(0), C.c_int32(0), C.c_int32(0)
    lib().orc_retrieve_tiered(_p(pr, C.c_int32), pr.size, _p(h, C.c_int32), h.size, int(prompt_len),
                              _p(rj, C.c_int32), rj.size, n_max, n_min, max_cont, _p(cont, C.c_int32),
                              C.byref(cl), C.byref(mn), C.byref(mp), C.byref(mt))
    return cont[:cl.value].copy(), cl.value, mn.value, mp.value, mt.value


def rejected_append(rejected, cap, hist, window, n_acc, n_draft, ctx_tokens=4):
    """Alg. 3's cache update for the rejected tier; returns the tier's new contents."""
    buf = np.full(cap, -1, np.int32)
    r = np.ascontiguousarray(rejected, dtype=np.int32)
    buf[:r.size] = r
    h = np.ascontiguousarray(hist, dtype=np.int32)
    w = np.ascontiguousarray(window, dtype=np.int32)
    n = lib().orc_rejected_append(_p(buf, C.c_int32), r.size, cap, _p(h, C.c_int32), h.size, _p(w, C.c_int32),
                                  int(n_acc), int(n_draft), int(ctx_tokens))
    return buf[:n].copy()
