"""Thin ctypes binding of libdbl.so (include/dbl.h): argument marshalling only.

Every function here has the name of the C entry point it calls.  PyTorch is used by
callers for device memory (`tensor.data_ptr()`) and streams; nothing in this module
computes anything, and there is no fallback: if the HIP library is missing or a
call fails, a DblError is raised.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdbl.so")

DBL_OK, DBL_EINVAL, DBL_ESTATE, DBL_ENOMEM, DBL_EHIP, DBL_ENODEV = 0, -1, -2, -3, -4, -5
DBL_F32, DBL_BF16 = 0, 1
DBL_GREEDY, DBL_SAMPLE = 0, 1
DBL_FLAG_VALIDATE_ONLY = 1
DBL_FLAG_PAGED_KV = 2
KV_PAGE = 256
T_EMB, T_LM, T_GF = 0, 1, 2
T_G1, T_WQ, T_WK, T_WV, T_GQ, T_GK, T_WO, T_G2, T_WG, T_WU, T_WD = range(10, 21)

EXPORTS = ["dbl_create", "dbl_destroy", "dbl_last_error", "dbl_set_weights", "dbl_get_weights", "dbl_reset", "dbl_truncate", "dbl_kv_fill",
           "dbl_kv_set", "dbl_kv_get", "dbl_attn_plan", "dbl_projection_plan", "dbl_tuning_default", "dbl_set_tuning",
           "dbl_build_guided_window", "dbl_merge", "dbl_history_tail", "dbl_history_splice", "dbl_catchup_window", "dbl_lengths_dev",
           "dbl_retrieve_tiered", "dbl_retrieve_tiered_static", "dbl_session_mark", "dbl_prior_set", "dbl_rejected_update", "dbl_rejected_get",
           "dbl_history_set", "dbl_history_get", "dbl_retrieve", "dbl_build_window", "dbl_verify_block", "dbl_verify_block_ragged", "dbl_accept",
           "dbl_kv_commit", "dbl_kv_len", "dbl_hist_len", "dbl_model_bytes", "dbl_debug_buffer",
           "dbl_bench_projection"]


class DblError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("libdbl error %d: %s" % (code, msg))
        self.code = code


class ModelCfg(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32),
                ("rms_eps", C.c_float), ("rope_base", C.c_float), ("qk_norm", C.c_int32), ("dtype", C.c_int32),
                ("max_batch", C.c_int32), ("max_ctx", C.c_int32), ("max_window", C.c_int32),
                ("max_hist", C.c_int32), ("flags", C.c_int32)]


class Tuning(C.Structure):
    """dbl_tuning of include/dbl_diag.h."""
    _fields_ = [(n, C.c_int32) for n in ("split_units", "wide_gate_up", "wide_residual", "wide_lm_head", "stream_16_rows", "attn_shared", "attn_blocks",
                                          "attn_p16", "attn_split_tokens", "verbose")]


_lib = None


def lib():
    """Load libdbl.so (built in-tree by build.py); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise DblError(DBL_EHIP, "libdbl.so is not built (run paper_2601_05524_amd/build.py); "
                                     "there is no fallback path")
        L = C.CDLL(LIB_PATH)
        vp, i32p, i = C.c_void_p, C.c_void_p, C.c_int
        L.dbl_create.argtypes = [C.POINTER(ModelCfg), C.c_uint64, vp, C.POINTER(vp)]
        L.dbl_destroy.argtypes = [vp]
        L.dbl_last_error.argtypes = [vp]
        L.dbl_last_error.restype = C.c_char_p
        L.dbl_set_weights.argtypes = [vp, i, i, vp, C.c_size_t]
        L.dbl_get_weights.argtypes = [vp, i, i, vp, C.c_size_t]
        L.dbl_reset.argtypes = [vp, i]
        L.dbl_truncate.argtypes = [vp, i, C.c_int32, C.c_int32]
        L.dbl_kv_fill.argtypes = [vp, i, C.c_int32, C.c_uint64]
        L.dbl_kv_set.argtypes = [vp, i, i, C.c_int32, C.c_int32, vp, vp]
        L.dbl_kv_get.argtypes = [vp, i, i, C.c_int32, C.c_int32, vp, vp]
        L.dbl_retrieve_tiered.argtypes = [vp, i, i, i, i, i32p, i32p, i32p, i32p, i32p]
        L.dbl_retrieve_tiered_static.argtypes = [vp, i, i, i, i, i32p, i32p, i32p, i32p, i32p]
        L.dbl_prior_set.argtypes = [vp, i32p, i]
        L.dbl_session_mark.argtypes = [vp, i, C.c_int32]
        L.dbl_rejected_update.argtypes = [vp, i32p]
        L.dbl_rejected_get.argtypes = [vp, i, i32p, i, C.POINTER(C.c_int32)]
        L.dbl_history_set.argtypes = [vp, i, vp, i]
        L.dbl_history_get.argtypes = [vp, i, vp, i, C.POINTER(C.c_int32)]
        L.dbl_retrieve.argtypes = [vp, i, i, i, i, i32p, i32p, i32p, i32p]
        L.dbl_build_window.argtypes = [vp, i, i, i, i32p, i32p, C.c_int32, i32p]
        L.dbl_build_guided_window.argtypes = [vp, i, i, i32p, i32p, i, i, i, i, C.c_int32, i32p, i32p]
        L.dbl_merge.argtypes = [vp, i, i, i32p, i32p, i32p, i32p, i32p, i, i, i32p, i32p, i32p, i32p, i32p, i32p, i32p]
        L.dbl_history_tail.argtypes = [vp, i, i32p, i, i32p, i32p]
        L.dbl_history_splice.argtypes = [vp, i, i32p, i32p, i32p, i, i32p]
        L.dbl_catchup_window.argtypes = [vp, i, i, C.c_int32, i32p, i32p]
        L.dbl_lengths_dev.argtypes = [vp, i, i32p, i32p]
        L.dbl_verify_block.argtypes = [vp, i32p, i, i, C.c_float, C.c_uint64, C.c_uint64, vp]
        L.dbl_verify_block_ragged.argtypes = [vp, i32p, i32p, i, i, C.c_float, C.c_uint64, C.c_uint64, vp]
        L.dbl_accept.argtypes = [vp, i, vp, i32p, i32p, i32p]
        L.dbl_kv_commit.argtypes = [vp, i32p]
        L.dbl_kv_len.argtypes = [vp, vp]
        L.dbl_hist_len.argtypes = [vp, vp]
        L.dbl_model_bytes.argtypes = [vp, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.dbl_bench_projection.argtypes = [vp, i, i, i, C.POINTER(C.c_float), C.POINTER(C.c_uint64)]
        L.dbl_attn_plan.argtypes = [vp, i, i, vp]
        L.dbl_projection_plan.argtypes = [vp, i, i, vp]
        L.dbl_tuning_default.argtypes = [C.POINTER(Tuning)]
        L.dbl_set_tuning.argtypes = [vp, C.POINTER(Tuning)]
        L.dbl_debug_buffer.argtypes = [vp, i, vp, C.c_size_t, C.POINTER(C.c_int32)]
        for n in EXPORTS:
            if n != "dbl_last_error":
                getattr(L, n).restype = C.c_int
        _lib = L
    return _lib


def _chk(ctx, rc, allow=()):
    if rc != DBL_OK and rc not in allow:
        msg = lib().dbl_last_error(ctx).decode() if ctx else ""
        raise DblError(rc, msg)
    return rc


def _ptr(x):
    """Device pointer of a torch tensor, host pointer of a numpy array, or None."""
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return C.c_void_p(x.data_ptr())
    return C.c_void_p(x.ctypes.data)


def dbl_create(cfg: ModelCfg, weight_seed: int, hip_stream: int = 0):
    h = C.c_void_p()
    rc = lib().dbl_create(C.byref(cfg), weight_seed, C.c_void_p(hip_stream), C.byref(h))
    if rc != DBL_OK:
        raise DblError(rc, "dbl_create failed")
    return h


def dbl_destroy(ctx):
    return _chk(None, lib().dbl_destroy(ctx))


def dbl_last_error(ctx) -> str:
    return lib().dbl_last_error(ctx).decode()


def dbl_set_weights(ctx, tensor_id, layer, host_array):
    return _chk(ctx, lib().dbl_set_weights(ctx, tensor_id, layer, _ptr(host_array), host_array.nbytes))


def dbl_get_weights(ctx, tensor_id, layer, host_array):
    return _chk(ctx, lib().dbl_get_weights(ctx, tensor_id, layer, _ptr(host_array), host_array.nbytes))


def dbl_reset(ctx, seq=-1):
    return _chk(ctx, lib().dbl_reset(ctx, seq))


def dbl_kv_fill(ctx, seq, n_tokens, seed):
    return _chk(ctx, lib().dbl_kv_fill(ctx, seq, int(n_tokens), int(seed)))


def dbl_kv_set(ctx, seq, layer, pos0, n, host_k, host_v):
    return _chk(ctx, lib().dbl_kv_set(ctx, seq, layer, int(pos0), int(n), _ptr(host_k), _ptr(host_v)))


def dbl_kv_get(ctx, seq, layer, pos0, n, host_k, host_v):
    return _chk(ctx, lib().dbl_kv_get(ctx, seq, layer, int(pos0), int(n), _ptr(host_k), _ptr(host_v)))


def dbl_truncate(ctx, seq, kv_len=-1, hist_len=-1):
    return _chk(ctx, lib().dbl_truncate(ctx, seq, int(kv_len), int(hist_len)))


def dbl_history_set(ctx, seq, host_tokens):
    return _chk(ctx, lib().dbl_history_set(ctx, seq, _ptr(host_tokens), int(host_tokens.size)))


def dbl_history_get(ctx, seq, host_out):
    n = C.c_int32(0)
    _chk(ctx, lib().dbl_history_get(ctx, seq, _ptr(host_out), int(host_out.size), C.byref(n)))
    return n.value


def dbl_retrieve(ctx, B, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos):
    return _chk(ctx, lib().dbl_retrieve(ctx, B, n_max, n_min, max_cont, _ptr(cont), _ptr(cont_len),
                                        _ptr(match_n), _ptr(match_pos)))


def dbl_retrieve_tiered(ctx, B, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos, match_tier):
    return _chk(ctx, lib().dbl_retrieve_tiered(ctx, B, n_max, n_min, max_cont, _ptr(cont), _ptr(cont_len),
                                               _ptr(match_n), _ptr(match_pos), _ptr(match_tier)))


def dbl_retrieve_tiered_static(ctx, B, n_max, n_min, max_cont, cont, cont_len, match_n, match_pos, match_tier):
    return _chk(ctx, lib().dbl_retrieve_tiered_static(ctx, B, n_max, n_min, max_cont, _ptr(cont), _ptr(cont_len),
                                                      _ptr(match_n), _ptr(match_pos), _ptr(match_tier)))


def dbl_session_mark(ctx, seq, prompt_len):
    return _chk(ctx, lib().dbl_session_mark(ctx, seq, int(prompt_len)))


def dbl_prior_set(ctx, host_tokens):
    return _chk(ctx, lib().dbl_prior_set(ctx, _ptr(host_tokens), int(host_tokens.size)))


def dbl_rejected_update(ctx, n_draft=None):
    return _chk(ctx, lib().dbl_rejected_update(ctx, _ptr(n_draft)))


def dbl_rejected_get(ctx, seq, host_out):
    n = C.c_int32(0)
    _chk(ctx, lib().dbl_rejected_get(ctx, seq, _ptr(host_out), int(host_out.size), C.byref(n)))
    return n.value


def dbl_build_window(ctx, B, k, max_cont, cont, cont_len, pad_id, window):
    return _chk(ctx, lib().dbl_build_window(ctx, B, k, max_cont, _ptr(cont), _ptr(cont_len), pad_id, _ptr(window)))


def dbl_build_guided_window(ctx, B, k, ahead, n_ahead, max_ahead, n_max, n_min, d, pad_id, window, n_draft):
    return _chk(ctx, lib().dbl_build_guided_window(ctx, B, k, _ptr(ahead), _ptr(n_ahead), max_ahead, n_max, n_min, d, pad_id,
                                                   _ptr(window), _ptr(n_draft)))


def dbl_merge(ctx, B, k, n_u, n_acc, emit, chain, n_chain, max_chain, max_u, base_len, u_out, n_u_out, text_out, n_text_out,
              splice_pos, record):
    return _chk(ctx, lib().dbl_merge(ctx, B, k, _ptr(n_u), _ptr(n_acc), _ptr(emit), _ptr(chain), _ptr(n_chain), max_chain, max_u,
                                     _ptr(base_len), _ptr(u_out), _ptr(n_u_out), _ptr(text_out), _ptr(n_text_out),
                                     _ptr(splice_pos), _ptr(record)))


def dbl_history_tail(ctx, B, from_pos, max_n, tokens_out, n_out):
    return _chk(ctx, lib().dbl_history_tail(ctx, B, _ptr(from_pos), max_n, _ptr(tokens_out), _ptr(n_out)))


def dbl_history_splice(ctx, B, pos, tokens, n, max_n, missing_out=None):
    return _chk(ctx, lib().dbl_history_splice(ctx, B, _ptr(pos), _ptr(tokens), _ptr(n), max_n, _ptr(missing_out)))


def dbl_catchup_window(ctx, B, k, pad_id, window, win_len):
    return _chk(ctx, lib().dbl_catchup_window(ctx, B, k, pad_id, _ptr(window), _ptr(win_len)))


def dbl_lengths_dev(ctx, B, kv_len_out=None, hist_len_out=None):
    return _chk(ctx, lib().dbl_lengths_dev(ctx, B, _ptr(kv_len_out), _ptr(hist_len_out)))


def dbl_verify_block(ctx, window, B, k, temperature=0.0, seed=0, step=0, logits_opt=None):
    return _chk(ctx, lib().dbl_verify_block(ctx, _ptr(window), B, k, temperature, seed, step, _ptr(logits_opt)))


def dbl_verify_block_ragged(ctx, window, win_len, B, k, temperature=0.0, seed=0, step=0, logits_opt=None):
    return _chk(ctx, lib().dbl_verify_block_ragged(ctx, _ptr(window), _ptr(win_len), B, k, temperature, seed, step,
                                                   _ptr(logits_opt)))


def dbl_accept(ctx, mode, q_probs, n_acc, emit, guide):
    return _chk(ctx, lib().dbl_accept(ctx, mode, _ptr(q_probs), _ptr(n_acc), _ptr(emit), _ptr(guide)))


def dbl_kv_commit(ctx, n_keep=None):
    return _chk(ctx, lib().dbl_kv_commit(ctx, _ptr(n_keep)))


def dbl_kv_len(ctx, host_out):
    return _chk(ctx, lib().dbl_kv_len(ctx, _ptr(host_out)))


def dbl_hist_len(ctx, host_out):
    return _chk(ctx, lib().dbl_hist_len(ctx, _ptr(host_out)))


def dbl_model_bytes(ctx):
    w, kv = C.c_uint64(0), C.c_uint64(0)
    _chk(ctx, lib().dbl_model_bytes(ctx, C.byref(w), C.byref(kv)))
    return w.value, kv.value


def dbl_bench_projection(ctx, which, M, iters):
    ms, nbytes = C.c_float(0), C.c_uint64(0)
    _chk(ctx, lib().dbl_bench_projection(ctx, which, M, iters, C.byref(ms), C.byref(nbytes)))
    return ms.value, nbytes.value


def dbl_attn_plan(ctx, B, k):
    """(form, query blocks per wave, waves per workgroup, splits) -- see include/dbl.h"""
    out = (C.c_int32 * 4)()
    _chk(ctx, lib().dbl_attn_plan(ctx, B, k, out))
    return tuple(out)


def dbl_projection_plan(ctx, which, M):
    """(kernel, tile rows per unit or slices, workgroups, split units) -- see include/dbl_diag.h"""
    out = (C.c_int32 * 4)()
    _chk(ctx, lib().dbl_projection_plan(ctx, which, M, out))
    return tuple(out)


def dbl_tuning_default() -> Tuning:
    t = Tuning()
    lib().dbl_tuning_default(C.byref(t))
    return t


def dbl_set_tuning(ctx, **fields):
    """Set the named fields of the tuning (the others keep their defaults)."""
    t = dbl_tuning_default()
    for k, v in fields.items():
        if not hasattr(t, k):
            raise KeyError(k)
        setattr(t, k, int(v))
    return _chk(ctx, lib().dbl_set_tuning(ctx, C.byref(t)))


def dbl_debug_buffer(ctx, which, host_out):
    ld = C.c_int32(0)
    _chk(ctx, lib().dbl_debug_buffer(ctx, which, _ptr(host_out), host_out.nbytes, C.byref(ld)))
    return ld.value


def make_cfg(*, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rms_eps=1e-5, rope_base=1e4,
             qk_norm=0, dtype=DBL_BF16, max_batch=1, max_ctx=4096, max_window=8, max_hist=4096, flags=0) -> ModelCfg:
    return ModelCfg(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rms_eps, rope_base, qk_norm,
                    dtype, max_batch, max_ctx, max_window, max_hist, flags)
