"""The C-ABI library loads without a GPU, exports what include/dbl.h declares, and checks
its arguments before touching the GPU (validate-only contexts compute nothing)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2601_05524_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    src = open(os.path.join(ROOT, "include", "dbl.h")).read() + open(os.path.join(ROOT, "include", "dbl_diag.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dbl_[a-z_0-9]+)\s*\(", src)))


def test_exports_every_declared_symbol():
    names = declared_symbols()
    assert set(names) == set(B.EXPORTS)
    L = C.CDLL(B.LIB_PATH)
    for n in names:
        assert getattr(L, n) is not None


def cfg(**kw):
    base = dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=688, vocab=2048,
                dtype=B.DBL_F32, max_batch=2, max_ctx=512, max_window=8, max_hist=1024,
                flags=B.DBL_FLAG_VALIDATE_ONLY)
    base.update(kw)
    return B.make_cfg(**base)


@pytest.mark.parametrize("bad", [dict(head_dim=48), dict(n_q_heads=3), dict(max_ctx=100), dict(dtype=7),
                                 dict(max_window=64), dict(max_batch=8, max_window=32), dict(d_model=8200 * 2),
                                 dict(vocab=1), dict(rms_eps=0.0), dict(max_hist=0), dict(d_model=250),
                                 dict(max_ctx=320, flags=B.DBL_FLAG_VALIDATE_ONLY | B.DBL_FLAG_PAGED_KV),   # paged: 256-token pages
                                 dict(flags=B.DBL_FLAG_VALIDATE_ONLY | (5 << 8))])                      # pool size without paging
def test_create_rejects_bad_configs(bad):
    with pytest.raises(B.DblError) as e:
        B.dbl_create(cfg(**bad), 1)
    assert e.value.code == B.DBL_EINVAL


def rc_of(fn, *a):
    try:
        return fn(*a)
    except B.DblError as e:
        return e.code


def test_validate_only_context_checks_arguments_and_order():
    ctx = B.dbl_create(cfg(), 1)
    L = B.lib()
    i32 = np.zeros(64, np.int32)
    p = C.c_void_p(i32.ctypes.data)      # never dereferenced: no GPU work happens
    ok = B.DBL_ENODEV                    # "arguments fine, nothing run"
    assert L.dbl_reset(ctx, -1) == ok
    assert L.dbl_reset(ctx, 5) == B.DBL_EINVAL
    assert L.dbl_history_set(ctx, 0, p, 10) == ok
    assert L.dbl_history_set(ctx, 0, p, 5000) == B.DBL_EINVAL
    assert L.dbl_history_set(ctx, 2, p, 1) == B.DBL_EINVAL
    assert L.dbl_retrieve(ctx, 1, 3, 1, 8, p, p, p, p) == ok
    assert L.dbl_retrieve(ctx, 3, 3, 1, 8, p, p, p, p) == B.DBL_EINVAL      # B > max_batch
    assert L.dbl_retrieve(ctx, 1, 1, 3, 8, p, p, p, p) == B.DBL_EINVAL      # n_min > n_max
    assert L.dbl_retrieve(ctx, 1, 3, 1, 0, p, p, p, p) == B.DBL_EINVAL
    assert L.dbl_retrieve(ctx, 1, 3, 1, 8, None, p, p, p) == B.DBL_EINVAL
    assert L.dbl_build_window(ctx, 1, 4, 8, p, p, 0, p) == ok
    assert L.dbl_build_window(ctx, 1, 9, 8, p, p, 0, p) == B.DBL_EINVAL
    assert L.dbl_build_window(ctx, 1, 4, 8, p, p, 5000, p) == B.DBL_EINVAL
    # order: accept / commit need a verify first
    assert L.dbl_accept(ctx, B.DBL_GREEDY, None, p, p, p) == B.DBL_ESTATE
    assert L.dbl_kv_commit(ctx, None) == B.DBL_ESTATE
    assert L.dbl_verify_block(ctx, None, 1, 4, 0.0, 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block(ctx, p, 1, 9, 0.0, 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block(ctx, p, 0, 4, 0.0, 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block(ctx, p, 1, 4, float("nan"), 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block_ragged(ctx, p, None, 1, 4, 0.0, 0, 0, None) == B.DBL_EINVAL   # lengths are required
    assert L.dbl_verify_block_ragged(ctx, None, p, 1, 4, 0.0, 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block_ragged(ctx, p, p, 1, 9, 0.0, 0, 0, None) == B.DBL_EINVAL
    assert L.dbl_verify_block_ragged(ctx, p, p, 1, 4, 0.0, 0, 0, None) == ok
    assert L.dbl_verify_block(ctx, p, 1, 4, 0.0, 0, 0, None) == ok
    assert L.dbl_kv_commit(ctx, None) == B.DBL_ESTATE                        # no accept yet
    assert L.dbl_accept(ctx, B.DBL_SAMPLE, None, p, p, p) == B.DBL_ESTATE    # verify was greedy
    assert L.dbl_accept(ctx, 3, None, p, p, p) == B.DBL_EINVAL
    assert L.dbl_accept(ctx, B.DBL_GREEDY, p, p, p, p) == B.DBL_EINVAL       # q in greedy mode
    assert L.dbl_accept(ctx, B.DBL_GREEDY, None, p, p, p) == ok
    assert L.dbl_kv_commit(ctx, None) == ok
    assert L.dbl_kv_commit(ctx, None) == B.DBL_ESTATE                        # consumed
    assert b"verify_block" in L.dbl_last_error(ctx)
    # capacity: the host-side upper bound of kv_len grows by k per commit
    n = 0
    while True:
        rc = L.dbl_verify_block(ctx, p, 1, 8, 0.7, 1, n, None)
        if rc != ok:
            break
        assert L.dbl_accept(ctx, B.DBL_SAMPLE, None, p, p, p) == ok
        assert L.dbl_kv_commit(ctx, None) == ok
        n += 1
    assert rc == B.DBL_EINVAL and n == (512 - 4) // 8
    assert b"max_ctx" in L.dbl_last_error(ctx)
    w = np.zeros(256, np.float32)
    assert L.dbl_set_weights(ctx, B.T_GF, 0, C.c_void_p(w.ctypes.data), w.nbytes) == ok
    assert L.dbl_set_weights(ctx, B.T_GF, 0, C.c_void_p(w.ctypes.data), 8) == B.DBL_EINVAL
    assert L.dbl_set_weights(ctx, 99, 0, C.c_void_p(w.ctypes.data), 8) == B.DBL_EINVAL
    assert L.dbl_set_weights(ctx, B.T_WQ, 2, C.c_void_p(w.ctypes.data), 8) == B.DBL_EINVAL
    wb, kvb = B.dbl_model_bytes(ctx)
    per_layer = (4 + 2 * 2) * 64 * 256 + 256 * 256 + 3 * 688 * 256
    assert wb == (2 * per_layer + 2048 * 256) * 4 and kvb == 2 * 2 * 128 * 4
    assert B.dbl_destroy(ctx) == 0


def test_validate_only_context_checks_the_datastore_and_rollback_calls():
    ctx = B.dbl_create(cfg(), 1)
    L = B.lib()
    i32 = np.zeros(64, np.int32)
    p = C.c_void_p(i32.ctypes.data)
    ok = B.DBL_ENODEV
    assert L.dbl_truncate(ctx, 0, 5, -1) == ok
    assert L.dbl_truncate(ctx, 2, 5, -1) == B.DBL_EINVAL                       # seq out of range
    assert L.dbl_retrieve_tiered(ctx, 2, 3, 1, 8, p, p, p, p, p) == ok
    assert L.dbl_retrieve_tiered(ctx, 1, 3, 1, 8, p, p, p, p, None) == B.DBL_EINVAL
    assert L.dbl_retrieve_tiered(ctx, 1, 33, 1, 8, p, p, p, p, p) == B.DBL_EINVAL
    assert L.dbl_retrieve_tiered(ctx, 1, 3, 1, 65, p, p, p, p, p) == B.DBL_EINVAL
    assert L.dbl_session_mark(ctx, 0, 3) == ok
    assert L.dbl_session_mark(ctx, 0, -1) == B.DBL_EINVAL
    assert L.dbl_session_mark(ctx, 9, 3) == B.DBL_EINVAL
    prior = np.array([1, 2, -1, 2047], np.int32)
    assert L.dbl_prior_set(ctx, C.c_void_p(prior.ctypes.data), 4) == ok
    assert L.dbl_prior_set(ctx, None, 0) == ok
    assert L.dbl_prior_set(ctx, None, 4) == B.DBL_EINVAL
    bad = np.array([1, 2048], np.int32)                                        # id == vocab
    assert L.dbl_prior_set(ctx, C.c_void_p(bad.ctypes.data), 2) == B.DBL_EINVAL
    bad = np.array([1, -2], np.int32)
    assert L.dbl_prior_set(ctx, C.c_void_p(bad.ctypes.data), 2) == B.DBL_EINVAL
    # the rejected tier is updated between accept and commit
    assert L.dbl_rejected_update(ctx, None) == B.DBL_ESTATE
    assert L.dbl_verify_block(ctx, p, 1, 4, 0.0, 0, 0, None) == ok
    assert L.dbl_rejected_update(ctx, None) == B.DBL_ESTATE                    # no accept yet
    assert L.dbl_accept(ctx, B.DBL_GREEDY, None, p, p, p) == ok
    assert L.dbl_rejected_update(ctx, p) == ok
    assert L.dbl_kv_commit(ctx, None) == ok
    assert L.dbl_rejected_update(ctx, None) == B.DBL_ESTATE                    # consumed by the commit
    n = C.c_int32(0)
    assert L.dbl_rejected_get(ctx, 0, p, 64, C.byref(n)) == ok
    assert L.dbl_rejected_get(ctx, 0, p, 64, None) == B.DBL_EINVAL
    assert L.dbl_rejected_get(ctx, 3, p, 64, C.byref(n)) == B.DBL_EINVAL
    # a rollback invalidates a pending verify: commit afterwards is refused
    assert L.dbl_verify_block(ctx, p, 1, 4, 0.0, 0, 0, None) == ok
    assert L.dbl_truncate(ctx, 0, 0, 0) == ok
    assert L.dbl_kv_commit(ctx, None) == B.DBL_ESTATE
    assert B.dbl_destroy(ctx) == 0


def test_new_entry_points_check_their_arguments():
    ctx = B.dbl_create(cfg(), 1)
    L = B.lib()
    i32 = np.zeros(64, np.int32)
    p = C.c_void_p(i32.ctypes.data)
    ok = B.DBL_ENODEV
    # the tiered retrieval on the library's static scratch: same checks as dbl_retrieve_tiered
    assert L.dbl_retrieve_tiered_static(ctx, 2, 3, 1, 8, p, p, p, p, p) == ok
    assert L.dbl_retrieve_tiered_static(ctx, 3, 3, 1, 8, p, p, p, p, p) == B.DBL_EINVAL       # B > max_batch
    assert L.dbl_retrieve_tiered_static(ctx, 129, 3, 1, 8, p, p, p, p, p) == B.DBL_EINVAL     # beyond the static array
    assert L.dbl_retrieve_tiered_static(ctx, 1, 3, 1, 65, p, p, p, p, p) == B.DBL_EINVAL
    assert L.dbl_retrieve_tiered_static(ctx, 1, 3, 1, 8, p, p, p, p, None) == B.DBL_EINVAL
    assert L.dbl_retrieve_tiered_static(None, 1, 3, 1, 8, p, p, p, p, p) == B.DBL_EINVAL
    # cache rows
    assert L.dbl_kv_set(ctx, 0, 1, 0, 4, p, p) == ok
    assert L.dbl_kv_get(ctx, 1, 0, 500, 12, p, p) == ok
    assert L.dbl_kv_set(ctx, 0, 2, 0, 4, p, p) == B.DBL_EINVAL          # layer
    assert L.dbl_kv_set(ctx, 2, 0, 0, 4, p, p) == B.DBL_EINVAL          # sequence
    assert L.dbl_kv_set(ctx, 0, 0, 510, 4, p, p) == B.DBL_EINVAL        # beyond max_ctx
    assert L.dbl_kv_get(ctx, 0, 0, -1, 4, p, p) == B.DBL_EINVAL
    assert L.dbl_kv_get(ctx, 0, 0, 0, 4, None, p) == B.DBL_EINVAL
    # attention plan: host logic only, works without a GPU
    out = (C.c_int32 * 4)()
    assert L.dbl_attn_plan(ctx, 1, 8, out) == B.DBL_OK and out[3] >= 1
    assert L.dbl_attn_plan(ctx, 3, 8, out) == B.DBL_EINVAL
    assert L.dbl_attn_plan(ctx, 1, 8, None) == B.DBL_EINVAL
    assert L.dbl_projection_plan(ctx, 2, 8, out) == B.DBL_OK and out[2] >= 1
    assert L.dbl_projection_plan(ctx, 5, 8, out) == B.DBL_EINVAL
    # tuning: forms can be forced or forbidden through the ABI; nonsense is refused
    t = B.dbl_tuning_default()
    assert (t.split_units, t.wide_gate_up, t.wide_residual, t.wide_lm_head, t.stream_16_rows, t.attn_shared, t.attn_blocks, t.attn_p16, t.attn_split_tokens) == (0, 1, 1, 1, 1, 1, 2, 1, 0)
    assert L.dbl_set_tuning(ctx, C.byref(t)) == B.DBL_OK
    before = tuple(out)
    assert B.dbl_set_tuning(ctx, split_units=1) == B.DBL_OK
    assert L.dbl_projection_plan(ctx, 2, 8, out) == B.DBL_OK and (out[3] == 1 or tuple(out) == before)
    t.attn_shared = 9
    assert L.dbl_set_tuning(ctx, C.byref(t)) == B.DBL_EINVAL
    assert L.dbl_set_tuning(ctx, None) == B.DBL_EINVAL
    assert B.dbl_destroy(ctx) == 0


def test_null_context():
    L = B.lib()
    assert L.dbl_destroy(None) == B.DBL_EINVAL
    assert L.dbl_kv_commit(None, None) == B.DBL_EINVAL
    assert L.dbl_last_error(None) == b"null context"
