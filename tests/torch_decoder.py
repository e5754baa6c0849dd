"""An independent decoder forward built from PyTorch CPU library routines in fp64
(F.rms_norm, F.scaled_dot_product_attention, F.silu, matmul, complex multiply for
the rotary embedding).  It recomputes the whole sequence from scratch, with no KV
cache and no row-by-row loop, so it shares neither code nor structure with the
oracle; tests use it to pin the oracle's forward.

acc="f32" runs the same contract the way a device would: every value before a bf16
rounding point is an fp32 number (fp32 weights times fp32 activations, the library's
blocked fp32 accumulation, fp32 norms and softmax; the rotary angles stay fp64-derived
fp32 tables).  It rounds at exactly the same points to exactly the same grid, so it is
a second exact-contract implementation; what separates it from the fp64 run is only
which side of a rounding boundary a value falls on.
"""
import numpy as np
import torch
import torch.nn.functional as F

import oracle as O


def np_round_bf16(x):
    b = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)
    drop = np.uint64(45)
    lsb = (b >> drop) & np.uint64(1)
    r = b + ((np.uint64(1) << np.uint64(44)) - np.uint64(1)) + lsb
    r &= ~((np.uint64(1) << drop) - np.uint64(1))
    return r.view(np.float64)


def _rnd(t, bf16):
    if not bf16:
        return t
    if t.dtype == torch.float32:
        return t.bfloat16().float()          # the library's round-to-nearest-even conversion
    return torch.from_numpy(np_round_bf16(t.numpy()).reshape(tuple(t.shape)))


def weights_of(model: O.Model, dtype=np.float64):
    c = model.cfg
    d, hd, H, Hkv, Fd, V = c.d_model, c.head_dim, c.n_q_heads, c.n_kv_heads, c.d_ffn, c.vocab

    def t(tid, layer, shape):
        # (fp32: a view of the model's own storage, no copy)
        return torch.from_numpy(model.tensor(tid, layer).astype(dtype, copy=False).reshape(shape))

    W = dict(emb=t(O.T_EMB, 0, (V, d)), lm=t(O.T_LM, 0, (V, d)), gf=t(O.T_GF, 0, (d,)), layers=[])
    for l in range(c.n_layers):
        W["layers"].append(dict(
            g1=t(O.T_G1, l, (d,)), wq=t(O.T_WQ, l, (H * hd, d)), wk=t(O.T_WK, l, (Hkv * hd, d)),
            wv=t(O.T_WV, l, (Hkv * hd, d)), gq=t(O.T_GQ, l, (hd,)), gk=t(O.T_GK, l, (hd,)),
            wo=t(O.T_WO, l, (d, H * hd)), g2=t(O.T_G2, l, (d,)), wg=t(O.T_WG, l, (Fd, d)),
            wu=t(O.T_WU, l, (Fd, d)), wd=t(O.T_WD, l, (d, Fd))))
    return W


def rope_complex(x, base):
    """x: [T, heads, hd]; pairs (i, i+hd/2) rotated by pos * base^(-2i/hd)."""
    T, _, hd = x.shape
    half = hd // 2
    inv = base ** (-2.0 * torch.arange(half, dtype=torch.float64) / hd)
    ang = torch.arange(T, dtype=torch.float64)[:, None] * inv[None, :]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]
    if x.dtype == torch.float32:
        rot = rot.to(torch.complex64)
    z = torch.complex(x[..., :half], x[..., half:]) * rot
    return torch.cat([z.real, z.imag], dim=-1)


def forward_full(model: O.Model, tokens, acc="f64"):
    """Logits [T][V] for the whole token sequence, full recompute; acc = "f64" or "f32"."""
    c = model.cfg
    W = weights_of(model, np.float64 if acc == "f64" else np.float32)
    bf = c.dtype == 1
    hd, H, Hkv = c.head_dim, c.n_q_heads, c.n_kv_heads
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    T = tok.numel()
    h = W["emb"][tok]
    for L in W["layers"]:
        a = _rnd(F.rms_norm(h, (c.d_model,), L["g1"], c.rms_eps), bf)
        q = (a @ L["wq"].T).view(T, H, hd)
        k = (a @ L["wk"].T).view(T, Hkv, hd)
        v = (a @ L["wv"].T).view(T, Hkv, hd)
        if c.qk_norm:
            q = F.rms_norm(q, (hd,), L["gq"], c.rms_eps)
            k = F.rms_norm(k, (hd,), L["gk"], c.rms_eps)
        q = _rnd(rope_complex(q, c.rope_base), bf)
        k = _rnd(rope_complex(k, c.rope_base), bf)
        v = _rnd(v, bf)
        g = H // Hkv
        kx = k.repeat_interleave(g, dim=1)
        vx = v.repeat_interleave(g, dim=1)
        att = F.scaled_dot_product_attention(q.transpose(0, 1)[None], kx.transpose(0, 1)[None],
                                             vx.transpose(0, 1)[None], is_causal=True)[0].transpose(0, 1)
        att = _rnd(att.reshape(T, H * hd), bf)
        h = h + att @ L["wo"].T
        m = _rnd(F.rms_norm(h, (c.d_model,), L["g2"], c.rms_eps), bf)
        act = _rnd(F.silu(m @ L["wg"].T) * (m @ L["wu"].T), bf)
        h = h + act @ L["wd"].T
    a = _rnd(F.rms_norm(h, (c.d_model,), W["gf"], c.rms_eps), bf)
    return (a @ W["lm"].T).numpy()
