"""Seeded synthetic inputs: token histories, draft windows, draft distributions.

These generators stand in for the prompts of the paper's benchmark suites
(Sec. 5.1 lists them), which are not available here; none of the suites' own
items appear anywhere.  The module holds no arithmetic of the method itself and
is the only code the GPU path's callers and the CPU oracle's callers share.
"""
from __future__ import annotations

import numpy as np

_M64 = (1 << 64) - 1

# Model shapes of the five workloads (layers / widths from the paper's model
# table, App. C.1; head counts, context and window sizes are this build's).
CONFIGS = {
    "tiny": dict(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=688,
                 vocab=2048, qk_norm=0, dtype=0, rms_eps=1e-5, rope_base=1e4),
    "llama1b": dict(n_layers=16, d_model=2048, n_q_heads=32, n_kv_heads=8, head_dim=64, d_ffn=8192,
                    vocab=128256, qk_norm=0, dtype=1, rms_eps=1e-5, rope_base=5e5),
    "llama70b": dict(n_layers=80, d_model=8192, n_q_heads=64, n_kv_heads=8, head_dim=128,
                     d_ffn=28672, vocab=128256, qk_norm=0, dtype=1, rms_eps=1e-5, rope_base=5e5),
    "qwen32b": dict(n_layers=64, d_model=5120, n_q_heads=64, n_kv_heads=8, head_dim=128,
                    d_ffn=25600, vocab=151936, qk_norm=1, dtype=1, rms_eps=1e-6, rope_base=1e6),
}
BASE_SEED = 20260105


def splitmix64(seed: int, n: int) -> np.ndarray:
    """n outputs of the splitmix64 stream started at `seed` (uint64)."""
    with np.errstate(over="ignore"):
        z = (np.uint64(seed & _M64) +
             np.uint64(0x9E3779B97F4A7C15) * np.arange(1, n + 1, dtype=np.uint64))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        return z ^ (z >> np.uint64(31))


def _unit(seed: int, n: int) -> np.ndarray:
    return (splitmix64(seed, n) >> np.uint64(11)).astype(np.float64) * (1.0 / (1 << 53))


def uniform_history(seed: int, length: int = 256, vocab: int = 2048, span: int = 8,
                    every: int = 32, tail: int = 4) -> np.ndarray:
    """Uniform ids; every `every` tokens a `span`-gram is copied from an earlier
    offset; the history ends `tail` tokens into one more copied span, so the
    first retrieval hits and its continuation (the rest of that span) is known."""
    r = splitmix64(seed, 3 * length + 8)
    h = (r[:length] % np.uint64(vocab)).astype(np.int32)
    j = length
    for dst in range(every, length - span - tail, every):
        src = int(r[j] % np.uint64(max(dst - span, 1)))
        j += 1
        h[dst:dst + span] = h[src:src + span]
    src = int(r[j] % np.uint64(length // 2))
    h[length - tail:] = h[src:src + tail]
    return h


def zipf_history(seed: int, length: int, vocab: int, s: float = 1.1, repeat_frac: float = 0.15,
                 span_lo: int = 16, span_hi: int = 16) -> np.ndarray:
    """Zipf(s) ids (rank -> id through a seeded permutation) with about
    `repeat_frac` of the positions inside spans copied from earlier text."""
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w)
    cdf /= cdf[-1]
    ranks = np.minimum(np.searchsorted(cdf, _unit(seed, length), side="right"), vocab - 1)
    perm = np.argsort(splitmix64(seed ^ 0x5EED, vocab), kind="stable")
    h = perm[ranks].astype(np.int32)
    r = splitmix64(seed ^ 0xC0FFEE, 4 * length + 16)
    covered = np.zeros(length, dtype=bool)
    j = 0
    target = int(repeat_frac * length)
    guard = 0
    while covered.sum() < target and guard < 8 * length:
        guard += 1
        n = span_lo + int(r[j] % np.uint64(span_hi - span_lo + 1)); j += 1
        if 2 * n + 1 >= length:
            break
        dst = n + int(r[j] % np.uint64(length - 2 * n)); j += 1
        src = int(r[j] % np.uint64(dst - n + 1)); j += 1
        if j + 3 >= r.size:
            break
        if covered[dst:dst + n].any():
            continue
        h[dst:dst + n] = h[src:src + n]
        covered[dst:dst + n] = True
    return h


def corrupt_drafts(seed: int, continuation: np.ndarray, vocab: int, alpha: float = 0.8) -> np.ndarray:
    """Drafts = a known continuation with one position, drawn Geometric(1-alpha),
    replaced by another id (so the accepted length varies over 0..len)."""
    c = np.array(continuation, dtype=np.int32)
    u = _unit(seed, 2)
    pos = int(np.floor(np.log(max(u[0], 1e-300)) / np.log(alpha)))
    if pos < c.size:
        c[pos] = (int(c[pos]) + 1 + int(u[1] * (vocab - 1))) % vocab
    return c


def dense_q(seed: int, rows: int, vocab: int, temperature: float, mix_logits=None) -> np.ndarray:
    """Draft distributions q[rows][vocab] (fp32, rows sum to 1): softmax(z/T) of
    seeded N(0, 1.5^2) scores, optionally averaged 50/50 with given logits so
    that q overlaps the target."""
    n = rows * vocab
    u1 = _unit(seed, n)
    u2 = _unit(seed ^ 0xABCDEF, n)
    z = 1.5 * np.sqrt(-2.0 * np.log(np.maximum(u1, 1e-300))) * np.cos(2 * np.pi * u2)
    z = z.reshape(rows, vocab)
    if mix_logits is not None:
        z = 0.5 * z + 0.5 * np.asarray(mix_logits, dtype=np.float64)[:rows]
    z = z / temperature
    z -= z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    return p.astype(np.float32)
