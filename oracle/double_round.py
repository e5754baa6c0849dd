"""TEST INFRASTRUCTURE ONLY -- reference orchestration of a full Double round on the oracle.

The two-model loop of the paper (Sec. 4.1 "Iterative Retrieval Drafter", "Synchronous Parallel
Execution"; Sec. 4.2 "Target-Guided Verification", Eq. 6; Alg. 1 / Alg. 2), greedy decoding and sampling,
written as plainly as possible on the oracle's sequences.  Nothing here is fast and nothing
runs concurrently: "parallel" steps are simply computed one after the other from the same
starting state, which is what makes them parallelisable.

Reading of Alg. 1 / Alg. 2 (their index ranges are garbled in places; this is the reading whose
output is token-identical to plain greedy decoding of the target, the invariant the paper states):

  state   x = text verified by the target; U = draft tokens appended after x that the target has
          not verified yet (Alg. 1's prev_tokens = |U|).  U empty <=> "pre-verify" mode, otherwise
          "post-verify".
  round   (a) target: one Retrieval Forward over  pending token + U + Y_p, where Y_p is the
              target-side retrieval (Sec. 4.2: Y_p = Retrieval(x, d)) continuing x + U; greedy
              acceptance gives E = accepted window tokens + the target's own next token.
          (b) draft, from x + U and without looking at (a): gamma chained Retrieval Forwards
              (Eq. 5), each appending the tokens the DRAFT model accepts plus its own next token;
              together X_q.
          (c) resolve.  x <- x + E always (every token of E is the target's greedy choice).
              If a token of U was rejected: U <- {} and the draft rolls back to x ("rollback
              both models").  Otherwise E = U + G with G = the part of Y_p that was accepted plus
              the target's next token: the draft's new chain X_q is checked against G (Alg. 1's
              pre-verify / Alg. 2's "check new tokens"); if X_q agrees with all of G and goes on,
              the rest of X_q becomes the new U (stay in / enter post-verify); at the first
              disagreement the target's tokens win (Eq. 6: verified draft prefix + target's
              suffix, which is x + E) and the draft rolls back.

T > 0 (Sec. 4.2 "Multi-token Pre-verify", Sec. 5.3 "Temperature Sampling", App. D.2 "Stochastic Sampling"): the same
round with the acceptance rule of speculative sampling in place of the equality test.  Every window token -- U as
well as Y_p -- is a proposal fixed before the target's randomness of this round is drawn, so it is tested as a point
proposal: kept with probability p(token), else replaced by a draw from p without that token, and nothing behind a
rejection is used (the guidance is discarded).  Conditional on the window this emits exact samples of the target,
whatever produced the window.  The draft model runs its own Retrieval Forwards the same way at the same temperature,
with its own seed, so its chain is a sample of the draft model.  Step (c) is unchanged: the tokens of E are now the
target's samples, and X_q survives only where it coincides with them.

Random numbers: an acceptance draws from Philox with the step word the caller names.  The target's acceptance of
round r uses step r; the draft's j-th Retrieval Forward of round r uses step r * gamma + j (seeds differ).
"""
import numpy as np

from . import accept_greedy, accept_sample, retrieve


def common_prefix(a, b):
    n = 0
    while n < len(a) and n < len(b) and int(a[n]) == int(b[n]):
        n += 1
    return n


def sync_to(seq, tokens):
    """Make `seq` hold `tokens` as its history with the KV of all but the last one, reusing
    whatever prefix of its cache is still valid and running the model over the rest."""
    tokens = [int(t) for t in tokens]
    keep = min(common_prefix(seq.history(), tokens), seq.kv_len, len(tokens) - 1)
    seq.truncate(kv_len=keep)
    seq.hist_set(tokens)
    rest = tokens[keep:len(tokens) - 1]
    if rest:
        seq.verify_block(rest)
        seq.commit(len(rest), [])


def padded_window(pending, tokens, k, pad_id=0):
    w = [int(pending)] + [int(t) for t in tokens[:k - 1]]
    return w + [pad_id] * (k - len(w))


def accept(logits, w, temperature, seed, step):
    """Acceptance over a padded window.  The padding tokens are proposals like any other: under the greedy rule one
    survives only if it is the model's own choice, under sampling with the probability the model gives it -- either
    way what is emitted is the model's."""
    if temperature <= 0.0:
        n, emit, _, _ = accept_greedy(logits, w)
    else:
        n, emit, _, _, _ = accept_sample(logits, w, None, temperature, seed, step, 0)
    return int(n), [int(t) for t in emit[:n + 1]]


def retrieval_forward(seq, k, n_max, n_min, d, temperature=0.0, seed=0, step=0):
    """One Retrieval Forward (Eq. 2) of the sequence's own model: retrieve, verify the window,
    keep what the model itself would have produced.  Returns the emitted tokens."""
    hist = seq.history()
    cont, cl, _, _ = retrieve(hist, n_max, n_min, min(d, k - 1)) if k > 1 else ([], 0, 0, -1)
    w = padded_window(hist[-1], cont[:cl], k)
    n, emit = accept(seq.verify_block(w), w, temperature, seed, step)
    seq.commit(n + 1, emit)
    return emit


def merge(U, E, Xq, max_u):
    """Step (c), Eq. 6.  U: the unverified drafts the target's window carried; E: what the target emitted (accepted
    window tokens + its own next token); Xq: the draft's new chain, which continues x + U.
    Returns (U_new, agree, valid): the next round's unverified drafts; how many leading tokens of Xq equal G (0 when
    a token of U was rejected); how much of the draft's text behind x (= U + Xq) is still a prefix of the new text
    x + E + U_new."""
    n = len(E) - 1                       # accepted window drafts
    if n < len(U):                       # a token of U was rejected: E = U[:n] + the target's replacement
        return [], 0, n
    G = E[len(U):]
    agree = common_prefix(Xq, G)
    if agree == len(G) and len(Xq) > len(G):
        U_new = [int(t) for t in Xq[len(G):][:max_u]]
        return U_new, agree, len(U) + len(G) + len(U_new)
    return [], agree, len(U) + agree


def double_decode(target, draft, prompt, max_new, gamma, k_p, k_q, n_max=3, n_min=1, d=10,
                  temperature=0.0, seed_target=0, seed_draft=0):
    """Decoding of `target` (an oracle Seq) helped by `draft` (an oracle Seq of another model with the same
    vocabulary): greedy, or sampling at `temperature` > 0.  Returns (new tokens, per-round records)."""
    x, U, rounds = [int(t) for t in prompt], [], []
    sync_to(target, x)
    sync_to(draft, x)
    while len(x) - len(prompt) < max_new:
        r = len(rounds)
        # (a) target: pending + U + its own retrieved guidance, padded to k_p rows
        room = k_p - 1 - len(U)
        Y = []
        if room > 0:
            cont, cl, _, _ = retrieve(np.asarray(x + U, np.int32), n_max, n_min, min(d, room))
            Y = [int(t) for t in cont[:cl]]
        W = padded_window(x[-1], U + Y, k_p)
        n, E = accept(target.verify_block(W), W, temperature, seed_target, r)
        # (b) draft: gamma chained Retrieval Forwards from x + U
        Xq = []
        for j in range(gamma):
            Xq += retrieval_forward(draft, k_q, n_max, n_min, d, temperature, seed_draft, r * gamma + j)
        # (c) resolve
        target.commit(n + 1, E)
        U_new, _, _ = merge(U, E, Xq, k_p - 1)
        rounds.append({"mode": "post" if U else "pre", "n_u": len(U), "n_acc": int(n), "emitted": len(E),
                       "drafted": len(Xq), "kept": len(U_new)})
        x = x + E
        U = U_new
        sync_to(draft, x + U)
    return x[len(prompt):], rounds


def autoregressive(seq, prompt, n_new):
    """Plain greedy decoding, one token per forward: the definition Double must reproduce."""
    x = [int(t) for t in prompt]
    sync_to(seq, x)
    out = []
    for _ in range(n_new):
        lg = seq.verify_block([x[-1]])
        t = int(np.argmax(lg[0]))
        seq.commit(1, [t])
        x.append(t)
        out.append(t)
    return out
