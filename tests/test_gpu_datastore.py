"""GPU parity of the hierarchical datastore (Alg. 3): tiered retrieval and the rejected tier's
update against the oracle, bit-exact."""
import numpy as np
import pytest
import torch

import oracle as O
from paper_2601_05524_amd import binding as B
from paper_2601_05524_amd import synth
from tests.gpu_util import Gpu, Ref

pytestmark = pytest.mark.gpu

SHAPE0 = dict(synth.CONFIGS["tiny"], n_layers=0)


def gpu_tiered(g, Bn, n_max, n_min, mc):
    cont = g.i32(Bn, mc, fill=-7)
    cl, mn, mp, mt = (g.i32(Bn, fill=-7) for _ in range(4))
    B.dbl_retrieve_tiered(g.ctx, Bn, n_max, n_min, mc, cont, cl, mn, mp, mt)
    torch.cuda.synchronize()
    return cont.cpu().numpy(), cl.cpu().numpy(), mn.cpu().numpy(), mp.cpu().numpy(), mt.cpu().numpy()


def test_tiered_retrieval_parity():
    Bn = 4
    g = Gpu(SHAPE0, seed=1, max_batch=Bn, max_ctx=64, max_window=4, max_hist=40000)
    rng = np.random.default_rng(3)
    tiers = set()
    for case in range(40):
        big = case % 8 == 7
        V = int(rng.integers(2, 7)) if not big else 300
        prior = rng.integers(0, V, int(rng.integers(0, 60)) if not big else 30000).astype(np.int32)
        if prior.size > 8:
            prior[rng.integers(0, prior.size, max(2, prior.size // 40))] = -1
        B.dbl_prior_set(g.ctx, prior)
        hists, plens = [], []
        for b in range(Bn):
            L = int(rng.integers(1, 50)) if not big else int(rng.integers(20000, 32768))
            h = rng.integers(0, V, L).astype(np.int32)
            if big:      # repeated spans, as in the long-context workload
                for _ in range(40):
                    n = int(rng.integers(8, 65)); s = int(rng.integers(0, L - n)); d = int(rng.integers(0, L - n))
                    h[d:d + n] = h[s:s + n]
            pl = int(rng.integers(0, L + 1))
            B.dbl_history_set(g.ctx, b, h)
            B.dbl_session_mark(g.ctx, b, pl)
            hists.append(h); plens.append(pl)
        n_max, mc = int(rng.integers(1, 6)), int(rng.integers(1, 11))
        cont, cl, mn, mp, mt = gpu_tiered(g, Bn, n_max, 1, mc)
        for b in range(Bn):
            # the rejected tier is empty here (filled in the next test)
            r = O.retrieve_tiered(prior, hists[b], plens[b], [], n_max, 1, mc)
            assert (cl[b], mn[b], mp[b], mt[b]) == (r[1], r[2], r[3], r[4]), (case, b)
            assert list(cont[b][:r[1]]) == list(r[0]) and (cont[b][r[1]:] == -1).all()
            tiers.add(int(mt[b]))
    assert tiers >= {0, 1, 3}
    g.close()


def test_rejected_tier_update_and_lookup_parity():
    """A zero-layer model (embedding -> norm -> LM head) decides what is accepted; windows carry
    its own next token for the first few drafts so that accepted lengths vary."""
    Bn, k = 2, 6
    g = Gpu(SHAPE0, seed=4, max_batch=Bn, max_ctx=256, max_window=k, max_hist=512)
    r = Ref(SHAPE0, seed=4, max_batch=Bn, max_ctx=256, max_hist=512)
    V = SHAPE0["vocab"]
    rng = np.random.default_rng(8)
    prompts = [rng.integers(0, 40, 12).astype(np.int32) for _ in range(Bn)]
    g.prefill(prompts, 4)
    r.prefill(prompts, 4)
    rej = [np.zeros(0, np.int32) for _ in range(Bn)]
    nd_dev = g.i32(Bn)
    seen_nonempty = False
    for step in range(24):
        ws, nds = [], []
        for b in range(Bn):
            s = r.seqs[b]
            good = int(rng.integers(0, 4))            # drafts that follow the model
            w = [int(s.history()[-1])]
            for _ in range(good):
                w.append(int(s.verify_block(w)[-1].argmax()))
            while len(w) < k:
                w.append(int(rng.integers(0, 40)))
            nds.append(int(rng.integers(good, k)))    # real drafts: the rest is padding
            ws.append(np.array(w, np.int32))
        g.verify(ws, want_logits=False)
        n_acc, emit, _ = g.accept(B.DBL_GREEDY)
        nd_dev.copy_(torch.as_tensor(np.array(nds, np.int32)))
        B.dbl_rejected_update(g.ctx, nd_dev)
        g.commit()
        for b in range(Bn):
            s = r.seqs[b]
            n_ref, e_ref, _, _ = O.accept_greedy(s.verify_block(ws[b]), ws[b])
            assert n_acc[b] == n_ref
            rej[b] = O.rejected_append(rej[b], 512, s.history(), ws[b], n_ref, nds[b], B_REJ_CTX)
            s.commit(n_ref + 1, e_ref[:n_ref + 1])
            buf = np.zeros(512, np.int32)
            n = B.dbl_rejected_get(g.ctx, b, buf)
            assert list(buf[:n]) == list(rej[b]), (step, b)
            seen_nonempty |= n > 0
        # lookups now see all tiers: no prior, generated text, rejected chains, the prompt
        cont, cl, mn, mp, mt = gpu_tiered(g, Bn, 3, 1, 5)
        for b in range(Bn):
            s = r.seqs[b]
            ref = O.retrieve_tiered([], s.history(), len(prompts[b]), rej[b], 3, 1, 5)
            assert (cl[b], mn[b], mp[b], mt[b]) == (ref[1], ref[2], ref[3], ref[4]), (step, b)
            assert list(cont[b][:ref[1]]) == list(ref[0])
    assert seen_nonempty
    B.dbl_reset(g.ctx, -1)
    assert B.dbl_rejected_get(g.ctx, 0, np.zeros(4, np.int32)) == 0
    g.close()


B_REJ_CTX = 4      # DBL_REJ_CTX of include/dbl.h
