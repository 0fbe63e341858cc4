"""DISC outer loop on the device: parity of ppv_disc_select with the oracle, and the whole method
(per-step constrained decoding with a model in the loop, then accept / reject / resample) on the
two-token construction of Theorem 2.1, whose exact output law can be enumerated."""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.stats import chisquare

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, to_dev
from test_oracle_pins import read_golden

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("K", [1, 2, 4, 8])
@pytest.mark.parametrize("reuse", [False, True])
def test_disc_select_parity(K, reuse):
    rng = np.random.default_rng(100 + K)
    Q = 20_000
    n_cand = K if reuse else 2 * K
    logx = np.log(rng.beta(1.5, 2.0, size=(n_cand, Q))).astype(np.float32)
    logx[:, :50] = -80.0 + rng.random((n_cand, 50)).astype(np.float32)          # tiny scores: always rejected
    au = rng.random((K, Q), dtype=np.float32)
    ru = rng.random(Q, dtype=np.float32)
    ch, nd, acc = oracle.disc_select(logx, K, au, ru, reuse_rejected=reuse)
    d_ch = torch.full((Q,), -3, dtype=torch.int32, device=DEV)
    d_nd = torch.full((Q,), -3, dtype=torch.int32, device=DEV)
    d_acc = torch.full((Q,), 9, dtype=torch.uint8, device=DEV)
    ppv.ppv_disc_select(to_dev(logx), K, to_dev(au), to_dev(ru), d_ch, d_nd, d_acc, reuse_rejected=reuse)
    torch.cuda.synchronize()
    g_ch, g_nd, g_acc = d_ch.cpu().numpy(), d_nd.cpu().numpy(), d_acc.cpu().numpy().astype(np.int32)
    bad = np.nonzero(g_ch != ch)[0]
    # a decision may differ only where exp(logx) and the uniform agree to the last bits of a double
    for q in bad:
        x = np.exp(logx[:K, q].astype(np.float64))
        assert (np.abs(x - au[:, q]) < 1e-12).any(), q
    assert len(bad) <= 1
    ok = g_ch == ch
    assert np.array_equal(g_nd[ok], nd[ok]) and np.array_equal(g_acc[ok], acc[ok])
    # optional outputs may be omitted
    ppv.ppv_disc_select(to_dev(logx), K, to_dev(au), to_dev(ru), d_ch, reuse_rejected=reuse)
    torch.cuda.synchronize()
    assert np.array_equal(d_ch.cpu().numpy(), g_ch)


def test_disc_end_to_end_on_theorem_2_1_toy():
    """Q queries x 2K candidates decoded by ppv_decode_step with the toy model in the loop (the second step's
    logits depend on the first sampled token), then ppv_disc_select.  The law of the returned sequence is
    (1 - r^K)/(1 - r) * P_L(a) + r^K * Qlaw(a), r = 1 - P_L(S), Qlaw enumerated over the K-tuples."""
    g = read_golden("thm21_construction.txt")
    pb, eps = g["p_b"], g["eps"]
    K, Q = 2, 60_000
    B = 2 * K * Q
    S = W.constraint_set_from_lists([[0, 0], [0, 1], [1, 0]], 2)
    index = ppv.ppv_build_index(S.tokens, S.offsets, 2)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    P = torch.full((B, 2), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    act = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ids = torch.zeros(B, dtype=torch.int32, device=DEV)
    ppv.ppv_decode_begin(index, P, lens, state, act, logx)
    buf = torch.zeros((B, 4), dtype=torch.float32, device=DEV)          # rows padded to 16 bytes
    logits = buf[:, :2]
    logits[:] = torch.log(torch.tensor([1 - pb, pb], device=DEV))
    ppv.ppv_decode_step(index, P, lens, act, logits, torch.rand(B, generator=gen, device=DEV), ids, None, logx,
                        state=state)
    second = torch.log(torch.tensor([[0.5, 0.5], [eps, 1 - eps]], device=DEV))
    logits[:] = second[ids.long()]                                       # the "model": next distribution given the token
    ppv.ppv_decode_step(index, P, lens, act, logits, torch.rand(B, generator=gen, device=DEV), ids, None, logx,
                        state=state)
    torch.cuda.synchronize()
    assert not act.any().item() and (lens == 2).all().item()
    seq_id = (P[:, 0] * 2 + P[:, 1]).cpu().numpy()                       # 0: v1v1, 1: v1v2, 2: v2v1
    assert set(np.unique(seq_id)) <= {0, 1, 2}
    # constrained decoding alone follows P^CD, with the scores the proof states
    pcd = np.array([g["pcd_v1v1"], g["pcd_v1v2"], g["pcd_v2v1"]])
    xs = np.array([g["x_v1v1"], g["x_v1v2"], g["x_v2v1"]])
    assert chisquare(np.bincount(seq_id, minlength=3), pcd * B).pvalue > 1e-4
    lx = logx.cpu().numpy()
    assert np.allclose(np.exp(lx), xs[seq_id], rtol=1e-5)
    # accept / reject / resample
    chosen = torch.zeros(Q, dtype=torch.int32, device=DEV)
    nd = torch.zeros(Q, dtype=torch.int32, device=DEV)
    acc = torch.zeros(Q, dtype=torch.uint8, device=DEV)
    ppv.ppv_disc_select(logx.view(2 * K, Q), K, torch.rand((K, Q), generator=gen, device=DEV),
                        torch.rand(Q, generator=gen, device=DEV), chosen, nd, acc)
    torch.cuda.synchronize()
    out = seq_id.reshape(2 * K, Q)[chosen.cpu().numpy(), np.arange(Q)]
    pl = pcd * xs
    r = 1 - pl.sum()
    qlaw = np.zeros(3)
    for tup in itertools.product(range(3), repeat=K):
        p = np.prod(pcd[list(tup)])
        w = xs[list(tup)]
        for j, a in enumerate(tup):
            qlaw[a] += p * w[j] / w.sum()
    law = (1 - r ** K) / (1 - r) * pl + r ** K * qlaw
    assert law.sum() == pytest.approx(1.0, abs=1e-12)
    assert chisquare(np.bincount(out, minlength=3), law * Q).pvalue > 1e-4
    # expected number of draws (Theorem 3.1 with p_b = r)
    want = (1 - r ** K) / (1 - r) + K * r ** K
    ndn = nd.cpu().numpy()
    assert abs(ndn.mean() - want) < 5 * ndn.std() / math.sqrt(Q)
    # DISC moves the law towards P_S: closer to it (in KL) than plain constrained decoding is
    ps = pl / pl.sum()
    kl = lambda p, q: float((p * np.log(p / q)).sum())
    assert kl(ps, law) < kl(ps, pcd)


def test_rows_that_cannot_draw_a_token_get_score_zero_and_are_never_returned():
    """A row whose valid tokens all have probability 0 stops outside S with logx = -inf (Algorithm 1's update
    multiplies x by a valid mass of 0), through ppv_decode_step and through ppv_decode_loop, as the oracle's loop
    says; ppv_disc_select then never returns it, and returns -1 when no candidate of a query is alive."""
    V = 4
    S = W.constraint_set_from_lists([[0, 1], [0, 2], [1, 3]], V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    B = 64
    rng = np.random.default_rng(12)
    un = rng.random((2, B), dtype=np.float32)
    first = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    after0 = np.array([0.3, -np.inf, -np.inf, 0.1], np.float32)      # both continuations of [0] have probability 0
    after1 = np.log(np.array([0.1, 0.2, 0.3, 0.4])).astype(np.float32)

    def logits_for_step(step, seqs_now, lens_now):
        if step == 0:
            return np.broadcast_to(first, (B, V)).copy()
        return np.stack([after0 if seqs_now[b, 0] == 0 else after1 for b in range(B)])
    ref = oracle.decode_loop(trie, B, logits_for_step, lambda s: un[s])
    assert ref.dead.any() and not ref.dead.all()
    step1 = logits_for_step(1, ref.seqs, ref.lens)
    lg = torch.stack([to_dev(np.broadcast_to(first, (B, V)).copy()), to_dev(step1)])
    for one_launch in (False, True):
        P = torch.full((B, 2), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        lens = torch.zeros(B, dtype=torch.int32, device=DEV)
        act = torch.zeros(B, dtype=torch.uint8, device=DEV)
        state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        logx = torch.zeros(B, dtype=torch.float32, device=DEV)
        ids = torch.full((2, B), -5, dtype=torch.int32, device=DEV)
        ppv.ppv_decode_begin(index, P, lens, state, act, logx)
        if one_launch:
            ppv.ppv_decode_loop(index, P, lens, act, lg, to_dev(un), ids, None, logx, state=state)
        else:
            for s in range(2):
                ppv.ppv_decode_step(index, P, lens, act, lg[s], to_dev(un[s]), ids[s], None, logx, state=state)
        torch.cuda.synchronize()
        glx, gl, gid = logx.cpu().numpy(), lens.cpu().numpy(), ids.cpu().numpy()
        assert not act.any().item()
        assert np.array_equal(gl, ref.lens) and np.array_equal(P.cpu().numpy()[:, 0], ref.seqs[:, 0])
        assert (glx[ref.dead] == -np.inf).all() and (gid[1][ref.dead] == -1).all()
        assert np.allclose(glx[~ref.dead], ref.logx[~ref.dead], atol=1e-5)
    # selection: 16 queries x 4 candidates (K = 2) made of these rows
    K, Q = 2, B // 4
    lx = glx.reshape(4, Q).copy()
    lx[:, 0] = -np.inf                                               # a query none of whose candidates is alive
    au = rng.random((K, Q), dtype=np.float32)
    au[:, 1::2] = 0.9999                                             # every second query goes to the fallback
    ru = rng.random(Q, dtype=np.float32)
    for reuse in (False, True):
        ch, nd, acc = oracle.disc_select(lx, K, au, ru, reuse_rejected=reuse)
        d_ch = torch.full((Q,), -3, dtype=torch.int32, device=DEV)
        d_nd = torch.full((Q,), -3, dtype=torch.int32, device=DEV)
        d_acc = torch.full((Q,), 9, dtype=torch.uint8, device=DEV)
        ppv.ppv_disc_select(to_dev(lx), K, to_dev(au), to_dev(ru), d_ch, d_nd, d_acc, reuse_rejected=reuse)
        torch.cuda.synchronize()
        g = d_ch.cpu().numpy()
        assert np.array_equal(g, ch) and np.array_equal(d_nd.cpu().numpy(), nd)
        assert np.array_equal(d_acc.cpu().numpy().astype(np.int32), acc)
        assert g[0] == -1
        alive = g >= 0
        assert np.isfinite(lx[g[alive], np.nonzero(alive)[0]]).all()
    index.free()
