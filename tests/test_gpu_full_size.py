"""Parity at the full sizes of the workload configs, in the launch configurations bench.py times:
C3 (N = 1M, V = 32k) as the whole decode loop replayed from a HIP graph, C4 (N ~ 10M, V = 1,024,
B = 4,096) and C5 (N = 5M, V = 256k, B = 1,024) as mask call + sample call.  The oracle is fast
enough here to check every row, so nothing is sampled."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, assert_query_parity, check_sample_rows, follow_loop, gpu_sample, logits_to_dev, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


_built = {}


def build_both(cfg):
    if cfg.name in _built:
        return _built[cfg.name]
    _built.clear()                                              # one full-size set at a time (host memory)
    _built[cfg.name] = _build_both(cfg)
    return _built[cfg.name]


def _build_both(cfg):
    say(f"{cfg.name}: generating S")
    S = W.make_constraint_set(cfg)
    say(f"{cfg.name}: oracle trie over {S.n} sequences")
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    say(f"{cfg.name}: device index")
    index = ppv.ppv_build_index(S.tokens, S.offsets, cfg.vocab)
    assert index.n_distinct == trie.n_members and index.l_max == trie.l_max
    assert index.n_prefixes == trie.n_nodes - 1
    return S, trie, index


def test_C3_full_decode_loop_graph():
    cfg = W.CONFIGS["C3"]
    S, trie, index = build_both(cfg)
    B, V, L = cfg.batch, cfg.vocab, index.l_max
    say("C3: logits for all steps")
    host_logits = [W.make_logits(cfg, step=s) for s in range(L)]
    host_un = [W.make_uniforms(cfg, step=s) for s in range(L)]
    logits = torch.empty((L, B, V), dtype=torch.bfloat16, device=DEV)
    uniforms = torch.empty((L, B), dtype=torch.float32, device=DEV)
    for s in range(L):
        logits[s] = logits_to_dev(cfg, host_logits[s])
        uniforms[s] = to_dev(host_un[s])
    prefixes = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    active = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ids = torch.zeros((L, B), dtype=torch.int32, device=DEV)
    lz = torch.zeros((L, B), dtype=torch.float32, device=DEV)
    step_logits = [logits[s] for s in range(L)]
    step_un = [uniforms[s] for s in range(L)]
    step_ids = [ids[s] for s in range(L)]
    step_lz = [lz[s] for s in range(L)]

    def loop():
        lens.zero_()
        ids.fill_(-5)
        ppv.ppv_decode_begin(index, prefixes, lens, state, active, logx)
        for s in range(L):
            ppv.ppv_decode_step(index, prefixes, lens, active, step_logits[s], step_un[s], step_ids[s], step_lz[s],
                                logx, state=state)

    loop()
    torch.cuda.synchronize()
    eager = [t.cpu().numpy().copy() for t in (prefixes, lens, ids, lz, logx)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        loop()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        loop()
    for rep in range(3):                       # every replay must reproduce the eager result bit for bit
        prefixes.fill_(W.PAD_TOKEN)
        logx.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in (prefixes, lens, ids, lz, logx)]
        for a, b in zip(eager, got):
            assert np.array_equal(a.view(np.int32) if a.dtype == np.float32 else a,
                                  b.view(np.int32) if b.dtype == np.float32 else b), rep
    gP, gL, gid, glz, glx = eager
    assert not active.cpu().numpy().any()

    # The batch sweep of bench.py runs the same loop on 1,024 and 4,096 rows, where a row gets 4 wavefronts instead
    # of 8.  Tiles and the order in which they are combined do not depend on that, so four replicas of this batch
    # in one launch must reproduce the 256-row result bit for bit -- per step and as one ppv_decode_loop launch.
    R = 4
    big_logits = logits.repeat(1, R, 1).contiguous()
    big_un = uniforms.repeat(1, R).contiguous()
    for single_launch in (False, True):
        bp = torch.full((B * R, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        bl = torch.zeros(B * R, dtype=torch.int32, device=DEV)
        ba = torch.zeros(B * R, dtype=torch.uint8, device=DEV)
        bs = torch.zeros((B * R, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        bx = torch.zeros(B * R, dtype=torch.float32, device=DEV)
        bid = torch.full((L, B * R), -5, dtype=torch.int32, device=DEV)
        blz = torch.zeros((L, B * R), dtype=torch.float32, device=DEV)
        ppv.ppv_decode_begin(index, bp, bl, bs, ba, bx)
        if single_launch:
            ppv.ppv_decode_loop(index, bp, bl, ba, big_logits, big_un, bid, blz, bx, state=bs)
        else:
            for s in range(L):
                ppv.ppv_decode_step(index, bp, bl, ba, big_logits[s], big_un[s], bid[s], blz[s], bx, state=bs)
        torch.cuda.synchronize()
        for r in range(R):
            rows = slice(r * B, (r + 1) * B)
            assert np.array_equal(bp[rows].cpu().numpy(), gP) and np.array_equal(bl[rows].cpu().numpy(), gL)
            assert np.array_equal(bid[:, rows].cpu().numpy(), gid), (single_launch, r)
            on = gid >= 0
            assert np.array_equal(blz[:, rows].cpu().numpy().view(np.int32)[on], glz.view(np.int32)[on])
            assert np.array_equal(bx[rows].cpu().numpy().view(np.int32), glx.view(np.int32))
    del big_logits, big_un

    say("C3: oracle loop")
    # the oracle makes its own choice at every step (recorded) but is kept on the HIP path's sequence, so
    # that a disagreement inside the CDF band at one step does not invalidate the comparison of later steps
    res = follow_loop(trie, B, lambda s, *_: W.logits_as_f32(cfg, host_logits[s]), lambda s: host_un[s],
                      lambda s: gid[s], threads=16)
    say("C3: comparing")
    excused = 0
    for s in range(res.steps):
        rows = np.nonzero(res.active_per_step[s])[0]
        assert (gid[s][~res.active_per_step[s]] == -5).all()

        class Sub:
            pass
        sub = Sub()
        sub.ids = res.ids_per_step[s][rows]
        sub.logZ_valid = res.logZ_per_step[s][rows]
        sub.logZ_all = None
        sub.cdf_lo = res.cdf_lo_per_step[s][rows]
        sub.cdf_hi = res.cdf_hi_per_step[s][rows]
        masks = {}

        def mask_of(i, s=s, rows=rows, masks=masks):
            if i not in masks:
                masks[i] = trie.query(res.seqs[rows[i]:rows[i] + 1], np.array([s], np.int32)).mask[0]
            return masks[i]
        excused += check_sample_rows(cfg.dtype, sub, mask_of, host_un[s][rows], gid[s][rows], glz[s][rows], None,
                                     rows=rows)
    for s in range(res.steps, L):
        assert (gid[s] == -5).all()
    assert np.array_equal(gL, res.lens)
    for b in range(B):
        assert np.array_equal(gP[b, :res.lens[b]], res.seqs[b, :res.lens[b]])
    assert np.allclose(glx, res.logx, rtol=1e-3, atol=1e-3)
    say(f"C3: {int(res.lens.sum())} prefix-steps compared, {excused} inside the CDF band")
    assert excused <= 0.01 * res.lens.sum()
    # every finished row is a member of S
    q = trie.query(gP, gL, want_mask=False)
    assert (q.member == 1).all()


@pytest.mark.parametrize("B", [4096, 16384])
def test_C3_decode_loop_at_the_batch_sizes_of_the_sweep(B):
    """bench.py's batch sweep runs the C3 decode loop on 4,096 and 16,384 rows (four wavefronts per row, several
    rows per compute unit).  Here the same launches are checked against the oracle: at six decode steps the logits
    come from the host generator and a few hundred active rows are compared (ids, log masses) with the oracle's step
    on the rows' prefixes at that point; the other steps run on logits drawn on the device, as in the sweep.  At the
    end every row must be a member of S whose tokens are all valid continuations."""
    cfg = W.CONFIGS["C3"]
    S, trie, index = build_both(cfg)
    V, L = cfg.vocab, index.l_max
    checked = (0, 1, 2, 4, 8, 14)
    n_rows = 400 if B == 4096 else 150
    gen = torch.Generator(device=DEV)
    gen.manual_seed(900 + B)
    rng = np.random.default_rng(B)
    P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    act = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ids = torch.zeros(B, dtype=torch.int32, device=DEV)
    lz = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.ppv_decode_begin(index, P, lens, state, act, logx)
    excused = compared = 0
    for s in range(L):
        on = act.cpu().numpy().astype(bool)
        if not on.any():
            break
        un = torch.rand(B, generator=gen, device=DEV)
        if s in checked:
            say(f"C3, B = {B}: step {s}, host logits")
            rows = np.nonzero(on)[0]
            rows = np.sort(rng.choice(rows, min(n_rows, len(rows)), replace=False))
            host = np.zeros((B, V), np.uint16)                   # rows that are not compared keep logit 0
            piece = W.make_logits(cfg, batch=len(rows), step=700 + s)
            host[rows] = piece
            lg = to_dev(host.view(np.int16)).view(torch.bfloat16)
            before_P, before_L = P.cpu().numpy()[rows], lens.cpu().numpy()[rows]
        else:
            lg = (torch.randn((B, V), generator=gen, device=DEV) * cfg.sigma).to(torch.bfloat16)
        ids.fill_(-5)
        ppv.ppv_decode_step(index, P, lens, act, lg, un, ids, lz, logx, state=state)
        torch.cuda.synchronize()
        if s in checked:
            unh = un.cpu().numpy()[rows]
            ref = trie.step(before_P, before_L, W.logits_as_f32(cfg, piece), unh, want_mask=True, threads=16)
            excused += check_sample_rows(cfg.dtype, ref, lambda i: ref.mask[i], unh, ids.cpu().numpy()[rows],
                                         lz.cpu().numpy()[rows], None, rows=rows)
            compared += len(rows)
        del lg
    assert not act.any().item()
    gP, gL = P.cpu().numpy(), lens.cpu().numpy()
    say(f"C3, B = {B}: {compared} prefix-steps compared with the oracle, {excused} inside the CDF band; membership of all rows")
    assert excused <= 0.01 * compared and compared >= 5 * n_rows // 2
    q = trie.query(gP, gL, want_mask=False, threads=16)
    assert (q.member == 1).all() and (gL >= 4).all()
    assert np.isfinite(logx.cpu().numpy()).all()


def test_C3_one_launch_loop_in_a_batch_above_1024_rows():
    """ppv_decode_loop picks another launch shape for batches above 1,024 rows (two wavefronts per row, the three-tile
    pipeline inside the loop kernel).  It must give, bit for bit, what one ppv_decode_step per step gives on the same
    logits -- whose results at such batch sizes are checked against the oracle in the test above."""
    cfg = W.CONFIGS["C3"]
    S, trie, index = build_both(cfg)
    V, L, B = cfg.vocab, index.l_max, 2048
    gen = torch.Generator(device=DEV)
    gen.manual_seed(77)
    logits = torch.empty((L, B, V), dtype=torch.bfloat16, device=DEV)
    for s in range(L):
        logits[s] = (torch.randn((B, V), generator=gen, device=DEV) * cfg.sigma).to(torch.bfloat16)
    un = torch.rand((L, B), generator=gen, device=DEV)

    def fresh():
        P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        lens = torch.zeros(B, dtype=torch.int32, device=DEV)
        act = torch.zeros(B, dtype=torch.uint8, device=DEV)
        state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        logx = torch.zeros(B, dtype=torch.float32, device=DEV)
        ids = torch.full((L, B), -7, dtype=torch.int32, device=DEV)
        lz = torch.full((L, B), 7.0, dtype=torch.float32, device=DEV)
        ppv.ppv_decode_begin(index, P, lens, state, act, logx)
        return P, lens, act, state, logx, ids, lz

    say("C3, B = 2048: one launch per step")
    P1, l1, a1, s1, x1, i1, z1 = fresh()
    for s in range(L):
        i1[s] = -7
        on = a1.clone()
        ppv.ppv_decode_step(index, P1, l1, a1, logits[s], un[s], i1[s], z1[s], x1, state=s1)
        i1[s][on == 0] = -7                                      # the loop kernel leaves retired rows' entries alone
        z1[s][on == 0] = 7.0
    say("C3, B = 2048: one launch for the loop")
    P2, l2, a2, s2, x2, i2, z2 = fresh()
    ppv.ppv_decode_loop(index, P2, l2, a2, logits, un, i2, z2, x2, state=s2)
    torch.cuda.synchronize()
    assert not a1.any().item() and not a2.any().item()
    assert torch.equal(P1, P2) and torch.equal(l1, l2)
    assert torch.equal(x1.view(torch.int32), x2.view(torch.int32))
    assert torch.equal(i1, i2)
    assert torch.equal(z1.view(torch.int32), z2.view(torch.int32))
    q = trie.query(P2.cpu().numpy(), l2.cpu().numpy(), want_mask=False, threads=16)
    assert (q.member == 1).all()


@pytest.mark.parametrize("name", ["C4", "C5"])
def test_full_size_mask_and_sample(name):
    cfg = W.CONFIGS[name]
    S, trie, index = build_both(cfg)
    pb = W.make_prefix_batch(cfg, S)
    say(f"{name}: masks / ranges / membership, B = {cfg.batch}")
    dmask, ref_q = assert_query_parity(index, trie, pb.prefixes, pb.lens, threads=16)
    say(f"{name}: logits")
    logits = W.make_logits(cfg)
    un = W.make_uniforms(cfg)
    say(f"{name}: oracle step")
    ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, want_mask=False, threads=16)
    say(f"{name}: HIP sample")
    ids, lzv, lza = gpu_sample(cfg, logits_to_dev(cfg, logits), dmask, un)
    ex = check_sample_rows(cfg.dtype, ref, lambda b: ref_q.mask[b], un, ids, lzv, lza)
    say(f"{name}: done, {ex} rows inside the CDF band")
    say(f"{name}: the same in one call, no mask written (ppv_sample_next)")
    B = cfg.batch
    ids1 = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv1 = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    ppv.ppv_sample_next(index, to_dev(pb.prefixes), to_dev(pb.lens), logits_to_dev(cfg, logits), to_dev(un), ids1, lzv1)
    torch.cuda.synchronize()
    ex1 = check_sample_rows(cfg.dtype, ref, lambda b: ref_q.mask[b], un, ids1.cpu().numpy(), lzv1.cpu().numpy(), None)
    say(f"{name}: done, {ex1} rows inside the CDF band")
    n_valid = int((ref.ids >= 0).sum())
    assert n_valid >= cfg.batch * cfg.valid_frac * 0.9
