"""Parity of the HIP path (through the C-ABI) with the CPU oracle, element by element, at sizes
the oracle finishes in seconds that still span several tiles and a ragged tail; plus edge cases."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import (DEV, assert_query_parity, check_sample_rows, follow_loop, gpu_query, gpu_sample, logits_to_dev,
                         to_dev, tuning, unpack_mask)

pytestmark = pytest.mark.gpu

# (config, |S|, batch): the five workload recipes, the larger ones scaled down
CASES = {
    "C1": (W.CONFIGS["C1"], 1_000, 16),
    "C2": (W.CONFIGS["C2"], 100_000, 64),
    "C3s": (W.CONFIGS["C3"], 60_000, 96),
    "C4s": (W.CONFIGS["C4"], 300_000, 512),
    "C5s": (W.CONFIGS["C5"], 80_000, 48),
}

_cache = {}


def setup_case(name):
    if name not in _cache:
        base, n, batch = CASES[name]
        cfg = W.scaled(base, n, batch, name=name)
        S = W.make_constraint_set(cfg)
        trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
        index = ppv.ppv_build_index(S.tokens, S.offsets, cfg.vocab)
        _cache[name] = (cfg, S, trie, index)
    return _cache[name]


@pytest.mark.parametrize("name", list(CASES))
def test_index_is_sorted_deduplicated_S(name):
    cfg, S, trie, index = setup_case(name)
    assert index.n_distinct == trie.n_members and index.l_max == trie.l_max and index.vocab == cfg.vocab
    assert index.n_prefixes == trie.n_nodes - 1
    tok, off = ppv.ppv_index_export(index)
    assert off[0] == 0 and off[-1] == tok.shape[0] and (np.diff(off) > 0).all()
    # rows strictly increasing in lexicographic order (prefix first): compare neighbours column by column
    n = index.n_distinct
    L = index.l_max
    M = np.full((n, L), -1, dtype=np.int64)
    lens = np.diff(off)
    M[np.arange(L)[None, :] < lens[:, None]] = tok
    a, b = M[:-1], M[1:]
    diff = a != b
    assert diff.any(axis=1).all(), "duplicate rows"
    first = diff.argmax(axis=1)
    r = np.arange(n - 1)
    assert (a[r, first] < b[r, first]).all(), "rows out of order"
    # same multiset of rows as the generator's S (S has no duplicates)
    if n <= 120_000:
        assert sorted(map(bytes, M.astype(np.int32))) == sorted(map(bytes, S.padded(-1)))


def test_index_build_with_duplicates_and_nesting():
    """Small alphabet, short ragged rows: many duplicates, many members that are prefixes of others.
    The exported rows must be exactly sorted(set(S)) in the order of Section 3.2 "Array Preparation"."""
    rng = np.random.default_rng(21)
    V = 5
    seqs = [rng.integers(0, V, size=int(rng.integers(1, 9))).tolist() for _ in range(30_000)]
    S = W.constraint_set_from_lists(seqs, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    want = sorted(set(map(tuple, seqs)))                       # tuple order: left to right, prefix first
    tok, off = ppv.ppv_index_export(index)
    got = [tuple(tok[off[i]:off[i + 1]].tolist()) for i in range(index.n_distinct)]
    assert got == want
    prefixes = {s[:k] for s in want for k in range(1, len(s) + 1)}
    assert index.n_prefixes == len(prefixes) and index.l_max == max(map(len, want))
    trie = oracle.Trie(S.tokens, S.offsets, V)
    q = [list(p) for p in list(prefixes)[:500]] + [list(p) + [4] for p in list(prefixes)[:200]] + [[]]
    stride = max(map(len, q))
    P = np.full((len(q), stride), W.PAD_TOKEN, np.int32)
    L = np.array([len(x) for x in q], np.int32)
    for i, x in enumerate(q):
        P[i, :len(x)] = x
    assert_query_parity(index, trie, P, L)


@pytest.mark.parametrize("name", list(CASES))
def test_mask_range_member_parity(name):
    cfg, S, trie, index = setup_case(name)
    for it in range(2):
        pb = W.make_prefix_batch(cfg, S, index=it)
        assert_query_parity(index, trie, pb.prefixes, pb.lens)


@pytest.mark.parametrize("name", list(CASES))
def test_constrained_sample_parity(name):
    cfg, S, trie, index = setup_case(name)
    pb = W.make_prefix_batch(cfg, S, index=3)
    dmask, _ = assert_query_parity(index, trie, pb.prefixes, pb.lens)
    logits = W.make_logits(cfg, step=3)
    un = W.make_uniforms(cfg, step=3)
    ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8)
    ids, lzv, lza = gpu_sample(cfg, logits_to_dev(cfg, logits), dmask, un)
    check_sample_rows(cfg.dtype, ref, lambda b: ref.mask[b], un, ids, lzv, lza)
    assert (lzv <= 1e-6).all()


@pytest.mark.parametrize("temperature", [0.05, 0.5, 1.7, 8.0, 100.0])
@pytest.mark.parametrize("name", list(CASES))
def test_constrained_sample_parity_with_temperature(name, temperature):
    """P = softmax(logits / T) (Algorithm 1's input T): masses, samples and logZ_all against the oracle at T != 1, and
    T = 1 passed explicitly gives bit for bit what the default gives."""
    cfg, S, trie, index = setup_case(name)
    pb = W.make_prefix_batch(cfg, S, index=5)
    dmask, _ = assert_query_parity(index, trie, pb.prefixes, pb.lens)
    logits = W.make_logits(cfg, step=5)
    un = W.make_uniforms(cfg, step=5)
    ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8, temperature=temperature)
    dl = logits_to_dev(cfg, logits)
    ids, lzv, lza = gpu_sample(cfg, dl, dmask, un, temperature=temperature)
    check_sample_rows(cfg.dtype, ref, lambda b: ref.mask[b], un, ids, lzv, lza)
    assert (lzv <= 1e-6).all()
    a, b = gpu_sample(cfg, dl, dmask, un), gpu_sample(cfg, dl, dmask, un, temperature=1.0)
    assert all(np.array_equal(x.view(np.int32), y.view(np.int32)) for x, y in zip(a, b))
    ref1 = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8)
    fin = np.isfinite(ref.logZ_valid)
    assert not np.allclose(ref.logZ_valid[fin], ref1.logZ_valid[fin])          # the temperature does something
    with pytest.raises(ppv.PPVError):
        gpu_sample(cfg, dl, dmask, un, temperature=0.0)


@pytest.mark.parametrize("name", ["C1", "C2", "C3s"])
def test_decode_step_equals_mask_plus_sample(name):
    cfg, S, trie, index = setup_case(name)
    pb = W.make_prefix_batch(cfg, S, index=5)
    B = pb.prefixes.shape[0]
    stride = pb.stride + 1                                   # room to append
    P = np.full((B, stride), W.PAD_TOKEN, np.int32)
    P[:, :pb.stride] = pb.prefixes
    logits = W.make_logits(cfg, step=5)
    un = W.make_uniforms(cfg, step=5)
    active = np.ones(B, np.uint8)
    active[1::7] = 0
    ref = trie.step(P, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8)
    dP, dL, dA = to_dev(P), to_dev(pb.lens), to_dev(active)
    ids = torch.full((B,), -9, dtype=torch.int32, device=DEV)
    lz = torch.full((B,), 5.0, dtype=torch.float32, device=DEV)
    logx = torch.full((B,), 0.25, dtype=torch.float32, device=DEV)
    ppv.ppv_decode_step(index, dP, dL, dA, logits_to_dev(cfg, logits), to_dev(un), ids, lz, logx)
    torch.cuda.synchronize()
    gP, gL, gA, gid, glz, glx = (t.cpu().numpy() for t in (dP, dL, dA, ids, lz, logx))
    on = active == 1
    # inactive rows untouched
    assert np.array_equal(gP[~on], P[~on]) and np.array_equal(gL[~on], pb.lens[~on])
    assert (gid[~on] == -9).all() and (glz[~on] == 5.0).all() and (glx[~on] == 0.25).all() and (gA[~on] == 0).all()
    rows = np.nonzero(on)[0]

    class Sub:
        pass
    sub = Sub()
    for k in ("ids", "logZ_valid", "logZ_all", "cdf_lo", "cdf_hi"):
        setattr(sub, k, getattr(ref, k)[rows])
    check_sample_rows(cfg.dtype, sub, lambda i: ref.mask[rows[i]], un[rows], gid[rows], glz[rows], None, rows=rows)
    for b in rows:
        if gid[b] < 0:
            assert gL[b] == pb.lens[b] and gA[b] == 0 and np.array_equal(gP[b], P[b]) and glx[b] == -np.inf
            continue
        assert gL[b] == pb.lens[b] + 1 and gP[b, pb.lens[b]] == gid[b]
        assert np.array_equal(np.delete(gP[b], pb.lens[b]), np.delete(P[b], pb.lens[b]))
        assert glx[b] == np.float32(0.25) + glz[b]
    # membership of the extended rows decides `active`
    ext = rows[gid[rows] >= 0]
    q = trie.query(gP[ext], gL[ext], want_mask=False)
    assert np.array_equal(gA[ext], (q.member == 0).astype(np.uint8))


@pytest.mark.parametrize("use_state,temperature", [(False, 1.0), (True, 1.0), (True, 0.6), (False, 2.5)])
def test_decode_loop_parity_small(use_state, temperature):
    """Algorithm 1's SampleCandidate loop on a scaled C3, step by step against the oracle's loop,
    with the cursor kept by ppv_decode_begin/ppv_decode_step and without it, at several temperatures."""
    cfg, S, trie, index = setup_case("C3s")
    B = 64
    stride = index.l_max
    dP = torch.full((B, stride), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    dL = torch.zeros(B, dtype=torch.int32, device=DEV)
    dA = torch.ones(B, dtype=torch.uint8, device=DEV)
    logx = torch.full((B,), 9.0, dtype=torch.float32, device=DEV)
    state = None
    if use_state:
        state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        dA.zero_()
        ppv.ppv_decode_begin(index, dP, dL, state, dA, logx)
    else:
        logx.zero_()
    ids = torch.zeros(B, dtype=torch.int32, device=DEV)
    lz = torch.zeros(B, dtype=torch.float32, device=DEV)
    gpu_ids, gpu_lz = [], []
    lg = lambda s, *_: W.logits_as_f32(cfg, W.make_logits(cfg, batch=B, step=100 + s))
    un = lambda s: W.make_uniforms(cfg, batch=B, step=100 + s)
    all_ids = []
    for s in range(index.l_max):
        act_before = dA.cpu().numpy().astype(bool)
        if not act_before.any():
            break
        ids.fill_(-5)
        ppv.ppv_decode_step(index, dP, dL, dA, logits_to_dev(cfg, W.make_logits(cfg, batch=B, step=100 + s)),
                            to_dev(un(s)), ids, lz, logx, state=state, temperature=temperature)
        torch.cuda.synchronize()
        all_ids.append((act_before, ids.cpu().numpy(), lz.cpu().numpy()))
    # the oracle makes its own choice at every step but is kept on the HIP path's sequence
    res = follow_loop(trie, B, lg, un, lambda s: all_ids[s][1], threads=8, temperature=temperature)
    assert res.steps == len(all_ids)
    excused = 0
    for s in range(res.steps):
        act_before, gid, glz = all_ids[s]
        assert np.array_equal(act_before, res.active_per_step[s]), s
        rows = np.nonzero(act_before)[0]
        q = trie.query(res.seqs[rows], np.full(len(rows), s, np.int32))   # oracle masks of this step's prefixes

        class Sub:
            pass
        sub = Sub()
        sub.ids = res.ids_per_step[s][rows]
        sub.logZ_valid = res.logZ_per_step[s][rows]
        sub.logZ_all = None
        sub.cdf_lo = res.cdf_lo_per_step[s][rows]
        sub.cdf_hi = res.cdf_hi_per_step[s][rows]
        excused += check_sample_rows(cfg.dtype, sub, lambda i: q.mask[i], un(s)[rows], gid[rows], glz[rows], None,
                                     rows=rows)
    assert excused <= 2
    assert not dA.cpu().numpy().any()
    assert np.array_equal(dL.cpu().numpy(), res.lens)
    gP = dP.cpu().numpy()
    for b in range(B):
        assert np.array_equal(gP[b, :res.lens[b]], res.seqs[b, :res.lens[b]])
    assert np.allclose(logx.cpu().numpy(), res.logx, rtol=1e-3, atol=1e-3)


@pytest.mark.parametrize("name,B,temperature", [("C3s", 96, 1.0), ("C1", 16, 1.0), ("C2", 64, 1.0), ("C3s", 40, 1.7)])
def test_decode_loop_launch_equals_single_steps(name, B, temperature):
    """ppv_decode_loop (one launch for all steps) gives bit for bit what the same number of
    ppv_decode_step calls give: tokens, lengths, flags, cursor, per-step ids / masses, logx."""
    cfg, S, trie, index = setup_case(name)
    L = index.l_max
    logits = torch.stack([logits_to_dev(cfg, W.make_logits(cfg, batch=B, step=200 + s)) for s in range(L)])
    un = torch.stack([to_dev(W.make_uniforms(cfg, batch=B, step=200 + s)) for s in range(L)])
    outs = []
    for use_loop in (False, True):
        P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        lens = torch.zeros(B, dtype=torch.int32, device=DEV)
        act = torch.zeros(B, dtype=torch.uint8, device=DEV)
        state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        logx = torch.zeros(B, dtype=torch.float32, device=DEV)
        ids = torch.full((L, B), -5, dtype=torch.int32, device=DEV)
        lz = torch.full((L, B), 2.0, dtype=torch.float32, device=DEV)
        ppv.ppv_decode_begin(index, P, lens, state, act, logx)
        if use_loop:
            ppv.ppv_decode_loop(index, P, lens, act, logits, un, ids, lz, logx, state=state, temperature=temperature)
        else:
            for s in range(L):
                ppv.ppv_decode_step(index, P, lens, act, logits[s], un[s], ids[s], lz[s], logx, state=state,
                                    temperature=temperature)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (P, lens, act, ids, lz.view(torch.int32), logx.view(torch.int32))]
                    + [state.cpu().numpy()[:, :4]])            # the cursor proper (the rest is its look-ahead cache)
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    assert not outs[0][2].any() and (outs[0][1] > 0).all()
    # a second launch on finished rows changes nothing; a launch of fewer steps than needed can be resumed
    P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    act = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.ppv_decode_begin(index, P, lens, state, act, logx)
    half = max(1, L // 3)
    ppv.ppv_decode_loop(index, P, lens, act, logits[:half], un[:half], None, None, logx, state=state, temperature=temperature)
    ppv.ppv_decode_loop(index, P, lens, act, logits[half:], un[half:], None, None, logx, state=state, temperature=temperature)
    torch.cuda.synchronize()
    assert np.array_equal(P.cpu().numpy(), outs[0][0]) and np.array_equal(lens.cpu().numpy(), outs[0][1])
    assert np.array_equal(logx.view(torch.int32).cpu().numpy(), outs[0][5])


def test_decode_begin_from_given_prefixes():
    """Resuming from arbitrary prefixes: active = (prefix of a member) and not (member); one step with
    the cursor equals one step without it."""
    cfg, S, trie, index = setup_case("C2")
    pb = W.make_prefix_batch(cfg, S, index=11)
    B = pb.prefixes.shape[0]
    full = [S.seq(i) for i in range(0, 40, 5)]                 # add some whole members (member => inactive)
    P = np.full((B + len(full), pb.stride + 1), W.PAD_TOKEN, np.int32)
    L = np.zeros(B + len(full), np.int32)
    P[:B, :pb.stride] = pb.prefixes
    L[:B] = pb.lens
    for i, q in enumerate(full):
        P[B + i, :len(q)] = q
        L[B + i] = len(q)
    n = B + len(full)
    ref = trie.query(P, L, want_mask=False)
    outs = []
    logits = W.make_logits(cfg, batch=n, step=12)
    un = W.make_uniforms(cfg, batch=n, step=12)
    for use_state in (True, False):
        dP, dL = to_dev(P), to_dev(L)
        dA = torch.full((n,), 3, dtype=torch.uint8, device=DEV)
        logx = torch.full((n,), 4.0, dtype=torch.float32, device=DEV)
        state = torch.zeros((n, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        ppv.ppv_decode_begin(index, dP, dL, state, dA, logx)
        torch.cuda.synchronize()
        want_active = ((ref.hi > ref.lo) & (ref.member == 0)).astype(np.uint8)
        assert np.array_equal(dA.cpu().numpy(), want_active)
        assert (logx.cpu().numpy() == 0).all()
        ids = torch.full((n,), -9, dtype=torch.int32, device=DEV)
        lz = torch.full((n,), 5.0, dtype=torch.float32, device=DEV)
        ppv.ppv_decode_step(index, dP, dL, dA, logits_to_dev(cfg, logits), to_dev(un), ids, lz, logx,
                            state=state if use_state else None)
        torch.cuda.synchronize()
        outs.append([t.cpu().numpy() for t in (dP, dL, dA, ids, lz, logx)])
    for a, b in zip(*outs):
        assert np.array_equal(a, b)
    assert (outs[0][3][want_active == 0] == -9).all() and (outs[0][3][want_active == 1] >= 0).all()


@pytest.mark.parametrize("name", ["C1", "C2", "C3s", "C4s", "C5s"])
def test_decode_begin_empty_is_decode_begin_on_empty_prefixes(name):
    """ppv_decode_begin_empty writes, without reading any prefix, what ppv_decode_begin writes for lens = 0: the same
    cursor words, flags and scores bit for bit, and the lengths; a decode step from either state gives the same rows."""
    cfg, S, trie, index = setup_case(name)
    B = 37
    L = max(index.l_max, 1)
    P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    outs = []
    logits = logits_to_dev(cfg, W.make_logits(cfg, batch=B, step=3))
    un = to_dev(W.make_uniforms(cfg, batch=B, step=3))
    for empty in (False, True):
        lens = torch.full((B,), 0 if not empty else 5, dtype=torch.int32, device=DEV)
        state = torch.full((B, ppv.PPV_STATE_WORDS), -7, dtype=torch.int32, device=DEV)
        act = torch.full((B,), 3, dtype=torch.uint8, device=DEV)
        logx = torch.full((B,), 4.0, dtype=torch.float32, device=DEV)
        if empty:
            ppv.ppv_decode_begin_empty(index, lens, state, act, logx)
        else:
            ppv.ppv_decode_begin(index, P, lens, state, act, logx)
        torch.cuda.synchronize()
        first = [t.clone() for t in (lens, state, act, logx)]
        rows = P.clone()
        ids = torch.full((B,), -9, dtype=torch.int32, device=DEV)
        lz = torch.full((B,), 5.0, dtype=torch.float32, device=DEV)
        ppv.ppv_decode_step(index, rows, lens, act, logits, un, ids, lz, logx, state=state)
        torch.cuda.synchronize()
        outs.append(first + [rows, lens, state, act, logx, ids, lz])
    for a, b in zip(*outs):
        assert torch.equal(a.view(torch.int32) if a.dtype == torch.float32 else a,
                           b.view(torch.int32) if b.dtype == torch.float32 else b)
    assert (outs[1][0] == 0).all() and (outs[1][2] == 1).all() and (outs[1][3] == 0).all()
    assert (outs[1][9] >= 0).all()                            # every row drew a token from the root's valid set


@pytest.mark.parametrize("name", ["C1", "C2", "C3s", "C4s", "C5s"])
@pytest.mark.parametrize("temperature", [1.0, 1.7])
def test_decode_first_step_is_begin_empty_plus_step(name, temperature):
    """ppv_decode_first_step = ppv_decode_begin_empty + ppv_decode_step in one launch: every output bit for bit, on rows
    whose buffers hold junk before the call (nothing of them may be read); one row is given logits of -inf only, so
    that it stops outside S in its first step."""
    cfg, S, trie, index = setup_case(name)
    B = 41
    L = max(index.l_max, 1)
    lg = W.make_logits(cfg, batch=B, step=5)
    if cfg.dtype == "bf16":
        lg[7, :] = 0xFF80
    else:
        lg[7, :] = -np.inf
    logits = logits_to_dev(cfg, lg)
    un = to_dev(W.make_uniforms(cfg, batch=B, step=5))
    outs = []
    for fused in (False, True):
        P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        lens = torch.full((B,), 9, dtype=torch.int32, device=DEV)
        state = torch.full((B, ppv.PPV_STATE_WORDS), -7, dtype=torch.int32, device=DEV)
        act = torch.full((B,), 0 if fused else 3, dtype=torch.uint8, device=DEV)
        logx = torch.full((B,), 4.0, dtype=torch.float32, device=DEV)
        ids = torch.full((B,), -9, dtype=torch.int32, device=DEV)
        lz = torch.full((B,), 5.0, dtype=torch.float32, device=DEV)
        if fused:
            ppv.ppv_decode_first_step(index, P, lens, act, logits, un, ids, lz, logx, state=state, temperature=temperature)
        else:
            ppv.ppv_decode_begin_empty(index, lens, state, act, logx)
            ppv.ppv_decode_step(index, P, lens, act, logits, un, ids, lz, logx, state=state, temperature=temperature)
        torch.cuda.synchronize()
        outs.append([P, lens, state, act, logx.view(torch.int32), ids, lz.view(torch.int32)])
    for a, b in zip(*outs):
        assert torch.equal(a, b)
    assert outs[1][5][7].item() == -1 and outs[1][3][7].item() == 0 and outs[1][1][7].item() == 0
    assert (outs[1][5][:7] >= 0).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_row_cut_out_of_a_padded_buffer(dtype):
    """A batch of one row whose vocabulary is no multiple of a 16-byte group, given as a slice of a padded buffer: the
    binding passes the buffer's row stride (which is what says the padding is there), not the vocabulary, and the
    sampling calls take it; values behind the row's end (+inf here) are never read as logits."""
    V = 2049
    rng = np.random.default_rng(3)
    seqs = [[int(v)] for v in rng.choice(V, size=300, replace=False)] + [[5, 7], [5, 2048]]
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    per = 8 if dtype == "bf16" else 4
    Vp = (V + per - 1) // per * per
    lg = rng.normal(0, 2, size=(1, V)).astype(np.float32)
    if dtype == "bf16":
        bits = W.f32_to_bf16_bits(lg)
        lf = W.bf16_bits_to_f32(bits)
        pad = np.full((1, Vp), 0x7F80, np.uint16)
        pad[:, :V] = bits
        ld = to_dev(pad.view(np.int16)).view(torch.bfloat16)[:, :V]
    else:
        lf = lg
        pad = np.full((1, Vp), np.inf, np.float32)
        pad[:, :V] = lg
        ld = to_dev(pad)[:, :V]
    for prefix in ([], [5]):
        P = np.full((1, 2), W.PAD_TOKEN, np.int32)
        P[0, :len(prefix)] = prefix
        Ln = np.array([len(prefix)], np.int32)
        un = np.array([0.37], np.float32)
        ref = trie.step(P, Ln, lf, un, want_mask=True)
        dmask = torch.zeros((1, index.n_words), dtype=torch.int32, device=DEV)
        ppv.ppv_next_token_mask(index, to_dev(P), to_dev(Ln), dmask)
        ids = torch.full((1,), -9, dtype=torch.int32, device=DEV)
        lz = torch.zeros(1, device=DEV)
        la = torch.zeros(1, device=DEV)
        ppv.constrained_sample(ld, dmask, to_dev(un), ids, lz, la)
        ids1 = torch.full((1,), -9, dtype=torch.int32, device=DEV)
        lz1 = torch.zeros(1, device=DEV)
        ppv.ppv_sample_next(index, to_dev(P), to_dev(Ln), ld, to_dev(un), ids1, lz1)
        torch.cuda.synchronize()
        check_sample_rows(dtype, ref, lambda b: ref.mask[b], un, ids.cpu().numpy(), lz.cpu().numpy(), la.cpu().numpy())
        check_sample_rows(dtype, ref, lambda b: ref.mask[b], un, ids1.cpu().numpy(), lz1.cpu().numpy())
    index.free()


# ------------------------------------------------------------------------------------------ edge cases
def brute_rows(S_lists, V, prefixes):
    from test_oracle_pins import brute
    return [brute(S_lists, V, p) for p in prefixes]


def test_adversarial_set_vs_bruteforce_and_oracle():
    V = 70
    Sl = [[5, 6, 7], [5, 6], [5, 6, 7, 69], [5, 6, 7, 0], [69], [0], [5, 6, 7, 69],
          [1, 1, 1, 1, 1, 1, 1, 2], [1, 1, 1, 1, 1, 1, 1, 3], [1, 1, 1, 1, 1, 1, 1], [33, 0, 33]]
    prefixes = [[], [5], [5, 6], [5, 6, 7], [5, 6, 7, 69], [5, 6, 7, 69, 1], [5, 6, 8], [5, 7], [4], [6],
                [69], [69, 0], [0], [70], [-1], [2 ** 31 - 1], [1, 1, 1, 1, 1, 1, 1], [1, 1, 1, 1, 1, 1, 1, 2],
                [1, 1, 1, 1, 1, 1, 1, 1], [1] * 12, [33], [33, 0], [33, 0, 33], [33, 0, 34], [33, 1], [5, 6, -5],
                [5, 6, 7, 0, 0, 0, 0, 0, 0, 0]]
    S = W.constraint_set_from_lists(Sl, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    assert index.n_distinct == 10 and index.l_max == 8
    stride = 12
    P = np.full((len(prefixes), stride), W.PAD_TOKEN, np.int32)
    L = np.zeros(len(prefixes), np.int32)
    for i, p in enumerate(prefixes):
        P[i, :len(p)] = np.array(p, dtype=np.int64).astype(np.int32)
        L[i] = len(p)
    assert_query_parity(index, trie, P, L)
    _, words, lo, hi, member = gpu_query(index, P, L)
    got = unpack_mask(words, V)
    for i, (m, blo, bhi, bmem) in enumerate(brute_rows(Sl, V, prefixes)):
        assert np.array_equal(got[i], m) and (lo[i], hi[i], member[i]) == (blo, bhi, bmem), (i, prefixes[i])


def test_wide_fanout_root_search_rounds():
    """A root with tens of thousands of children exercises the multi-round 64-way search and every
    insertion position (first, between, last)."""
    V = 262_144
    rng = np.random.default_rng(9)
    firsts = np.unique(rng.integers(1, V - 1, size=40_000))
    seqs = [[int(t), 1] for t in firsts]
    S = W.constraint_set_from_lists(seqs, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    q = np.concatenate([firsts[:300], firsts[-300:], rng.integers(0, V, size=1400), [0, V - 1, V, -1]]).astype(np.int64)
    P = np.full((len(q), 2), 1, np.int32)
    P[:, 0] = q.astype(np.int32)
    L = np.ones(len(q), np.int32)
    L[::3] = 2
    assert_query_parity(index, trie, P, L)
    assert_query_parity(index, trie, P[:4], np.zeros(4, np.int32))      # the root's own mask: 40k bits


def test_empty_batch_and_null_outputs():
    cfg, S, trie, index = setup_case("C1")
    ppv.ppv_next_token_mask(index, torch.zeros((0, 8), dtype=torch.int32, device=DEV),
                            torch.zeros(0, dtype=torch.int32, device=DEV),
                            torch.zeros((0, index.n_words), dtype=torch.int32, device=DEV))
    pb = W.make_prefix_batch(cfg, S)
    mask = torch.zeros((16, index.n_words), dtype=torch.int32, device=DEV)
    ppv.ppv_next_token_mask(index, to_dev(pb.prefixes), to_dev(pb.lens), mask)      # no lo/hi/member
    torch.cuda.synchronize()
    ref = trie.query(pb.prefixes, pb.lens)
    assert np.array_equal(unpack_mask(mask.cpu().numpy().view(np.uint32), cfg.vocab), ref.mask)


@pytest.mark.parametrize("name", list(CASES))
@pytest.mark.parametrize("temperature", [1.0, 0.7])
def test_sample_next_is_mask_plus_sample_without_the_mask(name, temperature):
    """ppv_sample_next (valid set read off the index inside the kernel, never written) against the oracle's step on
    every workload, invalid prefixes included; the caller's rows are left as they were."""
    cfg, S, trie, index = setup_case(name)
    pb = W.make_prefix_batch(cfg, S, index=3)
    B = pb.prefixes.shape[0]
    logits = W.make_logits(cfg, step=7)
    un = W.make_uniforms(cfg, step=7)
    ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8, temperature=temperature)
    dP, dL = to_dev(pb.prefixes), to_dev(pb.lens)
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    ppv.ppv_sample_next(index, dP, dL, logits_to_dev(cfg, logits), to_dev(un), ids, lzv, temperature=temperature)
    torch.cuda.synchronize()
    check_sample_rows(cfg.dtype, ref, lambda b: ref.mask[b], un, ids.cpu().numpy(), lzv.cpu().numpy(), None)
    assert np.array_equal(dP.cpu().numpy(), pb.prefixes) and np.array_equal(dL.cpu().numpy(), pb.lens)
    assert (ref.ids >= 0).any()
    # the mass is optional
    ids2 = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    ppv.ppv_sample_next(index, dP, dL, logits_to_dev(cfg, logits), to_dev(un), ids2, temperature=temperature)
    torch.cuda.synchronize()
    assert torch.equal(ids, ids2)


def test_sample_edge_cases():
    """Hand-made masks: empty row, single token, all tokens, valid tokens far below the maximum,
    -inf logits, u = 0 and u -> 1, V not a multiple of 32, padded row stride."""
    V = 1000
    rng = np.random.default_rng(4)
    B = 10
    lg = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    mask = (rng.random((B, V)) < 0.05).astype(np.uint8)
    un = rng.random(B, dtype=np.float32)
    mask[0] = 0                                   # empty
    mask[1] = 0; mask[1, 999] = 1                 # single (last token)
    mask[2] = 1                                   # everything
    lg[3, 5] = 60.0; mask[3, 5] = 0               # valid mass ~ e^-55
    lg[4, mask[4] == 1] = -np.inf; mask[4, 77] = 1; lg[4, 77] = 0.5    # valid tokens with zero weight
    un[5] = 0.0
    un[6] = np.float32(1.0) - np.float32(2 ** -24)
    lg[7] = 1.25                                   # constant logits: CDF cuts at multiples of 1/count
    lg[8, :] = -200.0; lg[8, 0] = 0.0; mask[8] = 0; mask[8, 500] = mask[8, 600] = 1   # mass ~ e^-200
    words = np.packbits(np.pad(mask, ((0, 0), (0, 24))), axis=1, bitorder="little").view(np.uint32)
    stride = 1008
    dl = torch.zeros((B, stride), dtype=torch.float32, device=DEV)
    dl[:, :V] = to_dev(lg)
    ids = torch.zeros(B, dtype=torch.int32, device=DEV)
    lzv = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.constrained_sample(dl[:, :V], to_dev(words.view(np.int32)), to_dev(un), ids, lzv)
    torch.cuda.synchronize()
    gid, glz = ids.cpu().numpy(), lzv.cpu().numpy()
    from test_oracle_pins import one_step
    for b in range(B):
        r = one_step(lg[b], mask[b], un[b])
        check_sample_rows("f32", r, lambda i: mask[b], un[b:b + 1], gid[b:b + 1], glz[b:b + 1], None, rows=[b])
    assert gid[0] == -1 and gid[1] == 999 and gid[4] == 77


@pytest.mark.parametrize("V", [10_000, 900])            # several tiles per row; the one-tile kernel
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_sample_wide_dynamic_range_inside_tiles(dtype, V):
    """Rows whose tiles hold values far apart: the tokens that the first lane of a wavefront holds lie far below,
    slightly below, or are the only finite ones of their tile, single spikes stand 30 to 90 above everything else, and
    whole tiles are -inf.  Sums must not depend on which token of a tile serves as the reference of its exponentials."""
    rng = np.random.default_rng(11)
    B = 12
    lg = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    epl = 4 if dtype == "f32" else 8                  # tokens per 16-byte load
    per_load = 64 * epl
    lane0 = (np.arange(V) % per_load) < epl           # the tokens lane 0 holds in every tile
    lg[0, lane0] = -100.0
    lg[1, lane0] = -39.0
    lg[2, lane0] = -41.5
    lg[3, lane0] = -np.inf
    lg[4, ~lane0] = -np.inf                           # lane 0 alone holds finite values
    lg[5, lane0] = 35.0                               # lane 0 far above the rest
    lg[6, rng.integers(0, V, 5)] = 30.0
    lg[7, rng.integers(0, V, 3)] = 90.0
    lg[8, :V * 2 // 5] = -np.inf                      # whole tiles without a finite value
    lg[9, V * 2 // 5:] = -np.inf
    lg[10] = lg[10] * 20                              # sigma = 40
    lg[11, lane0] = -60.0; lg[11, V // 2:V // 2 + 100] = 45.0
    mask = (rng.random((B, V)) < 0.3).astype(np.uint8)
    mask[5] = lane0.astype(np.uint8)                  # valid = exactly the reference tokens
    mask[6] = (~lane0).astype(np.uint8)
    un = rng.random(B, dtype=np.float32)
    stride = (V + 7) // 8 * 8                        # rows 16-byte aligned
    if dtype == "bf16":
        bits = W.f32_to_bf16_bits(lg)
        lg = W.bf16_bits_to_f32(bits)
        dl = torch.zeros((B, stride), dtype=torch.bfloat16, device=DEV)
        dl[:, :V] = to_dev(bits.view(np.int16)).view(torch.bfloat16)
    else:
        dl = torch.zeros((B, stride), dtype=torch.float32, device=DEV)
        dl[:, :V] = to_dev(lg)
    dl = dl[:, :V]
    words = np.packbits(np.pad(mask, ((0, 0), (0, (-V) % 32))), axis=1, bitorder="little").view(np.uint32)
    ids = torch.zeros(B, dtype=torch.int32, device=DEV)
    lzv = torch.zeros(B, dtype=torch.float32, device=DEV)
    lza = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.constrained_sample(dl, to_dev(words.view(np.int32)), to_dev(un), ids, lzv, lza)
    torch.cuda.synchronize()
    gid, glz, gla = ids.cpu().numpy(), lzv.cpu().numpy(), lza.cpu().numpy()
    from test_oracle_pins import one_step
    for b in range(B):
        r = one_step(lg[b], mask[b], un[b])
        check_sample_rows(dtype, r, lambda i: mask[b], un[b:b + 1], gid[b:b + 1], glz[b:b + 1], gla[b:b + 1], rows=[b])


def test_uniforms_outside_the_unit_interval_stay_defined():
    """uniforms are in [0, 1) by contract; 1, 2, -0.5, NaN and inf must still end in a valid token or -1."""
    for name in ("C2", "C1", "C5s"):                  # list and image rows, one-tile kernel, long rows
        cfg, S, trie, index = setup_case(name)
        pb = W.make_prefix_batch(cfg, S, index=6)
        dmask, _ = assert_query_parity(index, trie, pb.prefixes, pb.lens)
        full = trie.query(pb.prefixes, pb.lens).mask
        B = pb.prefixes.shape[0]
        un = np.resize(np.array([1.0, 2.0, -0.5, np.nan, np.inf, -np.inf, 0.999999], np.float32), B)
        ids, lzv, _ = gpu_sample(cfg, logits_to_dev(cfg, W.make_logits(cfg, step=6)), dmask, un)
        ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, W.make_logits(cfg, step=6)),
                        np.full(B, 0.5, np.float32), threads=8)
        for b in range(B):
            assert ids[b] == -1 or full[b, ids[b]] == 1, (name, b, ids[b], un[b])
            if ref.ids[b] >= 0 and un[b] >= 1.0:       # at or past the end of the CDF: the last valid token of positive weight
                lf = W.logits_as_f32(cfg, W.make_logits(cfg, step=6))[b]
                pos = np.nonzero((full[b] == 1) & (lf > -np.inf))[0]
                assert ids[b] == pos[-1], (name, b)
        fin = np.isfinite(ref.logZ_valid)
        tol = 1e-5 if cfg.dtype == "f32" else 1e-3     # the mass does not depend on the uniform
        assert np.all(np.abs(lzv[fin] - ref.logZ_valid[fin]) <= tol * np.maximum(1.0, np.abs(ref.logZ_valid[fin])))


def test_bf16_sample_matches_f32_on_same_values():
    cfg, S, trie, index = setup_case("C2")
    pb = W.make_prefix_batch(cfg, S, index=8)
    dmask, _ = assert_query_parity(index, trie, pb.prefixes, pb.lens)
    bits = W.make_logits(cfg, step=8)
    un = W.make_uniforms(cfg, step=8)
    a = gpu_sample(cfg, logits_to_dev(cfg, bits), dmask, un)
    b = gpu_sample(cfg, to_dev(W.bf16_bits_to_f32(bits)), dmask, un)
    # same values, different tiling (2048 vs 1024 tokens per tile): same samples, sums equal to rounding
    assert np.array_equal(a[0], b[0])
    fin = np.isfinite(a[1])
    assert np.array_equal(fin, np.isfinite(b[1]))
    assert np.allclose(a[1][fin], b[1][fin], rtol=2e-6, atol=2e-6) and np.allclose(a[2], b[2], rtol=2e-6, atol=2e-6)


def test_results_are_bit_repeatable():
    cfg, S, trie, index = setup_case("C5s")
    pb = W.make_prefix_batch(cfg, S, index=2)
    logits = logits_to_dev(cfg, W.make_logits(cfg, step=2))
    un = W.make_uniforms(cfg, step=2)
    runs = []
    for _ in range(3):
        dmask, words, lo, hi, member = gpu_query(index, pb.prefixes, pb.lens)
        ids, lzv, lza = gpu_sample(cfg, logits, dmask, un)
        runs.append((words.copy(), lo, hi, member, ids, lzv.view(np.uint32), lza.view(np.uint32)))
    for r in runs[1:]:
        for x, y in zip(runs[0], r):
            assert np.array_equal(x, y)


def test_binding_rejects_bad_arguments():
    cfg, S, trie, index = setup_case("C1")
    with pytest.raises(ppv.PPVError):
        ppv.ppv_build_index(np.array([1, 99999], np.int32), np.array([0, 2], np.int64), 1024)   # token out of range
    with pytest.raises(ppv.PPVError):
        ppv.ppv_build_index(np.array([1, 2], np.int32), np.array([0, 0, 2], np.int64), 1024)    # empty sequence
    with pytest.raises(TypeError):
        ppv.ppv_next_token_mask(index, torch.zeros((2, 8), dtype=torch.int64, device=DEV),
                                torch.zeros(2, dtype=torch.int32, device=DEV),
                                torch.zeros((2, index.n_words), dtype=torch.int32, device=DEV))
    with pytest.raises(ppv.PPVError):     # misaligned row stride for fp32 (not a multiple of 4 elements)
        base = torch.zeros((2, 1026), dtype=torch.float32, device=DEV)
        ppv.constrained_sample(base[:, :1022], torch.zeros((2, 32), dtype=torch.int32, device=DEV),
                               torch.zeros(2, device=DEV), torch.zeros(2, dtype=torch.int32, device=DEV),
                               torch.zeros(2, device=DEV))


@pytest.mark.parametrize("mode", ["weak", "off"])
def test_prefix_lookup_modes(mode):
    """Prefixes are located through a hash table whose hits are only hints.  PPV_TUNE_LOOKUP_WEAK = 1 builds the table
    with a single fingerprint, so that every probe returns some node and the exact check has to turn the wrong
    ones away; PPV_TUNE_LOOKUP = 0 builds none.  Masks, ranges and membership must not change, for valid, corrupted,
    random, over-long and empty prefixes alike."""
    cfg, S, trie, _ = setup_case("C2")
    with tuning(ppv.PPV_TUNE_LOOKUP_WEAK if mode == "weak" else ppv.PPV_TUNE_LOOKUP, 1 if mode == "weak" else 0):
        index = ppv.ppv_build_index(S.tokens, S.offsets, cfg.vocab)
    pb = W.make_prefix_batch(cfg, S)
    B = pb.prefixes.shape[0]
    stride = 80                                               # longer than a wavefront and than any member
    P = np.full((B + 4, stride), W.PAD_TOKEN, np.int32)
    L = np.zeros(B + 4, np.int32)
    P[:B, :pb.stride] = pb.prefixes
    L[:B] = pb.lens
    m0 = S.seq(0)
    P[B, :len(m0)] = m0                                       # a member followed by 70 more tokens
    P[B, len(m0):] = 1
    L[B] = stride
    P[B + 1, :len(m0)] = m0                                   # exactly a member
    L[B + 1] = len(m0)
    P[B + 2, :] = m0[0]                                       # one token repeated 80 times
    L[B + 2] = stride
    L[B + 3] = 0
    assert_query_parity(index, trie, P, L)
    index.free()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_largest_vocabulary_and_a_large_batch(dtype):
    """V = PPV_MAX_VOCAB (every per-row table at its limit: 256 fp32 tiles, 32 KB mask rows) with a root that
    has tens of thousands of children, and a batch larger than 65,535 rows on a small index."""
    V = ppv.PPV_MAX_VOCAB
    rng = np.random.default_rng(99)
    seqs = [[int(v)] for v in rng.choice(V, size=40_000, replace=False)]
    seqs += [[int(a), int(b)] for a, b in rng.integers(0, V, size=(5_000, 2))]
    seqs += [[V - 1, V - 1, V - 1], [0], [V - 1]]
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    assert index.n_distinct == trie.n_members
    B = 6
    P = np.full((B, 3), W.PAD_TOKEN, np.int32)
    L = np.array([0, 1, 2, 1, 0, 3], np.int32)
    P[1, 0] = seqs[40_000][0]
    P[2, :2] = [V - 1, V - 1]
    P[3, 0] = V - 1
    P[5, :3] = [V - 1, V - 1, V - 1]
    dmask, ref_q = assert_query_parity(index, trie, P, L)
    lg = rng.normal(0, 2, size=(B, V)).astype(np.float32)
    lg[4, :] = -30.0
    lg[4, V - 1] = 5.0                                        # the last token of the last tile carries the row
    un = rng.random(B).astype(np.float32)
    if dtype == "bf16":
        bits = ((lg.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
        lf = (bits.astype(np.uint32) << 16).view(np.float32)
        ld = to_dev(bits.view(np.int16)).view(torch.bfloat16)
    else:
        lf, ld = lg, to_dev(lg)
    ref = trie.step(P, L, lf, un, threads=4)
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.zeros(B, dtype=torch.float32, device=DEV)
    lza = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.constrained_sample(ld, dmask, to_dev(un), ids, lzv, lza)
    torch.cuda.synchronize()
    check_sample_rows(dtype, ref, lambda b: ref.mask[b], un, ids.cpu().numpy(), lzv.cpu().numpy(), lza.cpu().numpy())
    index.free()

    # 70,000 rows on the C1 index: the grid's first dimension goes past 65,535
    cfg, S1, trie1, index1 = setup_case("C1")
    pb = W.make_prefix_batch(cfg, S1)
    reps = 70_000 // pb.prefixes.shape[0] + 1
    Pb = np.tile(pb.prefixes, (reps, 1))[:70_000]
    Lb = np.tile(pb.lens, reps)[:70_000]
    assert_query_parity(index1, trie1, Pb, Lb, threads=8)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_nan_and_infinite_logits_do_not_derail_a_row(dtype):
    """NaN or +inf logits make a row's sums meaningless; what is asked of the library is that such a row ends
    in a defined state (a token of the valid set, or -1 and the row retires) and that its neighbours are not
    touched.  Regression test: a poisoned row used to be able to form a list position outside its list."""
    cfg, S, trie, index = setup_case("C3s")
    V, B = cfg.vocab, 8
    rng = np.random.default_rng(3)
    lg = rng.normal(0, 2, size=(B, V)).astype(np.float32)
    lg[0, :] = np.nan
    lg[1, ::7] = np.nan
    lg[2, ::5] = np.inf
    lg[3, :] = np.inf
    lg[4, 100] = -np.nan
    clean = [5, 6, 7]
    if dtype == "bf16":
        t = torch.from_numpy(lg).to(DEV).to(torch.bfloat16)
    else:
        t = torch.from_numpy(lg).to(DEV)
    un = torch.full((B,), 0.37, dtype=torch.float32, device=DEV)
    outs = []
    for rows in (list(range(B)), clean):
        n = len(rows)
        P = torch.full((n, index.l_max), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        L = torch.zeros(n, dtype=torch.int32, device=DEV)
        A = torch.zeros(n, dtype=torch.uint8, device=DEV)
        st = torch.zeros((n, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        lx = torch.zeros(n, dtype=torch.float32, device=DEV)
        ids = torch.full((4, n), -5, dtype=torch.int32, device=DEV)
        lz = torch.zeros((4, n), dtype=torch.float32, device=DEV)
        tl = t[rows].contiguous()
        ppv.ppv_decode_begin(index, P, L, st, A, lx)
        for s in range(4):                                    # step 0 at the root (image), then list steps
            ppv.ppv_decode_step(index, P, L, A, tl, un[:n], ids[s], lz[s], lx, state=st)
        mask = torch.zeros((n, index.n_words), dtype=torch.int32, device=DEV)
        ppv.ppv_next_token_mask(index, P, L, mask)
        sid = torch.full((n,), -5, dtype=torch.int32, device=DEV)
        slz = torch.zeros(n, dtype=torch.float32, device=DEV)
        ppv.constrained_sample(tl, mask, un[:n], sid, slz)
        top = torch.full((n, 50), -9, dtype=torch.int32, device=DEV)
        ppv.ppv_topm_mask(index, P, L, tl, 50, mask, top)
        torch.cuda.synchronize()
        outs.append((P.cpu().numpy(), L.cpu().numpy(), ids.cpu().numpy(), sid.cpu().numpy(), top.cpu().numpy()))
    P, L, ids, sid, top = outs[0]
    assert ((ids >= -5) & (ids < V)).all() and ((sid >= -1) & (sid < V)).all() and ((top >= 0) & (top < V)).all()
    q = trie.query(P, L, want_mask=False)
    assert (q.lo < q.hi).all()                                # every row is still a prefix of some member
    Pc, Lc, idc, sidc, topc = outs[1]
    assert np.array_equal(P[clean], Pc) and np.array_equal(L[clean], Lc) and np.array_equal(ids[:, clean], idc)
    assert np.array_equal(sid[clean], sidc) and np.array_equal(top[clean], topc)


@pytest.mark.parametrize("loop", [False, True])
def test_a_state_that_is_no_cursor_retires_the_row(loop):
    """The state is the caller's memory.  Words that are no cursor of this index (never initialised, or of another
    index) are recognised by the kernel's own range checks: the row samples nothing (id -1) and retires; the rows
    beside it, and later calls on the index, are not affected."""
    cfg, S, trie, index = setup_case("C3s")
    B, L = 32, index.l_max
    rng = np.random.default_rng(8)
    P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    lens = torch.zeros(B, dtype=torch.int32, device=DEV)
    act = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.ppv_decode_begin(index, P, lens, state, act, logx)
    good = state.cpu().numpy().copy()
    bad = good.copy()
    junk = rng.integers(0, 2 ** 32, size=(B, ppv.PPV_STATE_WORDS), dtype=np.uint64).astype(np.uint32).view(np.int32)
    rows = np.arange(0, B, 2)
    bad[rows] = junk[rows]
    bad[2, :4] = [5, 10, 3, -1]                  # children range that ends before it begins
    bad[4, :4] = [0, 0, 2_000_000_000, -1]       # a list far beyond the index
    bad[6, :4] = [1, 1, 2, 123456789]            # an image slot that does not exist
    bad[8, :4] = [-2, 0, 1, -1]                  # a node number beyond the index
    # good cursors whose look-ahead half claims to be filled in but cannot be one: it is ignored, the row goes on
    bad[1, 4:] = [cfg.vocab, 0, 1, 1]            # a token outside the vocabulary
    bad[3, 4:] = [7, 9, 3, 1]                    # a children range that ends before it begins
    bad[5, 4:] = [7, 0, 2_000_000_000, 1]        # ... that lies beyond the index
    bad[7, 4:] = junk[7, 4:]
    bad[9, 4:] = [7, 0, 1, 2]                    # flags that are neither 0 nor 1
    state.copy_(to_dev(bad))
    n = 3
    logits = torch.stack([logits_to_dev(cfg, W.make_logits(cfg, batch=B, step=300 + s)) for s in range(n)])
    un = torch.stack([to_dev(W.make_uniforms(cfg, batch=B, step=300 + s)) for s in range(n)])
    ids = torch.full((n, B), -5, dtype=torch.int32, device=DEV)
    if loop:
        ppv.ppv_decode_loop(index, P, lens, act, logits, un, ids, None, logx, state=state)
    else:
        for s in range(n):
            ppv.ppv_decode_step(index, P, lens, act, logits[s], un[s], ids[s], None, logx, state=state)
    torch.cuda.synchronize()
    gi, ga, gl = ids.cpu().numpy(), act.cpu().numpy(), lens.cpu().numpy()
    assert (gi[0, rows] == -1).all() and (ga[rows] == 0).all() and (gl[rows] == 0).all()
    others = np.setdiff1d(np.arange(B), rows)
    assert (gi[0, others] >= 0).all() and (gl[others] >= 1).all()
    # the index is as good as before
    pb = W.make_prefix_batch(cfg, S, index=4)
    assert_query_parity(index, trie, pb.prefixes, pb.lens)


def test_degenerate_sets():
    """One member; one token vocabulary; nothing but duplicates; one long chain; a set that is all single tokens."""
    cases = [
        ([[0]], 1, [[], [0], [0, 0], [5]]),
        ([[3, 1, 2]] * 500, 8, [[], [3], [3, 1], [3, 1, 2], [3, 1, 2, 0], [1]]),
        ([list(range(40))], 64, [[], list(range(39)), list(range(40)), list(range(1, 40))]),
        ([[v] for v in range(200)], 200, [[], [7], [199], [7, 7]]),
        ([[1], [1, 1], [1, 1, 1], [1, 1, 1, 1]], 2, [[], [1], [1, 1], [1, 1, 1, 1], [1, 1, 1, 1, 1], [0]]),
    ]
    for seqs, V, queries in cases:
        S = W.constraint_set_from_lists(seqs, V)
        trie = oracle.Trie(S.tokens, S.offsets, V)
        index = ppv.ppv_build_index(S.tokens, S.offsets, V)
        assert index.n_distinct == trie.n_members and index.n_prefixes == trie.n_nodes - 1
        stride = max(1, max(map(len, queries)))
        P = np.full((len(queries), stride), W.PAD_TOKEN, np.int32)
        L = np.array([len(q) for q in queries], np.int32)
        for i, q in enumerate(queries):
            P[i, :len(q)] = q
        dmask, ref_q = assert_query_parity(index, trie, P, L)
        # a sampling step on top (fp32 rows must be 16-byte aligned: pad the row stride)
        Vp = (V + 3) // 4 * 4
        rng = np.random.default_rng(V)
        lg = np.zeros((len(queries), Vp), np.float32)
        lg[:, :V] = rng.normal(0, 1, size=(len(queries), V))
        un = rng.random(len(queries)).astype(np.float32)
        ref = trie.step(P, L, lg[:, :V], un)
        ids = torch.full((len(queries),), -7, dtype=torch.int32, device=DEV)
        lzv = torch.zeros(len(queries), dtype=torch.float32, device=DEV)
        ppv.constrained_sample(to_dev(lg)[:, :V], dmask, to_dev(un), ids, lzv)
        torch.cuda.synchronize()
        check_sample_rows("f32", ref, lambda b: ref.mask[b], un, ids.cpu().numpy(), lzv.cpu().numpy())
        index.free()


def test_members_longer_than_a_wavefront():
    """Members of 80 to 150 tokens behind a common stem of 70: prefixes of 63, 64, 65 and more tokens (the look-up
    covers the first 64, the descent goes on from there), wrong tokens beyond position 64, and the decode loop to the end."""
    rng = np.random.default_rng(31)
    V = 50
    stem = rng.integers(0, V, 70).tolist()
    seqs = [stem + rng.integers(0, V, int(rng.integers(10, 81))).tolist() for _ in range(300)]
    seqs += [rng.integers(0, V, int(rng.integers(1, 140))).tolist() for _ in range(200)]
    seqs += [stem[:40], stem[:64], stem[:65]]
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    assert index.l_max == max(map(len, seqs)) and index.n_distinct == trie.n_members
    queries = []
    for s in seqs[:40]:
        for k in (0, 10, 63, 64, 65, 70, 71, 79, len(s) - 1, len(s)):
            queries.append(s[:k])
        bad = list(s)
        bad[66] = (bad[66] + 1) % V
        queries.append(bad[:75])
        bad = list(s)
        bad[-1] = (bad[-1] + 1) % V
        queries.append(bad)
        queries.append(s + [3])
    stride = max(map(len, queries))
    P = np.full((len(queries), stride), W.PAD_TOKEN, np.int32)
    L = np.array([len(q) for q in queries], np.int32)
    for i, q in enumerate(queries):
        P[i, :len(q)] = q
    assert_query_parity(index, trie, P, L)
    # the whole loop, one launch, from the empty prefix
    B, Lm = 64, index.l_max
    Vp = (V + 3) // 4 * 4
    lg = np.zeros((Lm, B, Vp), np.float32)
    lg[:, :, :V] = rng.normal(0, 1, size=(Lm, B, V))
    un = rng.random((Lm, B)).astype(np.float32)
    dP = torch.full((B, Lm), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
    dL = torch.zeros(B, dtype=torch.int32, device=DEV)
    dA = torch.zeros(B, dtype=torch.uint8, device=DEV)
    state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
    logx = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.ppv_decode_begin(index, dP, dL, state, dA, logx)
    ppv.ppv_decode_loop(index, dP, dL, dA, to_dev(lg)[:, :, :V], to_dev(un), None, None, logx, state=state)
    torch.cuda.synchronize()
    res = oracle.decode_loop(trie, B, lambda s, *_: lg[s, :, :V], lambda s: un[s], threads=8)
    gL, gP = dL.cpu().numpy(), dP.cpu().numpy()
    same = sum(int(gL[b] == res.lens[b] and np.array_equal(gP[b, :gL[b]], res.seqs[b, :res.lens[b]])) for b in range(B))
    assert same >= B - 1, same                                 # (a uniform on a CDF boundary may split one row)
    assert not dA.cpu().numpy().any() and (gL > 64).any()
    rows = [b for b in range(B) if gL[b] == res.lens[b] and np.array_equal(gP[b, :gL[b]], res.seqs[b, :res.lens[b]])]
    assert np.allclose(logx.cpu().numpy()[rows], res.logx[rows], rtol=1e-4, atol=1e-4)
    index.free()


def test_calls_on_two_streams_at_once():
    """An index is immutable after it is built: mask + sample pipelines on two streams, interleaved launch by
    launch over the same index, give what each gives alone."""
    cfg, S, trie, index = setup_case("C3s")
    pbs = [W.make_prefix_batch(cfg, S, index=i) for i in (11, 12)]
    logits = [logits_to_dev(cfg, W.make_logits(cfg, step=20 + i)) for i in range(2)]
    uns = [to_dev(W.make_uniforms(cfg, step=20 + i)) for i in range(2)]
    Ps = [to_dev(pb.prefixes) for pb in pbs]
    Ls = [to_dev(pb.lens) for pb in pbs]
    B = pbs[0].prefixes.shape[0]

    def buffers():
        return (torch.zeros((B, index.n_words), dtype=torch.int32, device=DEV),
                torch.full((B,), -7, dtype=torch.int32, device=DEV), torch.zeros(B, dtype=torch.float32, device=DEV))
    alone = []
    for i in range(2):
        m, ids, lz = buffers()
        ppv.ppv_next_token_mask(index, Ps[i], Ls[i], m)
        ppv.constrained_sample(logits[i], m, uns[i], ids, lz)
        torch.cuda.synchronize()
        alone.append((m.cpu().numpy(), ids.cpu().numpy(), lz.cpu().numpy().view(np.int32)))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    bufs = [buffers(), buffers()]
    torch.cuda.synchronize()
    for rep in range(20):
        for i in range(2):
            ppv.ppv_next_token_mask(index, Ps[i], Ls[i], bufs[i][0], stream=streams[i])
        for i in range(2):
            ppv.constrained_sample(logits[i], bufs[i][0], uns[i], bufs[i][1], bufs[i][2], stream=streams[i])
    torch.cuda.synchronize()
    for i in range(2):
        m, ids, lz = bufs[i]
        assert np.array_equal(m.cpu().numpy(), alone[i][0]) and np.array_equal(ids.cpu().numpy(), alone[i][1])
        assert np.array_equal(lz.cpu().numpy().view(np.int32), alone[i][2])


def test_many_small_random_sets():
    """A battery of small random sets of varied shape (vocabulary 1..300, lengths 1..12, heavy duplication,
    nesting, skewed tokens): index sizes, masks, ranges, membership, a sampling step and a top-M call each,
    all against the oracle.  Every set has its own index: this is mostly a test of the build."""
    rng = np.random.default_rng(2025)
    for trial in range(60):
        V = int(rng.choice([1, 2, 3, 7, 33, 64, 65, 300]))
        n = int(rng.choice([1, 2, 17, 400, 3000]))
        lmax = int(rng.integers(1, 13))
        skew = rng.random() < 0.5
        seqs = []
        for _ in range(n):
            ln = int(rng.integers(1, lmax + 1))
            t = (rng.integers(0, V, size=ln) if not skew else np.minimum(rng.geometric(0.4, size=ln) - 1, V - 1))
            seqs.append([int(x) for x in t])
        S = W.constraint_set_from_lists(seqs, V)
        trie = oracle.Trie(S.tokens, S.offsets, V)
        index = ppv.ppv_build_index(S.tokens, S.offsets, V)
        assert (index.n_distinct, index.l_max, index.n_prefixes) == (trie.n_members, trie.l_max, trie.n_nodes - 1), trial
        q = [[]] + [s[:int(rng.integers(0, len(s) + 1))] for s in seqs[:40]]
        q += [s + [int(rng.integers(0, V))] for s in seqs[:10]] + [[int(rng.integers(0, V + 2)) for _ in range(3)] for _ in range(5)]
        stride = max(1, max(map(len, q)))
        P = np.full((len(q), stride), W.PAD_TOKEN, np.int32)
        L = np.array([len(x) for x in q], np.int32)
        for i, x in enumerate(q):
            P[i, :len(x)] = x
        dmask, ref_q = assert_query_parity(index, trie, P, L)
        Vp = (V + 3) // 4 * 4
        lg = np.zeros((len(q), Vp), np.float32)
        lg[:, :V] = rng.normal(0, 2, size=(len(q), V))
        un = rng.random(len(q)).astype(np.float32)
        ref = trie.step(P, L, lg[:, :V], un)
        ld = to_dev(lg)[:, :V]
        ids = torch.full((len(q),), -7, dtype=torch.int32, device=DEV)
        lzv = torch.zeros(len(q), dtype=torch.float32, device=DEV)
        ppv.constrained_sample(ld, dmask, to_dev(un), ids, lzv)
        M = int(rng.choice([1, 5, 50]))
        tmask = torch.zeros_like(dmask)
        top = torch.zeros((len(q), M), dtype=torch.int32, device=DEV)
        ppv.ppv_topm_mask(index, to_dev(P), to_dev(L), ld, M, tmask, top)
        torch.cuda.synchronize()
        check_sample_rows("f32", ref, lambda b: ref.mask[b], un, ids.cpu().numpy(), lzv.cpu().numpy())
        m = min(M, V)
        order = np.argsort(-lg[:, :V].astype(np.float64), axis=1, kind="stable")[:, :m]
        want = np.zeros((len(q), V), np.uint8)
        np.put_along_axis(want, order, np.take_along_axis(ref_q.mask, order, axis=1), axis=1)
        assert np.array_equal(unpack_mask(tmask.cpu().numpy().view(np.uint32), V), want), trial
        assert np.array_equal(np.sort(order, axis=1), top.cpu().numpy()[:, :m]), trial
        index.free()
