"""Parity of ppv_topm_mask (Algorithm 2 with M candidates) with the oracle that follows the printed
algorithm on its own sorted array: candidate sets, verdicts and masks bit for bit; then the
sampling step of Algorithm 1 through that mask."""
import sys
import time

import numpy as np
import pytest
import torch

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, check_sample_rows, gpu_query, gpu_sample, logits_to_dev, to_dev, tuning, unpack_mask
from test_gpu_parity import setup_case

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

_sorted = {}


def say(msg):
    print(f"[{time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def sorted_array(name):
    if name not in _sorted:
        cfg, S, trie, index = setup_case(name)
        _sorted[name] = oracle.SortedArray(S.tokens, S.offsets, cfg.vocab)
    return _sorted[name]


def gpu_topm(index, prefixes, lens, logits_dev, M, specified=None):
    B = prefixes.shape[0]
    mask = torch.full((B, index.n_words), -1, dtype=torch.int32, device=DEV)
    top = torch.full((B, M), -9, dtype=torch.int32, device=DEV)
    mv = torch.full((B, M), 9, dtype=torch.uint8, device=DEV)
    ppv.ppv_topm_mask(index, to_dev(prefixes), to_dev(lens), logits_dev, M, mask, top, mv)
    torch.cuda.synchronize()
    # A caller that asks for the mask alone gets the same mask: prefixes with few children are then settled by
    # counting the tokens that come before each child instead of selecting the top M.
    alone = torch.full((B, index.n_words), -1, dtype=torch.int32, device=DEV)
    ppv.ppv_topm_mask(index, to_dev(prefixes), to_dev(lens), logits_dev, M, alone)
    torch.cuda.synchronize()
    differ = (alone != mask).any(dim=1).nonzero().flatten().tolist()
    if specified is not None:   # rows whose result is unspecified (NaN logits) only have to stay inside the full mask
        differ = [r for r in differ if r in set(int(x) for x in specified)]
    assert not differ, f"mask-only call differs from the call with candidates in rows {differ[:8]} (M={M})"
    return mask, top.cpu().numpy(), mv.cpu().numpy()


def assert_topm_parity(index, X, prefixes, lens, logits_f32, logits_dev, M, threads=8):
    V = index.vocab
    ref = X.topm(prefixes, lens, logits_f32, M, threads=threads)
    dmask, top, mv = gpu_topm(index, prefixes, lens, logits_dev, M)
    m = min(M, V)
    # the oracle lists candidates by decreasing probability, the library by increasing token id: same set,
    # and each candidate's verdict travels with it
    order = np.argsort(ref.top_ids[:, :m], axis=1, kind="stable")
    want_ids = np.take_along_axis(ref.top_ids[:, :m], order, axis=1)
    want_mv = np.take_along_axis(ref.mask_V[:, :m], order, axis=1)
    bad = np.nonzero((top[:, :m] != want_ids).any(axis=1))[0]
    assert bad.size == 0, f"candidate sets differ in rows {bad[:8]} (M={M})"
    assert np.array_equal(mv[:, :m], want_mv)
    assert (top[:, m:] == -1).all() and (mv[:, m:] == 0).all()
    got = unpack_mask(dmask.cpu().numpy().view(np.uint32), V)
    assert np.array_equal(got, ref.mask)
    return dmask, ref


@pytest.mark.parametrize("name", ["C1", "C2", "C3s", "C4s", "C5s"])
def test_topm_candidates_verdicts_and_mask(name):
    cfg, S, trie, index = setup_case(name)
    X = sorted_array(name)
    pb = W.make_prefix_batch(cfg, S)
    lens = pb.lens.copy()
    lens[:3] = 0                                              # the empty prefix: heavy node, image path
    logits = W.make_logits(cfg)
    lf = W.logits_as_f32(cfg, logits)
    ld = logits_to_dev(cfg, logits)
    for M in (1, 50, 100, 500, 1000, ppv.PPV_TOPM_MAX):
        say(f"{name}: M = {M}")
        dmask, ref = assert_topm_parity(index, X, pb.prefixes, lens, lf, ld, M)
        if M >= cfg.vocab:                                    # "in theory M = |V|": the full-vocabulary mask
            _, words, _, _, _ = gpu_query(index, pb.prefixes, lens)
            assert np.array_equal(dmask.cpu().numpy().view(np.uint32), words)
    # the top-M mask is the full mask restricted to the candidates (independent of the oracle above)
    dmask, top, mv = gpu_topm(index, pb.prefixes, lens, ld, 50)
    _, words, _, _, _ = gpu_query(index, pb.prefixes, lens)
    full = unpack_mask(words, cfg.vocab)
    m = min(50, cfg.vocab)
    assert np.array_equal(mv[:, :m], np.take_along_axis(full, top[:, :m].astype(np.int64), axis=1))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_topm_ties_special_values_and_ragged_rows(dtype):
    """Coarse logits (many equal values at the cut), -inf, +/-0, a vocabulary that is no multiple of anything."""
    ties_and_special_values(dtype)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("waves", [1, 2, 16])
def test_topm_any_number_of_wavefronts_per_row(dtype, waves):
    """The wavefronts per row are a launch detail (PPV_TUNE_TOPM_WAVES overrides the choice): with one or two, a wavefront's
    share no longer stays in registers between the two passes; with sixteen, shares are ragged or empty.  Same results."""
    with tuning(ppv.PPV_TUNE_TOPM_WAVES, waves):
        ties_and_special_values(dtype, Ms=(1, 7, 64, 128, 1000))


def ties_and_special_values(dtype, Ms=(1, 7, 64, 1000)):
    rng = np.random.default_rng(77)
    V = 5003
    seqs = [rng.integers(0, V, size=int(rng.integers(1, 5))).tolist() for _ in range(4000)]
    seqs += [[int(v)] for v in range(0, V, 2)]                # wide fan-out at the root
    S = W.constraint_set_from_lists(seqs, V)
    X = oracle.SortedArray(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    B = 24
    P = np.full((B, 4), W.PAD_TOKEN, np.int32)
    L = np.zeros(B, np.int32)
    for b in range(B):
        s = seqs[b]
        k = int(rng.integers(0, len(s) + 1))
        P[b, :k] = s[:k]
        L[b] = k
    lg = (rng.integers(-4, 5, size=(B, V)) * 0.5).astype(np.float32)
    lg[0, :] = 1.5                                            # every token equal: the first M ids
    lg[1, ::3] = -np.inf
    lg[2, ::2] = -0.0
    lg[2, 1::2] = 0.0
    lg[3, :] = -np.inf
    lg[3, 4000:] = -3.0
    lg[4, :] = np.linspace(-20, 20, V, dtype=np.float32)      # all distinct, increasing
    lg[5, :] = np.linspace(20, -20, V, dtype=np.float32)
    if dtype == "bf16":
        Vp = (V + 7) // 8 * 8                                 # rows must start 16-byte aligned
        bits = (lg.view(np.uint32) >> 16).astype(np.uint16)   # these values are exact in bf16 except the linspace rows
        lf = (bits.astype(np.uint32) << 16).view(np.float32)
        padded = np.zeros((B, Vp), np.uint16)
        padded[:, :V] = bits
        ld = to_dev(padded.view(np.int16)).view(torch.bfloat16)[:, :V]
    else:
        Vp = (V + 3) // 4 * 4
        lf = lg
        padded = np.zeros((B, Vp), np.float32)
        padded[:, :V] = lg
        ld = to_dev(padded)[:, :V]
    for M in Ms:
        assert_topm_parity(index, X, P, L, lf, ld, M)
    index.free()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_topm_long_rows_bound_from_the_first_chunks(dtype):
    """A wavefront's share of a long row does not stay in registers; the bound on the M-th largest token then comes
    from the chunks that each wavefront reads first, when the list has room for what that looser bound lets through
    (M = 50, 300), and from the whole row otherwise (M = 1000).  Rows whose first chunks say little about the rest:
    low there and high behind (the list overflows: whole-row select), high there and low behind (a short list),
    everything large in one wavefront's share, and plain noise."""
    rng = np.random.default_rng(4242)
    V = 40003
    seqs = [rng.integers(0, V, size=int(rng.integers(1, 4))).tolist() for _ in range(3000)]
    seqs += [[int(v)] for v in range(0, V, 3)]
    S = W.constraint_set_from_lists(seqs, V)
    X = oracle.SortedArray(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    B = 12
    P = np.full((B, 4), W.PAD_TOKEN, np.int32)
    L = np.zeros(B, np.int32)
    for b in range(B // 2, B):                                 # the second half of the batch: below the root
        s = seqs[b]
        P[b, :1] = s[:1]
        L[b] = 1
    per = 512 if dtype == "bf16" else 256                      # tokens per chunk
    lg = rng.normal(0.0, 2.0, size=(B, V)).astype(np.float32)
    for waves in (2, 4):
        n_chunks = (V + per - 1) // per
        share = (n_chunks + waves - 1) // waves * per         # tokens per wavefront
        first = np.zeros(V, bool)
        for w in range(waves):
            first[w * share: w * share + 8 * per] = True
        r = 0 if waves == 2 else 6
        lg[r, first] -= 6.0                                    # low where the bound is taken
        lg[r + 1, ~first] -= 6.0                               # high where the bound is taken
        lg[r + 2, share: 2 * share] += 9.0                     # everything large sits in the second wavefront's share
    if dtype == "bf16":
        Vp = (V + 7) // 8 * 8
        bits = (lg.view(np.uint32) >> 16).astype(np.uint16)
        lf = (bits.astype(np.uint32) << 16).view(np.float32)
        padded = np.zeros((B, Vp), np.uint16)
        padded[:, :V] = bits
        ld = to_dev(padded.view(np.int16)).view(torch.bfloat16)[:, :V]
    else:
        Vp = (V + 3) // 4 * 4
        lf = lg
        padded = np.zeros((B, Vp), np.float32)
        padded[:, :V] = lg
        ld = to_dev(padded)[:, :V]
    for waves in (2, 4):
        with tuning(ppv.PPV_TUNE_TOPM_WAVES, waves):
            for M in (50, 300, 1000):
                say(f"long rows {dtype} waves={waves} M={M}")
                assert_topm_parity(index, X, P, L, lf, ld, M)
    index.free()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("V", [200, 4104])
def test_topm_mask_alone_counts_the_tokens_before_each_child(dtype, V):
    """A mask-only call settles prefixes with at most eight children by counting, per child, the tokens that come
    before it (larger logit, or equal logit and smaller id).  Prefixes with 0 .. 12 children, on both sides of that
    limit and of the index's own limit for listed children (6 at V = 200); logits with many ties, among them the
    children's own values; M around the counts.  gpu_topm compares the mask-only call with the full one, and
    assert_topm_parity both with the oracle; switch 2 sends the mask-only call through the selection as well."""
    rng = np.random.default_rng(V)
    seqs = []
    for n in range(1, 13):                                    # prefix [n] has n children, [n, c] has one or two
        kids = np.sort(rng.choice(V, size=n, replace=False))
        for c in kids:
            seqs.append([n, int(c), int(rng.integers(0, V))])
            if c % 2:
                seqs.append([n, int(c), int(rng.integers(0, V))])
    seqs.append([V - 1])                                      # a member without continuation
    S = W.constraint_set_from_lists(seqs, V)
    X = oracle.SortedArray(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    rows = [[]] + [[n] for n in range(1, 13)] + [s[:2] for s in seqs[:40:3] if len(s) > 1] + [[V - 1], [V - 2, 3]]
    B = len(rows)
    P = np.full((B, 3), W.PAD_TOKEN, np.int32)
    L = np.zeros(B, np.int32)
    for b, r in enumerate(rows):
        P[b, :len(r)] = r
        L[b] = len(r)
    lg = (rng.integers(-3, 4, size=(B, V)) * 0.25).astype(np.float32)      # seven distinct values: ties everywhere
    lg[2, :] = 0.75                                           # every token equal: the first M ids
    lg[3, ::2] = -np.inf
    lg[4, :] = -np.inf
    lg[5, ::2] = -0.0
    lg[5, 1::2] = 0.0
    per = 8 if dtype == "bf16" else 4
    Vp = (V + per - 1) // per * per
    if dtype == "bf16":
        bits = (lg.view(np.uint32) >> 16).astype(np.uint16)   # exact in bf16
        padded = np.full((B, Vp), 0x7F80, np.uint16)          # +inf behind the row's end: must never be counted
        padded[:, :V] = bits
        ld = to_dev(padded.view(np.int16)).view(torch.bfloat16)[:, :V]
    else:
        padded = np.full((B, Vp), np.inf, np.float32)
        padded[:, :V] = lg
        ld = to_dev(padded)[:, :V]
    for M in (1, 2, 3, 17, 64, min(V // 2, 700), 1000):
        for waves in (0, 1, 16):
            with tuning(ppv.PPV_TUNE_TOPM_WAVES, waves):
                assert_topm_parity(index, X, P, L, lg, ld, M)
        with tuning(ppv.PPV_TUNE_TOPM_STREAMING, 2):
            assert_topm_parity(index, X, P, L, lg, ld, M)
    index.free()


def test_topm_largest_vocabulary():
    """V = PPV_MAX_VOCAB: the mask row fills the LDS that the histogram used; fp32 rows of 256 chunks per wavefront."""
    V = ppv.PPV_MAX_VOCAB
    rng = np.random.default_rng(5)
    seqs = [[int(v)] for v in rng.choice(V, size=30_000, replace=False)] + [[7, int(v)] for v in range(0, V, 997)] + [[7]]
    S = W.constraint_set_from_lists(seqs, V)
    X = oracle.SortedArray(S.tokens, S.offsets, V)
    index = ppv.ppv_build_index(S.tokens, S.offsets, V)
    P = np.full((3, 2), W.PAD_TOKEN, np.int32)
    L = np.array([0, 1, 1], np.int32)
    P[1, 0] = 7
    P[2, 0] = 8
    lg = rng.normal(0, 3, size=(3, V)).astype(np.float32)
    for M in (50, 1000):
        assert_topm_parity(index, X, P, L, lg, to_dev(lg), M)
    bits = ((lg.view(np.uint32) + 0x8000) >> 16).astype(np.uint16)
    lf = (bits.astype(np.uint32) << 16).view(np.float32)
    assert_topm_parity(index, X, P, L, lf, to_dev(bits.view(np.int16)).view(torch.bfloat16), 500)
    index.free()


def test_topm_whole_row_select_path():
    """The selection has two routes (bound + short list; radix select over the whole row when the list would not
    fit).  PPV_TUNE_TOPM_STREAMING = 1 sends every row down the second one: same results."""
    with tuning(ppv.PPV_TUNE_TOPM_STREAMING, 1):
        for name in ("C2", "C3s", "C5s"):
            cfg, S, trie, index = setup_case(name)
            X = sorted_array(name)
            pb = W.make_prefix_batch(cfg, S)
            logits = W.make_logits(cfg)
            lf = W.logits_as_f32(cfg, logits)
            ld = logits_to_dev(cfg, logits)
            for M in (1, 50, 1000):
                assert_topm_parity(index, X, pb.prefixes, pb.lens, lf, ld, M)


@pytest.mark.parametrize("waves", [2, 8])
def test_topm_rows_with_nans_stay_in_bounds(waves):
    """A row that holds NaNs has unspecified candidates, but its ids stay inside [0, V) or -1, its mask only holds
    tokens of the full mask, and the rows beside it are as the oracle says."""
    name = "C3s"
    cfg, S, trie, index = setup_case(name)
    X = sorted_array(name)
    pb = W.make_prefix_batch(cfg, S)
    logits = W.make_logits(cfg)
    lf = W.logits_as_f32(cfg, logits).copy()
    rng = np.random.default_rng(5)
    bad_rows = [1, 4, 9]
    lf[1, rng.integers(0, cfg.vocab, 500)] = np.nan
    lf[4, :] = np.nan
    lf[9, ::2] = np.nan
    lf[9, 1::2] = np.inf
    bits = W.f32_to_bf16_bits(lf)
    bits[np.isnan(lf)] = 0x7FC1                                # a quiet NaN in bf16, whatever the rounding made of it
    bits[9, 10::64] = 0xFFC0                                   # negative NaNs too
    ld = to_dev(bits.view(np.int16)).view(torch.bfloat16)
    lf = W.bf16_bits_to_f32(bits)
    good = np.setdiff1d(np.arange(lf.shape[0]), bad_rows)
    full = trie.query(pb.prefixes, pb.lens).mask
    for M in (50, 1000):
        with tuning(ppv.PPV_TUNE_TOPM_WAVES, waves):
            dmask, top, mv = gpu_topm(index, pb.prefixes, pb.lens, ld, M, specified=good)
            alone = torch.full_like(dmask, -1)
            ppv.ppv_topm_mask(index, to_dev(pb.prefixes), to_dev(pb.lens), ld, M, alone)
            torch.cuda.synchronize()
        assert not (unpack_mask(alone.cpu().numpy().view(np.uint32), cfg.vocab) & ~full).any()
        assert ((top >= -1) & (top < cfg.vocab)).all()
        got = unpack_mask(dmask.cpu().numpy().view(np.uint32), cfg.vocab)
        assert not (got & ~full).any()
        ref = X.topm(pb.prefixes[good], pb.lens[good], lf[good], M, threads=8)
        assert np.array_equal(got[good], ref.mask)
        assert np.array_equal(top[good], np.sort(ref.top_ids, axis=1))


def test_topm_then_sample_is_the_step_of_algorithm_1():
    """mask from ppv_topm_mask -> constrained_sample, against the oracle's top-M mask -> masked sample."""
    name = "C3s"
    cfg, S, trie, index = setup_case(name)
    X = sorted_array(name)
    pb = W.make_prefix_batch(cfg, S)
    lens = pb.lens.copy()
    lens[:8] = 0
    logits = W.make_logits(cfg)
    lf = W.logits_as_f32(cfg, logits)
    ld = logits_to_dev(cfg, logits)
    un = W.make_uniforms(cfg)
    for M in (50, 1000):
        dmask, ref_t = assert_topm_parity(index, X, pb.prefixes, lens, lf, ld, M)
        ref = oracle.masked_sample(lf, ref_t.mask, un, threads=8)
        ids, lzv, lza = gpu_sample(cfg, ld, dmask, un)
        check_sample_rows(cfg.dtype, ref, lambda b: ref_t.mask[b], un, ids, lzv, lza)
        assert (ref.ids >= 0).sum() > 0


def test_topm_full_size_C3():
    """|S| = 1M, V = 32k, B = 256, M = 50 and 1000 at the shape bench.py times, every row against the oracle."""
    cfg = W.CONFIGS["C3"]
    say("C3: S, sorted array, device index")
    S = W.make_constraint_set(cfg)
    X = oracle.SortedArray(S.tokens, S.offsets, cfg.vocab)
    index = ppv.ppv_build_index(S.tokens, S.offsets, cfg.vocab)
    assert X.n_rows == index.n_distinct
    pb = W.make_prefix_batch(cfg, S)
    lens = pb.lens.copy()
    lens[:16] = 0
    logits = W.make_logits(cfg)
    lf = W.logits_as_f32(cfg, logits)
    ld = logits_to_dev(cfg, logits)
    for M in (50, 1000):
        say(f"C3: M = {M}")
        assert_topm_parity(index, X, pb.prefixes, lens, lf, ld, M, threads=16)


def test_topm_full_size_C5():
    """|S| = 5M, V = 256k, B = 1,024 (4 wavefronts per row, 125 chunks each), M = 50 and 1000: every row."""
    cfg = W.CONFIGS["C5"]
    say("C5: S, sorted array, device index")
    S = W.make_constraint_set(cfg)
    X = oracle.SortedArray(S.tokens, S.offsets, cfg.vocab)
    index = ppv.ppv_build_index(S.tokens, S.offsets, cfg.vocab)
    assert X.n_rows == index.n_distinct
    pb = W.make_prefix_batch(cfg, S)
    logits = W.make_logits(cfg)
    lf = W.logits_as_f32(cfg, logits)
    ld = logits_to_dev(cfg, logits)
    for M in (50, 1000):
        say(f"C5: M = {M}")
        assert_topm_parity(index, X, pb.prefixes, pb.lens, lf, ld, M, threads=16)


def test_topm_bad_arguments():
    cfg, S, trie, index = setup_case("C1")
    B = 2
    P = torch.zeros((B, 4), dtype=torch.int32, device=DEV)
    L = torch.zeros(B, dtype=torch.int32, device=DEV)
    lg = torch.zeros((B, cfg.vocab), dtype=torch.float32, device=DEV)
    mask = torch.zeros((B, index.n_words), dtype=torch.int32, device=DEV)
    with pytest.raises(ppv.PPVError):
        ppv.ppv_topm_mask(index, P, L, lg, 0, mask)
    with pytest.raises(ppv.PPVError):
        ppv.ppv_topm_mask(index, P, L, lg, ppv.PPV_TOPM_MAX + 1, mask)
    with pytest.raises(ValueError):
        ppv.ppv_topm_mask(index, P, L, lg[:, :-1], 5, mask)
    ppv.ppv_topm_mask(index, P[:0], L[:0], lg[:0], 5, mask[:0])  # empty batch: nothing to do
    torch.cuda.synchronize()
