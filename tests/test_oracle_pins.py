"""Pins for the CPU oracle: it is checked against things other than itself -- the plain
definition by brute force, closed forms, library routines on special cases, invariants, and the
paper's worked examples -- so that a dropped term, a wrong sign/index or a transposed operand in
the oracle fails here.  No GPU needed."""
import math
import os

import numpy as np
import pytest
from scipy.special import logsumexp
from scipy.stats import chisquare

import oracle
from paper_2504_09135_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_golden(name):
    out = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split()
                out[k] = float(v)
    return out


# ------------------------------------------------------------------ brute force from the definition
def u32(t):
    return int(t) & 0xFFFFFFFF


def brute(S_lists, vocab, prefix):
    """Valid set A_{x,S} (Section 2.1), membership, and rank range by scanning S."""
    members = sorted({tuple(u32(t) for t in s) for s in S_lists})
    x = tuple(u32(t) for t in prefix)
    t = len(x)
    mask = np.zeros(vocab, dtype=np.uint8)
    for s in members:
        if len(s) > t and s[:t] == x:
            mask[s[t]] = 1
    lo = sum(1 for s in members if s < x)              # tuple order = lexicographic, prefix first
    cnt = sum(1 for s in members if s[:t] == x)
    return mask, lo, lo + cnt, int(x in set(members) and t > 0)


def as_lists(S: W.ConstraintSet):
    return [S.seq(i).tolist() for i in range(S.n)]


def check_against_brute(S_lists, vocab, prefixes):
    S = W.constraint_set_from_lists(S_lists, vocab)
    trie = oracle.Trie(S.tokens, S.offsets, vocab)
    stride = max(1, max(len(p) for p in prefixes))
    P = np.full((len(prefixes), stride), W.PAD_TOKEN, dtype=np.int32)
    L = np.zeros(len(prefixes), dtype=np.int32)
    for i, p in enumerate(prefixes):
        P[i, :len(p)] = np.array(p, dtype=np.int64).astype(np.int32)
        L[i] = len(p)
    r = trie.query(P, L)
    for i, p in enumerate(prefixes):
        m, lo, hi, mem = brute(S_lists, vocab, p)
        assert np.array_equal(r.mask[i], m), (i, p)
        assert (r.lo[i], r.hi[i], r.member[i]) == (lo, hi, mem), (i, p, r.lo[i], r.hi[i], r.member[i], lo, hi, mem)
    return trie


def test_mask_range_member_vs_bruteforce_C1():
    cfg = W.CONFIGS["C1"]
    S = W.make_constraint_set(cfg)
    assert S.n == 1000 and S.l_max == 8
    pb = W.make_prefix_batch(cfg, S, batch=64)
    prefixes = [pb.prefixes[b, :pb.lens[b]].tolist() for b in range(64)]
    prefixes += [[], S.seq(0).tolist(), S.seq(5).tolist() + [3]]
    trie = check_against_brute(as_lists(S), cfg.vocab, prefixes)
    assert trie.n_members == 1000 and trie.l_max == 8


def test_mask_range_member_adversarial_sets():
    V = 70  # not a multiple of 32; token V-1 in use
    # a member that is a proper prefix of another, a long shared prefix, duplicates, single tokens
    S = [[5, 6, 7], [5, 6], [5, 6, 7, 69], [5, 6, 7, 0], [69], [0], [5, 6, 7, 69],
         [1, 1, 1, 1, 1, 1, 1, 2], [1, 1, 1, 1, 1, 1, 1, 3], [1, 1, 1, 1, 1, 1, 1], [33, 0, 33]]
    prefixes = [[], [5], [5, 6], [5, 6, 7], [5, 6, 7, 69], [5, 6, 7, 69, 1], [5, 6, 8], [5, 7], [4], [6],
                [69], [69, 0], [0], [70], [-1], [2 ** 31 - 1], [1, 1, 1, 1, 1, 1, 1], [1, 1, 1, 1, 1, 1, 1, 2],
                [1, 1, 1, 1, 1, 1, 1, 1], [1] * 12, [33], [33, 0], [33, 0, 33], [33, 0, 34], [33, 1], [5, 6, -5],
                [5, 6, 7, 0, 0, 0, 0, 0, 0, 0]]
    check_against_brute(S, V, prefixes)


def test_single_sequence_set_and_duplicates():
    trie = check_against_brute([[3, 1, 2]] * 4, 8, [[], [3], [3, 1], [3, 1, 2], [3, 1, 2, 0], [0], [7], [3, 0], [3, 2]])
    assert trie.n_members == 1


def test_mask_empty_iff_not_in_S_or_leaf():
    """mask empty <=> (lo == hi) or (the prefix is a member with no extension)."""
    cfg = W.scaled(W.CONFIGS["C2"], 3000)
    S = W.make_constraint_set(cfg)
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    pb = W.make_prefix_batch(cfg, S, batch=400)
    r = trie.query(pb.prefixes, pb.lens)
    empty = r.mask.sum(axis=1) == 0
    expect = (r.lo == r.hi) | ((r.hi - r.lo == 1) & (r.member == 1))
    assert np.array_equal(empty, expect)
    assert empty.any() and (~empty).any()
    # rows drawn as proper prefixes of members are in S's prefix closure: never an empty range
    assert ((r.hi > r.lo) | ~pb.drawn_valid).all()


def test_rejects_bad_sets():
    for toks, offs, V in [([], [0], 4), ([1, 2], [0, 0, 2], 4), ([1, 4], [0, 2], 4), ([1, -1], [0, 2], 4)]:
        with pytest.raises(ValueError):
            oracle.Trie(np.array(toks, dtype=np.int32), np.array(offs, dtype=np.int64), V)


def test_ranges_second_route_sorted_matrix():
    """Ranks from the trie's subtree counts == ranks from numpy sorting of the padded matrix
    (pad below every token), an independent route."""
    cfg = W.scaled(W.CONFIGS["C3"], 20000)
    S = W.make_constraint_set(cfg)
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    M = S.padded(pad=-1).astype(np.int64)
    order = np.lexsort(M.T[::-1])
    M = M[order]
    pb = W.make_prefix_batch(W.scaled(cfg, cfg.n_seq, batch=200), S)
    # make a fifth of them invalid
    pb.prefixes[::5, 0] = (pb.prefixes[::5, 0] + 7) % cfg.vocab
    pb.lens[::5] = np.maximum(pb.lens[::5], 1)
    r = trie.query(pb.prefixes, pb.lens, want_mask=False)
    for b in range(200):
        t = int(pb.lens[b])
        x = pb.prefixes[b, :t].astype(np.int64)
        less = np.zeros(S.n, dtype=bool)
        eq = np.ones(S.n, dtype=bool)
        for c in range(t):
            less |= eq & (M[:, c] < x[c])
            eq &= M[:, c] == x[c]
        lo = int(less.sum())
        assert (r.lo[b], r.hi[b]) == (lo, lo + int(eq.sum()))


# ------------------------------------------------------------------ masked log-softmax
def one_step(logits, mask_bytes, u):
    """Run the oracle's masked step on a hand-made mask via a one-level S = {[v] : mask[v]}."""
    V = len(logits)
    valid = np.nonzero(mask_bytes)[0]
    if len(valid) == 0:
        seqs, prefix = [[0, 0]], [1]            # prefix [1] is not in S: empty mask
    else:
        seqs, prefix = [[int(v)] for v in valid], []
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    P = np.full((1, 1), W.PAD_TOKEN, dtype=np.int32)
    if prefix:
        P[0, 0] = prefix[0]
    r = trie.step(P, np.array([len(prefix)], dtype=np.int32), np.asarray(logits, dtype=np.float32)[None, :],
                  np.array([u], dtype=np.float32))
    assert np.array_equal(r.mask[0], np.asarray(mask_bytes, dtype=np.uint8))
    return r


def test_logZ_matches_library_logsumexp_and_closed_forms():
    rng = np.random.default_rng(1)
    V = 257
    l = (rng.standard_normal(V) * 3).astype(np.float32)
    mask = (rng.random(V) < 0.3).astype(np.uint8)
    r = one_step(l, mask, 0.5)
    ld = l.astype(np.float64)
    assert r.logZ_all[0] == pytest.approx(logsumexp(ld), abs=1e-12)
    assert r.logZ_valid[0] == pytest.approx(logsumexp(ld[mask == 1]) - logsumexp(ld), abs=1e-12)
    assert r.logZ_valid[0] <= 0
    # mask = everything => mass 1
    assert one_step(l, np.ones(V, np.uint8), 0.5).logZ_valid[0] == pytest.approx(0.0, abs=1e-12)
    # mask = {v} => log softmax(l)_v
    one = np.zeros(V, np.uint8)
    one[123] = 1
    r1 = one_step(l, one, 0.9)
    assert r1.logZ_valid[0] == pytest.approx(ld[123] - logsumexp(ld), abs=1e-12) and r1.ids[0] == 123
    # complement identity: the two masses add up to 1
    rc = one_step(l, 1 - mask, 0.5)
    assert math.exp(r.logZ_valid[0]) + math.exp(rc.logZ_valid[0]) == pytest.approx(1.0, abs=1e-12)
    # shift invariance (exact shift in fp32: integers)
    li = np.round(l * 8).astype(np.float32)
    a, b = one_step(li, mask, 0.5), one_step(li + 64, mask, 0.5)
    assert a.logZ_valid[0] == pytest.approx(b.logZ_valid[0], abs=1e-12) and a.ids[0] == b.ids[0]
    # constant logits: mass = (#valid)/V
    rcst = one_step(np.full(V, 1.5, np.float32), mask, 0.5)
    assert rcst.logZ_valid[0] == pytest.approx(math.log(mask.sum() / V), abs=1e-12)
    # empty mask
    re = one_step(l, np.zeros(V, np.uint8), 0.5)
    assert re.ids[0] == -1 and re.logZ_valid[0] == -np.inf


def test_temperature_closed_forms_and_exact_rescaling():
    """Algorithm 1 takes a temperature T: P = softmax(logits / T).  Pins: the library log-sum-exp of l/T; the
    two-token logistic closed form; T = 2 on even integers equals T = 1 on their halves bit for bit (the division is
    exact); probabilities p^(1/T) renormalised for a known p; large T tends to the uniform distribution."""
    rng = np.random.default_rng(21)
    V = 129
    l = (rng.standard_normal(V) * 3).astype(np.float32)
    mask = (rng.random(V) < 0.4).astype(np.uint8)
    S = W.constraint_set_from_lists([[int(v)] for v in np.nonzero(mask)[0]], V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    P0, L0 = np.full((1, 1), W.PAD_TOKEN, np.int32), np.zeros(1, np.int32)

    def step(lg, u, T):
        return trie.step(P0, L0, np.asarray(lg, np.float32)[None, :], np.array([u], np.float32), temperature=T)
    for T in (0.5, 0.7, 1.0, 3.0):
        r = step(l, 0.4, T)
        ld = l.astype(np.float64) / T
        assert r.logZ_all[0] == pytest.approx(logsumexp(ld), abs=1e-12)
        assert r.logZ_valid[0] == pytest.approx(logsumexp(ld[mask == 1]) - logsumexp(ld), abs=1e-12)
        # the sample: inverse CDF over the valid tokens' weights exp(l/T), written out with numpy
        w = np.exp(ld[mask == 1] - ld[mask == 1].max())
        cdf = np.cumsum(w) / w.sum()
        assert r.ids[0] == np.nonzero(mask)[0][np.searchsorted(cdf, 0.4, side="right")]
        # and through the other entry point
        m = oracle.masked_sample(l[None, :], mask[None, :], np.array([0.4], np.float32), temperature=T)
        assert m.ids[0] == r.ids[0] and m.logZ_valid[0] == r.logZ_valid[0] and m.logZ_all[0] == r.logZ_all[0]
    # exact rescaling: even integers at T = 2 are their halves at T = 1
    le = (np.round(l * 4) * 2).astype(np.float32)
    a, b = step(le, 0.61, 2.0), step(le / 2, 0.61, 1.0)
    assert a.logZ_valid[0] == b.logZ_valid[0] and a.logZ_all[0] == b.logZ_all[0] and a.ids[0] == b.ids[0]
    assert a.cdf_lo[0] == b.cdf_lo[0] and a.cdf_hi[0] == b.cdf_hi[0]
    # two valid tokens: P(first | valid) = 1 / (1 + exp((l_b - l_a) / T)), so u just below / above it picks a / b
    S2 = W.constraint_set_from_lists([[3], [9]], 16)
    t2 = oracle.Trie(S2.tokens, S2.offsets, 16)
    l2 = np.zeros(16, np.float32)
    l2[3], l2[9] = 1.0, 2.5
    for T in (0.5, 1.0, 4.0):
        pa = 1.0 / (1.0 + math.exp((2.5 - 1.0) / T))
        for u, want in ((pa - 1e-4, 3), (pa + 1e-4, 9)):
            r = t2.step(P0, L0, l2[None, :], np.array([u], np.float32), temperature=T)
            assert r.ids[0] == want
            assert r.cdf_hi[0] == pytest.approx(pa, abs=1e-12) if want == 3 else r.cdf_lo[0] == pytest.approx(pa, abs=1e-12)
        mass = (math.exp(1.0 / T) + math.exp(2.5 / T)) / (14.0 + math.exp(1.0 / T) + math.exp(2.5 / T))
        assert r.logZ_valid[0] == pytest.approx(math.log(mass), abs=1e-12)
    # known probabilities: softmax(log p / T) = p^(1/T) / sum p^(1/T)
    p = np.array([0.1, 0.2, 0.3, 0.4])
    lp = np.log(p).astype(np.float32)
    S4 = W.constraint_set_from_lists([[0], [2]], 4)
    t4 = oracle.Trie(S4.tokens, S4.offsets, 4)
    q = p ** 2 / (p ** 2).sum()                        # T = 0.5
    r = t4.step(P0, L0, lp[None, :], np.array([0.5], np.float32), temperature=0.5)
    assert r.logZ_valid[0] == pytest.approx(math.log(q[0] + q[2]), abs=1e-6)
    assert r.cdf_hi[0] == pytest.approx(1.0, abs=1e-9) and r.cdf_lo[0] == pytest.approx(q[0] / (q[0] + q[2]), abs=1e-6) and r.ids[0] == 2
    # T large: uniform over the vocabulary, mass = |valid| / V
    r = step(l, 0.5, 1e9)
    assert r.logZ_valid[0] == pytest.approx(math.log(mask.sum() / V), abs=1e-6)
    assert r.ids[0] == np.nonzero(mask)[0][mask.sum() // 2]


def test_decode_loop_temperature_is_the_per_step_temperature():
    """The loop passes T to every step: its log importance score is the sum of the steps' tempered masses."""
    S = W.constraint_set_from_lists([[1, 2, 3], [1, 2, 4], [1, 5], [6, 7, 8, 9]], 12)
    trie = oracle.Trie(S.tokens, S.offsets, 12)
    rng = np.random.default_rng(3)
    B = 6
    lg = [(rng.standard_normal((B, 12)) * 2).astype(np.float32) for _ in range(trie.l_max)]
    un = [rng.random(B, dtype=np.float32) for _ in range(trie.l_max)]
    for T in (0.6, 1.0, 2.0):
        res = oracle.decode_loop(trie, B, lambda s, *_: lg[s], lambda s: un[s], temperature=T)
        for b in range(B):
            a, lx = [], 0.0
            while a not in ([1, 2, 3], [1, 2, 4], [1, 5], [6, 7, 8, 9]):
                r = trie.step(np.array([a + [W.PAD_TOKEN] * (4 - len(a))], np.int32), np.array([len(a)], np.int32),
                              lg[len(a)][b:b + 1], un[len(a)][b:b + 1], temperature=T)
                lx += r.logZ_valid[0]
                a.append(int(r.ids[0]))
            assert list(res.seqs[b, :res.lens[b]]) == a and res.logx[b] == pytest.approx(lx, abs=1e-12)
    # different temperatures give different scores on the same draws
    r1 = oracle.decode_loop(trie, B, lambda s, *_: lg[s], lambda s: un[s], temperature=1.0)
    r2 = oracle.decode_loop(trie, B, lambda s, *_: lg[s], lambda s: un[s], temperature=2.0)
    assert not np.allclose(r1.logx, r2.logx)


def test_logZ_far_below_max_does_not_underflow():
    l = np.full(64, -900.0, np.float32)
    l[0] = 0.0
    mask = np.zeros(64, np.uint8)
    mask[10] = mask[20] = 1
    r = one_step(l, mask, 0.75)
    assert r.logZ_valid[0] == pytest.approx(-900.0 + math.log(2.0), abs=1e-6)  # logsumexp(all) ~ 0
    assert r.ids[0] == 20


def test_inverse_cdf_known_boundaries():
    p = np.array([0.1, 0.2, 0.3, 0.4])
    l = np.log(p).astype(np.float32)
    allm = np.ones(4, np.uint8)
    for u, want in [(0.0, 0), (0.05, 0), (0.15, 1), (0.29, 1), (0.35, 2), (0.59, 2), (0.65, 3), (0.999, 3)]:
        assert one_step(l, allm, u).ids[0] == want
    m = np.array([1, 0, 1, 1], np.uint8)               # renormalised (0.1, 0.3, 0.4)/0.8: cuts 0.125, 0.5
    for u, want in [(0.0, 0), (0.12, 0), (0.13, 2), (0.49, 2), (0.51, 3), (0.9999, 3)]:
        r = one_step(l, m, u)
        assert r.ids[0] == want
        assert r.cdf_lo[0] <= u < r.cdf_hi[0]
    r = one_step(l, m, 0.3)
    assert r.cdf_lo[0] == pytest.approx(0.125, abs=1e-7) and r.cdf_hi[0] == pytest.approx(0.5, abs=1e-7)
    assert r.logZ_valid[0] == pytest.approx(math.log(0.8), abs=1e-7)
    # a zero-weight valid token is never chosen: u = 0 skips it, u -> 1 falls back to the last positive one
    lz = np.array([-np.inf, 0.0, 0.0, -np.inf], np.float32)
    assert one_step(lz, allm, 0.0).ids[0] == 1
    assert one_step(lz, allm, np.float32(1.0) - np.float32(2 ** -24)).ids[0] == 2


def test_sampling_distribution_chi_square():
    rng = np.random.default_rng(7)
    V = 16
    l = rng.standard_normal(V).astype(np.float32)
    mask = np.array([1, 1, 0, 1, 0, 0, 1, 1, 1, 0, 1, 1, 0, 1, 1, 0], np.uint8)
    S = W.constraint_set_from_lists([[int(v)] for v in np.nonzero(mask)[0]], V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    n = 200_000
    us = rng.random(n, dtype=np.float32)
    P = np.full((n, 1), W.PAD_TOKEN, np.int32)
    r = trie.step(P, np.zeros(n, np.int32), np.broadcast_to(l, (n, V)), us, want_mask=False, threads=4)
    p = np.exp(l.astype(np.float64)) * mask
    p /= p.sum()
    counts = np.bincount(r.ids, minlength=V)
    assert counts[mask == 0].sum() == 0
    stat = chisquare(counts[mask == 1], p[mask == 1] * n)
    assert stat.pvalue > 1e-4


# ------------------------------------------------------------------ loop identities
def toy_lm(prefix, V, seed=11):
    """Deterministic stand-in for L(a, T): logits are a seeded function of the prefix."""
    h = seed
    for t in prefix:
        h = (h * 1000003 + int(t) + 1) % (2 ** 61 - 1)
    return np.random.default_rng(h).standard_normal(V).astype(np.float32) * 1.5


def test_identity_sum_over_S_of_PL_over_x_is_one():
    """sum_{a in S} P_L(a)/x(a) = 1 and P^CD(a) = P_L(a)/x(a) (appendix, proof of Theorem 3.1),
    on a prefix-free toy S; a missing or extra valid token anywhere breaks the sum."""
    V = 6
    rng = np.random.default_rng(3)
    seqs = {tuple(rng.integers(0, V, size=3).tolist()) for _ in range(60)}      # fixed length => prefix-free
    seqs = sorted(seqs)
    S = W.constraint_set_from_lists([list(s) for s in seqs], V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    total = 0.0
    accept = 0.0
    for a in seqs:
        logp, logx = 0.0, 0.0
        for i in range(len(a)):
            l = toy_lm(a[:i], V)
            P = np.full((1, 3), W.PAD_TOKEN, np.int32)
            P[0, :i] = a[:i]
            r = trie.step(P, np.array([i], np.int32), l[None, :], np.array([0.5], np.float32))
            logp += float(l[a[i]]) - r.logZ_all[0]
            logx += r.logZ_valid[0]
        total += math.exp(logp - logx)
        accept += math.exp(logp)            # = P^CD(a) * x(a)
    assert total == pytest.approx(1.0, abs=1e-9)
    # acceptance probability of one draw = P_L(S) <= 1
    assert 0 < accept < 1


def test_decode_loop_law_is_PL_over_x():
    V = 5
    seqs = [[0, 1], [0, 2, 3], [0, 2, 4], [1], [2, 0, 0, 1], [2, 0, 0, 2], [3, 3]]
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    B = 60_000
    rng = np.random.default_rng(5)
    us = [rng.random(B, dtype=np.float32) for _ in range(4)]

    def logits_for_step(step, seqs_now, lens_now):
        out = np.zeros((B, V), np.float32)
        cache = {}
        for b in range(B):
            key = tuple(seqs_now[b, :lens_now[b]].tolist())
            if key not in cache:
                cache[key] = toy_lm(key, V)
            out[b] = cache[key]
        return out

    res = oracle.decode_loop(trie, B, logits_for_step, lambda s: us[s], threads=4)
    seqs_arr, lens, logx = res.seqs, res.lens, res.logx
    # expected law: P^CD(a) = P_L(a)/x(a)
    expect, xs = [], []
    for a in seqs:
        logp, lx = 0.0, 0.0
        for i in range(len(a)):
            l = toy_lm(tuple(a[:i]), V).astype(np.float64)
            r = trie.step(np.array([a[:i] + [W.PAD_TOKEN] * (4 - i)], np.int32), np.array([i], np.int32),
                          l[None, :].astype(np.float32), np.array([0.5], np.float32))
            logp += l[a[i]] - r.logZ_all[0]
            lx += r.logZ_valid[0]
        expect.append(math.exp(logp - lx))
        xs.append(lx)
    assert sum(expect) == pytest.approx(1.0, abs=1e-9)
    counts = []
    for a, lx in zip(seqs, xs):
        hit = (lens == len(a)) & (seqs_arr[:, :len(a)] == np.array(a)).all(axis=1)
        counts.append(int(hit.sum()))
        assert np.allclose(logx[hit], lx, atol=1e-9)
    assert sum(counts) == B
    assert chisquare(counts, np.array(expect) * B).pvalue > 1e-4


def test_decode_loop_function_runs_and_stops_at_first_member():
    V = 4
    seqs = [[1], [1, 2], [0, 3], [0, 3, 3]]     # [1] and [0,3] are members with extensions
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    B = 64
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((3, B, V)).astype(np.float32)
    un = rng.random((3, B), dtype=np.float32)
    r = oracle.decode_loop(trie, B, lambda s, *_: lg[s], lambda s: un[s])
    got = {tuple(r.seqs[b, :r.lens[b]].tolist()) for b in range(B)}
    assert got == {(1,), (0, 3)}                # stops the first time the row is in S (Algorithm 1)
    assert r.steps == 2
    assert (r.logx <= 1e-12).all()


# ------------------------------------------------------------------ the paper's worked examples
def run_toy_chain(seqs, V, cond_probs, path):
    """Valid masses along `path` with conditional next-token probabilities given per prefix."""
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    masses, pcd, pl = [], 1.0, 1.0
    for i in range(len(path)):
        p = np.array(cond_probs[tuple(path[:i])], dtype=np.float64)
        with np.errstate(divide="ignore"):
            l = np.log(p).astype(np.float32)
        P = np.full((1, 4), W.PAD_TOKEN, np.int32)
        P[0, :i] = path[:i]
        r = trie.step(P, np.array([i], np.int32), l[None, :], np.array([0.5], np.float32))
        mass = math.exp(r.logZ_valid[0])
        masses.append(mass)
        pcd *= p[path[i]] / mass
        pl *= p[path[i]]
    return masses, pcd, pl


def test_theorem_2_1_construction():
    g = read_golden("thm21_construction.txt")
    pb, eps = g["p_b"], g["eps"]
    seqs = [[0, 0], [0, 1], [1, 0]]
    cond = {(): [1 - pb, pb], (0,): [0.5, 0.5], (1,): [eps, 1 - eps]}
    tol = 1e-7  # logits pass through fp32
    m, pcd, pl = run_toy_chain(seqs, 2, cond, [0, 0])
    assert m == pytest.approx([g["mass_root"], g["mass_after_v1"]], abs=tol)
    assert pcd == pytest.approx(g["pcd_v1v1"], abs=tol)
    m, pcd2, pl2 = run_toy_chain(seqs, 2, cond, [0, 1])
    assert pcd2 == pytest.approx(g["pcd_v1v2"], abs=tol)
    m, pcd3, pl3 = run_toy_chain(seqs, 2, cond, [1, 0])
    assert m == pytest.approx([g["mass_root"], g["mass_after_v2"]], abs=tol)
    assert pcd3 == pytest.approx(g["pcd_v2v1"], abs=tol)
    assert m[0] * m[1] == pytest.approx(g["x_v2v1"], abs=tol)
    # acceptance = sum_a P^CD(a) x(a) = P_L(S)
    acc = pcd * g["x_v1v1"] + pcd2 * g["x_v1v2"] + pcd3 * g["x_v2v1"]
    assert acc == pytest.approx(g["accept"], abs=tol)
    assert pl + pl2 + pl3 == pytest.approx(g["accept"], abs=tol)
    # the valid sets the proof states: both tokens at the root and after v1, only v1 after v2
    S = W.constraint_set_from_lists(seqs, 2)
    trie = oracle.Trie(S.tokens, S.offsets, 2)
    q = trie.query(np.array([[9, 9], [0, 9], [1, 9]], np.int32), np.array([0, 1, 1], np.int32))
    assert q.mask.tolist() == [[1, 1], [1, 1], [1, 0]]


def test_figure_1_caption_numbers():
    g = read_golden("fig1_caption.txt")
    soccer, used, gloves, shoes, shirts = range(5)
    seqs = [[soccer, gloves], [used, shirts], [used, soccer, shoes]]
    z = 0.0
    cond = {(): [0.6, 0.4, z, z, z], (soccer,): [z, z, 0.1, 0.9, z], (used,): [0.9, z, z, z, 0.1],
            (used, soccer): [z, z, 0.1, 0.9, z]}
    tol = 1e-7
    m, pcd, pl = run_toy_chain(seqs, 5, cond, [soccer, gloves])
    assert pl == pytest.approx(g["pl_soccer_gloves"], abs=tol)
    assert pcd == pytest.approx(g["pcd_soccer_gloves"], abs=tol)
    assert m == pytest.approx([g["mass_root"], g["mass_after_soccer"]], abs=tol)
    m, pcd, pl = run_toy_chain(seqs, 5, cond, [used, soccer, shoes])
    assert pl == pytest.approx(g["pl_used_soccer_shoes"], abs=tol)
    assert pcd == pytest.approx(g["pcd_used_soccer_shoes"], abs=tol)
    assert m == pytest.approx([g["mass_root"], g["mass_after_used"], g["mass_after_used_soccer"]], abs=tol)


# ------------------------------------------------------------------ DISC outer loop (accept / reject / resample)
def test_disc_expected_number_of_draws_closed_form():
    """E[k] = (1 - p_b^K)/(1 - p_b) + K p_b^K (Theorem 3.1) when every draw is accepted with probability
    1 - p_b independently: scores x ~ Beta(2, 3) have mean 0.4, so p_b = 0.6."""
    rng = np.random.default_rng(12)
    Q = 120_000
    for K in (1, 2, 4):
        x = rng.beta(2.0, 3.0, size=(2 * K, Q))
        ch, nd, acc = oracle.disc_select(np.log(x), K, rng.random((K, Q)), rng.random(Q))
        pb = 0.6
        want = (1 - pb ** K) / (1 - pb) + K * pb ** K
        se = nd.std() / math.sqrt(Q)
        assert abs(nd.mean() - want) < 5 * se + 1e-9, (K, nd.mean(), want)
        assert abs(acc.mean() - (1 - pb ** K)) < 5 * math.sqrt(pb ** K * (1 - pb ** K) / Q)
        assert ((ch < K) == (acc == 1)).all() and ((nd == 2 * K) == (acc == 0)).all()


def test_disc_accepted_samples_follow_P_S_on_the_theorem_2_1_toy():
    """Candidates drawn from P^CD of the two-token construction with their scores x(a): a sample returned
    by an accept round has law P_S = P_L(a)/P_L(S) (appendix, "Unbiased distribution for the accepted sample")."""
    g = read_golden("thm21_construction.txt")
    pcd = np.array([g["pcd_v1v1"], g["pcd_v1v2"], g["pcd_v2v1"]])
    xs = np.array([g["x_v1v1"], g["x_v1v2"], g["x_v2v1"]])
    pl = pcd * xs
    ps = pl / pl.sum()
    assert pl.sum() == pytest.approx(g["accept"], abs=1e-12)
    rng = np.random.default_rng(13)
    Q, K = 150_000, 3
    cand = rng.choice(3, size=(2 * K, Q), p=pcd)
    ch, nd, acc = oracle.disc_select(np.log(xs)[cand], K, rng.random((K, Q)), rng.random(Q))
    out = cand[ch, np.arange(Q)]
    got = np.bincount(out[acc == 1], minlength=3)
    assert chisquare(got, ps * got.sum()).pvalue > 1e-4
    # every round accepts with probability P_L(S)
    assert abs((nd[acc == 1] == 1).sum() / Q - g["accept"]) < 5 * math.sqrt(g["accept"] * (1 - g["accept"]) / Q)
    # the fallback is importance resampling among K fresh candidates: exact law by enumeration of the K-tuples
    import itertools
    qlaw = np.zeros(3)
    for tup in itertools.product(range(3), repeat=K):
        p = np.prod(pcd[list(tup)])
        w = xs[list(tup)]
        for j, a in enumerate(tup):
            qlaw[a] += p * w[j] / w.sum()
    rej = np.bincount(out[acc == 0], minlength=3)
    assert rej.sum() > 200 and chisquare(rej, qlaw * rej.sum()).pvalue > 1e-4


def test_disc_fallback_is_proportional_to_scores_and_K1_reuse_is_plain_constrained_decoding():
    rng = np.random.default_rng(14)
    Q, K = 60_000, 4
    x = np.array([0.05, 0.2, 0.4, 0.1, 0.3, 0.15, 0.05, 0.5])
    logx = np.log(np.tile(x[:, None], (1, Q)))
    never = np.ones((K, Q))                                    # epsilon = 1: x > 1 never holds
    ch, nd, acc = oracle.disc_select(logx, K, never, rng.random(Q))
    assert (acc == 0).all() and (nd == 2 * K).all() and (ch >= K).all()
    assert chisquare(np.bincount(ch - K, minlength=K), x[K:] / x[K:].sum() * Q).pvalue > 1e-4
    ch, nd, acc = oracle.disc_select(logx, K, never, rng.random(Q), reuse_rejected=True)
    assert (nd == K).all() and chisquare(np.bincount(ch, minlength=K), x[:K] / x[:K].sum() * Q).pvalue > 1e-4
    # K = 1, reuse: whatever happens, the one constrained-decoding sample is returned
    ch, nd, acc = oracle.disc_select(logx[:1], 1, rng.random((1, Q)), rng.random(Q), reuse_rejected=True)
    assert (ch == 0).all() and (nd == 1).all()
    # u = 0 picks the first fallback candidate, u -> 1 the last
    ch, _, _ = oracle.disc_select(logx[:, :2], K, never[:, :2], np.array([0.0, 1.0 - 2 ** -40]))
    assert ch.tolist() == [K, 2 * K - 1]


# ------------------------------------------------------------------ Algorithm 2 as printed (top-M candidates)
def brute_topm(S_lists, prefix, logits_row, M):
    """Top M by python's sort (larger logit first, smaller id first on ties); a candidate is valid iff some
    member of S starts with prefix + [t] -- the definition, by scanning S."""
    V = len(logits_row)
    order = sorted(range(V), key=lambda v: (-float(logits_row[v]), v))[:min(M, V)]
    x = [u32(t) for t in prefix]
    verdict = []
    for t in order:
        c = x + [t]
        verdict.append(int(any(len(s) >= len(c) and [u32(a) for a in s[:len(c)]] == c for s in S_lists)))
    return order, verdict


def test_topm_vs_bruteforce_tiny_sets():
    rng = np.random.default_rng(11)
    for trial in range(30):
        V = int(rng.integers(3, 40))
        n = int(rng.integers(1, 60))
        S_lists = [rng.integers(0, V, size=int(rng.integers(1, 6))).tolist() for _ in range(n)]
        S = W.constraint_set_from_lists(S_lists, V)
        X = oracle.SortedArray(S.tokens, S.offsets, V)
        assert X.n_rows == len({tuple(s) for s in S_lists})
        prefixes = [[]] + [s[:k] for s in S_lists[:8] for k in range(len(s) + 1)] + [[V + 5], [0, 0, 0, 0, 0, 0, 0]]
        # coarse logits so that ties at the cut are common
        for M in (1, 2, V // 2 + 1, V, V + 3):
            for p in prefixes:
                lg = (rng.integers(-3, 4, size=V) * 0.5).astype(np.float32)
                P = np.full((1, 8), W.PAD_TOKEN, dtype=np.int32)
                P[0, :len(p)] = p
                r = X.topm(P, np.array([len(p)], np.int32), lg[None, :], M)
                order, verdict = brute_topm(S_lists, p, lg, M)
                m = len(order)
                assert r.top_ids[0, :m].tolist() == order and (r.top_ids[0, m:] == -1).all()
                assert r.mask_V[0, :m].tolist() == verdict and (r.mask_V[0, m:] == 0).all()
                want = np.zeros(V, np.uint8)
                for t, ok in zip(order, verdict):
                    want[t] = ok
                assert np.array_equal(r.mask[0], want)


def test_topm_mask_is_full_mask_intersected_with_top_M_second_route():
    """mask_topM = A_{a,S} restricted to the top-M tokens: the printed algorithm (sorted array + binary search per
    candidate) against the prefix tree's full mask and numpy's stable argsort -- two routes that share no code."""
    cfg = W.CONFIGS["C2"]
    S = W.make_constraint_set(cfg)
    X = oracle.SortedArray(S.tokens, S.offsets, cfg.vocab)
    trie = oracle.Trie(S.tokens, S.offsets, cfg.vocab)
    assert X.n_rows == trie.n_members
    pb = W.make_prefix_batch(cfg, S)
    B = min(cfg.batch, 48)
    P, L = pb.prefixes[:B], pb.lens[:B]
    L = L.copy()
    L[:4] = 0                                            # the root too (largest fan-out)
    lg = W.logits_as_f32(cfg, W.make_logits(cfg))[:B]
    full = trie.query(P, L).mask
    for M in (1, 50, 500, 1000, cfg.vocab):
        r = X.topm(P, L, lg, M, threads=4)
        m = min(M, cfg.vocab)
        for b in range(B):
            order = np.argsort(-lg[b].astype(np.float64), kind="stable")[:m]     # stable: ties keep increasing id
            assert np.array_equal(r.top_ids[b, :m], order)
            want = np.zeros(cfg.vocab, np.uint8)
            want[order] = full[b, order]
            assert np.array_equal(r.mask[b], want)
            assert np.array_equal(r.mask_V[b, :m], full[b, order])
        if M == cfg.vocab:
            assert np.array_equal(r.mask, full)           # "in theory M = |V|": nothing is missed


def test_topm_ties_and_signed_zero():
    """Equal probabilities are ordered by token id; -0.0 and +0.0 are the same logit."""
    S = W.constraint_set_from_lists([[0], [1], [2], [3], [4], [5]], 6)
    X = oracle.SortedArray(S.tokens, S.offsets, 6)
    lg = np.array([[0.0, -0.0, 1.0, -0.0, 0.0, -1.0]], np.float32)
    r = X.topm(np.zeros((1, 1), np.int32), np.zeros(1, np.int32), lg, 3)
    assert r.top_ids[0].tolist() == [2, 0, 1]
    assert r.mask_V[0].tolist() == [1, 1, 1]


def test_masked_sample_with_topm_mask_matches_renormalised_top_M_distribution():
    """With every token valid in S, sampling through the top-M mask is sampling from P renormalised over the top
    M tokens, and the reported mass is their total probability (checked against scipy)."""
    V, M = 50, 7
    S = W.constraint_set_from_lists([[v] for v in range(V)], V)
    X = oracle.SortedArray(S.tokens, S.offsets, V)
    rng = np.random.default_rng(5)
    lg = rng.normal(0, 2, size=(1, V)).astype(np.float32)
    r = X.topm(np.zeros((1, 1), np.int32), np.zeros(1, np.int32), lg, M)
    top = np.sort(r.top_ids[0])
    logp = lg[0].astype(np.float64) - logsumexp(lg[0].astype(np.float64))
    p_top = np.exp(logp[top])
    for u in (0.0, 0.3, 0.77, 0.999):
        s = oracle.masked_sample(lg, r.mask, np.array([u], np.float32))
        assert abs(s.logZ_valid[0] - math.log(p_top.sum())) < 1e-12
        cdf = np.cumsum(p_top) / p_top.sum()
        assert s.ids[0] == top[np.searchsorted(cdf, np.float32(u), side="right")]


# ------------------------------------------------------------------ rows that cannot draw a token
def test_valid_tokens_all_of_probability_zero_sample_nothing():
    """Algorithm 1 samples from P (.) mask / |P (.) mask|_1, which is undefined when the mass is 0.  The reading:
    a valid set that is not empty but whose tokens all have logit -inf yields no token (id -1) and log mass -inf,
    for every u, while the log-sum-exp over the whole vocabulary is still the library's.  The neighbouring case,
    one valid token of positive probability among such ones, yields that token for every u, with mass = its
    softmax probability.  Expected values are written out here, not taken from the oracle's formula."""
    rng = np.random.default_rng(16)
    V = 37
    l = (rng.standard_normal(V) * 2).astype(np.float32)
    mask = np.zeros(V, np.uint8)
    valid = [3, 4, 17, 36]
    mask[valid] = 1
    dead = l.copy()
    dead[valid] = -np.inf
    lse_all = logsumexp(dead.astype(np.float64))
    for u in (0.0, 0.25, 0.5, float(np.float32(1.0) - np.float32(2 ** -24))):
        r = one_step(dead, mask, u)
        assert r.ids[0] == -1 and r.logZ_valid[0] == -np.inf
        assert r.logZ_all[0] == pytest.approx(lse_all, abs=1e-12)
        m = oracle.masked_sample(dead[None, :], mask[None, :], np.array([u], np.float32))
        assert m.ids[0] == -1 and m.logZ_valid[0] == -np.inf and m.logZ_all[0] == pytest.approx(lse_all, abs=1e-12)
    one = dead.copy()
    one[17] = 0.7
    lse_one = logsumexp(one.astype(np.float64))
    for u in (0.0, 0.25, 0.5, float(np.float32(1.0) - np.float32(2 ** -24))):
        r = one_step(one, mask, u)
        assert r.ids[0] == 17
        assert r.logZ_valid[0] == pytest.approx(float(np.float32(0.7)) - lse_one, abs=1e-12)
        assert r.cdf_lo[0] == 0.0 and r.cdf_hi[0] == 1.0
        assert r.logZ_all[0] == pytest.approx(lse_one, abs=1e-12)
    # a single valid token at -inf: the same
    single = np.zeros(V, np.uint8)
    single[9] = 1
    l9 = l.copy()
    l9[9] = -np.inf
    r = one_step(l9, single, 0.4)
    assert r.ids[0] == -1 and r.logZ_valid[0] == -np.inf


def test_decode_loop_row_without_valid_mass_stops_outside_S_with_score_zero():
    """Algorithm 1's update multiplies x by the valid mass; when that mass is 0 the row can neither draw a token
    nor ever be accepted.  The loop leaves such a row where it is, outside S, with logx = -inf, and the rows
    beside it are unaffected."""
    V = 4
    seqs = [[0, 1], [0, 2], [1, 3]]
    S = W.constraint_set_from_lists(seqs, V)
    trie = oracle.Trie(S.tokens, S.offsets, V)
    B = 40
    rng = np.random.default_rng(2)
    un = rng.random((2, B), dtype=np.float32)
    first = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    after0 = np.array([0.3, -np.inf, -np.inf, 0.1], np.float32)      # both continuations of [0] have probability 0
    after1 = np.log(np.array([0.1, 0.2, 0.3, 0.4])).astype(np.float32)

    def logits_for_step(step, seqs_now, lens_now):
        if step == 0:
            return np.broadcast_to(first, (B, V)).copy()
        return np.stack([after0 if seqs_now[b, 0] == 0 else after1 for b in range(B)])
    res = oracle.decode_loop(trie, B, logits_for_step, lambda s: un[s])
    went0 = un[0] < 0.5 / 0.75                                       # P(0 | valid) = 0.5 / (0.5 + 0.25)
    assert went0.any() and (~went0).any()
    assert np.array_equal(res.dead, went0)
    assert (res.lens[went0] == 1).all() and (res.seqs[went0, 0] == 0).all() and (res.logx[went0] == -np.inf).all()
    assert (res.lens[~went0] == 2).all() and (res.seqs[~went0, 1] == 3).all()
    assert np.allclose(res.logx[~went0], math.log(0.75) + math.log(0.4), atol=1e-7)
    assert res.steps == 2
    # the outer loop never returns such a candidate: not through an accept round (x = 0 > epsilon is false also
    # for epsilon = 0), not through the resampling (weight 0)
    K = 2
    logx = np.array([[-np.inf, -np.inf, math.log(0.3), -np.inf],
                     [math.log(0.2), -np.inf, -np.inf, -np.inf],
                     [-np.inf, -np.inf, math.log(0.3), math.log(0.01)],
                     [math.log(0.6), -np.inf, -np.inf, -np.inf]])     # [2K candidates, Q = 4 queries]
    zero = np.zeros((K, 4))
    for u in (0.0, 0.3, 0.7, 0.999999):
        ch, nd, acc = oracle.disc_select(logx, K, zero, np.full(4, u))
        assert list(ch[:3]) == [1, -1, 0] and list(acc[:3]) == [1, 0, 1] and list(nd[:3]) == [2, 4, 1]
        assert ch[3] == 2 and acc[3] == 0 and nd[3] == 4             # rejected twice (eps = 1 below), then the only live one
        ch, nd, acc = oracle.disc_select(logx, K, np.full((K, 4), 0.999999), np.full(4, u))
        assert ch[0] == 3 and ch[1] == -1 and ch[3] == 2 and not acc.any() and (nd == 4).all()
        ch, nd, acc = oracle.disc_select(logx, K, np.full((K, 4), 0.999999), np.full(4, u), reuse_rejected=True)
        assert list(ch) == [1, -1, 0, -1] and (nd == 2).all()
    # ... and with probability proportional to the scores among the live ones (0.3 : 0.01 in the last query's
    # fallback would need candidates 2, 3 of query 3: they are (log 0.01, -inf) above, so take a direct case)
    lx = np.log(np.array([[0.5], [1e-300], [0.2], [0.6]]))
    lx[1, 0] = -np.inf
    us = (np.arange(1000) + 0.5) / 1000
    picks = [int(oracle.disc_select(np.repeat(lx, 1, axis=1), 2, np.full((2, 1), 0.999999), np.array([u]))[0][0]) for u in us]
    assert set(picks) == {2, 3} and picks.count(2) == 250            # 0.2 / (0.2 + 0.6)


def test_loading_the_oracle_starts_no_process_and_refuses_a_stale_library(monkeypatch, tmp_path):
    """The oracle is loaded inside processes that have a GPU open; nothing may be compiled (no child process at
    all) from there.  A library built from another source file is refused, not rebuilt."""
    import importlib
    import subprocess

    def forbidden(*a, **k):
        raise AssertionError("a process was started while loading the oracle")
    for mod, name in ((subprocess, "Popen"), (subprocess, "run"), (os, "system"), (os, "fork"), (os, "posix_spawn"),
                      (os, "execv"), (os, "execve"), (os, "popen")):
        monkeypatch.setattr(mod, name, forbidden)
    fresh = importlib.reload(oracle)
    try:
        assert fresh._lib is None
        assert fresh.max_threads() >= 1                               # first call: loads the library
        S = W.constraint_set_from_lists([[1, 2], [3]], 5)
        t = fresh.Trie(S.tokens, S.offsets, 5)
        assert t.n_members == 2
        # another source file: refused
        other = tmp_path / "ppv_oracle.c"
        other.write_bytes(open(fresh._SRC, "rb").read() + b"\n/* changed */\n")
        monkeypatch.setattr(fresh, "_SRC", str(other))
        monkeypatch.setattr(fresh, "_lib", None)
        with pytest.raises(RuntimeError, match="built from another"):
            fresh.max_threads()
        # no library at all: refused
        monkeypatch.setattr(fresh, "_LIB", str(tmp_path / "missing.so"))
        with pytest.raises(RuntimeError, match="missing"):
            fresh.max_threads()
    finally:
        monkeypatch.undo()
        importlib.reload(oracle)
