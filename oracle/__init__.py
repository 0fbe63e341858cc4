"""CPU oracle (test infrastructure only): ctypes front for ``ppv_oracle.c``.

Only tests, the smoke check and the CPU-baseline leg of the benchmark may import this
package; the HIP path never does, and this package imports nothing from the HIP path.

``Trie``            pointer-based prefix tree over S (Section 2.1, "Prefix-tree")
``Trie.query``      valid-next-token masks, rank ranges [lo,hi) in sorted S, membership
``Trie.step``       query + one constrained decoding step per row (Algorithm 1, SampleCandidate body)
``decode_loop``     Algorithm 1's SampleCandidate for a batch of rows: extend until the row is in S
``SortedArray``     Algorithm 2 as printed: sorted array X, top-M candidates, one binary search per candidate
``masked_sample``   masked softmax mass + inverse-CDF sample for given masks
``disc_select``     Algorithm 1 after SampleCandidate: accept / reject rounds and the resampling fallback
"""
from __future__ import annotations

import ctypes as C
import hashlib
import os
from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def source_digest() -> str:
    """SHA-256 of ppv_oracle.c as it is on disk; the build stamps the same digest into liboracle.so."""
    with open(_SRC, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()


def _load():
    """Load liboracle.so.  Never compiles: a process that checks the HIP path has the GPU open, and no compiler
    (no child process at all) is started from there.  The library is built by `python -m oracle.build`
    (`__graft_entry__.build()` runs it); a missing library, or one built from another ppv_oracle.c, is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB):
        raise RuntimeError(f"{_LIB} is missing: build it first with `python -m oracle.build`")
    lib = C.CDLL(_LIB)
    lib.oracle_source_digest.restype = C.c_char_p
    built_from = lib.oracle_source_digest().decode()
    if built_from != source_digest():
        raise RuntimeError(f"{_LIB} was built from another ppv_oracle.c (digest {built_from[:12]}..., source "
                           f"{source_digest()[:12]}...): rebuild it with `python -m oracle.build`")
    p = C.c_void_p
    lib.oracle_trie_build.restype = p
    lib.oracle_trie_build.argtypes = [p, p, C.c_int64, C.c_int32]
    lib.oracle_trie_free.argtypes = [p]
    lib.oracle_trie_members.restype = C.c_int64
    lib.oracle_trie_members.argtypes = [p]
    lib.oracle_trie_nodes.restype = C.c_int64
    lib.oracle_trie_nodes.argtypes = [p]
    lib.oracle_trie_lmax.restype = C.c_int32
    lib.oracle_trie_lmax.argtypes = [p]
    lib.oracle_step_batch.restype = None
    lib.oracle_step_batch.argtypes = [p, p, C.c_int32, p, C.c_int32, p, p, p, p, p, p, p, p, p, p, p, C.c_int32,
                                      C.c_double]
    lib.oracle_max_threads.restype = C.c_int32
    lib.oracle_sorted_build.restype = p
    lib.oracle_sorted_build.argtypes = [p, p, C.c_int64, C.c_int32]
    lib.oracle_sorted_free.argtypes = [p]
    lib.oracle_sorted_rows.restype = C.c_int64
    lib.oracle_sorted_rows.argtypes = [p]
    lib.oracle_topm_batch.restype = None
    lib.oracle_topm_batch.argtypes = [p, p, C.c_int32, p, C.c_int32, p, C.c_int32, p, p, p, C.c_int32]
    lib.oracle_sample_batch.restype = None
    lib.oracle_sample_batch.argtypes = [p, C.c_int64, p, p, C.c_int32, p, p, p, p, p, C.c_int32, C.c_double]
    _lib = lib
    return lib


def max_threads() -> int:
    return int(_load().oracle_max_threads())


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


@dataclass
class StepResult:
    mask: np.ndarray          # uint8 [B, V], one byte per token
    lo: np.ndarray            # int64 [B]
    hi: np.ndarray            # int64 [B]
    member: np.ndarray        # int32 [B]
    ids: Optional[np.ndarray] = None          # int32 [B]
    logZ_valid: Optional[np.ndarray] = None   # float64 [B]
    logZ_all: Optional[np.ndarray] = None     # float64 [B]
    cdf_lo: Optional[np.ndarray] = None       # float64 [B]
    cdf_hi: Optional[np.ndarray] = None       # float64 [B]


class Trie:
    def __init__(self, tokens: np.ndarray, offsets: np.ndarray, vocab: int):
        lib = _load()
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        self.vocab = int(vocab)
        self._h = lib.oracle_trie_build(_ptr(tokens), _ptr(offsets), int(offsets.shape[0] - 1), int(vocab))
        if not self._h:
            raise ValueError("oracle_trie_build rejected S (empty set, empty sequence or token out of range)")
        self.n_members = int(lib.oracle_trie_members(self._h))
        self.n_nodes = int(lib.oracle_trie_nodes(self._h))
        self.l_max = int(lib.oracle_trie_lmax(self._h))

    def close(self):
        if getattr(self, "_h", None):
            _load().oracle_trie_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _run(self, prefixes, lens, logits, uniforms, want_mask, threads, temperature=1.0) -> StepResult:
        assert temperature > 0.0
        prefixes = np.ascontiguousarray(prefixes, dtype=np.int32)
        if prefixes.ndim == 1:
            prefixes = prefixes[None, :]
        lens = np.ascontiguousarray(lens, dtype=np.int32)
        B, stride = prefixes.shape
        assert lens.shape == (B,) and (lens >= 0).all() and (lens <= stride).all()
        V = self.vocab
        mask = np.empty((B, V), dtype=np.uint8) if want_mask else None
        lo = np.empty(B, dtype=np.int64)
        hi = np.empty(B, dtype=np.int64)
        member = np.empty(B, dtype=np.int32)
        res = StepResult(mask, lo, hi, member)
        if logits is not None:
            logits = np.ascontiguousarray(logits, dtype=np.float32)
            uniforms = np.ascontiguousarray(uniforms, dtype=np.float32)
            assert logits.shape == (B, V) and uniforms.shape == (B,)
            res.ids = np.empty(B, dtype=np.int32)
            res.logZ_valid = np.empty(B, dtype=np.float64)
            res.logZ_all = np.empty(B, dtype=np.float64)
            res.cdf_lo = np.empty(B, dtype=np.float64)
            res.cdf_hi = np.empty(B, dtype=np.float64)
        _load().oracle_step_batch(self._h, _ptr(prefixes), stride, _ptr(lens), B, _ptr(logits), _ptr(uniforms),
                                  _ptr(mask), _ptr(lo), _ptr(hi), _ptr(member), _ptr(res.ids),
                                  _ptr(res.logZ_valid), _ptr(res.logZ_all), _ptr(res.cdf_lo), _ptr(res.cdf_hi),
                                  int(threads), float(temperature))
        return res

    def query(self, prefixes, lens, want_mask: bool = True, threads: int = 1) -> StepResult:
        """mask / [lo,hi) / member for a batch of prefixes (int32 [B, stride], lens int32 [B])."""
        return self._run(prefixes, lens, None, None, want_mask, threads, 1.0)

    def step(self, prefixes, lens, logits_f32, uniforms, want_mask: bool = True, threads: int = 1,
             temperature: float = 1.0) -> StepResult:
        """query + masked softmax mass + inverse-CDF sample per row, with P = softmax(logits / temperature)."""
        return self._run(prefixes, lens, logits_f32, uniforms, want_mask, threads, temperature)


@dataclass
class TopMResult:
    top_ids: np.ndarray       # int32 [B, M] candidates in order of decreasing probability (ties: smaller id first), -1 beyond min(M, V)
    mask_V: np.ndarray        # uint8 [B, M] verdict per candidate
    mask: Optional[np.ndarray]  # uint8 [B, V] the extended mask


class SortedArray:
    """Algorithm 2 as printed: the members of S as a lexicographically sorted array, searched per candidate."""

    def __init__(self, tokens: np.ndarray, offsets: np.ndarray, vocab: int):
        lib = _load()
        tokens = np.ascontiguousarray(tokens, dtype=np.int32)
        offsets = np.ascontiguousarray(offsets, dtype=np.int64)
        self.vocab = int(vocab)
        self._h = lib.oracle_sorted_build(_ptr(tokens), _ptr(offsets), int(offsets.shape[0] - 1), int(vocab))
        if not self._h:
            raise ValueError("oracle_sorted_build rejected S")
        self.n_rows = int(lib.oracle_sorted_rows(self._h))

    def close(self):
        if getattr(self, "_h", None):
            _load().oracle_sorted_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def topm(self, prefixes, lens, logits_f32, M: int, want_mask: bool = True, threads: int = 1) -> TopMResult:
        prefixes = np.ascontiguousarray(prefixes, dtype=np.int32)
        if prefixes.ndim == 1:
            prefixes = prefixes[None, :]
        lens = np.ascontiguousarray(lens, dtype=np.int32)
        logits = np.ascontiguousarray(logits_f32, dtype=np.float32)
        B, stride = prefixes.shape
        assert lens.shape == (B,) and (lens >= 0).all() and (lens <= stride).all()
        assert logits.shape == (B, self.vocab) and M >= 1
        top = np.empty((B, M), dtype=np.int32)
        mv = np.empty((B, M), dtype=np.uint8)
        mask = np.empty((B, self.vocab), dtype=np.uint8) if want_mask else None
        _load().oracle_topm_batch(self._h, _ptr(prefixes), stride, _ptr(lens), B, _ptr(logits), int(M), _ptr(top),
                                  _ptr(mv), _ptr(mask), int(threads))
        return TopMResult(top, mv, mask)


def masked_sample(logits_f32: np.ndarray, mask: np.ndarray, uniforms: np.ndarray, threads: int = 1,
                  temperature: float = 1.0) -> StepResult:
    """Algorithm 1's "sample a token from P (.) mask / |P (.) mask|_1" and its mass for given masks (uint8 [B, V])."""
    logits = np.ascontiguousarray(logits_f32, dtype=np.float32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    un = np.ascontiguousarray(uniforms, dtype=np.float32)
    B, V = logits.shape
    assert mask.shape == (B, V) and un.shape == (B,) and temperature > 0.0
    res = StepResult(mask, None, None, None)
    res.ids = np.empty(B, dtype=np.int32)
    res.logZ_valid = np.empty(B, dtype=np.float64)
    res.logZ_all = np.empty(B, dtype=np.float64)
    res.cdf_lo = np.empty(B, dtype=np.float64)
    res.cdf_hi = np.empty(B, dtype=np.float64)
    _load().oracle_sample_batch(_ptr(logits), V, _ptr(mask), _ptr(un), B, _ptr(res.ids), _ptr(res.logZ_valid),
                                _ptr(res.logZ_all), _ptr(res.cdf_lo), _ptr(res.cdf_hi), int(threads), float(temperature))
    return res


@dataclass
class LoopResult:
    seqs: np.ndarray        # int32 [B, l_max] generated sequences (unused slots = -1)
    lens: np.ndarray        # int32 [B]
    logx: np.ndarray        # float64 [B]: log of the importance score x = prod of per-step valid masses
    steps: int              # decode steps run until every row had stopped
    ids_per_step: list      # list of int32 [B] (-1 for rows already finished)
    logZ_per_step: list     # list of float64 [B] (nan for rows already finished)
    cdf_lo_per_step: list
    cdf_hi_per_step: list
    active_per_step: list   # list of bool [B]: row took part in that step
    dead: np.ndarray        # bool [B]: the row stopped outside S (see decode_loop); its logx is -inf


def decode_loop(trie: Trie, B: int, logits_f32_for_step: Callable[[int, np.ndarray, np.ndarray], np.ndarray],
                uniforms_for_step: Callable[[int], np.ndarray], threads: int = 1,
                temperature: float = 1.0) -> LoopResult:
    """Algorithm 1, SampleCandidate, for B independent rows: start from the empty sequence and
    repeat {distribution, mask, sample, append, x *= valid mass} while the row is not in S.
    A row stops the first time it is a member, also when that member has extensions.
    `logits_f32_for_step(step, seqs, lens)` returns the [B, V] logits of that step (the stand-in
    for L(a, T); it may look at the rows' current sequences).

    A row whose valid tokens all have probability 0 cannot draw a token: the update of Algorithm 1 multiplies
    its x by |P (.) mask|_1 = 0, so the row stops where it is, outside S, with logx = -inf (`dead`): the
    accept test x > epsilon of the outer loop can never pass for it and it has weight 0 in the resampling."""
    l_max = trie.l_max
    seqs = np.full((B, l_max), -1, dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    logx = np.zeros(B, dtype=np.float64)
    active = np.ones(B, dtype=bool)
    dead = np.zeros(B, dtype=bool)
    out = LoopResult(seqs, lens, logx, 0, [], [], [], [], [], dead)
    step = 0
    while active.any():
        assert step < l_max, "a row outlived the longest member of S"
        rows = np.nonzero(active)[0]
        lg = logits_f32_for_step(step, seqs, lens)[rows]
        un = uniforms_for_step(step)[rows]
        r = trie.step(seqs[rows], lens[rows], lg, un, want_mask=False, threads=threads, temperature=temperature)
        ids = np.full(B, -1, dtype=np.int32)
        lz = np.full(B, np.nan)
        cl = np.full(B, np.nan)
        ch = np.full(B, np.nan)
        ids[rows], lz[rows], cl[rows], ch[rows] = r.ids, r.logZ_valid, r.cdf_lo, r.cdf_hi
        out.ids_per_step.append(ids.copy())
        out.logZ_per_step.append(lz)
        out.cdf_lo_per_step.append(cl)
        out.cdf_hi_per_step.append(ch)
        out.active_per_step.append(active.copy())
        took = rows[ids[rows] >= 0]
        stuck = rows[ids[rows] < 0]
        dead[stuck] = True
        logx[stuck] = -np.inf
        active[stuck] = False
        seqs[took, lens[took]] = ids[took]
        lens[took] += 1
        logx[took] += lz[took]
        q = trie.query(seqs[took], lens[took], want_mask=False, threads=threads)
        active[took] = q.member == 0
        step += 1
    out.steps = step
    return out


def disc_select(logx: np.ndarray, K: int, accept_u: np.ndarray, resample_u: np.ndarray, reuse_rejected: bool = False):
    """Algorithm 1 after SampleCandidate: the accept / reject rounds and the importance-resampling fallback,
    for Q independent queries whose candidates have already been drawn.

    logx[c, q]      log importance score of candidate c of query q (x = exp(logx) in (0, 1]); candidates
                    0..K-1 are the ones offered to the accept/reject rounds, in order; candidates K..2K-1 are
                    the K fresh ones of the fallback (not needed when reuse_rejected)
    accept_u[k, q]  the uniform epsilon of round k: candidate k is accepted iff x > epsilon
    resample_u[q]   the uniform that drives the fallback: among its K candidates, in order, the first whose
                    cumulative score exceeds u * (sum of scores), i.e. candidate j with probability x_j / sum x
                    (the paper fixes no procedure; the last candidate of positive score if rounding lets none
                    exceed it).  A candidate of score 0 (logx = -inf: it stopped outside S) is never returned;
                    when all K scores are 0 nothing can be returned and chosen[q] = -1
    reuse_rejected  False: the fallback draws K new candidates, as the algorithm is printed;
                    True: it resamples among the K rejected ones (the reading under which K = 1 coincides with
                    plain constrained decoding, Section 4.1 "Methods")
    Returns chosen[q] (candidate index), n_draws[q] (candidates consumed: k+1 on acceptance in round k, else
    2K, or K when reusing), accepted[q] (1 iff returned by an accept round).  Double precision throughout."""
    logx = np.asarray(logx, dtype=np.float64)
    accept_u = np.asarray(accept_u, dtype=np.float64)
    resample_u = np.asarray(resample_u, dtype=np.float64)
    n_cand, Q = logx.shape
    assert accept_u.shape == (K, Q) and resample_u.shape == (Q,)
    assert n_cand >= (K if reuse_rejected else 2 * K)
    chosen = np.empty(Q, dtype=np.int32)
    n_draws = np.empty(Q, dtype=np.int32)
    accepted = np.zeros(Q, dtype=np.int32)
    for q in range(Q):
        done = False
        for k in range(K):
            if np.exp(logx[k, q]) > accept_u[k, q]:
                chosen[q], n_draws[q], accepted[q] = k, k + 1, 1
                done = True
                break
        if done:
            continue
        first = 0 if reuse_rejected else K
        lw = logx[first:first + K, q]
        n_draws[q] = K if reuse_rejected else 2 * K
        if lw.max() == -np.inf:                 # every score is 0: x_k / sum x is undefined, nothing is returned
            chosen[q] = -1
            continue
        w = np.exp(lw - lw.max())
        tau = resample_u[q] * w.sum()
        c, pick = 0.0, -1
        for j in range(K):
            c += w[j]
            if w[j] > 0.0:
                pick = j
                if c > tau:
                    break
        chosen[q] = first + pick
    return chosen, n_draws, accepted
