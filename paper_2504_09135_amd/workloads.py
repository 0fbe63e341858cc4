"""Seeded synthetic workloads: constraint sets S, prefix batches, logits and uniforms.

This module only *makes inputs*.  It holds none of the method's arithmetic (no
sorting of S into an index, no prefix lookup, no softmax, no sampling): both the
CPU oracle's tests and the HIP path's tests/bench draw their inputs from here so
that the two sides see identical bits.

The constraint sets stand in for the Wikipedia-title corpora of the paper's
Table 1 ("Task Statistics": 4.6-5.9 M sequences, 7.7-9.5 tokens on average,
vocabularies of 50,264 and 128,256 tokens), which are not available here; the
logits stand in for the language model L(a, T) of Algorithm 1.

Every draw comes from a counter-based generator (numpy's Philox) keyed by
``(seed, stream, index)``, so any slice (for example the logits of one decode
step) can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional, Tuple

import numpy as np

BASE_SEED = 20250409
STREAM_S, STREAM_PREFIX, STREAM_LOGITS, STREAM_UNIFORM = 1, 2, 3, 4
PAD_TOKEN = 0x7FFFFFF0  # fills prefix slots past lens[b]; never a real token


def rng_for(seed: int, stream: int, index: int = 0) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(stream) << np.uint64(32)) | np.uint64(index)],
                   dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


# --------------------------------------------------------------------------- configs
@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_seq: int                 # number of sequences drawn for S (distinct unless top_up=False)
    vocab: int
    len_kind: str              # "fixed" | "geometric" | "uniform"
    len_a: int                 # fixed: length; geometric: mean; uniform: low
    len_b: int                 # geometric: cap; uniform: high (inclusive)
    tok_kind: str              # "uniform" | "zipf" | "codebook"
    zipf_s: float = 0.0
    top_up: bool = True        # redraw until exactly n_seq distinct sequences
    batch: int = 16
    valid_frac: float = 1.0    # fraction of rows drawn as prefixes of members
    dtype: str = "f32"         # "f32" | "bf16"
    sigma: float = 1.0         # std of the normal logits
    loop: bool = False         # full decode loop from the empty prefix
    seed: int = BASE_SEED

    @property
    def l_max(self) -> int:
        return self.len_a if self.len_kind == "fixed" else self.len_b


CONFIGS: Dict[str, WorkloadConfig] = {
    "C1": WorkloadConfig("C1", 1_000, 1_024, "fixed", 8, 8, "uniform",
                         batch=16, valid_frac=0.75, dtype="f32", sigma=1.0),
    "C2": WorkloadConfig("C2", 100_000, 32_000, "geometric", 8, 16, "zipf", 1.1,
                         batch=64, valid_frac=0.90, dtype="bf16", sigma=2.0),
    "C3": WorkloadConfig("C3", 1_000_000, 32_000, "uniform", 4, 32, "zipf", 1.1,
                         batch=256, valid_frac=1.0, dtype="bf16", sigma=2.0, loop=True),
    "C4": WorkloadConfig("C4", 10_000_000, 1_024, "fixed", 4, 4, "codebook",
                         top_up=False, batch=4_096, valid_frac=1.0, dtype="f32", sigma=1.0),
    "C5": WorkloadConfig("C5", 5_000_000, 256_000, "uniform", 2, 24, "zipf", 1.05,
                         batch=1_024, valid_frac=0.95, dtype="bf16", sigma=3.0),
}


def scaled(cfg: WorkloadConfig, n_seq: int, batch: Optional[int] = None, name: Optional[str] = None
           ) -> WorkloadConfig:
    """Same recipe at a smaller |S| / batch (for cases the oracle finishes in seconds)."""
    from dataclasses import replace
    return replace(cfg, n_seq=n_seq, batch=batch if batch is not None else cfg.batch,
                   name=name or f"{cfg.name}@{n_seq}")


# --------------------------------------------------------------------------- S
@dataclass
class ConstraintSet:
    """S in CSR form on the host: sequence i is tokens[offsets[i]:offsets[i+1]]; order is shuffled."""
    tokens: np.ndarray      # int32 [sum len]
    offsets: np.ndarray     # int64 [n+1]
    vocab: int
    l_max: int

    @property
    def n(self) -> int:
        return int(self.offsets.shape[0] - 1)

    def lengths(self) -> np.ndarray:
        return np.diff(self.offsets)

    def seq(self, i: int) -> np.ndarray:
        return self.tokens[self.offsets[i]:self.offsets[i + 1]]

    def padded(self, pad: int = -1) -> np.ndarray:
        """[n, l_max] int32 matrix, rows padded with `pad` (host convenience for generators/tests)."""
        lens = self.lengths()
        out = np.full((self.n, self.l_max), pad, dtype=np.int32)
        col = np.arange(self.l_max)[None, :]
        out[col < lens[:, None]] = self.tokens
        return out


def _zipf_cdf(vocab: int, s: float) -> np.ndarray:
    w = np.arange(1, vocab + 1, dtype=np.float64) ** (-s)
    c = np.cumsum(w)
    return c / c[-1]


def _draw_lengths(cfg: WorkloadConfig, rng: np.random.Generator, n: int) -> np.ndarray:
    if cfg.len_kind == "fixed":
        return np.full(n, cfg.len_a, dtype=np.int64)
    if cfg.len_kind == "geometric":
        g = rng.geometric(1.0 / cfg.len_a, size=n)          # support {1,2,...}, mean len_a
        return np.minimum(g, cfg.len_b).astype(np.int64)
    if cfg.len_kind == "uniform":
        return rng.integers(cfg.len_a, cfg.len_b + 1, size=n, dtype=np.int64)
    raise ValueError(cfg.len_kind)


def _draw_padded(cfg: WorkloadConfig, rng: np.random.Generator, n: int,
                 zipf_cdf: Optional[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """n sequences as a [n, l_max] matrix padded with -1, plus their lengths."""
    lens = _draw_lengths(cfg, rng, n)
    L = cfg.l_max
    if cfg.tok_kind == "uniform":
        toks = rng.integers(0, cfg.vocab, size=(n, L), dtype=np.int32)
    elif cfg.tok_kind == "zipf":
        u = rng.random(size=(n, L))
        toks = np.searchsorted(zipf_cdf, u, side="right").astype(np.int32)
        np.minimum(toks, cfg.vocab - 1, out=toks)
    elif cfg.tok_kind == "codebook":
        per = cfg.vocab // L                                   # 256 codes per level
        toks = rng.integers(0, per, size=(n, L), dtype=np.int32)
        toks += (np.arange(L, dtype=np.int32) * per)[None, :]
    else:
        raise ValueError(cfg.tok_kind)
    toks[np.arange(L)[None, :] >= lens[:, None]] = -1
    return toks, lens


def _row_fingerprint(padded: np.ndarray) -> np.ndarray:
    """64-bit fingerprint per padded row; equal rows always get equal fingerprints."""
    h = np.full(padded.shape[0], 0x9E3779B97F4A7C15, dtype=np.uint64)
    mul = np.uint64(0xD1342543DE82EF95)
    with np.errstate(over="ignore"):
        for c in range(padded.shape[1]):
            h = (h ^ (padded[:, c].astype(np.int64).astype(np.uint64) + np.uint64(0x632BE59BD9B4E019))) * mul
            h ^= h >> np.uint64(29)
    return h


def make_constraint_set(cfg: WorkloadConfig) -> ConstraintSet:
    """Draw S for a config.  Rows are pairwise distinct (kept rows have pairwise distinct
    fingerprints, which implies distinct rows) and handed over in shuffled order."""
    cdf = _zipf_cdf(cfg.vocab, cfg.zipf_s) if cfg.tok_kind == "zipf" else None
    chunks, fps = [], np.empty(0, dtype=np.uint64)
    have, round_ = 0, 0
    while have < cfg.n_seq:
        rng = rng_for(cfg.seed, STREAM_S, round_)
        want = cfg.n_seq - have
        draw = want if round_ == 0 else max(1024, int(want * 1.5))
        padded, _ = _draw_padded(cfg, rng, draw, cdf)
        fp = _row_fingerprint(padded)
        _, first = np.unique(fp, return_index=True)             # dedupe inside this draw
        first.sort()
        padded, fp = padded[first], fp[first]
        if fps.size:
            fresh = ~np.isin(fp, fps)
            padded, fp = padded[fresh], fp[fresh]
        if padded.shape[0] > want:
            padded, fp = padded[:want], fp[:want]
        chunks.append(padded)
        fps = np.concatenate([fps, fp])
        have += padded.shape[0]
        round_ += 1
        if not cfg.top_up:
            break
    allp = np.concatenate(chunks, axis=0) if len(chunks) > 1 else chunks[0]
    perm = rng_for(cfg.seed, STREAM_S, 1_000_003).permutation(allp.shape[0])
    allp = allp[perm]
    lens = (allp >= 0).sum(axis=1).astype(np.int64)
    offsets = np.zeros(allp.shape[0] + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    tokens = allp[allp >= 0].astype(np.int32)                   # row-major => CSR order
    return ConstraintSet(tokens=tokens, offsets=offsets, vocab=cfg.vocab, l_max=cfg.l_max)


def constraint_set_from_lists(seqs, vocab: int) -> ConstraintSet:
    """Hand-written S (tests): list of token lists -> CSR."""
    lens = np.array([len(s) for s in seqs], dtype=np.int64)
    offsets = np.zeros(len(seqs) + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    tokens = np.array([t for s in seqs for t in s], dtype=np.int32)
    return ConstraintSet(tokens, offsets, vocab, int(lens.max()) if len(seqs) else 0)


# --------------------------------------------------------------------------- prefixes
@dataclass
class PrefixBatch:
    prefixes: np.ndarray    # int32 [B, stride], slots past lens[b] hold PAD_TOKEN
    lens: np.ndarray        # int32 [B]
    drawn_valid: np.ndarray  # bool [B]: row was drawn as a prefix of a member (not corrupted)

    @property
    def stride(self) -> int:
        return int(self.prefixes.shape[1])


def make_prefix_batch(cfg: WorkloadConfig, S: ConstraintSet, batch: Optional[int] = None,
                      index: int = 0) -> PrefixBatch:
    """B prefixes.  A `valid_frac` share are the first k ~ U{0..len-1} tokens of a uniformly
    chosen member.  The rest are corruptions, half of each kind:
      (a) such a prefix with k >= 1 whose last token is replaced by a different uniform token,
      (b) a uniform random token string of length U{1..l_max-1}.
    A corruption can land in S by chance (likely only at depth 1); nothing here checks, the
    oracle decides what is valid."""
    B = cfg.batch if batch is None else batch
    rng = rng_for(cfg.seed, STREAM_PREFIX, index)
    stride = max(S.l_max, 1)
    out = np.full((B, stride), PAD_TOKEN, dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    n_valid = int(round(B * cfg.valid_frac))
    kinds = np.zeros(B, dtype=np.int8)                         # 0 valid, 1 corrupt-last, 2 random
    n_bad = B - n_valid
    kinds[n_valid:n_valid + (n_bad + 1) // 2] = 1
    kinds[n_valid + (n_bad + 1) // 2:] = 2
    kinds = kinds[rng.permutation(B)]
    members = rng.integers(0, S.n, size=B)
    slens = S.lengths()
    for b in range(B):
        L = int(slens[members[b]])
        row = S.seq(int(members[b]))
        if kinds[b] == 0:
            k = int(rng.integers(0, L))
            out[b, :k] = row[:k]
        elif kinds[b] == 1:
            k = int(rng.integers(1, L + 1)) if L >= 1 else 1
            out[b, :k] = row[:k]
            repl = int(rng.integers(0, cfg.vocab - 1))
            out[b, k - 1] = repl if repl < row[k - 1] else repl + 1
        else:
            k = int(rng.integers(1, max(2, stride)))
            out[b, :k] = rng.integers(0, cfg.vocab, size=k, dtype=np.int32)
        lens[b] = k
    return PrefixBatch(out, lens, kinds == 0)


# --------------------------------------------------------------------------- logits / uniforms
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((b >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((b + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_logits(cfg: WorkloadConfig, batch: Optional[int] = None, step: int = 0) -> np.ndarray:
    """[B, V] logits ~ N(0, sigma) drawn in fp32; float32 array for "f32" configs, uint16 bf16 bit
    patterns (round-to-nearest-even of the fp32 draw) for "bf16" configs.  `step` selects an
    independent draw (one per decode step of the loop config)."""
    B = cfg.batch if batch is None else batch
    rng = rng_for(cfg.seed, STREAM_LOGITS, step)
    x = rng.standard_normal(size=(B, cfg.vocab), dtype=np.float32)
    if cfg.sigma != 1.0:
        x *= np.float32(cfg.sigma)
    return f32_to_bf16_bits(x) if cfg.dtype == "bf16" else x


def logits_as_f32(cfg: WorkloadConfig, logits: np.ndarray) -> np.ndarray:
    """The exact fp32 values of a logits array from make_logits (what the CPU side consumes)."""
    return bf16_bits_to_f32(logits) if cfg.dtype == "bf16" else logits


def make_uniforms(cfg: WorkloadConfig, batch: Optional[int] = None, step: int = 0) -> np.ndarray:
    """[B] fp32 uniforms in [0, 1)."""
    B = cfg.batch if batch is None else batch
    return rng_for(cfg.seed, STREAM_UNIFORM, step).random(size=B, dtype=np.float32)
