"""Helpers shared by the GPU parity tests: run the HIP path through the C-ABI binding and compare
with the CPU oracle under the stated tolerances."""
from __future__ import annotations

import contextlib

import numpy as np
import torch

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

# logZ_valid: |gpu - ref| <= tol * max(1, |ref|); fp32 logits 1e-5, bf16 logits 1e-3
LOGZ_TOL = {"f32": 1e-5, "bf16": 1e-3}
# sampled ids must match except where u lies within this distance of a CDF boundary
CDF_BAND = 1e-6

DEV = "cuda:0"


@contextlib.contextmanager
def tuning(knob: int, value: int):
    """A tuning / test switch of the library set for the duration of a block, then put back."""
    before = ppv.ppv_tuning_get(knob)
    ppv.ppv_tuning_set(knob, value)
    try:
        yield
    finally:
        ppv.ppv_tuning_set(knob, before)


def to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def logits_to_dev(cfg: W.WorkloadConfig, logits: np.ndarray) -> torch.Tensor:
    if cfg.dtype == "bf16":
        return to_dev(logits.view(np.int16)).view(torch.bfloat16)
    return to_dev(logits)


def unpack_mask(words: np.ndarray, V: int) -> np.ndarray:
    """uint32 [B, W] packed (bit v&31 of word v>>5, LSB first) -> uint8 [B, V]; also checks pad bits."""
    B = words.shape[0]
    bits = np.unpackbits(np.ascontiguousarray(words).view(np.uint8).reshape(B, -1), axis=1, bitorder="little")
    assert not bits[:, V:].any(), "bits at positions >= V must be zero"
    return bits[:, :V]


def gpu_query(index, prefixes: np.ndarray, lens: np.ndarray):
    B = prefixes.shape[0]
    mask = torch.full((B, index.n_words), -1, dtype=torch.int32, device=DEV)
    lo = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    hi = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    member = torch.full((B,), 7, dtype=torch.uint8, device=DEV)
    ppv.ppv_next_token_mask(index, to_dev(prefixes), to_dev(lens), mask, lo, hi, member)
    torch.cuda.synchronize()
    return (mask, mask.cpu().numpy().view(np.uint32), lo.cpu().numpy().view(np.uint32).astype(np.int64),
            hi.cpu().numpy().view(np.uint32).astype(np.int64), member.cpu().numpy().astype(np.int32))


def assert_query_parity(index, trie: oracle.Trie, prefixes, lens, threads=8):
    """Bit-exact masks, ranges and membership.  Returns (device mask, oracle result)."""
    dmask, words, lo, hi, member = gpu_query(index, prefixes, lens)
    ref = trie.query(prefixes, lens, want_mask=True, threads=threads)
    got = unpack_mask(words, index.vocab)
    bad = np.nonzero((got != ref.mask).any(axis=1))[0]
    assert bad.size == 0, f"mask rows differ: {bad[:8]} (lens {lens[bad[:8]]})"
    assert np.array_equal(lo, ref.lo), np.nonzero(lo != ref.lo)[0][:8]
    assert np.array_equal(hi, ref.hi), np.nonzero(hi != ref.hi)[0][:8]
    assert np.array_equal(member, ref.member), np.nonzero(member != ref.member)[0][:8]
    return dmask, ref


def check_sample_rows(dtype: str, ref, ref_mask_rows, uniforms, ids, lzv, lza=None, rows=None):
    """Compare ids / logZ_valid / logZ_all of the HIP path with an oracle StepResult.
    ref_mask_rows(b) must return the oracle's uint8 mask of row b (used only for excused rows)."""
    tol = LOGZ_TOL[dtype]
    n = len(ref.ids)
    excused = 0
    for b in range(n):
        r_id, g_id = int(ref.ids[b]), int(ids[b])
        name = b if rows is None else rows[b]
        if r_id < 0:
            assert g_id == -1 and lzv[b] == -np.inf, (name, g_id, lzv[b])
            continue
        r_lz = ref.logZ_valid[b]
        assert abs(float(lzv[b]) - r_lz) <= tol * max(1.0, abs(r_lz)), (name, float(lzv[b]), r_lz)
        if lza is not None:
            r_la = ref.logZ_all[b]
            assert abs(float(lza[b]) - r_la) <= tol * max(1.0, abs(r_la)), (name, float(lza[b]), r_la)
        if g_id == r_id:
            continue
        u = float(uniforms[b])
        valid = np.nonzero(ref_mask_rows(b))[0]
        pos = int(np.searchsorted(valid, r_id))
        ok = False
        if u - ref.cdf_lo[b] < CDF_BAND and pos > 0 and g_id == valid[pos - 1]:
            ok = True
        if ref.cdf_hi[b] - u < CDF_BAND and pos + 1 < len(valid) and g_id == valid[pos + 1]:
            ok = True
        assert ok, (name, "id", g_id, "oracle", r_id, "u", u, "cdf", ref.cdf_lo[b], ref.cdf_hi[b])
        excused += 1
    return excused


def gpu_sample(cfg, logits_dev, dmask, uniforms: np.ndarray, temperature: float = 1.0):
    B = logits_dev.shape[0]
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    lza = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    ppv.constrained_sample(logits_dev, dmask, to_dev(uniforms), ids, lzv, lza, temperature=temperature)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lzv.cpu().numpy(), lza.cpu().numpy()


def follow_loop(trie: oracle.Trie, B: int, logits_f32_for_step, uniforms_for_step, taken_ids_for_step, threads: int = 1,
                temperature: float = 1.0) -> oracle.LoopResult:
    """The oracle's own choice at every step of the decode loop (one Trie.step per decode step, recorded), with the
    rows then moved along the tokens the HIP path took (`taken_ids_for_step(step)` -> int32 [B]), so that one
    excused disagreement inside the CDF band does not invalidate the comparison of the steps after it.  The
    free-running loop is oracle.decode_loop; this one exists for the parity tests only."""
    l_max = trie.l_max
    seqs = np.full((B, l_max), -1, dtype=np.int32)
    lens = np.zeros(B, dtype=np.int32)
    logx = np.zeros(B, dtype=np.float64)
    active = np.ones(B, dtype=bool)
    dead = np.zeros(B, dtype=bool)
    out = oracle.LoopResult(seqs, lens, logx, 0, [], [], [], [], [], dead)
    step = 0
    while active.any():
        assert step < l_max, "a row outlived the longest member of S"
        rows = np.nonzero(active)[0]
        r = trie.step(seqs[rows], lens[rows], logits_f32_for_step(step, seqs, lens)[rows], uniforms_for_step(step)[rows],
                      want_mask=False, threads=threads, temperature=temperature)
        ids = np.full(B, -1, dtype=np.int32)
        lz, cl, ch = np.full(B, np.nan), np.full(B, np.nan), np.full(B, np.nan)
        ids[rows], lz[rows], cl[rows], ch[rows] = r.ids, r.logZ_valid, r.cdf_lo, r.cdf_hi
        out.ids_per_step.append(ids)
        out.logZ_per_step.append(lz)
        out.cdf_lo_per_step.append(cl)
        out.cdf_hi_per_step.append(ch)
        out.active_per_step.append(active.copy())
        stuck = rows[ids[rows] < 0]                 # the oracle found nothing to sample: the row stops outside S
        took = rows[ids[rows] >= 0]
        dead[stuck] = True
        logx[stuck] = -np.inf
        active[stuck] = False
        taken = np.asarray(taken_ids_for_step(step))[took]
        assert (taken >= 0).all(), "the HIP path sampled nothing where the oracle sampled a token"
        seqs[took, lens[took]] = taken
        lens[took] += 1
        logx[took] += lz[took]
        q = trie.query(seqs[took], lens[took], want_mask=False, threads=threads)
        active[took] = q.member == 0
        step += 1
    out.steps = step
    return out
