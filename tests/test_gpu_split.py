"""Rows spread over several workgroups (small batches): every number of workgroups per row gives bit for bit the
result of one workgroup per row, which in turn is checked against the oracle.  The split is a launch detail
(PPV_TUNE_ROW_SPLIT forces it; the library picks it from the batch size and the row length otherwise)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, check_sample_rows, logits_to_dev, to_dev, tuning
from test_gpu_parity import setup_case

pytestmark = pytest.mark.gpu

SPLITS = (1, 2, 4, 8, 16)


def pack(mask: np.ndarray) -> np.ndarray:
    B, V = mask.shape
    pad = (-V) % 32
    return np.packbits(np.pad(mask, ((0, 0), (0, pad))), axis=1, bitorder="little").view(np.uint32).view(np.int32)


def sample_all_splits(logits_dev, words_dev, un_dev, temperature=1.0, waves=0):
    """constrained_sample with 1, 2, ... workgroups per row; returns the unsplit result after checking that every
    split reproduces its bits."""
    B = logits_dev.shape[0]
    base = None
    for k in SPLITS:
        ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
        lzv = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
        lza = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
        with tuning(ppv.PPV_TUNE_ROW_SPLIT, k), tuning(ppv.PPV_TUNE_WAVES_PER_ROW, waves):
            ppv.constrained_sample(logits_dev, words_dev, un_dev, ids, lzv, lza, temperature=temperature)
        torch.cuda.synchronize()
        got = (ids.cpu().numpy(), lzv.cpu().numpy(), lza.cpu().numpy())
        if base is None:
            base = got
            continue
        assert np.array_equal(got[0], base[0]), (k, np.nonzero(got[0] != base[0])[0][:8])
        assert np.array_equal(got[1].view(np.int32), base[1].view(np.int32)), k
        assert np.array_equal(got[2].view(np.int32), base[2].view(np.int32)), k
    return base


@pytest.mark.parametrize("name", ["C2", "C5s", "C3s"])
def test_split_rows_on_the_workloads(name):
    cfg, S, trie, index = setup_case(name)
    pb = W.make_prefix_batch(cfg, S)
    logits = W.make_logits(cfg)
    un = W.make_uniforms(cfg)
    ref = trie.step(pb.prefixes, pb.lens, W.logits_as_f32(cfg, logits), un, threads=8)
    ids, lzv, lza = sample_all_splits(logits_to_dev(cfg, logits), to_dev(pack(ref.mask)), to_dev(un))
    check_sample_rows(cfg.dtype, ref, lambda b: ref.mask[b], un, ids, lzv, lza)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("waves", [0, 1, 2])
def test_split_rows_hand_made_masks(dtype, waves):
    """List rows of 0, 1, 63, 64, 65, 700 and 1,000 valid tokens, image rows, an image row whose valid mass lies far
    below the row maximum (the second pass over the row), rows with -inf tiles, a ragged last tile; several tiles per
    workgroup and fewer tiles than wavefronts."""
    V = 128_256                                               # the vocabulary of the paper's larger model (Table 1)
    rng = np.random.default_rng(31)
    counts = [0, 1, 63, 64, 65, 700, 1000, 1100, 5000, V // 2, 300, 40, 4000, 1]
    B = len(counts)
    lg = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    mask = np.zeros((B, V), np.uint8)
    for b, c in enumerate(counts):
        mask[b, rng.choice(V, c, replace=False)] = 1
    lg[10, mask[10] == 1] -= 150.0                            # list row, mass ~ e^-150
    lg[12, mask[12] == 1] -= 60.0                             # image row, mass ~ e^-55: sums are redone
    lg[11, : V // 3] = -np.inf                                # whole tiles without a finite value
    lg[13, mask[13] == 1] = -np.inf                           # the only valid token has probability 0
    un = rng.random(B, dtype=np.float32)
    un[2], un[3] = 0.0, np.float32(1.0) - np.float32(2 ** -24)
    if dtype == "bf16":
        bits = W.f32_to_bf16_bits(lg)
        lf = W.bf16_bits_to_f32(bits)
        ld = to_dev(bits.view(np.int16)).view(torch.bfloat16)
    else:
        lf, ld = lg, to_dev(lg)
    ids, lzv, lza = sample_all_splits(ld, to_dev(pack(mask)), to_dev(un), waves=waves)
    ref = oracle.masked_sample(lf, mask, un, threads=8)
    check_sample_rows(dtype, ref, lambda b: mask[b], un, ids, lzv, lza)
    assert ids[0] == -1 and ids[13] == -1 and lzv[13] == -np.inf


def test_split_rows_with_temperature_and_a_second_smaller_call():
    """The scratch area keeps what the last call left: a second, smaller call right after a larger one, at another
    temperature and on other rows, must not see any of it."""
    cfg, S, trie, index = setup_case("C2")
    pb = W.make_prefix_batch(cfg, S)
    for step, (rows, T) in enumerate([(slice(0, 64), 0.7), (slice(5, 22), 1.9), (slice(0, 64), 1.0)]):
        logits = W.make_logits(cfg, step=40 + step)[rows]
        un = W.make_uniforms(cfg, step=40 + step)[rows]
        P, L = pb.prefixes[rows], pb.lens[rows]
        ref = trie.step(P, L, W.logits_as_f32(cfg, logits), un, threads=8, temperature=T)
        ids, lzv, lza = sample_all_splits(logits_to_dev(cfg, logits), to_dev(pack(ref.mask)), to_dev(un), temperature=T)
        check_sample_rows(cfg.dtype, ref, lambda b: ref.mask[b], un, ids, lzv, lza)


@pytest.mark.parametrize("use_state", [True, False])
def test_split_rows_in_the_decode_step(use_state):
    """The fused decode step with its rows split: the whole loop, every split, bit for bit the unsplit loop."""
    cfg, S, trie, index = setup_case("C3s")
    B, L = 48, index.l_max
    logits = torch.stack([logits_to_dev(cfg, W.make_logits(cfg, batch=B, step=300 + s)) for s in range(L)])
    un = torch.stack([to_dev(W.make_uniforms(cfg, batch=B, step=300 + s)) for s in range(L)])
    base = None
    for k in SPLITS:
        P = torch.full((B, L), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        lens = torch.zeros(B, dtype=torch.int32, device=DEV)
        act = torch.ones(B, dtype=torch.uint8, device=DEV)
        state = None
        logx = torch.zeros(B, dtype=torch.float32, device=DEV)
        if use_state:
            state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
            ppv.ppv_decode_begin(index, P, lens, state, act, logx)
        ids = torch.full((L, B), -5, dtype=torch.int32, device=DEV)
        lz = torch.full((L, B), 2.0, dtype=torch.float32, device=DEV)
        with tuning(ppv.PPV_TUNE_ROW_SPLIT, k):
            for s in range(L):
                ppv.ppv_decode_step(index, P, lens, act, logits[s], un[s], ids[s], lz[s], logx, state=state)
        torch.cuda.synchronize()
        got = [t.cpu().numpy() for t in (P, lens, act, ids, lz.view(torch.int32), logx.view(torch.int32))]
        if base is None:
            base = got
            assert not got[2].any() and (got[1] > 0).all()
            q = trie.query(got[0], got[1], want_mask=False)
            assert (q.member == 1).all()                       # every row ended on a member of S
            continue
        for a, b in zip(got, base):
            assert np.array_equal(a, b), k


def test_split_rows_under_graph_capture():
    """A stream that is being captured cannot allocate its scratch area: without one the rows are simply not
    split; with one (the stream made a call before the capture) they are.  Replays equal the eager result."""
    cfg, S, trie, index = setup_case("C2")
    pb = W.make_prefix_batch(cfg, S)
    logits = logits_to_dev(cfg, W.make_logits(cfg))
    un = to_dev(W.make_uniforms(cfg))
    ref = trie.query(pb.prefixes, pb.lens)
    words = to_dev(pack(ref.mask))
    B = logits.shape[0]
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.constrained_sample(logits, words, un, ids, lzv)
    torch.cuda.synchronize()
    want = (ids.cpu().numpy().copy(), lzv.cpu().numpy().copy())
    for warm in (False, True):
        side = torch.cuda.Stream()
        if warm:
            with torch.cuda.stream(side):
                ppv.constrained_sample(logits, words, un, ids, lzv)
            side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ppv.constrained_sample(logits, words, un, ids, lzv)
        for _ in range(3):
            ids.fill_(-9)
            lzv.fill_(7.0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(ids.cpu().numpy(), want[0])
            assert np.array_equal(lzv.cpu().numpy().view(np.int32), want[1].view(np.int32))
