"""constrained_sample_noalloc, the entry point for callers that cannot allocate (graph capture, serving loops): it
meets in a fixed scratch array instead of an allocated one and must give constrained_sample's results bit for bit,
also on a second, smaller call that finds the array as the first call left it."""
import numpy as np
import pytest
import torch

from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, to_dev, tuning

pytestmark = pytest.mark.gpu


def make_case(B, V, dtype, seed):
    rng = np.random.default_rng(seed)
    lg = (rng.standard_normal((B, V)) * 2).astype(np.float32)
    mask = np.zeros((B, V), np.uint8)
    for b in range(B):
        c = min([0, 1, 5, 64, 65, 900, 3000, V // 3][b % 8], V // 2)
        mask[b, rng.choice(V, c, replace=False)] = 1
    words = np.packbits(np.pad(mask, ((0, 0), (0, (-V) % 32))), axis=1, bitorder="little").view(np.int32)
    un = rng.random(B, dtype=np.float32)
    if dtype == "bf16":
        ld = to_dev(W.f32_to_bf16_bits(lg).view(np.int16)).view(torch.bfloat16)
    else:
        ld = to_dev(lg)
    return ld, to_dev(words), to_dev(un)


def run(fn, ld, words, un, T):
    B = ld.shape[0]
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    lza = torch.full((B,), 3.0, dtype=torch.float32, device=DEV)
    fn(ld, words, un, ids, lzv, lza, temperature=T)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lzv.cpu().numpy().view(np.int32), lza.cpu().numpy().view(np.int32)


@pytest.mark.parametrize("split", [0, 4, 16, 1])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_noalloc_equals_constrained_sample_on_two_calls_in_a_row(dtype, split):
    """Two calls in a row on the same GPU, the second with fewer and shorter rows; each must equal the allocating
    entry point bit for bit, with the library's own choice of workgroups per row and with forced ones."""
    with tuning(ppv.PPV_TUNE_ROW_SPLIT, split):
        for B, V, T, seed in ((40, 128_256, 1.0, 1), (9, 50_264, 0.7, 2), (40, 128_256, 1.3, 3), (3, 1_000, 1.0, 4)):
            ld, words, un = make_case(B, V, dtype, seed)
            want = run(ppv.constrained_sample, ld, words, un, T)
            got = run(ppv.constrained_sample_noalloc, ld, words, un, T)
            for g, w in zip(got, want):
                assert np.array_equal(g, w), (B, V, T)
            assert (want[0][np.arange(B) % 8 == 0] == -1).all() and (want[0][np.arange(B) % 8 != 0] >= 0).all()


def test_noalloc_under_graph_capture_and_its_largest_batch():
    """The call can be captured (its first call on the device has been made above or is made here, outside the
    capture) and replayed; a batch beyond PPV_NOALLOC_MAX_ROWS is refused with PPV_ERANGE."""
    ld, words, un = make_case(24, 128_256, "bf16", 7)
    want = run(ppv.constrained_sample, ld, words, un, 1.0)
    B = ld.shape[0]
    ids = torch.full((B,), -7, dtype=torch.int32, device=DEV)
    lzv = torch.zeros(B, dtype=torch.float32, device=DEV)
    lza = torch.zeros(B, dtype=torch.float32, device=DEV)
    ppv.constrained_sample_noalloc(ld, words, un, ids, lzv, lza)          # resolves the array's address
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):                                          # a stream that never made a call before
        ppv.constrained_sample_noalloc(ld, words, un, ids, lzv, lza)
    for _ in range(3):
        ids.fill_(-9)
        lzv.fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(ids.cpu().numpy(), want[0])
        assert np.array_equal(lzv.cpu().numpy().view(np.int32), want[1])
        assert np.array_equal(lza.cpu().numpy().view(np.int32), want[2])
    big = ppv.PPV_NOALLOC_MAX_ROWS + 1
    ld, words, un = make_case(big, 4_096, "bf16", 8)
    out = [torch.zeros(big, dtype=torch.int32, device=DEV), torch.zeros(big, device=DEV)]
    with pytest.raises(ppv.PPVError) as e:
        ppv.constrained_sample_noalloc(ld, words, un, out[0], out[1])
    assert e.value.status == -4
    ld, words, un = make_case(ppv.PPV_NOALLOC_MAX_ROWS, 4_096, "bf16", 9)  # the largest batch itself is fine
    want = run(ppv.constrained_sample, ld, words, un, 1.0)
    got = run(ppv.constrained_sample_noalloc, ld, words, un, 1.0)
    for g, w in zip(got, want):
        assert np.array_equal(g, w)
