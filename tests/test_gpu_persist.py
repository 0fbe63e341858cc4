"""ppv_index_save / ppv_index_load: a loaded index answers exactly like the one that was saved (and like the
oracle); damaged or structurally wrong files are refused instead of reaching a kernel."""
import numpy as np
import pytest
import torch

from paper_2504_09135_amd import binding as ppv
from paper_2504_09135_amd import workloads as W

from gpu_helpers import DEV, assert_query_parity, gpu_query, logits_to_dev, to_dev
from test_gpu_parity import setup_case

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]

MASK64 = (1 << 64) - 1


@pytest.mark.parametrize("name", ["C2", "C3s", "C4s"])
def test_save_load_round_trip(name, tmp_path):
    cfg, S, trie, index = setup_case(name)
    path = str(tmp_path / f"{name}.ppv")
    ppv.ppv_index_save(index, path)
    loaded = ppv.ppv_index_load(path)
    assert ppv.ppv_index_info(loaded) == ppv.ppv_index_info(index)
    t0, o0 = ppv.ppv_index_export(index)
    t1, o1 = ppv.ppv_index_export(loaded)
    assert np.array_equal(t0, t1) and np.array_equal(o0, o1)
    pb = W.make_prefix_batch(cfg, S)
    lens = pb.lens.copy()
    lens[:2] = 0
    a = gpu_query(index, pb.prefixes, lens)
    b = gpu_query(loaded, pb.prefixes, lens)
    for x, y in zip(a[1:], b[1:]):
        assert np.array_equal(x, y)
    assert_query_parity(loaded, trie, pb.prefixes, lens)
    # the fused decode step (cursor, heavy images rebuilt at load) gives the same tokens on both
    B = pb.prefixes.shape[0]
    logits = logits_to_dev(cfg, W.make_logits(cfg))
    un = to_dev(W.make_uniforms(cfg))
    outs = []
    for ix in (index, loaded):
        P = torch.full((B, ix.l_max + 1), W.PAD_TOKEN, dtype=torch.int32, device=DEV)
        L = torch.zeros(B, dtype=torch.int32, device=DEV)
        active = torch.zeros(B, dtype=torch.uint8, device=DEV)
        state = torch.zeros((B, ppv.PPV_STATE_WORDS), dtype=torch.int32, device=DEV)
        logx = torch.zeros(B, dtype=torch.float32, device=DEV)
        ids = torch.full((B,), -5, dtype=torch.int32, device=DEV)
        lz = torch.zeros(B, dtype=torch.float32, device=DEV)
        ppv.ppv_decode_begin(ix, P, L, state, active, logx)
        for _ in range(3):
            ppv.ppv_decode_step(ix, P, L, active, logits, un, ids, lz, logx, state=state)
        torch.cuda.synchronize()
        outs.append((P.cpu().numpy(), L.cpu().numpy(), lz.cpu().numpy().view(np.int32)))
    for x, y in zip(*outs):
        assert np.array_equal(x, y)
    loaded.free()


def test_damaged_files_are_refused(tmp_path):
    cfg, S, trie, index = setup_case("C1")
    path = tmp_path / "c1.ppv"
    ppv.ppv_index_save(index, str(path))
    good = path.read_bytes()
    assert int.from_bytes(good[48:56], "little") == file_checksum_of_sections(good, index)

    def status_of(data: bytes):
        p = tmp_path / "damaged.ppv"
        p.write_bytes(data)
        try:
            ppv.ppv_index_load(str(p)).free()
            return 0
        except ppv.PPVError as e:
            return e.status
    assert status_of(good) == 0
    flipped = bytearray(good)
    flipped[len(good) // 2] ^= 0x10
    assert status_of(bytes(flipped)) == -1                      # checksum
    assert status_of(good[:-4]) == -1                           # length
    assert status_of(good + b"\0\0\0\0") == -1
    assert status_of(good[:100]) == -1


def section_bounds(index):
    n_nodes = index.n_prefixes + 1
    tok, off = ppv.ppv_index_export(index)
    sizes = [(n_nodes + 1) * 8, n_nodes * 4, n_nodes * 4, (index.n_distinct + 1) * 8, tok.shape[0] * 4]
    starts = np.concatenate([[128], 128 + np.cumsum(sizes)]).tolist()
    return starts


def file_checksum_of_sections(data: bytes, index) -> int:
    """The file format's checksum (a format rule, restated here to craft test files): over the sections in file
    order, per 8-byte little-endian word (a section's tail zero-padded to a word), h = (h ^ w) * 0x100000001B3
    mod 2^64, then h ^= h >> 29."""
    st = section_bounds(index)
    h = 0xCBF29CE484222325
    for a, b in zip(st[:-1], st[1:]):
        payload = data[a:b]
        for i in range(0, len(payload), 8):
            w = int.from_bytes(payload[i:i + 8].ljust(8, b"\0"), "little")
            h = ((h ^ w) * 0x100000001B3) & MASK64
            h ^= h >> 29
    assert st[-1] == len(data)
    return h


def test_structurally_wrong_files_with_a_correct_checksum_are_refused(tmp_path):
    """A file that was wrong when it was written passes the checksum; the device pass must catch what could
    send a kernel out of bounds: child offsets, ranks, tokens, row offsets."""
    cfg, S, trie, index = setup_case("C1")
    path = tmp_path / "c1.ppv"
    ppv.ppv_index_save(index, str(path))
    good = path.read_bytes()
    st = section_bounds(index)
    n_nodes = index.n_prefixes + 1

    def status_with(patch_at: int, value: int, width: int = 4):
        data = bytearray(good)
        data[patch_at:patch_at + width] = int(value).to_bytes(width, "little")
        data[48:56] = file_checksum_of_sections(bytes(data), index).to_bytes(8, "little")
        p = tmp_path / "wrong.ppv"
        p.write_bytes(bytes(data))
        try:
            ppv.ppv_index_load(str(p)).free()
            return 0
        except ppv.PPVError as e:
            return e.status
    ent = st[0]
    assert status_with(ent + 8 * 5 + 4, 0x7FFFFFFF) == -1       # a child offset far outside
    assert status_with(ent + 8 * 5 + 4, 2) == -1                # children before their parent
    assert status_with(ent + 8 * n_nodes + 4, n_nodes - 1) == -1  # the sentinel does not close the offsets
    assert status_with(ent + 8 * 3, cfg.vocab + 7) == -1        # a token outside the vocabulary
    assert status_with(ent + 8 * 3, 0x40000000 | 1) == -1       # a stored heavy flag
    assert status_with(st[1] + 4 * 2, index.n_distinct + 5) == -1  # rank range outside S
    assert status_with(st[3] + 8 * 1, 0, 8) == -1               # row offsets not increasing
    assert status_with(st[4] + 4 * 2, cfg.vocab, 4) == -1       # a member token outside the vocabulary
    assert status_with(ent + 4, 1) == 0                         # (patching a value with itself still loads)
