"""The C-ABI library loads, exports every function include/ppv.h declares, and rejects bad
arguments with status codes before touching a device.  No GPU needed."""
import ctypes as C
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ppv.h")


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(ppv_\w+|constrained_sample\w*)\s*\(", src)) - {"ppv_index"})


@pytest.fixture(scope="module")
def lib():
    from paper_2504_09135_amd import binding
    return binding.load_library()


def test_header_and_binding_agree(lib):
    from paper_2504_09135_amd import binding
    names = declared_functions()
    assert set(names) == set(binding.SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None
    hdr = open(HEADER).read()
    assert int(re.search(r"#define PPV_MAX_VOCAB (\d+)", hdr).group(1)) == binding.PPV_MAX_VOCAB


def test_status_strings(lib):
    for s in (0, -1, -2, -3, -4, -5, 77):
        assert isinstance(lib.ppv_status_string(s), bytes)


def test_argument_errors_without_device(lib):
    from paper_2504_09135_amd.binding import PPV_MAX_VOCAB
    out = C.c_void_p()
    tok = np.array([1, 2, 3], dtype=np.int32)
    off = np.array([0, 2, 3], dtype=np.int64)
    tp, op = tok.ctypes.data_as(C.c_void_p), off.ctypes.data_as(C.c_void_p)
    EINVAL, ERANGE = -1, -4
    assert lib.ppv_build_index(None, op, 2, 8, C.byref(out)) == EINVAL
    assert lib.ppv_build_index(tp, None, 2, 8, C.byref(out)) == EINVAL
    assert lib.ppv_build_index(tp, op, 0, 8, C.byref(out)) == EINVAL
    assert lib.ppv_build_index(tp, op, 2, 0, C.byref(out)) == EINVAL
    assert lib.ppv_build_index(tp, op, 2, 8, None) == EINVAL
    assert lib.ppv_build_index(tp, op, 2, PPV_MAX_VOCAB + 1, C.byref(out)) == ERANGE
    assert out.value is None
    assert lib.ppv_index_info(None, None, None, None, None, None) == EINVAL
    assert lib.ppv_index_export(None, None, None, None) == EINVAL
    lib.ppv_free_index(None)
    assert lib.ppv_next_token_mask(None, None, 0, None, 0, None, None, None, None, None) == EINVAL
    assert lib.constrained_sample(None, 0, 8, None, None, 1, 8, None, None, None, 1.0, None) == EINVAL
    assert lib.constrained_sample(None, 0, 8, None, None, -1, 8, None, None, None, 1.0, None) == EINVAL
    assert lib.constrained_sample(None, 0, 8, None, None, 0, 8, None, None, None, 1.0, None) == 0
    for bad_t in (0.0, -1.0, float("inf"), float("nan")):       # the temperature is checked before anything is launched
        assert lib.constrained_sample(None, 0, 8, None, None, 0, 8, None, None, None, bad_t, None) == EINVAL
    # the entry point that allocates nothing: same checks, and a largest batch
    assert lib.constrained_sample_noalloc(None, 0, 8, None, None, 1, 8, None, None, None, 1.0, None) == EINVAL
    assert lib.constrained_sample_noalloc(None, 0, 8, None, None, 0, 8, None, None, None, 1.0, None) == 0
    never = C.c_void_p(16)   # never dereferenced: the size check comes first
    assert lib.constrained_sample_noalloc(never, 0, 8, never, never, 513, 8, never, never, None, 1.0, None) == ERANGE
    assert lib.ppv_sample_next(None, None, 0, None, 0, None, 0, 8, None, None, None, 1.0, None) == EINVAL
    assert lib.ppv_sample_next(never, None, 0, None, 0, None, 0, 8, None, None, None, 1.0, None) == 0      # B = 0
    assert lib.ppv_sample_next(never, None, 0, None, 1, None, 0, 8, None, None, None, 1.0, None) == EINVAL
    assert lib.ppv_decode_step(None, None, 0, None, None, None, None, 0, 0, None, 0, None, None, None, 1.0, None) == EINVAL
    assert lib.ppv_decode_begin(None, None, 0, None, 0, None, None, None, None) == EINVAL
    assert lib.ppv_decode_begin_empty(None, 1, None, None, None, None, None) == EINVAL
    assert lib.ppv_decode_first_step(None, None, 0, None, None, None, None, 0, 0, None, 0, None, None, None, 1.0, None) == EINVAL
    assert lib.ppv_decode_first_step(never, never, 4, never, never, None, never, 0, 8, never, 1, None, None, None, 1.0, None) == EINVAL   # no state
    assert lib.ppv_decode_begin_empty(never, 0, None, None, None, None, None) == 0          # B = 0
    assert lib.ppv_decode_begin_empty(never, 1, None, None, None, None, None) == EINVAL
    assert lib.ppv_disc_select(None, 2, 1, 5, None, None, 0, None, None, None, None) == EINVAL
    assert lib.ppv_disc_select(None, 1, 1, 5, None, None, 0, None, None, None, None) == EINVAL
    EIO = -5
    assert lib.ppv_index_save(None, b"/tmp/x") == EINVAL
    assert lib.ppv_index_load(None, C.byref(out)) == EINVAL
    assert lib.ppv_index_load(b"/nonexistent/dir/index.ppv", C.byref(out)) == EIO
    assert lib.ppv_index_load(b"/nonexistent/dir/index.ppv", None) == EINVAL
    fake = C.c_void_p(16)   # never dereferenced: the checks below come first
    assert lib.ppv_topm_mask(None, None, 0, None, None, 0, 8, 5, 1, None, None, None, None) == EINVAL
    assert lib.ppv_topm_mask(fake, None, 0, None, None, 0, 8, 0, 0, None, None, None, None) == EINVAL
    assert lib.ppv_topm_mask(fake, None, 0, None, None, 0, 8, 1025, 0, None, None, None, None) == ERANGE
    assert lib.ppv_topm_mask(fake, None, 0, None, None, 0, 8, 5, 0, None, None, None, None) == 0
    assert lib.ppv_decode_loop(None, None, 0, None, None, None, None, 0, 0, 0, None, 1, 1, None, None, None, 1.0, None) == EINVAL


def test_tuning_switches(lib):
    """Switches are set and read back through the ABI; unknown knobs and values out of range are refused."""
    from paper_2504_09135_amd import binding
    v = C.c_int32(-7)
    for knob in range(6):
        assert lib.ppv_tuning_get(knob, C.byref(v)) == 0 and v.value >= 0
    assert lib.ppv_tuning_get(6, C.byref(v)) == -1 and lib.ppv_tuning_get(0, None) == -1
    assert lib.ppv_tuning_set(-1, 0) == -1 and lib.ppv_tuning_set(6, 0) == -1
    assert lib.ppv_tuning_set(binding.PPV_TUNE_WAVES_PER_ROW, 17) == -4
    before = binding.ppv_tuning_get(binding.PPV_TUNE_TOPM_WAVES)
    binding.ppv_tuning_set(binding.PPV_TUNE_TOPM_WAVES, 2)
    assert binding.ppv_tuning_get(binding.PPV_TUNE_TOPM_WAVES) == 2
    binding.ppv_tuning_set(binding.PPV_TUNE_TOPM_WAVES, before)


def test_index_load_rejects_files_that_are_not_an_index(lib, tmp_path):
    """Everything that can be told from the header and the file's length is refused before any device call."""
    out = C.c_void_p()
    EINVAL, ERANGE = -1, -4
    junk = tmp_path / "junk.ppv"
    junk.write_bytes(b"not an index")
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == EINVAL and out.value is None
    junk.write_bytes(bytes(4096))
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == EINVAL

    def header(vocab=8, l_max=2, n_rows=2, n_nodes=4, n_tokens=3, version=1):
        h = bytearray(128)
        h[0:8] = b"PPVIDX\x00\x01"
        h[8:12] = np.uint32(version).tobytes()
        h[12:16] = np.uint32(128).tobytes()
        h[16:20] = np.int32(vocab).tobytes()
        h[20:24] = np.int32(l_max).tobytes()
        h[24:32] = np.uint64(n_rows).tobytes()
        h[32:40] = np.uint64(n_nodes).tobytes()
        h[40:48] = np.uint64(n_tokens).tobytes()
        return bytes(h)
    junk.write_bytes(header(version=2) + bytes(200))
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == EINVAL
    junk.write_bytes(header(vocab=0) + bytes(200))
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == EINVAL
    junk.write_bytes(header(vocab=1 << 20) + bytes(200))
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == ERANGE
    junk.write_bytes(header() + bytes(7))                     # sections shorter than the header promises
    assert lib.ppv_index_load(str(junk).encode(), C.byref(out)) == EINVAL
    assert out.value is None


def test_binding_fails_loudly_without_the_library(monkeypatch):
    """No fallback: with the shared library gone, the first call raises and names the build step."""
    from paper_2504_09135_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libppv_hip.so")
    with pytest.raises(FileNotFoundError, match="no fallback"):
        binding.load_library()
    with pytest.raises(FileNotFoundError):
        binding.ppv_build_index(np.array([1], np.int32), np.array([0, 1], np.int64), 4)
