"""Thin ctypes binding of libppv_hip.so: argument marshalling only.

Same names as the C ABI in include/ppv.h.  Tensors are torch tensors on the GPU (torch provides
device memory and the current stream, nothing else); every step of the path runs in the library's
own kernels.  There is no fallback: if the library is missing or a call fails, this raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libppv_hip.so")

PPV_OK = 0
PPV_F32, PPV_BF16 = 0, 1
PPV_MAX_VOCAB = 262144
PPV_TOPM_MAX = 1024

PPV_STATE_WORDS = 8

SYMBOLS = ("ppv_status_string", "ppv_build_index", "ppv_index_info", "ppv_index_export", "ppv_free_index",
           "ppv_index_save", "ppv_index_load",
           "ppv_next_token_mask", "constrained_sample", "ppv_decode_begin", "ppv_decode_step", "ppv_decode_loop", "ppv_topm_mask",
           "ppv_disc_select", "ppv_tuning_set", "ppv_tuning_get", "constrained_sample_noalloc",
           "ppv_sample_next", "ppv_decode_begin_empty", "ppv_decode_first_step")
PPV_NOALLOC_MAX_ROWS = 512

# tuning / test switches (ppv_tuning_set)
(PPV_TUNE_WAVES_PER_ROW, PPV_TUNE_TOPM_WAVES, PPV_TUNE_TOPM_STREAMING, PPV_TUNE_LOOKUP, PPV_TUNE_LOOKUP_WEAK,
 PPV_TUNE_ROW_SPLIT) = range(6)

_lib = None


class PPVError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__(f"{what}: status {status} ({status_string(status)})")


def load_library() -> C.CDLL:
    """Load libppv_hip.so (built by paper_2504_09135_amd.build); raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is missing: run `python -m paper_2504_09135_amd.build` "
                                "(or __graft_entry__.build()) first; there is no fallback path")
    lib = C.CDLL(LIB_PATH)
    p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.ppv_status_string.restype = C.c_char_p
    lib.ppv_status_string.argtypes = [C.c_int]
    lib.ppv_build_index.restype = C.c_int
    lib.ppv_build_index.argtypes = [p, p, i64, i32, C.POINTER(p)]
    lib.ppv_index_info.restype = C.c_int
    lib.ppv_index_info.argtypes = [p, C.POINTER(i64), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64), C.POINTER(i64)]
    lib.ppv_index_export.restype = C.c_int
    lib.ppv_index_export.argtypes = [p, p, p, C.POINTER(i64)]
    lib.ppv_index_save.restype = C.c_int
    lib.ppv_index_save.argtypes = [p, C.c_char_p]
    lib.ppv_index_load.restype = C.c_int
    lib.ppv_index_load.argtypes = [C.c_char_p, C.POINTER(p)]
    lib.ppv_free_index.restype = None
    lib.ppv_free_index.argtypes = [p]
    lib.ppv_next_token_mask.restype = C.c_int
    lib.ppv_next_token_mask.argtypes = [p, p, i32, p, i32, p, p, p, p, p]
    lib.constrained_sample.restype = C.c_int
    lib.constrained_sample.argtypes = [p, C.c_int, i64, p, p, i32, i32, p, p, p, C.c_float, p]
    lib.constrained_sample_noalloc.restype = C.c_int
    lib.constrained_sample_noalloc.argtypes = lib.constrained_sample.argtypes
    lib.ppv_sample_next.restype = C.c_int
    lib.ppv_sample_next.argtypes = [p, p, i32, p, i32, p, C.c_int, i64, p, p, p, C.c_float, p]
    lib.ppv_decode_begin.restype = C.c_int
    lib.ppv_decode_begin.argtypes = [p, p, i32, p, i32, p, p, p, p]
    lib.ppv_decode_begin_empty.restype = C.c_int
    lib.ppv_decode_begin_empty.argtypes = [p, i32, p, p, p, p, p]
    lib.ppv_decode_step.restype = C.c_int
    lib.ppv_decode_step.argtypes = [p, p, i32, p, p, p, p, C.c_int, i64, p, i32, p, p, p, C.c_float, p]
    lib.ppv_decode_first_step.restype = C.c_int
    lib.ppv_decode_first_step.argtypes = [p, p, i32, p, p, p, p, C.c_int, i64, p, i32, p, p, p, C.c_float, p]
    lib.ppv_decode_loop.restype = C.c_int
    lib.ppv_decode_loop.argtypes = [p, p, i32, p, p, p, p, C.c_int, i64, i64, p, i32, i32, p, p, p, C.c_float, p]
    lib.ppv_topm_mask.restype = C.c_int
    lib.ppv_topm_mask.argtypes = [p, p, i32, p, p, C.c_int, i64, i32, i32, p, p, p, p]
    lib.ppv_disc_select.restype = C.c_int
    lib.ppv_disc_select.argtypes = [p, i32, i32, i32, p, p, i32, p, p, p, p]
    lib.ppv_tuning_set.restype = C.c_int
    lib.ppv_tuning_set.argtypes = [i32, i32]
    lib.ppv_tuning_get.restype = C.c_int
    lib.ppv_tuning_get.argtypes = [i32, C.POINTER(i32)]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().ppv_status_string(int(status)).decode()


def _check(status: int, what: str):
    if status != PPV_OK:
        raise PPVError(status, what)


def _dev(t: Optional[torch.Tensor], dtype, what: str):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{what}: need a contiguous GPU tensor of {dtype}, got {t.dtype} on {t.device}")
    return C.c_void_p(t.data_ptr())


def _stream(stream) -> C.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class PPVIndex:
    """Owner of a ppv_index_t handle."""

    def __init__(self, handle: int):
        self._h = C.c_void_p(handle)
        self.n_distinct, self.l_max, self.vocab, self.n_prefixes, self.device_bytes = ppv_index_info(self)
        self.n_words = (self.vocab + 31) // 32

    @property
    def handle(self) -> C.c_void_p:
        if not self._h:
            raise ValueError("index already freed")
        return self._h

    def free(self):
        if self._h:
            load_library().ppv_free_index(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def ppv_build_index(tokens: np.ndarray, offsets: np.ndarray, vocab: int) -> PPVIndex:
    """S as host CSR arrays (int32 tokens, int64 offsets) -> device index."""
    lib = load_library()
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    offsets = np.ascontiguousarray(offsets, dtype=np.int64)
    out = C.c_void_p()
    st = lib.ppv_build_index(tokens.ctypes.data_as(C.c_void_p), offsets.ctypes.data_as(C.c_void_p),
                             int(offsets.shape[0]) - 1, int(vocab), C.byref(out))
    _check(st, "ppv_build_index")
    return PPVIndex(out.value)


def ppv_index_save(index: PPVIndex, path: str) -> None:
    """Write the index to a file (ppv_index_load reads it back)."""
    _check(load_library().ppv_index_save(index.handle, os.fsencode(path)), "ppv_index_save")


def ppv_index_load(path: str) -> PPVIndex:
    """Read an index written by ppv_index_save onto the current device."""
    out = C.c_void_p()
    _check(load_library().ppv_index_load(os.fsencode(path), C.byref(out)), "ppv_index_load")
    return PPVIndex(out.value)


def ppv_index_info(index: PPVIndex) -> Tuple[int, int, int, int, int]:
    n, l, v, g, by = C.c_int64(), C.c_int32(), C.c_int32(), C.c_int64(), C.c_int64()
    _check(load_library().ppv_index_info(index.handle, C.byref(n), C.byref(l), C.byref(v), C.byref(g), C.byref(by)),
           "ppv_index_info")
    return n.value, l.value, v.value, g.value, by.value


def ppv_index_export(index: PPVIndex) -> Tuple[np.ndarray, np.ndarray]:
    """Sorted, de-duplicated S as host CSR arrays."""
    lib = load_library()
    nt = C.c_int64()
    _check(lib.ppv_index_export(index.handle, None, None, C.byref(nt)), "ppv_index_export")
    tokens = np.empty(nt.value, dtype=np.int32)
    offsets = np.empty(index.n_distinct + 1, dtype=np.int64)
    _check(lib.ppv_index_export(index.handle, tokens.ctypes.data_as(C.c_void_p),
                                offsets.ctypes.data_as(C.c_void_p), None), "ppv_index_export")
    return tokens, offsets


def ppv_free_index(index: PPVIndex) -> None:
    index.free()


def ppv_next_token_mask(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, mask: torch.Tensor,
                        range_lo: Optional[torch.Tensor] = None, range_hi: Optional[torch.Tensor] = None,
                        member: Optional[torch.Tensor] = None, stream=None) -> None:
    """prefixes int32 [B, stride], lens int32 [B] -> mask int32 [B, ceil(V/32)] (bit pattern of
    uint32 words), range_lo/range_hi int32 [B] (bit pattern of uint32), member uint8 [B]."""
    B, stride = (int(prefixes.shape[0]), int(prefixes.shape[1])) if prefixes.dim() == 2 else (0, 0)
    if prefixes.dim() != 2 or tuple(lens.shape) != (B,) or tuple(mask.shape) != (B, index.n_words):
        raise ValueError("ppv_next_token_mask: shape mismatch")
    for t, nm in ((range_lo, "range_lo"), (range_hi, "range_hi"), (member, "member")):
        if t is not None and tuple(t.shape) != (B,):
            raise ValueError(f"ppv_next_token_mask: {nm} must have shape [B]")
    st = load_library().ppv_next_token_mask(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"), B,
        _dev(mask, torch.int32, "mask"), _dev(range_lo, torch.int32, "range_lo"),
        _dev(range_hi, torch.int32, "range_hi"), _dev(member, torch.uint8, "member"), _stream(stream))
    _check(st, "ppv_next_token_mask")


def _logits_args(logits: torch.Tensor):
    if logits.dim() != 2 or not logits.is_cuda or logits.stride(1) != 1:
        raise ValueError("logits: need a 2-D GPU tensor with unit stride along the vocabulary")
    if logits.dtype == torch.float32:
        dt = PPV_F32
    elif logits.dtype == torch.bfloat16:
        dt = PPV_BF16
    else:
        raise TypeError(f"logits: float32 or bfloat16, got {logits.dtype}")
    # a single row: torch's stride of a size-1 dimension carries no meaning unless it covers the row (a row cut out
    # of a padded buffer keeps the buffer's stride, which is what says that the padding is there)
    row_stride = int(logits.stride(0))
    if logits.shape[0] <= 1 and row_stride < int(logits.shape[1]):
        row_stride = int(logits.shape[1])
    return C.c_void_p(logits.data_ptr()), dt, row_stride


def constrained_sample(logits: torch.Tensor, mask: torch.Tensor, uniforms: torch.Tensor, ids: torch.Tensor,
                       logZ_valid: torch.Tensor, logZ_all: Optional[torch.Tensor] = None, stream=None,
                       temperature: float = 1.0, _noalloc: bool = False) -> None:
    """logits [B, V] f32/bf16, mask int32 [B, ceil(V/32)], uniforms f32 [B] -> ids int32 [B],
    logZ_valid f32 [B], logZ_all f32 [B] (optional); P = softmax(logits / temperature)."""
    ptr, dt, row_stride = _logits_args(logits)
    B, V = int(logits.shape[0]), int(logits.shape[1])
    if tuple(mask.shape) != (B, (V + 31) // 32) or tuple(uniforms.shape) != (B,) or tuple(ids.shape) != (B,) \
            or tuple(logZ_valid.shape) != (B,) or (logZ_all is not None and tuple(logZ_all.shape) != (B,)):
        raise ValueError("constrained_sample: shape mismatch")
    fn = load_library().constrained_sample_noalloc if _noalloc else load_library().constrained_sample
    st = fn(ptr, dt, row_stride, _dev(mask, torch.int32, "mask"), _dev(uniforms, torch.float32, "uniforms"), B, V,
            _dev(ids, torch.int32, "ids"), _dev(logZ_valid, torch.float32, "logZ_valid"),
            _dev(logZ_all, torch.float32, "logZ_all"), float(temperature), _stream(stream))
    _check(st, "constrained_sample_noalloc" if _noalloc else "constrained_sample")


def constrained_sample_noalloc(logits: torch.Tensor, mask: torch.Tensor, uniforms: torch.Tensor, ids: torch.Tensor,
                               logZ_valid: torch.Tensor, logZ_all: Optional[torch.Tensor] = None, stream=None,
                               temperature: float = 1.0) -> None:
    """constrained_sample through the entry point that allocates nothing (at most PPV_NOALLOC_MAX_ROWS rows)."""
    constrained_sample(logits, mask, uniforms, ids, logZ_valid, logZ_all, stream, temperature, _noalloc=True)


def ppv_decode_begin(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, state: torch.Tensor,
                     active: torch.Tensor, logx: Optional[torch.Tensor] = None, stream=None) -> None:
    """Locate every row's current prefix once: writes state int32 [B, PPV_STATE_WORDS], active uint8 [B]
    and zeroes logx f32 [B]."""
    B, stride = int(prefixes.shape[0]), int(prefixes.shape[1])
    if tuple(lens.shape) != (B,) or tuple(state.shape) != (B, PPV_STATE_WORDS) or tuple(active.shape) != (B,) \
            or (logx is not None and tuple(logx.shape) != (B,)):
        raise ValueError("ppv_decode_begin: shape mismatch")
    st = load_library().ppv_decode_begin(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"), B,
        _dev(state, torch.int32, "state"), _dev(active, torch.uint8, "active"), _dev(logx, torch.float32, "logx"),
        _stream(stream))
    _check(st, "ppv_decode_begin")


def ppv_decode_begin_empty(index: PPVIndex, lens: torch.Tensor, state: torch.Tensor, active: torch.Tensor,
                           logx: Optional[torch.Tensor] = None, stream=None) -> None:
    """SampleCandidate initialisation from the empty candidate for every row: lens int32 [B] (written 0),
    state int32 [B, PPV_STATE_WORDS], active uint8 [B], logx f32 [B] (optional) are written."""
    B = int(lens.shape[0])
    if tuple(lens.shape) != (B,) or tuple(state.shape) != (B, PPV_STATE_WORDS) or tuple(active.shape) != (B,) \
            or (logx is not None and tuple(logx.shape) != (B,)):
        raise ValueError("ppv_decode_begin_empty: shape mismatch")
    st = load_library().ppv_decode_begin_empty(
        index.handle, B, _dev(lens, torch.int32, "lens"), _dev(state, torch.int32, "state"),
        _dev(active, torch.uint8, "active"), _dev(logx, torch.float32, "logx"), _stream(stream))
    _check(st, "ppv_decode_begin_empty")


def ppv_decode_step(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, active: torch.Tensor,
                    logits: torch.Tensor, uniforms: torch.Tensor, ids: Optional[torch.Tensor] = None,
                    logZ_valid: Optional[torch.Tensor] = None, logx: Optional[torch.Tensor] = None,
                    state: Optional[torch.Tensor] = None, stream=None, temperature: float = 1.0,
                    _first: bool = False) -> None:
    """One fused constrained decoding step, in place on prefixes / lens / active / logx (and on
    state int32 [B, PPV_STATE_WORDS] from ppv_decode_begin when given); P = softmax(logits / temperature)."""
    ptr, dt, row_stride = _logits_args(logits)
    B, stride = int(prefixes.shape[0]), int(prefixes.shape[1])
    if int(logits.shape[0]) != B or int(logits.shape[1]) != index.vocab or tuple(lens.shape) != (B,) \
            or tuple(active.shape) != (B,) or tuple(uniforms.shape) != (B,) \
            or (state is not None and tuple(state.shape) != (B, PPV_STATE_WORDS)):
        raise ValueError("ppv_decode_step: shape mismatch")
    for t, nm in ((ids, "ids"), (logZ_valid, "logZ_valid"), (logx, "logx")):
        if t is not None and tuple(t.shape) != (B,):
            raise ValueError(f"ppv_decode_step: {nm} must have shape [B]")
    fn = load_library().ppv_decode_first_step if _first else load_library().ppv_decode_step
    st = fn(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"),
        _dev(active, torch.uint8, "active"), _dev(state, torch.int32, "state"), ptr, dt, row_stride,
        _dev(uniforms, torch.float32, "uniforms"), B, _dev(ids, torch.int32, "ids"),
        _dev(logZ_valid, torch.float32, "logZ_valid"), _dev(logx, torch.float32, "logx"), float(temperature),
        _stream(stream))
    _check(st, "ppv_decode_first_step" if _first else "ppv_decode_step")


def ppv_decode_first_step(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, active: torch.Tensor,
                          logits: torch.Tensor, uniforms: torch.Tensor, ids: Optional[torch.Tensor] = None,
                          logZ_valid: Optional[torch.Tensor] = None, logx: Optional[torch.Tensor] = None,
                          state: Optional[torch.Tensor] = None, stream=None, temperature: float = 1.0) -> None:
    """ppv_decode_begin_empty and the first ppv_decode_step in one launch (state is required)."""
    ppv_decode_step(index, prefixes, lens, active, logits, uniforms, ids, logZ_valid, logx, state, stream, temperature,
                    _first=True)


def ppv_decode_loop(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, active: torch.Tensor,
                    logits: torch.Tensor, uniforms: torch.Tensor, ids: Optional[torch.Tensor] = None,
                    logZ_valid: Optional[torch.Tensor] = None, logx: Optional[torch.Tensor] = None,
                    state: Optional[torch.Tensor] = None, stream=None, temperature: float = 1.0) -> None:
    """The whole decode loop in one launch: logits [n_steps, B, V] (f32/bf16), uniforms f32 [n_steps, B],
    ids int32 / logZ_valid f32 [n_steps, B] (optional); everything else as ppv_decode_step."""
    if logits.dim() != 3 or not logits.is_cuda or logits.stride(2) != 1:
        raise ValueError("logits: need a 3-D GPU tensor [n_steps, B, V] with unit stride along the vocabulary")
    n_steps, B, V = (int(x) for x in logits.shape)
    dt = {torch.float32: PPV_F32, torch.bfloat16: PPV_BF16}.get(logits.dtype)
    if dt is None:
        raise TypeError(f"logits: float32 or bfloat16, got {logits.dtype}")
    stride = int(prefixes.shape[1])
    if int(prefixes.shape[0]) != B or V != index.vocab or tuple(lens.shape) != (B,) or tuple(active.shape) != (B,) \
            or tuple(uniforms.shape) != (n_steps, B) \
            or (state is not None and tuple(state.shape) != (B, PPV_STATE_WORDS)) \
            or (logx is not None and tuple(logx.shape) != (B,)):
        raise ValueError("ppv_decode_loop: shape mismatch")
    for t, nm in ((ids, "ids"), (logZ_valid, "logZ_valid")):
        if t is not None and tuple(t.shape) != (n_steps, B):
            raise ValueError(f"ppv_decode_loop: {nm} must have shape [n_steps, B]")
    st = load_library().ppv_decode_loop(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"),
        _dev(active, torch.uint8, "active"), _dev(state, torch.int32, "state"), C.c_void_p(logits.data_ptr()), dt,
        int(logits.stride(1)), int(logits.stride(0)), _dev(uniforms, torch.float32, "uniforms"), n_steps, B,
        _dev(ids, torch.int32, "ids"), _dev(logZ_valid, torch.float32, "logZ_valid"),
        _dev(logx, torch.float32, "logx"), float(temperature), _stream(stream))
    _check(st, "ppv_decode_loop")


def ppv_topm_mask(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, logits: torch.Tensor, M: int,
                  mask: torch.Tensor, top_ids: Optional[torch.Tensor] = None, mask_V: Optional[torch.Tensor] = None,
                  stream=None) -> None:
    """Algorithm 2 with M candidates: prefixes int32 [B, stride], lens int32 [B], logits [B, V] f32/bf16 ->
    mask int32 [B, ceil(V/32)], top_ids int32 [B, M] (optional), mask_V uint8 [B, M] (optional)."""
    ptr, dt, row_stride = _logits_args(logits)
    B, stride = (int(prefixes.shape[0]), int(prefixes.shape[1])) if prefixes.dim() == 2 else (0, 0)
    if prefixes.dim() != 2 or tuple(lens.shape) != (B,) or tuple(mask.shape) != (B, index.n_words) \
            or tuple(logits.shape) != (B, index.vocab):
        raise ValueError("ppv_topm_mask: shape mismatch")
    for t, nm in ((top_ids, "top_ids"), (mask_V, "mask_V")):
        if t is not None and tuple(t.shape) != (B, M):
            raise ValueError(f"ppv_topm_mask: {nm} must have shape [B, M]")
    st = load_library().ppv_topm_mask(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"), ptr, dt,
        row_stride, int(M), B, _dev(top_ids, torch.int32, "top_ids"), _dev(mask_V, torch.uint8, "mask_V"),
        _dev(mask, torch.int32, "mask"), _stream(stream))
    _check(st, "ppv_topm_mask")


def ppv_disc_select(logx: torch.Tensor, K: int, accept_u: torch.Tensor, resample_u: torch.Tensor,
                    chosen: torch.Tensor, n_draws: Optional[torch.Tensor] = None,
                    accepted: Optional[torch.Tensor] = None, reuse_rejected: bool = False, stream=None) -> None:
    """DISC accept/reject rounds + importance-resampling fallback: logx f32 [n_candidates, Q], accept_u f32 [K, Q],
    resample_u f32 [Q] -> chosen int32 [Q], n_draws int32 [Q], accepted uint8 [Q]."""
    n_cand, Q = int(logx.shape[0]), int(logx.shape[1])
    if tuple(accept_u.shape) != (K, Q) or tuple(resample_u.shape) != (Q,) or tuple(chosen.shape) != (Q,):
        raise ValueError("ppv_disc_select: shape mismatch")
    st = load_library().ppv_disc_select(
        _dev(logx, torch.float32, "logx"), n_cand, int(K), Q, _dev(accept_u, torch.float32, "accept_u"),
        _dev(resample_u, torch.float32, "resample_u"), 1 if reuse_rejected else 0,
        _dev(chosen, torch.int32, "chosen"), _dev(n_draws, torch.int32, "n_draws"),
        _dev(accepted, torch.uint8, "accepted"), _stream(stream))
    _check(st, "ppv_disc_select")


def ppv_tuning_set(knob: int, value: int) -> None:
    """Set a process-wide tuning / test switch (PPV_TUNE_*)."""
    _check(load_library().ppv_tuning_set(int(knob), int(value)), "ppv_tuning_set")


def ppv_tuning_get(knob: int) -> int:
    v = C.c_int32()
    _check(load_library().ppv_tuning_get(int(knob), C.byref(v)), "ppv_tuning_get")
    return v.value


def ppv_sample_next(index: PPVIndex, prefixes: torch.Tensor, lens: torch.Tensor, logits: torch.Tensor,
                    uniforms: torch.Tensor, ids: torch.Tensor, logZ_valid: Optional[torch.Tensor] = None, stream=None,
                    temperature: float = 1.0) -> None:
    """Mask + sample fused, nothing of the caller's rows changed: prefixes int32 [B, stride], lens int32 [B],
    logits [B, V] f32/bf16, uniforms f32 [B] -> ids int32 [B], logZ_valid f32 [B] (optional)."""
    ptr, dt, row_stride = _logits_args(logits)
    B, stride = (int(prefixes.shape[0]), int(prefixes.shape[1])) if prefixes.dim() == 2 else (0, 0)
    if prefixes.dim() != 2 or tuple(lens.shape) != (B,) or tuple(logits.shape) != (B, index.vocab) \
            or tuple(uniforms.shape) != (B,) or tuple(ids.shape) != (B,) \
            or (logZ_valid is not None and tuple(logZ_valid.shape) != (B,)):
        raise ValueError("ppv_sample_next: shape mismatch")
    st = load_library().ppv_sample_next(
        index.handle, _dev(prefixes, torch.int32, "prefixes"), stride, _dev(lens, torch.int32, "lens"), B, ptr, dt,
        row_stride, _dev(uniforms, torch.float32, "uniforms"), _dev(ids, torch.int32, "ids"),
        _dev(logZ_valid, torch.float32, "logZ_valid"), float(temperature), _stream(stream))
    _check(st, "ppv_sample_next")
