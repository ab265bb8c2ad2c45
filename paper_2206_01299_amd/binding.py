"""Thin ctypes binding over ``libaqsgd.so`` (the C ABI in ``include/aqsgd.h``).

Argument marshalling only: every step of the codec runs in the HIP kernels.
torch supplies device memory (``tensor.data_ptr()``) and the stream
(``torch.cuda.current_stream()``); no tensor maths happens here.  There is no
CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

import os

_HERE = Path(__file__).resolve().parent
# AQSGD_LIB names another build of the same library (used to compare two builds in one session)
LIB_PATH = Path(os.environ["AQSGD_LIB"]) if os.environ.get("AQSGD_LIB") else _HERE / "libaqsgd.so"

F32, F16, BF16 = 0, 1, 2
NEAREST, STOCHASTIC = 0, 1

DTYPE_CODE = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}
DTYPE_NAME = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

EXPORTS = ("aqsgd_codes_bytes", "aqsgd_scales_count", "aqsgd_encode", "aqsgd_decode",
           "aqsgd_grad_quant", "aqsgd_grad_dequant", "aqsgd_run_jobs", "aqsgd_seed", "aqsgd_encode_seen",
           "aqsgd_decode_seen", "aqsgd_lowbit_row_bytes",
           "aqsgd_encode_lowbit", "aqsgd_decode_lowbit", "aqsgd_tier_create", "aqsgd_tier_create_file",
           "aqsgd_tier_prefetch",
           "aqsgd_tier_acquire", "aqsgd_tier_release", "aqsgd_tier_drain", "aqsgd_tier_destroy",
           "aqsgd_topk_bitmap_bytes", "aqsgd_topk_codes_bytes", "aqsgd_grad_topk_quant",
           "aqsgd_grad_topk_dequant", "aqsgd_check_ids", "aqsgd_set_launch_shape",
           "aqsgd_profile_next_launch", "aqsgd_strerror", "aqsgd_version")


class Desc(ctypes.Structure):
    """Mirror of ``aqsgd_desc``."""
    _fields_ = [("batch", ctypes.c_int64), ("n_per", ctypes.c_int64), ("n_samples", ctypes.c_int64),
                ("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("rounding", ctypes.c_int32), ("rng_seed", ctypes.c_uint64)]


JOB_ENCODE, JOB_DECODE, JOB_GRAD_QUANT, JOB_GRAD_DEQUANT, JOB_ENCODE_SEEN, JOB_DECODE_SEEN = 0, 1, 2, 3, 4, 5


class Job(ctypes.Structure):
    """Mirror of ``aqsgd_job``."""
    _fields_ = [("kind", ctypes.c_int32), ("desc", Desc), ("src", ctypes.c_void_p),
                ("sample_ids", ctypes.c_void_p), ("m_buf", ctypes.c_void_p), ("codes", ctypes.c_void_p),
                ("scales", ctypes.c_void_p), ("out", ctypes.c_void_p), ("seen", ctypes.c_void_p),
                ("first", ctypes.c_void_p), ("full", ctypes.c_void_p), ("stamp", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]


class AqsgdError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"aqsgd status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load the HIP library built by ``python -m paper_2206_01299_amd.build``."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2206_01299_amd.build` "
                "(there is no fallback path)")
        L = ctypes.CDLL(str(LIB_PATH))
        vp, dp = ctypes.c_void_p, ctypes.POINTER(Desc)
        L.aqsgd_codes_bytes.restype = ctypes.c_size_t
        L.aqsgd_codes_bytes.argtypes = [dp]
        L.aqsgd_scales_count.restype = ctypes.c_size_t
        L.aqsgd_scales_count.argtypes = [dp]
        L.aqsgd_encode.restype = ctypes.c_int
        L.aqsgd_encode.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.aqsgd_decode.restype = ctypes.c_int
        L.aqsgd_decode.argtypes = [dp, vp, vp, vp, vp, vp, vp]
        L.aqsgd_grad_quant.restype = ctypes.c_int
        L.aqsgd_grad_quant.argtypes = [dp, vp, vp, vp, vp]
        L.aqsgd_grad_dequant.restype = ctypes.c_int
        L.aqsgd_grad_dequant.argtypes = [dp, vp, vp, vp, vp]
        L.aqsgd_seed.restype = ctypes.c_int
        L.aqsgd_seed.argtypes = [dp, vp, vp, vp, vp]
        L.aqsgd_encode_seen.restype = ctypes.c_int
        L.aqsgd_encode_seen.argtypes = [dp, vp, vp, vp, vp, ctypes.c_uint32, vp, vp, vp, vp]
        L.aqsgd_decode_seen.restype = ctypes.c_int
        L.aqsgd_decode_seen.argtypes = [dp, vp, vp, vp, vp, vp, vp, ctypes.c_uint32, vp, vp]
        L.aqsgd_run_jobs.restype = ctypes.c_int
        L.aqsgd_run_jobs.argtypes = [ctypes.POINTER(Job), ctypes.c_int32, vp]
        L.aqsgd_lowbit_row_bytes.restype = ctypes.c_size_t
        L.aqsgd_lowbit_row_bytes.argtypes = [dp, ctypes.c_int32]
        L.aqsgd_encode_lowbit.restype = ctypes.c_int
        L.aqsgd_encode_lowbit.argtypes = [dp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp]
        L.aqsgd_decode_lowbit.restype = ctypes.c_int
        L.aqsgd_decode_lowbit.argtypes = [dp, ctypes.c_int32, vp, vp, vp, vp, vp, vp, vp]
        L.aqsgd_topk_bitmap_bytes.restype = ctypes.c_size_t
        L.aqsgd_topk_bitmap_bytes.argtypes = [dp]
        L.aqsgd_topk_codes_bytes.restype = ctypes.c_size_t
        L.aqsgd_topk_codes_bytes.argtypes = [dp, ctypes.c_int32]
        L.aqsgd_grad_topk_quant.restype = ctypes.c_int
        L.aqsgd_grad_topk_quant.argtypes = [dp, ctypes.c_int32, vp, vp, vp, vp, vp]
        L.aqsgd_grad_topk_dequant.restype = ctypes.c_int
        L.aqsgd_grad_topk_dequant.argtypes = [dp, ctypes.c_int32, vp, vp, vp, vp, vp]
        L.aqsgd_tier_create.restype = ctypes.c_int
        L.aqsgd_tier_create.argtypes = [ctypes.POINTER(vp), vp, vp, vp, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_int32, ctypes.c_int32]
        L.aqsgd_tier_create_file.restype = ctypes.c_int
        L.aqsgd_tier_create_file.argtypes = [ctypes.POINTER(vp), ctypes.c_char_p, ctypes.c_int32, vp, vp, vp,
                                             ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
        L.aqsgd_tier_prefetch.restype = ctypes.c_int
        L.aqsgd_tier_prefetch.argtypes = [vp, ctypes.c_int32, vp, vp]
        L.aqsgd_tier_acquire.restype = ctypes.c_int
        L.aqsgd_tier_acquire.argtypes = [vp, ctypes.c_int32, vp, ctypes.POINTER(vp)]
        L.aqsgd_tier_release.restype = ctypes.c_int
        L.aqsgd_tier_release.argtypes = [vp, ctypes.c_int32, vp, vp]
        L.aqsgd_tier_drain.restype = ctypes.c_int
        L.aqsgd_tier_drain.argtypes = [vp]
        L.aqsgd_tier_destroy.restype = None
        L.aqsgd_tier_destroy.argtypes = [vp]
        L.aqsgd_check_ids.restype = ctypes.c_int
        L.aqsgd_check_ids.argtypes = [vp, ctypes.c_int64, ctypes.c_int64, vp, vp]
        L.aqsgd_set_launch_shape.restype = ctypes.c_int
        L.aqsgd_set_launch_shape.argtypes = [ctypes.c_int64, ctypes.c_int32]
        L.aqsgd_profile_next_launch.restype = ctypes.c_int
        L.aqsgd_profile_next_launch.argtypes = [vp, vp]
        L.aqsgd_strerror.restype = ctypes.c_char_p
        L.aqsgd_strerror.argtypes = [ctypes.c_int]
        L.aqsgd_version.restype = ctypes.c_char_p
        L.aqsgd_version.argtypes = []
        _lib = L
    return _lib


def version() -> str:
    return lib().aqsgd_version().decode()


def strerror(status: int) -> str:
    return lib().aqsgd_strerror(status).decode()


def make_desc(*, batch: int, n_per: int, n_samples: int = 0, bits: int, group: int, dtype,
              rounding: int = NEAREST, rng_seed: int = 0) -> Desc:
    code = DTYPE_CODE[dtype] if isinstance(dtype, torch.dtype) else DTYPE_CODE[DTYPE_NAME[dtype]]
    return Desc(batch, n_per, n_samples, bits, group, code, rounding, rng_seed & 0xFFFFFFFFFFFFFFFF)


def codes_bytes(desc: Desc) -> int:
    return int(lib().aqsgd_codes_bytes(ctypes.byref(desc)))


def scales_count(desc: Desc) -> int:
    return int(lib().aqsgd_scales_count(ctypes.byref(desc)))


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _dev(t: torch.Tensor, what: str) -> ctypes.c_void_p:
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{what} must be a contiguous device tensor")
    return ctypes.c_void_p(t.data_ptr())


_TORCH_OF_CODE = {code: dt for dt, code in DTYPE_CODE.items()}

# When set (``check_ids_always(True)``), every call that takes sample ids first runs
# ``aqsgd_check_ids`` on them and waits for its verdict: a debugging aid, it
# synchronises the stream.
_debug_ids = False


def check_ids_always(on: bool = True) -> None:
    global _debug_ids
    _debug_ids = bool(on)


def _want(t: torch.Tensor, what: str, dtype, numel: int, exact: bool) -> None:
    """The kernels index these tensors from the descriptor alone; a tensor of another
    element type or a smaller size would be read or written out of bounds."""
    if t.dtype != dtype:
        raise ValueError(f"{what} must be {dtype}, got {t.dtype}")
    if (t.numel() != numel) if exact else (t.numel() < numel):
        raise ValueError(f"{what} must hold {'exactly' if exact else 'at least'} {numel} elements, "
                         f"got {t.numel()}")


def _check(desc: Desc, *, rows=(), ids=None, m_buf=None, codes=None, scales=None, stream=None) -> None:
    """Shapes and element types of one codec call against its descriptor.
    ``rows``: (tensor, name) pairs of [batch, n_per] tensors in the descriptor's dtype."""
    if desc.dtype not in _TORCH_OF_CODE:
        return                                  # the library reports the bad descriptor
    td = _TORCH_OF_CODE[desc.dtype]
    n = desc.batch * desc.n_per
    for t, what in rows:
        _want(t, what, td, n, exact=True)
    if m_buf is not None:
        _want(m_buf, "m_buf", td, desc.n_samples * desc.n_per, exact=True)
    if ids is not None:
        _want(ids, "sample_ids", torch.int64, desc.batch, exact=True)
    if codes is not None:
        _want(codes, "codes", torch.uint8, codes_bytes(desc), exact=False)
    if scales is not None:
        _want(scales, "scales", torch.float32, scales_count(desc), exact=False)
    if ids is not None and _debug_ids and desc.batch > 0:
        flag = torch.zeros(1, dtype=torch.int32, device=ids.device)
        check_ids(ids, desc.n_samples, flag, stream)
        bad = int(flag.item())
        if bad:
            raise ValueError("sample_ids: " + " and ".join(
                w for b, w in ((1, "an id is outside [0, n_samples)"), (2, "two ids are equal")) if bad & b))


def _raise(status: int):
    if status != 0:
        raise AqsgdError(status, strerror(status))


def encode(desc: Desc, act, sample_ids, m_buf, codes, scales, stream=None) -> None:
    """``aqsgd_encode``: updates ``m_buf`` in place, fills ``codes`` and ``scales``."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales, stream=stream)
    _raise(lib().aqsgd_encode(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                              _dev(m_buf, "m_buf"), _dev(codes, "codes"), _dev(scales, "scales"),
                              _stream(stream)))


def decode(desc: Desc, codes, scales, sample_ids, m_buf, out, stream=None) -> None:
    """``aqsgd_decode``: updates ``m_buf`` in place, fills ``out``."""
    _check(desc, rows=[(out, "out")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales, stream=stream)
    _raise(lib().aqsgd_decode(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                              _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"), _dev(out, "out"),
                              _stream(stream)))


def grad_quant(desc: Desc, grad, codes, scales, stream=None) -> None:
    _check(desc, rows=[(grad, "grad")], codes=codes, scales=scales)
    _raise(lib().aqsgd_grad_quant(ctypes.byref(desc), _dev(grad, "grad"), _dev(codes, "codes"),
                                  _dev(scales, "scales"), _stream(stream)))


def grad_dequant(desc: Desc, codes, scales, out, stream=None) -> None:
    _check(desc, rows=[(out, "out")], codes=codes, scales=scales)
    _raise(lib().aqsgd_grad_dequant(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                                    _dev(out, "out"), _stream(stream)))


def seed(desc: Desc, act, sample_ids, m_buf, stream=None) -> None:
    """``aqsgd_seed``: uncompressed first visit, ``m_buf[sample_ids] <- act``."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, m_buf=m_buf, stream=stream)
    _raise(lib().aqsgd_seed(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                            _dev(m_buf, "m_buf"), _stream(stream)))


def _copy_desc(desc: Desc) -> Desc:
    return Desc(desc.batch, desc.n_per, desc.n_samples, desc.bits, desc.group, desc.dtype, desc.rounding,
                desc.rng_seed)


def encode_job(desc: Desc, act, sample_ids, m_buf, codes, scales) -> Job:
    """An ``aqsgd_encode`` call as one job of :func:`run_jobs` (the descriptor is copied)."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales)
    return Job(JOB_ENCODE, _copy_desc(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
               _dev(m_buf, "m_buf"), _dev(codes, "codes"), _dev(scales, "scales"), None)


def decode_job(desc: Desc, codes, scales, sample_ids, m_buf, out) -> Job:
    _check(desc, rows=[(out, "out")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales)
    return Job(JOB_DECODE, _copy_desc(desc), None, _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"),
               _dev(codes, "codes"), _dev(scales, "scales"), _dev(out, "out"))


def grad_quant_job(desc: Desc, grad, codes, scales) -> Job:
    _check(desc, rows=[(grad, "grad")], codes=codes, scales=scales)
    return Job(JOB_GRAD_QUANT, _copy_desc(desc), _dev(grad, "grad"), None, None, _dev(codes, "codes"),
               _dev(scales, "scales"), None)


def grad_dequant_job(desc: Desc, codes, scales, out) -> Job:
    _check(desc, rows=[(out, "out")], codes=codes, scales=scales)
    return Job(JOB_GRAD_DEQUANT, _copy_desc(desc), None, None, None, _dev(codes, "codes"),
               _dev(scales, "scales"), _dev(out, "out"))


def encode_seen_job(desc: Desc, act, sample_ids, m_buf, seen, stamp: int, first, codes, scales) -> Job:
    """An ``aqsgd_encode_seen`` call as one job of :func:`run_jobs`."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales)
    _want(seen, "seen", torch.int32, desc.n_samples, exact=True)
    _want(first, "first", torch.int32, desc.batch, exact=True)
    return Job(JOB_ENCODE_SEEN, _copy_desc(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
               _dev(m_buf, "m_buf"), _dev(codes, "codes"), _dev(scales, "scales"), None,
               _dev(seen, "seen"), _dev(first, "first"), None, stamp & 0xFFFFFFFF, 0)


def decode_seen_job(desc: Desc, codes, scales, full, sample_ids, m_buf, seen, stamp: int, out) -> Job:
    """An ``aqsgd_decode_seen`` call as one job of :func:`run_jobs`."""
    _check(desc, rows=[(out, "out"), (full, "full")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales)
    _want(seen, "seen", torch.int32, desc.n_samples, exact=True)
    return Job(JOB_DECODE_SEEN, _copy_desc(desc), None, _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"),
               _dev(codes, "codes"), _dev(scales, "scales"), _dev(out, "out"),
               _dev(seen, "seen"), None, _dev(full, "full"), stamp & 0xFFFFFFFF, 0)


def run_jobs(jobs, stream=None) -> None:
    """``aqsgd_run_jobs``: independent messages (built with the ``*_job`` helpers) in as few
    launches as possible.  The tensors the jobs point at must stay alive until the stream
    has run them, as for the single calls."""
    arr = (Job * len(jobs))(*jobs)
    _raise(lib().aqsgd_run_jobs(arr, len(jobs), _stream(stream)))


def encode_seen(desc: Desc, act, sample_ids, m_buf, seen, stamp: int, first, codes, scales, stream=None) -> None:
    """``aqsgd_encode_seen``: Algorithm 1's sender with the first-visit branch.  ``seen`` is an
    int32 tensor (one 32-bit word per sample, zero = never visited); ``stamp`` a non-zero
    32-bit number that no earlier call on this buffer has used."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, m_buf=m_buf, codes=codes, scales=scales, stream=stream)
    _want(seen, "seen", torch.int32, desc.n_samples, exact=True)
    _want(first, "first", torch.int32, desc.batch, exact=True)
    _raise(lib().aqsgd_encode_seen(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                                   _dev(m_buf, "m_buf"), _dev(seen, "seen"), stamp & 0xFFFFFFFF,
                                   _dev(first, "first"), _dev(codes, "codes"), _dev(scales, "scales"),
                                   _stream(stream)))


def decode_seen(desc: Desc, codes, scales, full, sample_ids, m_buf, seen, stamp: int, out, stream=None) -> None:
    """``aqsgd_decode_seen``: Algorithm 1's receiver with the first-visit branch."""
    _check(desc, rows=[(out, "out"), (full, "full")], ids=sample_ids, m_buf=m_buf, codes=codes,
           scales=scales, stream=stream)
    _want(seen, "seen", torch.int32, desc.n_samples, exact=True)
    _raise(lib().aqsgd_decode_seen(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                                   _dev(full, "full"), _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"),
                                   _dev(seen, "seen"), stamp & 0xFFFFFFFF, _dev(out, "out"), _stream(stream)))


def lowbit_row_bytes(desc: Desc, m_bits: int) -> int:
    return int(lib().aqsgd_lowbit_row_bytes(ctypes.byref(desc), m_bits))


def _check_lowbit_store(desc: Desc, m_bits: int, m_codes, m_scales) -> None:
    row = lowbit_row_bytes(desc, m_bits)
    if row:                                     # 0: the library reports the bad descriptor
        _want(m_codes, "m_codes", torch.uint8, desc.n_samples * row, exact=True)
        _want(m_scales, "m_scales", torch.float32, desc.n_samples * (desc.n_per // desc.group), exact=True)


def encode_lowbit(desc: Desc, m_bits: int, act, sample_ids, m_codes, m_scales, codes, scales,
                  stream=None) -> None:
    """``aqsgd_encode_lowbit``: sender with z-bit storage of the previous messages."""
    _check(desc, rows=[(act, "act")], ids=sample_ids, codes=codes, scales=scales, stream=stream)
    _check_lowbit_store(desc, m_bits, m_codes, m_scales)
    _raise(lib().aqsgd_encode_lowbit(ctypes.byref(desc), m_bits, _dev(act, "act"),
                                     _dev(sample_ids, "sample_ids"), _dev(m_codes, "m_codes"),
                                     _dev(m_scales, "m_scales"), _dev(codes, "codes"),
                                     _dev(scales, "scales"), _stream(stream)))


def decode_lowbit(desc: Desc, m_bits: int, codes, scales, sample_ids, m_codes, m_scales, out,
                  stream=None) -> None:
    """``aqsgd_decode_lowbit``: receiver with z-bit storage of the previous messages."""
    _check(desc, rows=[(out, "out")], ids=sample_ids, codes=codes, scales=scales, stream=stream)
    _check_lowbit_store(desc, m_bits, m_codes, m_scales)
    _raise(lib().aqsgd_decode_lowbit(ctypes.byref(desc), m_bits, _dev(codes, "codes"),
                                     _dev(scales, "scales"), _dev(sample_ids, "sample_ids"),
                                     _dev(m_codes, "m_codes"), _dev(m_scales, "m_scales"),
                                     _dev(out, "out"), _stream(stream)))


def topk_bitmap_bytes(desc: Desc) -> int:
    return int(lib().aqsgd_topk_bitmap_bytes(ctypes.byref(desc)))


def topk_codes_bytes(desc: Desc, keep: int) -> int:
    return int(lib().aqsgd_topk_codes_bytes(ctypes.byref(desc), keep))


def _check_topk(desc: Desc, keep: int, rows, what: str, bitmap, codes, scales) -> None:
    nb = topk_bitmap_bytes(desc)
    if nb:                                      # 0: the library reports the bad descriptor
        _check(desc, rows=[(rows, what)], scales=scales)
        _want(bitmap, "bitmap", torch.uint8, nb, exact=False)
        nc = topk_codes_bytes(desc, keep)
        if nc:
            _want(codes, "codes", torch.uint8, nc, exact=False)


def grad_topk_quant(desc: Desc, keep: int, grad, bitmap, codes, scales, stream=None) -> None:
    """``aqsgd_grad_topk_quant``: the ``keep`` largest entries per group, at 8 bits."""
    _check_topk(desc, keep, grad, "grad", bitmap, codes, scales)
    _raise(lib().aqsgd_grad_topk_quant(ctypes.byref(desc), keep, _dev(grad, "grad"), _dev(bitmap, "bitmap"),
                                       _dev(codes, "codes"), _dev(scales, "scales"), _stream(stream)))


def grad_topk_dequant(desc: Desc, keep: int, bitmap, codes, scales, out, stream=None) -> None:
    """``aqsgd_grad_topk_dequant``: kept entries reconstructed, the rest +0."""
    _check_topk(desc, keep, out, "out", bitmap, codes, scales)
    _raise(lib().aqsgd_grad_topk_dequant(ctypes.byref(desc), keep, _dev(bitmap, "bitmap"),
                                         _dev(codes, "codes"), _dev(scales, "scales"), _dev(out, "out"),
                                         _stream(stream)))


def check_ids(sample_ids, n_samples: int, flag, stream=None) -> None:
    """``aqsgd_check_ids``: bit 0 of ``flag`` (one zeroed device int32) is set if an id is
    out of range, bit 1 if two ids are equal."""
    _want(sample_ids, "sample_ids", torch.int64, sample_ids.numel(), exact=True)
    _want(flag, "flag", torch.int32, 1, exact=False)
    _raise(lib().aqsgd_check_ids(_dev(sample_ids, "sample_ids"), sample_ids.numel(), n_samples,
                                 _dev(flag, "flag"), _stream(stream)))


def set_launch_shape(max_blocks: int = 0, dequant_unroll: int = 0) -> None:
    """``aqsgd_set_launch_shape``: bound the workgroups per launch / pick the dequantising
    kernel's unroll for this process; 0 restores the environment's or the built-in value."""
    _raise(lib().aqsgd_set_launch_shape(max_blocks, dequant_unroll))


def profile_next_launch(start: "torch.cuda.Event", stop: "torch.cuda.Event") -> None:
    """Have the next codec launch of this thread stamp two timing events with the
    kernel's own begin and end.  The events must already exist on the device
    (a torch event is created by its first ``record()``)."""
    _raise(lib().aqsgd_profile_next_launch(ctypes.c_void_p(start.cuda_event),
                                           ctypes.c_void_p(stop.cuda_event)))


class Tier:
    """Handle of ``aqsgd_tier``: previous messages below HBM, ``slots`` windows of ``batch``
    rows in HBM.  Host tier: ``host_rows`` pinned [N, row] holds every row.  File tier
    (``path`` given): the rows live in that file and ``host_rows`` pinned [slots*batch, row]
    is the staging memory; ``n_samples`` is then the number of rows of the file.  The
    tensors are the caller's memory (``dev_rows`` [slots*batch, row], ``dev_row_ids`` int64
    [slots*batch]); this object only forwards calls and keeps them alive."""

    def __init__(self, host_rows, dev_rows, dev_row_ids, slots: int, batch: int, path: str | None = None,
                 n_samples: int | None = None, direct_io: bool = False):
        if not host_rows.is_pinned() or host_rows.is_cuda or not host_rows.is_contiguous():
            raise ValueError("host_rows must be a contiguous pinned host tensor")
        if dev_rows.shape[0] != slots * batch or dev_row_ids.numel() != slots * batch:
            raise ValueError("dev_rows / dev_row_ids must hold slots * batch rows")
        if dev_row_ids.dtype != torch.int64:
            raise ValueError("dev_row_ids must be int64")
        self.host_rows, self.dev_rows, self.dev_row_ids = host_rows, dev_rows, dev_row_ids
        self.slots, self.batch = slots, batch
        row_bytes = host_rows[0].numel() * host_rows.element_size()
        if dev_rows[0].numel() * dev_rows.element_size() != row_bytes:
            raise ValueError("host and device rows differ in size")
        self._h = ctypes.c_void_p()
        if path is None:
            _raise(lib().aqsgd_tier_create(ctypes.byref(self._h), ctypes.c_void_p(host_rows.data_ptr()),
                                           _dev(dev_rows, "dev_rows"), _dev(dev_row_ids, "dev_row_ids"),
                                           host_rows.shape[0], row_bytes, slots, batch))
        else:
            if host_rows.shape[0] != slots * batch or not n_samples:
                raise ValueError("the file tier needs slots * batch staging rows and the file's row count")
            _raise(lib().aqsgd_tier_create_file(ctypes.byref(self._h), str(path).encode(), int(direct_io),
                                                ctypes.c_void_p(host_rows.data_ptr()), _dev(dev_rows, "dev_rows"),
                                                _dev(dev_row_ids, "dev_row_ids"), n_samples, row_bytes, slots,
                                                batch))

    def prefetch(self, slot: int, host_ids, copy_stream) -> None:
        """``host_ids``: host int64 tensor of ``batch`` distinct sample ids."""
        if host_ids.is_cuda or host_ids.dtype != torch.int64 or host_ids.numel() != self.batch:
            raise ValueError("host_ids must be a host int64 tensor with one id per row of the window")
        _raise(lib().aqsgd_tier_prefetch(self._h, slot, ctypes.c_void_p(host_ids.data_ptr()),
                                         _stream(copy_stream)))

    def acquire(self, slot: int, compute_stream=None):
        """Returns the window's sample ids (a view of ``dev_row_ids``) for the codec call."""
        p = ctypes.c_void_p()
        _raise(lib().aqsgd_tier_acquire(self._h, slot, _stream(compute_stream), ctypes.byref(p)))
        ids = self.dev_row_ids[slot * self.batch:(slot + 1) * self.batch]
        assert ids.data_ptr() == p.value
        return ids

    def release(self, slot: int, compute_stream, copy_stream) -> None:
        _raise(lib().aqsgd_tier_release(self._h, slot, _stream(compute_stream), _stream(copy_stream)))

    def drain(self) -> None:
        _raise(lib().aqsgd_tier_drain(self._h))

    def close(self) -> None:
        if self._h:
            lib().aqsgd_tier_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
