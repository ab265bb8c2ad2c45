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

_HERE = Path(__file__).resolve().parent
LIB_PATH = _HERE / "libaqsgd.so"

F32, F16, BF16 = 0, 1, 2
NEAREST, STOCHASTIC = 0, 1

DTYPE_CODE = {torch.float32: F32, torch.float16: F16, torch.bfloat16: BF16}
DTYPE_NAME = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}

EXPORTS = ("aqsgd_codes_bytes", "aqsgd_scales_count", "aqsgd_encode", "aqsgd_decode",
           "aqsgd_grad_quant", "aqsgd_grad_dequant", "aqsgd_seed", "aqsgd_encode_seen",
           "aqsgd_decode_seen", "aqsgd_lowbit_row_bytes",
           "aqsgd_encode_lowbit", "aqsgd_decode_lowbit", "aqsgd_tier_create", "aqsgd_tier_prefetch",
           "aqsgd_tier_acquire", "aqsgd_tier_release", "aqsgd_tier_drain", "aqsgd_tier_destroy",
           "aqsgd_topk_bitmap_bytes", "aqsgd_topk_codes_bytes", "aqsgd_grad_topk_quant",
           "aqsgd_grad_topk_dequant", "aqsgd_check_ids", "aqsgd_set_launch_shape",
           "aqsgd_profile_next_launch", "aqsgd_strerror", "aqsgd_version")


class Desc(ctypes.Structure):
    """Mirror of ``aqsgd_desc``."""
    _fields_ = [("batch", ctypes.c_int64), ("n_per", ctypes.c_int64), ("n_samples", ctypes.c_int64),
                ("bits", ctypes.c_int32), ("group", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("rounding", ctypes.c_int32), ("rng_seed", ctypes.c_uint64)]


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
        L.aqsgd_encode_seen.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.aqsgd_decode_seen.restype = ctypes.c_int
        L.aqsgd_decode_seen.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, vp]
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


def _raise(status: int):
    if status != 0:
        raise AqsgdError(status, strerror(status))


def encode(desc: Desc, act, sample_ids, m_buf, codes, scales, stream=None) -> None:
    """``aqsgd_encode``: updates ``m_buf`` in place, fills ``codes`` and ``scales``."""
    _raise(lib().aqsgd_encode(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                              _dev(m_buf, "m_buf"), _dev(codes, "codes"), _dev(scales, "scales"),
                              _stream(stream)))


def decode(desc: Desc, codes, scales, sample_ids, m_buf, out, stream=None) -> None:
    """``aqsgd_decode``: updates ``m_buf`` in place, fills ``out``."""
    _raise(lib().aqsgd_decode(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                              _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"), _dev(out, "out"),
                              _stream(stream)))


def grad_quant(desc: Desc, grad, codes, scales, stream=None) -> None:
    _raise(lib().aqsgd_grad_quant(ctypes.byref(desc), _dev(grad, "grad"), _dev(codes, "codes"),
                                  _dev(scales, "scales"), _stream(stream)))


def grad_dequant(desc: Desc, codes, scales, out, stream=None) -> None:
    _raise(lib().aqsgd_grad_dequant(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                                    _dev(out, "out"), _stream(stream)))


def seed(desc: Desc, act, sample_ids, m_buf, stream=None) -> None:
    """``aqsgd_seed``: uncompressed first visit, ``m_buf[sample_ids] <- act``."""
    _raise(lib().aqsgd_seed(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                            _dev(m_buf, "m_buf"), _stream(stream)))


def encode_seen(desc: Desc, act, sample_ids, m_buf, seen, first, codes, scales, stream=None) -> None:
    """``aqsgd_encode_seen``: Algorithm 1's sender with the first-visit branch."""
    _raise(lib().aqsgd_encode_seen(ctypes.byref(desc), _dev(act, "act"), _dev(sample_ids, "sample_ids"),
                                   _dev(m_buf, "m_buf"), _dev(seen, "seen"), _dev(first, "first"),
                                   _dev(codes, "codes"), _dev(scales, "scales"), _stream(stream)))


def decode_seen(desc: Desc, codes, scales, full, sample_ids, m_buf, seen, out, stream=None) -> None:
    """``aqsgd_decode_seen``: Algorithm 1's receiver with the first-visit branch."""
    _raise(lib().aqsgd_decode_seen(ctypes.byref(desc), _dev(codes, "codes"), _dev(scales, "scales"),
                                   _dev(full, "full"), _dev(sample_ids, "sample_ids"), _dev(m_buf, "m_buf"),
                                   _dev(seen, "seen"), _dev(out, "out"), _stream(stream)))


def lowbit_row_bytes(desc: Desc, m_bits: int) -> int:
    return int(lib().aqsgd_lowbit_row_bytes(ctypes.byref(desc), m_bits))


def encode_lowbit(desc: Desc, m_bits: int, act, sample_ids, m_codes, m_scales, codes, scales,
                  stream=None) -> None:
    """``aqsgd_encode_lowbit``: sender with z-bit storage of the previous messages."""
    _raise(lib().aqsgd_encode_lowbit(ctypes.byref(desc), m_bits, _dev(act, "act"),
                                     _dev(sample_ids, "sample_ids"), _dev(m_codes, "m_codes"),
                                     _dev(m_scales, "m_scales"), _dev(codes, "codes"),
                                     _dev(scales, "scales"), _stream(stream)))


def decode_lowbit(desc: Desc, m_bits: int, codes, scales, sample_ids, m_codes, m_scales, out,
                  stream=None) -> None:
    """``aqsgd_decode_lowbit``: receiver with z-bit storage of the previous messages."""
    _raise(lib().aqsgd_decode_lowbit(ctypes.byref(desc), m_bits, _dev(codes, "codes"),
                                     _dev(scales, "scales"), _dev(sample_ids, "sample_ids"),
                                     _dev(m_codes, "m_codes"), _dev(m_scales, "m_scales"),
                                     _dev(out, "out"), _stream(stream)))


def topk_bitmap_bytes(desc: Desc) -> int:
    return int(lib().aqsgd_topk_bitmap_bytes(ctypes.byref(desc)))


def topk_codes_bytes(desc: Desc, keep: int) -> int:
    return int(lib().aqsgd_topk_codes_bytes(ctypes.byref(desc), keep))


def grad_topk_quant(desc: Desc, keep: int, grad, bitmap, codes, scales, stream=None) -> None:
    """``aqsgd_grad_topk_quant``: the ``keep`` largest entries per group, at 8 bits."""
    _raise(lib().aqsgd_grad_topk_quant(ctypes.byref(desc), keep, _dev(grad, "grad"), _dev(bitmap, "bitmap"),
                                       _dev(codes, "codes"), _dev(scales, "scales"), _stream(stream)))


def grad_topk_dequant(desc: Desc, keep: int, bitmap, codes, scales, out, stream=None) -> None:
    """``aqsgd_grad_topk_dequant``: kept entries reconstructed, the rest +0."""
    _raise(lib().aqsgd_grad_topk_dequant(ctypes.byref(desc), keep, _dev(bitmap, "bitmap"),
                                         _dev(codes, "codes"), _dev(scales, "scales"), _dev(out, "out"),
                                         _stream(stream)))


def check_ids(sample_ids, n_samples: int, flag, stream=None) -> None:
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
    """Handle of ``aqsgd_tier``: previous messages in pinned host memory, ``slots``
    windows of ``batch`` rows in HBM.  The three tensors are the caller's memory
    (``host_rows`` pinned [N, row], ``dev_rows`` [slots*batch, row], ``dev_row_ids``
    int64 [slots*batch]); this object only forwards calls and keeps them alive."""

    def __init__(self, host_rows, dev_rows, dev_row_ids, slots: int, batch: int):
        if not host_rows.is_pinned() or host_rows.is_cuda or not host_rows.is_contiguous():
            raise ValueError("host_rows must be a contiguous pinned host tensor")
        if dev_rows.shape[0] != slots * batch or dev_row_ids.numel() != slots * batch:
            raise ValueError("dev_rows / dev_row_ids must hold slots * batch rows")
        self.host_rows, self.dev_rows, self.dev_row_ids = host_rows, dev_rows, dev_row_ids
        self.slots, self.batch = slots, batch
        row_bytes = host_rows[0].numel() * host_rows.element_size()
        self._h = ctypes.c_void_p()
        _raise(lib().aqsgd_tier_create(ctypes.byref(self._h), ctypes.c_void_p(host_rows.data_ptr()),
                                       _dev(dev_rows, "dev_rows"), _dev(dev_row_ids, "dev_row_ids"),
                                       host_rows.shape[0], row_bytes, slots, batch))

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
