"""Python face of the CPU oracle (``aqsgd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by the smoke check and by the
CPU-baseline leg of ``bench.py``; never by the product package.  Arrays are
numpy, on the host; float16 travels as ``np.float16``, bfloat16 as ``np.uint16``
bit patterns, float32 as ``np.float32``.

The shared object is built on demand with gcc (``build()``), with floating-point
contraction off so that every written operation rounds once.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "aqsgd_oracle.c"
_LIB = _HERE / "libaqsgd_oracle.so"

F32, F16, BF16 = 0, 1, 2
NEAREST, STOCHASTIC = 0, 1
DTYPE_CODE = {"f32": F32, "f16": F16, "bf16": BF16}
_NP_OF = {F32: np.float32, F16: np.float16, BF16: np.uint16}

_CFLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp",
           "-ffp-contract=off", "-fno-fast-math", "-Wall", "-Wextra"]


def build(force: bool = False) -> Path:
    """Compile the oracle if the library is missing or older than its source."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.run(["gcc", *_CFLAGS, str(_SRC), "-o", str(tmp), "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        i32, i64, u64 = ctypes.c_int, ctypes.c_int64, ctypes.c_uint64
        vp = ctypes.c_void_p
        L.aqsgd_oracle_half_to_float.restype = ctypes.c_float
        L.aqsgd_oracle_half_to_float.argtypes = [ctypes.c_uint16]
        L.aqsgd_oracle_float_to_half.restype = ctypes.c_uint16
        L.aqsgd_oracle_float_to_half.argtypes = [ctypes.c_float]
        L.aqsgd_oracle_bf16_to_float.restype = ctypes.c_float
        L.aqsgd_oracle_bf16_to_float.argtypes = [ctypes.c_uint16]
        L.aqsgd_oracle_float_to_bf16.restype = ctypes.c_uint16
        L.aqsgd_oracle_float_to_bf16.argtypes = [ctypes.c_float]
        L.aqsgd_oracle_philox4x32_10.restype = None
        L.aqsgd_oracle_philox4x32_10.argtypes = [vp, vp, vp]
        L.aqsgd_oracle_uniform.restype = ctypes.c_float
        L.aqsgd_oracle_uniform.argtypes = [u64, u64]
        L.aqsgd_oracle_pack.restype = None
        L.aqsgd_oracle_pack.argtypes = [vp, i64, i32, vp]
        L.aqsgd_oracle_unpack.restype = None
        L.aqsgd_oracle_unpack.argtypes = [vp, i64, i32, vp]
        L.aqsgd_oracle_quantize_group.restype = None
        L.aqsgd_oracle_quantize_group.argtypes = [vp, vp, i64, i32, vp, vp, vp]
        L.aqsgd_oracle_dequantize_group.restype = None
        L.aqsgd_oracle_dequantize_group.argtypes = [vp, ctypes.c_float, i64, i32, vp]
        L.aqsgd_oracle_encode.restype = i32
        L.aqsgd_oracle_encode.argtypes = [i32, i32, i64, i32, u64, i64, i64, vp, vp, vp, vp, vp]
        L.aqsgd_oracle_seed.restype = i32
        L.aqsgd_oracle_seed.argtypes = [i32, i64, i64, vp, vp, vp]
        L.aqsgd_oracle_encode_lowbit.restype = i32
        L.aqsgd_oracle_encode_lowbit.argtypes = [i32, i32, i32, i64, i32, u64, i64, i64, vp, vp, vp, vp, vp, vp]
        L.aqsgd_oracle_decode_lowbit.restype = i32
        L.aqsgd_oracle_decode_lowbit.argtypes = [i32, i32, i32, i64, i64, i64, vp, vp, vp, vp, vp, vp]
        L.aqsgd_oracle_decode.restype = i32
        L.aqsgd_oracle_decode.argtypes = [i32, i32, i64, i64, i64, vp, vp, vp, vp, vp]
        L.aqsgd_oracle_grad_quant.restype = i32
        L.aqsgd_oracle_grad_quant.argtypes = [i32, i32, i64, i32, u64, i64, i64, vp, vp, vp]
        L.aqsgd_oracle_grad_dequant.restype = i32
        L.aqsgd_oracle_grad_dequant.argtypes = [i32, i32, i64, i64, i64, vp, vp, vp]
        _lib = L
    return _lib


def set_threads(n: int) -> None:
    """Number of OpenMP threads the group loops use (1 = serial)."""
    omp = ctypes.CDLL("libgomp.so.1")
    omp.omp_set_num_threads(int(n))


def max_threads() -> int:
    omp = ctypes.CDLL("libgomp.so.1")
    return int(omp.omp_get_max_threads())


def _ptr(a: np.ndarray) -> ctypes.c_void_p:
    return ctypes.c_void_p(a.ctypes.data)


def _check(a: np.ndarray, dtype, what: str) -> np.ndarray:
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{what}: need C-contiguous {np.dtype(dtype)}, got {a.dtype}")
    return a


def codes_bytes(n: int, bits: int) -> int:
    return n * bits // 8


# -- building blocks (used by the pins) ------------------------------------
def half_to_float(h: int) -> float:
    return float(lib().aqsgd_oracle_half_to_float(int(h)))


def float_to_half(x) -> int:
    return int(lib().aqsgd_oracle_float_to_half(ctypes.c_float(x)))


def bf16_to_float(b: int) -> float:
    return float(lib().aqsgd_oracle_bf16_to_float(int(b)))


def float_to_bf16(x) -> int:
    return int(lib().aqsgd_oracle_float_to_bf16(ctypes.c_float(x)))


def philox4x32_10(ctr, key) -> np.ndarray:
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    out = np.zeros(4, dtype=np.uint32)
    lib().aqsgd_oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def uniform(seed: int, j: int) -> np.float32:
    return np.float32(lib().aqsgd_oracle_uniform(seed, j))


def pack(q: np.ndarray, bits: int) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int32)
    out = np.zeros((q.size * bits + 7) // 8, dtype=np.uint8)
    lib().aqsgd_oracle_pack(_ptr(q), q.size, bits, _ptr(out))
    return out


def unpack(b: np.ndarray, count: int, bits: int) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint8)
    q = np.zeros(count, dtype=np.int32)
    lib().aqsgd_oracle_unpack(_ptr(b), count, bits, _ptr(q))
    return q


def quantize_group(d: np.ndarray, bits: int, r: np.ndarray | None = None):
    """Q on one group. ``r``: rounding offsets (default 1/2 = nearest).

    Returns (q int32[G], scale float32, dhat float32[G]).
    """
    d = np.ascontiguousarray(d, dtype=np.float32)
    r = np.full(d.size, 0.5, dtype=np.float32) if r is None \
        else np.ascontiguousarray(r, dtype=np.float32)
    q = np.zeros(d.size, dtype=np.int32)
    s = np.zeros(1, dtype=np.float32)
    dhat = np.zeros(d.size, dtype=np.float32)
    lib().aqsgd_oracle_quantize_group(_ptr(d), _ptr(r), d.size, bits, _ptr(q), _ptr(s), _ptr(dhat))
    return q, s[0], dhat


def dequantize_group(q: np.ndarray, scale, bits: int) -> np.ndarray:
    q = np.ascontiguousarray(q, dtype=np.int32)
    dhat = np.zeros(q.size, dtype=np.float32)
    lib().aqsgd_oracle_dequantize_group(_ptr(q), ctypes.c_float(scale), q.size, bits, _ptr(dhat))
    return dhat


# -- the four boundary calls ------------------------------------------------
def encode(act: np.ndarray, ids: np.ndarray, m_buf: np.ndarray, *, dtype: str, bits: int,
           group: int, rounding: int = NEAREST, seed: int = 0):
    """Sender side.  Updates ``m_buf`` in place; returns (codes, scales)."""
    dt = DTYPE_CODE[dtype]
    _check(act, _NP_OF[dt], "act"); _check(m_buf, _NP_OF[dt], "m_buf")
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    batch = ids.size
    assert m_buf.ndim >= 2, "m_buf must be [rows, ...sample shape]"
    n_rows = m_buf.shape[0]
    n_per = m_buf.size // n_rows
    assert act.size == batch * n_per
    assert batch == 0 or (ids.min() >= 0 and ids.max() < n_rows), "sample id out of range"
    assert len(np.unique(ids)) == batch, "duplicate sample ids in one call"
    n = batch * n_per
    codes = np.zeros(codes_bytes(n, bits), dtype=np.uint8)
    scales = np.zeros(n // group, dtype=np.float32)
    rc = lib().aqsgd_oracle_encode(dt, bits, group, rounding, seed, batch, n_per,
                                   _ptr(act), _ptr(ids), _ptr(m_buf), _ptr(codes), _ptr(scales))
    if rc:
        raise ValueError(f"oracle encode rejected its arguments (rc={rc})")
    return codes, scales


def seed(act: np.ndarray, ids: np.ndarray, m_buf: np.ndarray, *, dtype: str) -> None:
    """Uncompressed first visit: ``m_buf[ids] <- act`` in place."""
    dt = DTYPE_CODE[dtype]
    _check(act, _NP_OF[dt], "act"); _check(m_buf, _NP_OF[dt], "m_buf")
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    batch = ids.size
    assert m_buf.ndim >= 2, "m_buf must be [rows, ...sample shape]"
    n_rows = m_buf.shape[0]
    n_per = m_buf.size // n_rows
    assert act.size == batch * n_per
    assert batch == 0 or (ids.min() >= 0 and ids.max() < n_rows), "sample id out of range"
    assert len(np.unique(ids)) == batch, "duplicate sample ids in one call"
    rc = lib().aqsgd_oracle_seed(dt, batch, n_per, _ptr(act), _ptr(ids), _ptr(m_buf))
    if rc:
        raise ValueError(f"oracle seed rejected its arguments (rc={rc})")


def decode(codes: np.ndarray, scales: np.ndarray, ids: np.ndarray, m_buf: np.ndarray, *,
           dtype: str, bits: int, group: int) -> np.ndarray:
    """Receiver side.  Updates ``m_buf`` in place; returns the activation [B*n_per]."""
    dt = DTYPE_CODE[dtype]
    _check(codes, np.uint8, "codes"); _check(scales, np.float32, "scales")
    _check(m_buf, _NP_OF[dt], "m_buf")
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    batch = ids.size
    assert m_buf.ndim >= 2, "m_buf must be [rows, ...sample shape]"
    n_rows = m_buf.shape[0]
    n_per = m_buf.size // n_rows
    assert batch == 0 or (ids.min() >= 0 and ids.max() < n_rows), "sample id out of range"
    assert len(np.unique(ids)) == batch, "duplicate sample ids in one call"
    assert codes.size == codes_bytes(batch * n_per, bits)
    assert scales.size == batch * n_per // group
    out = np.zeros(batch * n_per, dtype=_NP_OF[dt])
    rc = lib().aqsgd_oracle_decode(dt, bits, group, batch, n_per, _ptr(codes), _ptr(scales),
                                   _ptr(ids), _ptr(m_buf), _ptr(out))
    if rc:
        raise ValueError(f"oracle decode rejected its arguments (rc={rc})")
    return out


def grad_quant(grad: np.ndarray, *, dtype: str, bits: int, group: int,
               rounding: int = NEAREST, seed: int = 0):
    dt = DTYPE_CODE[dtype]
    _check(grad, _NP_OF[dt], "grad")
    n = grad.size
    codes = np.zeros(codes_bytes(n, bits), dtype=np.uint8)
    scales = np.zeros(n // group, dtype=np.float32)
    rc = lib().aqsgd_oracle_grad_quant(dt, bits, group, rounding, seed, 1, n,
                                       _ptr(grad), _ptr(codes), _ptr(scales))
    if rc:
        raise ValueError(f"oracle grad_quant rejected its arguments (rc={rc})")
    return codes, scales


def grad_dequant(codes: np.ndarray, scales: np.ndarray, *, dtype: str, bits: int,
                 group: int) -> np.ndarray:
    dt = DTYPE_CODE[dtype]
    _check(codes, np.uint8, "codes"); _check(scales, np.float32, "scales")
    n = scales.size * group
    assert codes.size == codes_bytes(n, bits)
    out = np.zeros(n, dtype=_NP_OF[dt])
    rc = lib().aqsgd_oracle_grad_dequant(dt, bits, group, 1, n, _ptr(codes), _ptr(scales), _ptr(out))
    if rc:
        raise ValueError(f"oracle grad_dequant rejected its arguments (rc={rc})")
    return out


# -- previous messages kept at low precision ("m z") --------------------------
def lowbit_state(n_rows: int, n_per: int, m_bits: int, group: int):
    """All-zero storage for ``n_rows`` samples: (m_codes uint8 [rows, n_per*z/8],
    m_scales float32 [rows, n_per/group])."""
    return (np.zeros((n_rows, n_per * m_bits // 8), dtype=np.uint8),
            np.zeros((n_rows, n_per // group), dtype=np.float32))


def _lowbit_shapes(ids, m_codes, m_scales, m_bits, group):
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    _check(m_codes, np.uint8, "m_codes"); _check(m_scales, np.float32, "m_scales")
    n_rows = m_codes.shape[0]
    n_per = m_codes.shape[1] * 8 // m_bits
    assert m_scales.shape == (n_rows, n_per // group)
    assert ids.size == 0 or (ids.min() >= 0 and ids.max() < n_rows), "sample id out of range"
    assert len(np.unique(ids)) == ids.size, "duplicate sample ids in one call"
    return ids, n_per


def encode_lowbit(act: np.ndarray, ids: np.ndarray, m_codes: np.ndarray, m_scales: np.ndarray, *,
                  dtype: str, bits: int, m_bits: int, group: int, rounding: int = NEAREST, seed: int = 0):
    """Sender with z-bit storage of m.  Updates the storage in place; returns (codes, scales)."""
    dt = DTYPE_CODE[dtype]
    _check(act, _NP_OF[dt], "act")
    ids, n_per = _lowbit_shapes(ids, m_codes, m_scales, m_bits, group)
    n = ids.size * n_per
    assert act.size == n
    codes = np.zeros(codes_bytes(n, bits), dtype=np.uint8)
    scales = np.zeros(n // group, dtype=np.float32)
    rc = lib().aqsgd_oracle_encode_lowbit(dt, bits, m_bits, group, rounding, seed, ids.size, n_per,
                                          _ptr(act), _ptr(ids), _ptr(m_codes), _ptr(m_scales),
                                          _ptr(codes), _ptr(scales))
    if rc:
        raise ValueError(f"oracle encode_lowbit rejected its arguments (rc={rc})")
    return codes, scales


def decode_lowbit(codes: np.ndarray, scales: np.ndarray, ids: np.ndarray, m_codes: np.ndarray,
                  m_scales: np.ndarray, *, dtype: str, bits: int, m_bits: int, group: int) -> np.ndarray:
    """Receiver with z-bit storage of m.  Updates the storage in place; returns the activation."""
    dt = DTYPE_CODE[dtype]
    _check(codes, np.uint8, "codes"); _check(scales, np.float32, "scales")
    ids, n_per = _lowbit_shapes(ids, m_codes, m_scales, m_bits, group)
    n = ids.size * n_per
    assert codes.size == codes_bytes(n, bits) and scales.size == n // group
    out = np.zeros(n, dtype=_NP_OF[dt])
    rc = lib().aqsgd_oracle_decode_lowbit(dt, bits, m_bits, group, ids.size, n_per, _ptr(codes),
                                          _ptr(scales), _ptr(ids), _ptr(m_codes), _ptr(m_scales), _ptr(out))
    if rc:
        raise ValueError(f"oracle decode_lowbit rejected its arguments (rc={rc})")
    return out


# -- sparsified backward message (top-k + b-bit, Appendix H.6) ------------------
def grad_topk_quant(grad: np.ndarray, *, dtype: str, bits: int, group: int, keep: int,
                    rounding: int = NEAREST, seed: int = 0):
    """Returns (bitmap uint8[n/8], codes uint8[n_groups*keep*bits/8], scales float32[n_groups])."""
    dt = DTYPE_CODE[dtype]
    _check(grad, _NP_OF[dt], "grad")
    n = grad.size
    bitmap = np.zeros(n // 8, dtype=np.uint8)
    codes = np.zeros(n // group * keep * bits // 8, dtype=np.uint8)
    scales = np.zeros(n // group, dtype=np.float32)
    L = lib()
    L.aqsgd_oracle_grad_topk_quant.restype = ctypes.c_int
    L.aqsgd_oracle_grad_topk_quant.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                               ctypes.c_int, ctypes.c_uint64, ctypes.c_int64] + [ctypes.c_void_p] * 4
    rc = L.aqsgd_oracle_grad_topk_quant(dt, bits, group, keep, rounding, seed, n, _ptr(grad), _ptr(bitmap),
                                        _ptr(codes), _ptr(scales))
    if rc:
        raise ValueError(f"oracle grad_topk_quant rejected its arguments (rc={rc})")
    return bitmap, codes, scales


def grad_topk_dequant(bitmap: np.ndarray, codes: np.ndarray, scales: np.ndarray, *, dtype: str,
                      bits: int, group: int, keep: int) -> np.ndarray:
    dt = DTYPE_CODE[dtype]
    _check(bitmap, np.uint8, "bitmap"); _check(codes, np.uint8, "codes"); _check(scales, np.float32, "scales")
    n = scales.size * group
    assert bitmap.size == n // 8 and codes.size == scales.size * keep * bits // 8
    out = np.zeros(n, dtype=_NP_OF[dt])
    L = lib()
    L.aqsgd_oracle_grad_topk_dequant.restype = ctypes.c_int
    L.aqsgd_oracle_grad_topk_dequant.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                                 ctypes.c_int64] + [ctypes.c_void_p] * 4
    rc = L.aqsgd_oracle_grad_topk_dequant(dt, bits, group, keep, n, _ptr(bitmap), _ptr(codes), _ptr(scales),
                                          _ptr(out))
    if rc:
        raise ValueError(f"oracle grad_topk_dequant rejected its arguments (rc={rc})")
    return out


# -- Algorithm 1 with its first-visit branch --------------------------------------
def _seen_args(ids, m_buf, seen):
    ids = np.ascontiguousarray(ids, dtype=np.int64)
    assert m_buf.ndim >= 2, "m_buf must be [rows, ...sample shape]"
    n_rows = m_buf.shape[0]
    _check(seen, np.uint8, "seen")
    assert seen.size == n_rows
    assert ids.size == 0 or (ids.min() >= 0 and ids.max() < n_rows), "sample id out of range"
    assert len(np.unique(ids)) == ids.size, "duplicate sample ids in one call"
    return ids, m_buf.size // n_rows


def encode_seen(act: np.ndarray, ids: np.ndarray, m_buf: np.ndarray, seen: np.ndarray, *, dtype: str,
                bits: int, group: int, rounding: int = NEAREST, seed: int = 0, fill: int = 0):
    """Sender side of Algorithm 1.  Updates ``m_buf`` and ``seen`` in place; returns
    (first int32[batch], codes, scales); slices of first-visit samples keep ``fill``."""
    dt = DTYPE_CODE[dtype]
    _check(act, _NP_OF[dt], "act"); _check(m_buf, _NP_OF[dt], "m_buf")
    ids, n_per = _seen_args(ids, m_buf, seen)
    batch = ids.size
    assert act.size == batch * n_per
    n = batch * n_per
    codes = np.full(codes_bytes(n, bits), fill, dtype=np.uint8)
    scales = np.full(n // group, float(fill), dtype=np.float32)
    first = np.zeros(batch, dtype=np.int32)
    L = lib()
    L.aqsgd_oracle_encode_seen.restype = ctypes.c_int
    L.aqsgd_oracle_encode_seen.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int,
                                           ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64] + [ctypes.c_void_p] * 7
    rc = L.aqsgd_oracle_encode_seen(dt, bits, group, rounding, seed, batch, n_per, _ptr(act), _ptr(ids),
                                    _ptr(m_buf), _ptr(seen), _ptr(first), _ptr(codes), _ptr(scales))
    if rc:
        raise ValueError(f"oracle encode_seen rejected its arguments (rc={rc})")
    return first, codes, scales


def decode_seen(codes: np.ndarray, scales: np.ndarray, full: np.ndarray, ids: np.ndarray, m_buf: np.ndarray,
                seen: np.ndarray, *, dtype: str, bits: int, group: int) -> np.ndarray:
    """Receiver side of Algorithm 1.  Updates ``m_buf`` and ``seen`` in place; returns out."""
    dt = DTYPE_CODE[dtype]
    _check(codes, np.uint8, "codes"); _check(scales, np.float32, "scales")
    _check(full, _NP_OF[dt], "full"); _check(m_buf, _NP_OF[dt], "m_buf")
    ids, n_per = _seen_args(ids, m_buf, seen)
    batch = ids.size
    assert full.size == batch * n_per and scales.size == batch * n_per // group
    out = np.zeros(batch * n_per, dtype=_NP_OF[dt])
    L = lib()
    L.aqsgd_oracle_decode_seen.restype = ctypes.c_int
    L.aqsgd_oracle_decode_seen.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int64, ctypes.c_int64,
                                           ctypes.c_int64] + [ctypes.c_void_p] * 7
    rc = L.aqsgd_oracle_decode_seen(dt, bits, group, batch, n_per, _ptr(codes), _ptr(scales), _ptr(full),
                                    _ptr(ids), _ptr(m_buf), _ptr(seen), _ptr(out))
    if rc:
        raise ValueError(f"oracle decode_seen rejected its arguments (rc={rc})")
    return out
