"""Seeded synthetic activation / gradient streams for the stage-boundary codec.

This module only *draws inputs*.  It holds none of the codec's arithmetic (no
delta, scale, rounding, packing or buffer update) and is the one piece of code
that both the CPU oracle's tests and the HIP path's tests feed from.

The streams stand in for the fine-tuning activations of the paper's GPT2-1.5B
and DeBERTa-1.5B runs (Section 4.1 and Appendix C give sequence lengths and
micro-batch structure; the datasets and checkpoints themselves are not used).
What is reproduced is the property the method relies on (Figure 1b): the
activation of one training sample changes only a little between two visits,
so the change is much smaller than the activation.  Sample ``xi`` at epoch
``t`` has the fp32 pre-image

    z_t(xi) = z_0(xi) + drift * sum_{tau=1..t} e_tau(xi),

with ``z_0`` and every ``e_tau`` drawn from the configuration's law by a
generator seeded with ``(seed, xi, tau)``; any (sample, epoch) can therefore
be produced on its own, without state, in any order.

Arrays are returned in the storage dtype of the boundary: ``float32`` and
``float16`` as numpy arrays of that dtype, ``bf16`` as ``uint16`` bit patterns
(numpy has no bfloat16); see :func:`to_torch` for the device-side view.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Iterator, List, Sequence, Tuple

import numpy as np

NEAREST = 0
STOCHASTIC = 1

_DTYPE_BYTES = {"f32": 4, "f16": 2, "bf16": 2}


@dataclass(frozen=True)
class BoundaryConfig:
    """One pipeline-stage boundary: shapes, codec settings and input law."""

    name: str
    n_samples: int          # N rows in the previous-message buffer m
    batch: int              # B samples per call (micro-batch)
    seq: int                # S
    hidden: int             # H
    dtype: str              # "f32" | "f16" | "bf16" (act, m, out)
    fwd_bits: int
    fwd_group: int
    fwd_rounding: int
    bwd_bits: int
    bwd_group: int
    bwd_rounding: int
    law: str                # "normal" | "student_t3" | "laplace"
    drift: float
    epochs: int
    outlier_channel_frac: float = 0.0   # channels scaled by outlier_scale
    outlier_token_frac: float = 0.0     # token rows scaled by outlier_scale
    outlier_scale: float = 1.0
    grad_scale: float = 1e-3
    shuffle_ids: bool = False
    seed: int = 0

    @property
    def n_per(self) -> int:
        return self.seq * self.hidden

    @property
    def n(self) -> int:
        return self.batch * self.n_per

    @property
    def elem_bytes(self) -> int:
        return _DTYPE_BYTES[self.dtype]

    def scaled(self, **kw) -> "BoundaryConfig":
        return replace(self, **kw)


def tiny() -> BoundaryConfig:
    return BoundaryConfig(
        name="tiny", n_samples=64, batch=4, seq=128, hidden=256, dtype="f32",
        fwd_bits=4, fwd_group=256, fwd_rounding=NEAREST,
        bwd_bits=8, bwd_group=256, bwd_rounding=NEAREST,
        law="normal", drift=0.01, epochs=3, seed=0)


def gpt2_4bit() -> BoundaryConfig:
    return BoundaryConfig(
        name="gpt2_1p5b_fw4_bw8", n_samples=8192, batch=4, seq=1024, hidden=1600,
        dtype="f16", fwd_bits=4, fwd_group=1600, fwd_rounding=NEAREST,
        bwd_bits=8, bwd_group=1600, bwd_rounding=NEAREST,
        law="normal", drift=0.05, epochs=2,
        outlier_channel_frac=0.01, outlier_scale=20.0, seed=1)


def gpt2_2bit_stochastic() -> BoundaryConfig:
    return BoundaryConfig(
        name="gpt2_1p5b_fw2_bw4_stochastic", n_samples=8192, batch=4, seq=1024,
        hidden=1600, dtype="f16", fwd_bits=2, fwd_group=128,
        fwd_rounding=STOCHASTIC, bwd_bits=4, bwd_group=128,
        bwd_rounding=STOCHASTIC, law="normal", drift=0.05, epochs=4,
        outlier_channel_frac=0.01, outlier_scale=20.0, shuffle_ids=True, seed=2)


def deberta_3bit() -> BoundaryConfig:
    return BoundaryConfig(
        name="deberta_1p5b_fw3_bw6", n_samples=100_000, batch=32, seq=256,
        hidden=1536, dtype="bf16", fwd_bits=3, fwd_group=64,
        fwd_rounding=NEAREST, bwd_bits=6, bwd_group=64, bwd_rounding=NEAREST,
        law="student_t3", drift=0.05, epochs=2, seed=3)


def stress(bits: int = 4, index: int = 0) -> BoundaryConfig:
    return BoundaryConfig(
        name=f"stress_b{bits}_boundary{index}", n_samples=256, batch=8, seq=2048,
        hidden=4096, dtype="f32", fwd_bits=bits, fwd_group=4096,
        fwd_rounding=NEAREST, bwd_bits=8, bwd_group=4096, bwd_rounding=NEAREST,
        law="laplace", drift=0.05, epochs=2, outlier_token_frac=0.005,
        outlier_scale=100.0, seed=40 + index)


STRESS_BITS = (2, 4, 8, 2, 4, 8, 2, 4)


def all_configs() -> List[BoundaryConfig]:
    return [tiny(), gpt2_4bit(), gpt2_2bit_stochastic(), deberta_3bit()] + [
        stress(b, i) for i, b in enumerate(STRESS_BITS)]


# --------------------------------------------------------------------------
# dtype helpers (input preparation only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns via torch's CPU conversion (RNE)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def storage_to_f32(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "bf16":
        return bf16_bits_to_f32(x)
    return x.astype(np.float32)


def storage_numpy_dtype(dtype: str):
    return {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype]


def to_torch(x: np.ndarray, dtype: str, device="cpu"):
    """numpy storage array -> torch tensor of the matching torch dtype."""
    import torch
    if dtype == "bf16":
        t = torch.from_numpy(x.view(np.int16)).view(torch.bfloat16)
    else:
        t = torch.from_numpy(x)
    return t.to(device)


def from_torch(t, dtype: str) -> np.ndarray:
    """torch tensor (any device) -> numpy storage array (bf16 as uint16 bits)."""
    import torch
    t = t.detach().cpu().contiguous()
    if dtype == "bf16":
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


# --------------------------------------------------------------------------
# the streams
# --------------------------------------------------------------------------
def _draw(rng: np.random.Generator, law: str, shape) -> np.ndarray:
    if law == "normal":
        return rng.standard_normal(shape, dtype=np.float32)
    if law == "student_t3":
        return rng.standard_t(3.0, shape).astype(np.float32)
    if law == "laplace":
        return rng.laplace(0.0, 1.0, shape).astype(np.float32)
    raise ValueError(law)


@dataclass
class ActivationStream:
    """Stateless, seeded source of activations and gradients for one boundary.

    ``visited`` optionally restricts an epoch to a subset of sample ids (the
    parity tests visit a few dozen rows of a buffer that is allocated at full
    size); it must hold a multiple of ``cfg.batch`` distinct ids.
    """

    cfg: BoundaryConfig
    visited: Sequence[int] | None = None
    _chan: np.ndarray = field(init=False, repr=False)

    def __post_init__(self):
        c = self.cfg
        rng = np.random.default_rng([c.seed, 0xC0FFEE])
        chan = np.ones(c.hidden, dtype=np.float32)
        k = int(round(c.outlier_channel_frac * c.hidden))
        if k > 0:
            chan[rng.choice(c.hidden, size=k, replace=False)] = c.outlier_scale
        self._chan = chan
        ids = np.arange(c.n_samples, dtype=np.int64) if self.visited is None \
            else np.asarray(self.visited, dtype=np.int64)
        if len(ids) % c.batch or len(np.unique(ids)) != len(ids):
            raise ValueError("visited ids must be distinct and fill whole calls")
        if len(ids) and (ids.min() < 0 or ids.max() >= c.n_samples):
            raise ValueError("visited id out of range")
        self._ids = ids

    # -- which samples each call of an epoch touches ------------------------
    def calls_per_epoch(self) -> int:
        return len(self._ids) // self.cfg.batch

    def epoch_ids(self, epoch: int) -> np.ndarray:
        """int64[calls, B]: sample ids of every call of this epoch."""
        c = self.cfg
        ids = self._ids
        if c.shuffle_ids:
            rng = np.random.default_rng([c.seed, 0x1D5, epoch])
            ids = rng.permutation(ids)
        return ids.reshape(-1, c.batch).copy()

    # -- one sample ---------------------------------------------------------
    def _token_scale(self, sample: int) -> np.ndarray | None:
        c = self.cfg
        if c.outlier_token_frac <= 0.0:
            return None
        rng = np.random.default_rng([c.seed, 0x70C, int(sample)])
        tok = np.ones((c.seq, 1), dtype=np.float32)
        k = max(1, int(round(c.outlier_token_frac * c.seq)))
        tok[rng.choice(c.seq, size=k, replace=False)] = c.outlier_scale
        return tok

    def sample_f32(self, sample: int, epoch: int) -> np.ndarray:
        """fp32 pre-image z_t(sample) * channel/token scales, shape [S, H]."""
        c = self.cfg
        z = _draw(np.random.default_rng([c.seed, int(sample), 0]), c.law,
                  (c.seq, c.hidden))
        for tau in range(1, epoch + 1):
            e = _draw(np.random.default_rng([c.seed, int(sample), tau]), c.law,
                      (c.seq, c.hidden))
            z += np.float32(c.drift) * e
        z *= self._chan[None, :]
        tok = self._token_scale(sample)
        if tok is not None:
            z *= tok
        return z

    def activations(self, ids: np.ndarray, epoch: int) -> np.ndarray:
        """Storage-dtype activations [B, S, H] of one call."""
        c = self.cfg
        out = np.empty((len(ids), c.seq, c.hidden), dtype=np.float32)
        for i, s in enumerate(ids):
            out[i] = self.sample_f32(int(s), epoch)
        return to_storage(out, c.dtype)

    def gradients(self, ids: np.ndarray, epoch: int) -> np.ndarray:
        """Storage-dtype backward activation-gradients [B, S, H] of one call."""
        c = self.cfg
        out = np.empty((len(ids), c.seq, c.hidden), dtype=np.float32)
        for i, s in enumerate(ids):
            rng = np.random.default_rng([c.seed, int(s), 0x6AAD, epoch])
            g = _draw(rng, c.law, (c.seq, c.hidden)) * np.float32(c.grad_scale)
            g *= self._chan[None, :]
            out[i] = g
        return to_storage(out, c.dtype)

    def __iter__(self) -> Iterator[Tuple[int, int, np.ndarray, np.ndarray]]:
        """Yield (epoch, call, ids, activations) over the whole stream."""
        for t in range(self.cfg.epochs):
            for k, ids in enumerate(self.epoch_ids(t)):
                yield t, k, ids, self.activations(ids, t)


def call_seed(cfg: BoundaryConfig, epoch: int, call: int, backward: bool = False) -> int:
    """rng_seed handed to the codec for one call (fresh for every message)."""
    base = (cfg.seed + 1) * 0x9E3779B97F4A7C15 & 0xFFFFFFFFFFFFFFFF
    k = (epoch * 1_000_003 + call) * 2 + (1 if backward else 0)
    return (base + k) & 0xFFFFFFFFFFFFFFFF


def parity_ids(cfg: BoundaryConfig, calls: int, seed: int = 7) -> np.ndarray:
    """A small set of distinct sample ids that spans the whole buffer.

    Always holds row 0 and row N-1 (first and last byte of the buffer; for the
    large buffers the last row's offset is far beyond 2^32 elements).
    """
    k = calls * cfg.batch
    if k > cfg.n_samples:
        raise ValueError("more ids requested than samples")
    rng = np.random.default_rng([seed, cfg.seed])
    pool = rng.permutation(np.arange(1, cfg.n_samples - 1, dtype=np.int64))[:max(0, k - 2)]
    ids = np.concatenate([[0], pool, [cfg.n_samples - 1]]).astype(np.int64)[:k]
    return rng.permutation(ids)
