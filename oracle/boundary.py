"""Sender and receiver of one stage boundary on the host, through the oracle.

TEST INFRASTRUCTURE ONLY, like the rest of this package: used by the GPU parity
tests, the smoke check and the CPU-baseline leg of ``bench.py``.  It holds only
the rows of the previous-message buffer that a run visits, so the large
configurations (tens of GB per replica on the device) fit in host memory.

``cfg`` is any object with the fields of a boundary configuration: ``batch``,
``n_per``, ``dtype`` ("f32" | "f16" | "bf16"), ``fwd_bits``, ``fwd_group``,
``fwd_rounding``, ``bwd_bits``, ``bwd_group``, ``bwd_rounding``.
"""
from __future__ import annotations

import numpy as np

import oracle

_NUMPY_OF = {"f32": np.float32, "f16": np.float16, "bf16": np.uint16}


class OracleBoundary:
    """Algorithm 2's two machines, each with its own copy of m (visited rows only)."""

    def __init__(self, cfg, visited: np.ndarray):
        self.cfg = cfg
        self.order = np.sort(np.asarray(visited, dtype=np.int64))
        self.local = {int(s): i for i, s in enumerate(self.order)}
        npdt = _NUMPY_OF[cfg.dtype]
        self.m_send = np.zeros((len(self.order), cfg.n_per), dtype=npdt)
        self.m_recv = np.zeros((len(self.order), cfg.n_per), dtype=npdt)

    def forward(self, act_np: np.ndarray, ids_np: np.ndarray, seed: int):
        """Network a encodes against its copy, network b decodes into its own."""
        c = self.cfg
        loc = np.array([self.local[int(s)] for s in ids_np], dtype=np.int64)
        act = np.ascontiguousarray(act_np.reshape(c.batch, c.n_per))
        codes, scales = oracle.encode(act, loc, self.m_send, dtype=c.dtype, bits=c.fwd_bits,
                                      group=c.fwd_group, rounding=c.fwd_rounding, seed=seed)
        out = oracle.decode(codes, scales, loc, self.m_recv, dtype=c.dtype, bits=c.fwd_bits,
                            group=c.fwd_group)
        return codes, scales, out

    def backward(self, grad_np: np.ndarray, seed: int):
        """The backward message: direct quantisation and its reconstruction."""
        c = self.cfg
        g = np.ascontiguousarray(grad_np.reshape(-1))
        codes, scales = oracle.grad_quant(g, dtype=c.dtype, bits=c.bwd_bits, group=c.bwd_group,
                                          rounding=c.bwd_rounding, seed=seed)
        out = oracle.grad_dequant(codes, scales, dtype=c.dtype, bits=c.bwd_bits, group=c.bwd_group)
        return codes, scales, out
