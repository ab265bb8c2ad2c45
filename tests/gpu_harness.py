"""Shared driver for the GPU parity tests: replays a seeded stream through the
HIP library (sender and receiver buffers on the device) and through the CPU
oracle (compact copies of the visited rows on the host) and compares every
output byte: codes, scales, both copies of m, the receiver's activation, and the
backward message and its reconstruction.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
from oracle.boundary import OracleBoundary
from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W


def dev() -> torch.device:
    return torch.device("cuda:0")


def same_bytes(a: np.ndarray, b: np.ndarray) -> bool:
    return a.shape == b.shape and np.array_equal(a.view(np.uint8), b.view(np.uint8))


def first_diff(a: np.ndarray, b: np.ndarray) -> str:
    a8, b8 = a.reshape(-1).view(np.uint8), b.reshape(-1).view(np.uint8)
    if a8.size != b8.size:
        return f"sizes differ: {a8.size} vs {b8.size} bytes"
    bad = np.nonzero(a8 != b8)[0]
    if bad.size == 0:
        return "identical"
    k = int(bad[0])
    return (f"{bad.size} of {a8.size} bytes differ; first at byte {k}: "
            f"got {a8[k:k + 8].tolist()} want {b8[k:k + 8].tolist()}")


class DeviceBoundary:
    """Sender and receiver state of one boundary on the GPU."""

    def __init__(self, cfg: W.BoundaryConfig, stream: torch.cuda.Stream | None = None):
        self.cfg = cfg
        self.tdtype = B.DTYPE_NAME[cfg.dtype]
        self.stream = stream
        d = dev()
        self.m_send = torch.zeros((cfg.n_samples, cfg.n_per), dtype=self.tdtype, device=d)
        self.m_recv = torch.zeros((cfg.n_samples, cfg.n_per), dtype=self.tdtype, device=d)
        torch.cuda.synchronize()          # the zero fill ran on the default stream

    def desc(self, backward: bool, seed: int) -> B.Desc:
        c = self.cfg
        if backward:
            return B.make_desc(batch=c.batch, n_per=c.n_per, n_samples=c.n_samples, bits=c.bwd_bits,
                               group=c.bwd_group, dtype=c.dtype, rounding=c.bwd_rounding, rng_seed=seed)
        return B.make_desc(batch=c.batch, n_per=c.n_per, n_samples=c.n_samples, bits=c.fwd_bits,
                           group=c.fwd_group, dtype=c.dtype, rounding=c.fwd_rounding, rng_seed=seed)

    def forward(self, act_np: np.ndarray, ids_np: np.ndarray, seed: int):
        """encode on the sender copy, decode on the receiver copy; returns device tensors."""
        c, d = self.cfg, dev()
        with torch.cuda.stream(self.stream) if self.stream is not None else _null():
            desc = self.desc(False, seed)
            act = W.to_torch(act_np.reshape(c.batch, c.n_per), c.dtype, d)
            ids = torch.from_numpy(ids_np).to(d)
            codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
            scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
            out = torch.empty((c.batch, c.n_per), dtype=self.tdtype, device=d)
            B.encode(desc, act, ids, self.m_send, codes, scales)
            B.decode(desc, codes, scales, ids, self.m_recv, out)
        return codes, scales, out, (act, ids)

    def backward(self, grad_np: np.ndarray, seed: int):
        c, d = self.cfg, dev()
        with torch.cuda.stream(self.stream) if self.stream is not None else _null():
            desc = self.desc(True, seed)
            grad = W.to_torch(grad_np.reshape(c.batch, c.n_per), c.dtype, d)
            codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
            scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
            out = torch.empty((c.batch, c.n_per), dtype=self.tdtype, device=d)
            B.grad_quant(desc, grad, codes, scales)
            B.grad_dequant(desc, codes, scales, out)
        return codes, scales, out, (grad,)

    def rows(self, which: str, ids: np.ndarray) -> np.ndarray:
        buf = self.m_send if which == "send" else self.m_recv
        idx = torch.from_numpy(np.asarray(ids, dtype=np.int64)).to(dev())
        return W.from_torch(buf.index_select(0, idx), self.cfg.dtype)


class _null:
    def __enter__(self): return self
    def __exit__(self, *a): return False


def compare_call(tag: str, cfg, got, want) -> None:
    """got: device (codes, scales, out, ...); want: oracle (codes, scales, out)."""
    g_codes = got[0].cpu().numpy()
    g_scales = got[1].cpu().numpy()
    g_out = W.from_torch(got[2], cfg.dtype).reshape(-1)
    assert same_bytes(g_scales, want[1]), f"{tag}: scales: {first_diff(g_scales, want[1])}"
    assert same_bytes(g_codes, want[0]), f"{tag}: codes: {first_diff(g_codes, want[0])}"
    assert same_bytes(g_out, want[2]), f"{tag}: out: {first_diff(g_out, want[2])}"


def replay_and_compare(cfg: W.BoundaryConfig, calls_per_epoch: int, epochs: int | None = None,
                       backward: bool = True, log=print) -> dict:
    """Full parity protocol for one boundary; returns a few statistics."""
    visited = W.parity_ids(cfg, calls_per_epoch)
    stream = W.ActivationStream(cfg, visited=visited)
    gpu = DeviceBoundary(cfg)
    cpu = OracleBoundary(cfg, visited)
    epochs = cfg.epochs if epochs is None else epochs
    stats = {"calls": 0, "mean_scale": []}
    for t in range(epochs):
        for k, ids in enumerate(stream.epoch_ids(t)):
            log(f"[{cfg.name}] epoch {t} call {k} ids {ids.tolist()}", flush=True)
            act = stream.activations(ids, t)
            seed = W.call_seed(cfg, t, k)
            got = gpu.forward(act, ids, seed)
            want = cpu.forward(act, ids, seed)
            torch.cuda.synchronize()
            compare_call(f"{cfg.name} fwd e{t} c{k}", cfg, got, want)
            stats["mean_scale"].append((t, float(want[1].mean())))
            if backward:
                grad = stream.gradients(ids, t)
                bseed = W.call_seed(cfg, t, k, backward=True)
                gotb = gpu.backward(grad, bseed)
                wantb = cpu.backward(grad, bseed)
                torch.cuda.synchronize()
                compare_call(f"{cfg.name} bwd e{t} c{k}", cfg, gotb, wantb)
            stats["calls"] += 1
        # both copies of m, every visited row, after each epoch
        for which, want_m in (("send", cpu.m_send), ("recv", cpu.m_recv)):
            got_m = gpu.rows(which, cpu.order)
            assert same_bytes(got_m, want_m), f"{cfg.name} m_{which} e{t}: {first_diff(got_m, want_m)}"
    # rows nobody visited are still zero (spot check around the visited ones)
    probe = np.setdiff1d(np.clip(np.concatenate([visited + 1, visited - 1]), 0, cfg.n_samples - 1), visited)
    if probe.size:
        assert not gpu.rows("send", probe[:8]).any() and not gpu.rows("recv", probe[:8]).any()
    return stats
