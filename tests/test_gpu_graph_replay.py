"""The codec calls recorded into a HIP graph (as bench.py does) must give, on every
replay, exactly what the same calls give when launched eagerly: the kernels take
all their state through pointers, use no host-side memset or allocation, and so
replay cleanly.  Eager work and synchronisation sit between the replays."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W


def test_graph_replays_match_eager_launches():
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    B.lib()
    d = torch.device("cuda:0")
    cfg = W.gpt2_2bit_stochastic().scaled(n_samples=24, seq=64)        # stochastic: seeds are baked in too
    stream = W.ActivationStream(cfg)
    steps = 3
    ids_np = stream.epoch_ids(0)[:steps]
    fdesc = [B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=cfg.fwd_bits,
                         group=cfg.fwd_group, dtype=cfg.dtype, rounding=cfg.fwd_rounding, rng_seed=100 + k)
             for k in range(steps)]
    bdesc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, bits=cfg.bwd_bits, group=cfg.bwd_group,
                        dtype=cfg.dtype, rounding=cfg.bwd_rounding, rng_seed=7)

    def fresh():
        st = {"m_send": torch.zeros((cfg.n_samples, cfg.n_per), dtype=torch.float16, device=d),
              "m_recv": torch.zeros((cfg.n_samples, cfg.n_per), dtype=torch.float16, device=d),
              "act": torch.empty((steps, cfg.batch, cfg.n_per), dtype=torch.float16, device=d),
              "grad": torch.empty((steps, cfg.batch, cfg.n_per), dtype=torch.float16, device=d),
              "ids": torch.from_numpy(ids_np.copy()).to(d),
              "codes": torch.zeros((steps, B.codes_bytes(fdesc[0])), dtype=torch.uint8, device=d),
              "scales": torch.zeros((steps, B.scales_count(fdesc[0])), dtype=torch.float32, device=d),
              "out": torch.zeros((steps, cfg.batch, cfg.n_per), dtype=torch.float16, device=d),
              "bcodes": torch.zeros((steps, B.codes_bytes(bdesc)), dtype=torch.uint8, device=d),
              "bscales": torch.zeros((steps, B.scales_count(bdesc)), dtype=torch.float32, device=d),
              "gout": torch.zeros((steps, cfg.batch, cfg.n_per), dtype=torch.float16, device=d)}
        return st

    def launch_all(st):
        for k in range(steps):
            B.encode(fdesc[k], st["act"][k], st["ids"][k], st["m_send"], st["codes"][k], st["scales"][k])
            B.decode(fdesc[k], st["codes"][k], st["scales"][k], st["ids"][k], st["m_recv"], st["out"][k])
            B.grad_quant(bdesc, st["grad"][k], st["bcodes"][k], st["bscales"][k])
            B.grad_dequant(bdesc, st["bcodes"][k], st["bscales"][k], st["gout"][k])

    def load_inputs(st, epoch):
        for k in range(steps):
            a = stream.activations(ids_np[k], epoch).reshape(cfg.batch, cfg.n_per)
            g = stream.gradients(ids_np[k], epoch).reshape(cfg.batch, cfg.n_per)
            st["act"][k].copy_(torch.from_numpy(a))
            st["grad"][k].copy_(torch.from_numpy(g))

    eager, graphed = fresh(), fresh()
    load_inputs(graphed, 0)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        launch_all(graphed)                      # recorded, not run
    torch.cuda.synchronize()
    assert not graphed["m_send"].any()           # capture itself changed nothing

    for epoch in range(4):                       # every replay sees new activations for the same samples
        load_inputs(eager, epoch)
        load_inputs(graphed, epoch)              # eager copies between replays
        torch.cuda.synchronize()
        launch_all(eager)
        g.replay()
        torch.cuda.synchronize()
        for key in ("codes", "scales", "out", "bcodes", "bscales", "gout", "m_send", "m_recv"):
            assert torch.equal(eager[key], graphed[key]), f"replay {epoch}: {key} differs from eager"
        assert torch.equal(graphed["m_send"], graphed["m_recv"])
        assert bool(graphed["scales"].any())
