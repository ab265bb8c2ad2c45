"""Parity in the launch configurations that bench.py times: the GPT2-1.5B-shaped
boundary at full size (8192-sample buffers, float16 [4, 1024, 1600] micro-batches),
every stream's part of the steps recorded into a HIP graph of its own with bench.py's own
enqueueing code, and the graphs replayed twice on their streams: the default (one launch
per time slot of the two stages, micro-batches dealt over two streams), the per-stage
launches, and the four single calls on four streams; and the default schedule on the
2-bit stochastic GPT2 boundary and on the DeBERTa-shaped boundary (100,000-sample
bfloat16 buffers), whose slot launches share a workgroup budget.  Every output of every
step, and every visited row of both copies of m, must equal the oracle's after each
replay."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W


CASES = [("gpt2_4bit", "pipeline", 2), ("gpt2_4bit", "stage", 2), ("gpt2_4bit", "calls", 4),
         ("gpt2_4bit", "pipeline", 1), ("gpt2_2bit_stochastic", "pipeline", 2), ("deberta_3bit", "pipeline", 2)]


@pytest.mark.parametrize("config,schedule,n_streams", CASES, ids=[f"{c}-{s}-{n}" for c, s, n in CASES])
def test_graph_at_full_size_matches_the_oracle(config, schedule, n_streams):
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    B.lib()
    import bench
    import gpu_harness as H
    cfg = getattr(W, config)()
    print("bench launches", config, schedule, n_streams, flush=True)
    steps = 8
    wl = bench.Workload(cfg, pool=steps)                 # m starts at zero: replay 1 = first visits
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    graphs = []
    for i, st in enumerate(streams):                     # the enqueueing code of bench.timed_steps
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            bench.stream_part(wl, i, n_streams, 0, steps, schedule)
        graphs.append(g)
    torch.cuda.synchronize()
    assert not bool(wl.m_send[wl.ids[0]].any())          # capture ran nothing

    ids = wl.ids[:steps].cpu().numpy()
    acts = [W.from_torch(wl.act[k], cfg.dtype).reshape(cfg.batch, cfg.n_per) for k in range(steps)]
    grads = [W.from_torch(wl.grad[k], cfg.dtype).reshape(cfg.batch, cfg.n_per) for k in range(steps)]
    cpu = H.OracleBoundary(cfg, ids.reshape(-1))
    for replay in range(2):
        for g, st in zip(graphs, streams):
            with torch.cuda.stream(st):
                g.replay()
        torch.cuda.synchronize()
        for k in range(steps):
            want = cpu.forward(acts[k], ids[k], 0x5EED0000 + 2 * k)    # bench.py's key per message
            H.compare_call(f"replay {replay} step {k} fwd", cfg, (wl.codes[k], wl.scales[k], wl.out[k]), want)
            wantb = cpu.backward(grads[k], 0x5EED0001 + 2 * k)
            H.compare_call(f"replay {replay} step {k} bwd", cfg, (wl.bcodes[k], wl.bscales[k], wl.gout[k]), wantb)
        order = torch.from_numpy(cpu.order).to(wl.dev)
        for name, dev_m, want_m in (("send", wl.m_send, cpu.m_send), ("recv", wl.m_recv, cpu.m_recv)):
            got = W.from_torch(dev_m[order], cfg.dtype).reshape(len(cpu.order), cfg.n_per)
            assert H.same_bytes(got, want_m), f"replay {replay} m_{name}: {H.first_diff(got, want_m)}"
        if replay == 0:
            assert bool(wl.scales[0].any())
