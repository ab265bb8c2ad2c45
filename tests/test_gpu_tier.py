"""GPU test of the tiers below HBM for the previous messages (Section 3.3 and Appendix G
of the paper: m(xi) in host memory or on an SSD, prefetched before its sample's forward
pass and written back after the update).  The codec must produce the same bytes whether
m lives in one big HBM array or is paged through a few HBM windows from pinned host
memory or from a file."""
import time

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W


@pytest.fixture(scope="module")
def H():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the MI355X; run them with -m gpu on the GPU box")
    B.lib()
    import oracle
    oracle.build()
    import gpu_harness
    return gpu_harness


def _tier(cfg, slots, d, path=None, direct_io=False):
    """Host tier, or (with a path) the file tier with its rows in that file."""
    td = B.DTYPE_NAME[cfg.dtype]
    dev = torch.zeros((slots * cfg.batch, cfg.n_per), dtype=td, device=d)
    row_ids = torch.empty(slots * cfg.batch, dtype=torch.int64, device=d)
    if path is None:
        host = torch.zeros((cfg.n_samples, cfg.n_per), dtype=td).pin_memory()
        return B.Tier(host, dev, row_ids, slots, cfg.batch)
    staging = torch.zeros((slots * cfg.batch, cfg.n_per), dtype=td).pin_memory()
    return B.Tier(staging, dev, row_ids, slots, cfg.batch, path=str(path), n_samples=cfg.n_samples,
                  direct_io=direct_io)


def _file_rows(path, cfg):
    return np.fromfile(str(path), dtype=np.float16).reshape(cfg.n_samples, cfg.n_per)


@pytest.mark.parametrize("kind", ["host", "file", "file_direct"])
def test_tiered_m_gives_the_same_bytes_as_resident_m(H, kind, tmp_path):
    import oracle
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(name="tier", n_samples=48, seq=96, epochs=3, shuffle_ids=True)
    slots = 3
    stream = W.ActivationStream(cfg)
    path = None if kind == "host" else tmp_path / "m_rows.bin"
    try:
        tier = _tier(cfg, slots, d, path, direct_io=kind == "file_direct")
    except B.AqsgdError as e:
        if kind == "file_direct" and e.status == -8:
            pytest.skip("this file system refuses unbuffered (O_DIRECT) files")
        raise
    resident = torch.zeros((cfg.n_samples, cfg.n_per), dtype=torch.float16, device=d)
    m_host = np.zeros((cfg.n_samples, cfg.n_per), dtype=np.float16)       # the oracle's m
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    win_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=slots * cfg.batch, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    res_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    calls = [(t, k, ids) for t in range(cfg.epochs) for k, ids in enumerate(stream.epoch_ids(t))]
    keep = []
    tier.prefetch(0, torch.from_numpy(calls[0][2].copy()), copy)
    for n, (t, k, ids) in enumerate(calls):
        slot = n % slots
        nxt = calls[n + 1][2] if n + 1 < len(calls) else None
        # The next micro-batch's rows travel while this one computes, unless the two share a
        # sample (possible across an epoch boundary): then its row must be written back first.
        early = nxt is not None and not (set(nxt.tolist()) & set(ids.tolist()))
        if early:
            tier.prefetch((n + 1) % slots, torch.from_numpy(nxt.copy()), copy)
        act_np = stream.activations(ids, t).reshape(cfg.batch, cfg.n_per)
        with torch.cuda.stream(compute):
            act = W.to_torch(act_np, "f16", d)
            codes = torch.empty(B.codes_bytes(win_desc), dtype=torch.uint8, device=d)
            scales = torch.empty(B.scales_count(win_desc), dtype=torch.float32, device=d)
            win_ids = tier.acquire(slot, compute)
            B.encode(win_desc, act, win_ids, tier.dev_rows, codes, scales, stream=compute)
            tier.release(slot, compute, copy)
            if nxt is not None and not early:
                tier.prefetch((n + 1) % slots, torch.from_numpy(nxt.copy()), copy)
            # the same call against the resident array
            codes2 = torch.empty_like(codes)
            scales2 = torch.empty_like(scales)
            B.encode(res_desc, act, torch.from_numpy(ids).to(d), resident, codes2, scales2, stream=compute)
        wc, ws = oracle.encode(act_np, ids, m_host, dtype="f16", bits=4, group=cfg.fwd_group)
        keep.append((codes, scales, codes2, scales2, wc, ws, act))
    tier.drain()
    torch.cuda.synchronize()
    for n, (codes, scales, codes2, scales2, wc, ws, _) in enumerate(keep):
        assert H.same_bytes(codes.cpu().numpy(), wc), f"call {n}: tiered codes differ from the oracle"
        assert H.same_bytes(scales.cpu().numpy(), ws), f"call {n}: tiered scales differ from the oracle"
        assert torch.equal(codes, codes2) and torch.equal(scales, scales2)
    assert H.same_bytes(resident.cpu().numpy(), m_host)
    if path is None:
        assert H.same_bytes(tier.host_rows.numpy(), m_host)               # host tier is current
        tier.close()
    else:
        tier.close()
        assert H.same_bytes(_file_rows(path, cfg), m_host)                # and so is the file


def test_tier_protocol_errors(H):
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=16, seq=8)
    tier = _tier(cfg, 2, d)
    s = torch.cuda.Stream()
    ids = torch.tensor([3, 1, 0, 7], dtype=torch.int64)
    with pytest.raises(B.AqsgdError) as e:
        tier.acquire(0, s)                          # nothing prefetched
    assert e.value.status == -5
    tier.prefetch(0, ids, s)
    with pytest.raises(B.AqsgdError):
        tier.prefetch(0, ids, s)                    # window not released
    with pytest.raises(B.AqsgdError):
        tier.prefetch(1, torch.tensor([3, 1, 0, 16], dtype=torch.int64), s)   # id out of range
    with pytest.raises(B.AqsgdError):
        tier.prefetch(1, torch.tensor([9, 8, 7, 6], dtype=torch.int64), s)    # sample 7 sits in window 0
    with pytest.raises(B.AqsgdError):
        tier.prefetch(1, torch.tensor([9, 8, 9, 6], dtype=torch.int64), s)    # twice in one call
    with pytest.raises(B.AqsgdError):
        tier.release(1, s, s)                       # empty window
    assert list(tier.acquire(0, s).cpu().numpy()) == [0, 1, 2, 3]
    tier.release(0, s, s)
    tier.prefetch(0, ids, s)                        # released: may be filled again
    tier.release(0, s, s)
    tier.drain()
    tier.close()


def test_tier_traffic_hides_behind_compute(H, capsys):
    """Section 3.3's claim, on this machine: with the next micro-batch's rows prefetched
    and the previous one's written back on a copy stream, a stage that computes between
    codec calls runs as fast as with the whole m resident in HBM.  The stand-in for the
    stage's forward pass is ~3 ms of elementwise work per micro-batch (the paper's budget
    is 44 ms, so this is the harder case)."""
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=64)
    slots, calls = 3, 32
    rng = np.random.default_rng(3)
    sweep = rng.permutation(cfg.n_samples).reshape(-1, cfg.batch)               # 16 disjoint micro-batches
    ids_all = np.concatenate([sweep, sweep])[:calls]                            # neighbours never share a sample
    act = torch.randn((cfg.batch, cfg.n_per), device=d).to(torch.float16)
    work = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=d)          # 256 MB
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    win_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=slots * cfg.batch, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    res_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    codes = torch.empty(B.codes_bytes(win_desc), dtype=torch.uint8, device=d)
    scales = torch.empty(B.scales_count(win_desc), dtype=torch.float32, device=d)

    def stage_compute():
        for _ in range(24):
            work.mul_(1.0000001)

    def run_resident():
        m = torch.zeros((cfg.n_samples, cfg.n_per), dtype=torch.float16, device=d)
        dev_ids = [torch.from_numpy(i.copy()).to(d) for i in ids_all]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        with torch.cuda.stream(compute):
            for n in range(calls):
                stage_compute()
                B.encode(res_desc, act, dev_ids[n], m, codes, scales, stream=compute)
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    def run_tiered():
        tier = _tier(cfg, slots, d)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        tier.prefetch(0, torch.from_numpy(ids_all[0].copy()), copy)
        with torch.cuda.stream(compute):
            for n in range(calls):
                if n + 1 < calls:
                    tier.prefetch((n + 1) % slots, torch.from_numpy(ids_all[n + 1].copy()), copy)
                stage_compute()
                win_ids = tier.acquire(n % slots, compute)
                B.encode(win_desc, act, win_ids, tier.dev_rows, codes, scales, stream=compute)
                tier.release(n % slots, compute, copy)
        tier.drain()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        tier.close()
        return dt

    run_resident(); run_tiered()                                                 # warm-up
    t_res = min(run_resident() for _ in range(3))
    t_tier = min(run_tiered() for _ in range(3))
    with capsys.disabled():
        print(f"\n[tier] {calls} micro-batches with {t_res / calls * 1e3:.2f} ms of stage compute each: "
              f"resident m {t_res * 1e3:.1f} ms, host-tiered m {t_tier * 1e3:.1f} ms "
              f"({t_tier / t_res:.3f}x)")
    assert t_tier < 1.25 * t_res


def test_file_tier_hides_behind_the_papers_compute_budget(H, capsys, tmp_path):
    """Appendix G keeps m on an SSD: loading a micro-batch's rows takes 12 ms there against
    44 ms of forward compute.  Here the rows of the GPT2 shape (4 x 3.28 MB per micro-batch)
    come from a file on this machine's disk through the read-ahead worker and go back
    through the write-behind, with a stand-in of about 11 ms of stage compute per
    micro-batch (a quarter of the paper's budget); the run must take about as long as with
    m resident in HBM."""
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=64)
    slots, calls = 3, 24
    rng = np.random.default_rng(4)
    sweep = rng.permutation(cfg.n_samples).reshape(-1, cfg.batch)
    ids_all = np.concatenate([sweep, sweep])[:calls]
    act = torch.randn((cfg.batch, cfg.n_per), device=d).to(torch.float16)
    work = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=d)
    compute, copy = torch.cuda.Stream(), torch.cuda.Stream()
    win_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=slots * cfg.batch, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    res_desc = B.make_desc(batch=cfg.batch, n_per=cfg.n_per, n_samples=cfg.n_samples, bits=4,
                           group=cfg.fwd_group, dtype="f16")
    codes = torch.empty(B.codes_bytes(win_desc), dtype=torch.uint8, device=d)
    scales = torch.empty(B.scales_count(win_desc), dtype=torch.float32, device=d)

    def stage_compute():
        for _ in range(150):
            work.mul_(1.0000001)

    def run(tier):
        dev_ids = [torch.from_numpy(i.copy()).to(d) for i in ids_all]
        m = torch.zeros((cfg.n_samples, cfg.n_per), dtype=torch.float16, device=d) if tier is None else None
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        if tier is not None:
            tier.prefetch(0, torch.from_numpy(ids_all[0].copy()), copy)
            tier.prefetch(1, torch.from_numpy(ids_all[1].copy()), copy)
        with torch.cuda.stream(compute):
            for n in range(calls):
                if tier is None:
                    stage_compute()
                    B.encode(res_desc, act, dev_ids[n], m, codes, scales, stream=compute)
                    continue
                stage_compute()
                win_ids = tier.acquire(n % slots, compute)
                B.encode(win_desc, act, win_ids, tier.dev_rows, codes, scales, stream=compute)
                tier.release(n % slots, compute, copy)
                if n + 2 < calls:                        # read two micro-batches ahead
                    tier.prefetch((n + 2) % slots, torch.from_numpy(ids_all[n + 2].copy()), copy)
        if tier is not None:
            tier.drain()
        torch.cuda.synchronize()
        return time.perf_counter() - t0

    run(None)
    t_res = min(run(None) for _ in range(2))
    results = {}
    for kind in ("file_direct", "file"):
        try:
            tier = _tier(cfg, slots, d, tmp_path / f"rows_{kind}.bin", direct_io=kind == "file_direct")
        except B.AqsgdError as e:
            if e.status == -8:
                continue
            raise
        run(tier)
        results[kind] = min(run(tier) for _ in range(2))
        tier.close()
    assert "file" in results
    with capsys.disabled():
        msg = ", ".join(f"{k} {v * 1e3:.1f} ms ({v / t_res:.3f}x)" for k, v in results.items())
        print(f"\n[tier] {calls} micro-batches with {t_res / calls * 1e3:.1f} ms of stage compute each: "
              f"resident m {t_res * 1e3:.1f} ms; rows from a file: {msg}")
    assert min(results.values()) < 1.25 * t_res


def test_file_tier_reports_a_file_it_cannot_open(H):
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=16, seq=8)
    with pytest.raises(B.AqsgdError) as e:
        _tier(cfg, 2, d, "/nonexistent_dir/rows.bin")
    assert e.value.status == -8
    with pytest.raises(B.AqsgdError) as e:             # rows of 25600 bytes are not whole 4 KiB blocks
        _tier(cfg, 2, d, "/tmp/aqsgd_never_made.bin", direct_io=True)
    assert e.value.status == -6


def test_tier_refuses_a_second_copy_stream(H):
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=16, seq=8)
    tier = _tier(cfg, 2, d)
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    tier.prefetch(0, torch.tensor([3, 1, 0, 7], dtype=torch.int64), s1)
    with pytest.raises(B.AqsgdError) as e:
        tier.prefetch(1, torch.tensor([4, 5, 6, 8], dtype=torch.int64), s2)
    assert e.value.status == -5
    tier.acquire(0, s1)
    with pytest.raises(B.AqsgdError):
        tier.release(0, s1, s2)
    tier.release(0, s1, s1)
    tier.drain()
    tier.close()


def test_tier_copy_rate_against_the_papers_budget(H, capsys):
    """The paper hides 0.2 ms of loading per micro-batch behind 44 ms of forward
    compute.  Here: rows of the GPT2 shape (3.2 MB each, 4 per micro-batch) in and
    out over the host link; the round trip must be far below that budget."""
    d = H.dev()
    cfg = W.gpt2_4bit().scaled(n_samples=256)
    slots = 4
    tier = _tier(cfg, slots, d)
    copy = torch.cuda.Stream()
    rng = np.random.default_rng(0)
    perm = rng.permutation(cfg.n_samples).reshape(-1, cfg.batch)
    torch.cuda.synchronize()
    reps = len(perm)
    t0 = time.perf_counter()
    for n in range(reps):
        slot = n % slots
        tier.prefetch(slot, torch.from_numpy(perm[n].copy()), copy)
        tier.acquire(slot, copy)
        tier.release(slot, copy, copy)
    tier.drain()
    dt = (time.perf_counter() - t0) / reps
    moved = 2 * cfg.batch * cfg.n_per * 2
    with capsys.disabled():
        print(f"\n[tier] {cfg.batch} rows x {cfg.n_per * 2 / 1e6:.2f} MB in and out: {dt * 1e3:.3f} ms per "
              f"micro-batch, {moved / dt / 1e9:.1f} GB/s over the host link")
    assert dt < 5e-3            # << 44 ms of forward compute per micro-batch in the paper's setting
    tier.close()
