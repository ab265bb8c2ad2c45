"""GPU parity: the HIP library against the CPU oracle, byte for byte.

Bar (integer codes, binary32 scales, stored m and out): bit-exact, 0 ulp.  Both
sides decide every level in binary32 with the same operation order, so there is
no tolerance to state.
"""
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
    B.lib()                                    # fails loudly if the library is not built
    import oracle
    oracle.build()
    import gpu_harness
    return gpu_harness


# ---------------------------------------------------------------------------
# element-by-element sweeps at sizes the oracle finishes in well under a second:
# every dtype x bits x rounding, group sizes that hit every kernel shape
# (sub-wave teams, one wave with 1-4 chunks per lane, multi-wave teams, the
# any-shape fallback), group counts that leave ragged tails in every tiling.
# ---------------------------------------------------------------------------
GROUPS = [8, 24, 64, 128, 200, 256, 520, 1000, 1536, 1600, 2048, 4096, 8200, 16384, 32768]
ODD_GROUPS = {2: [4, 12, 20], 3: [], 4: [2, 6, 100], 6: [4, 12, 100], 8: [1, 3, 7, 50]}     # not multiples of 8
HUGE_GROUPS = [40000]                                                       # beyond a workgroup


def _case_cfg(dtype, bits, group, rounding, groups_per_sample, batch=3, n_samples=7):
    return W.BoundaryConfig(
        name=f"sweep_{dtype}_b{bits}_g{group}_r{rounding}", n_samples=n_samples, batch=batch,
        seq=groups_per_sample, hidden=group, dtype=dtype, fwd_bits=bits, fwd_group=group,
        fwd_rounding=rounding, bwd_bits=bits, bwd_group=group, bwd_rounding=rounding,
        law="normal", drift=0.05, epochs=2, shuffle_ids=True, seed=1000 + bits * 7 + group)


def _sweep(H, dtype, bits, group, rounding, gps):
    cfg = _case_cfg(dtype, bits, group, rounding, gps)
    quiet = lambda *a, **k: None
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=2, log=quiet)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_sweep_group_sizes_nearest(H, dtype, bits):
    for group in GROUPS:
        gps = 37 if group <= 2048 else 5
        print(f"sweep {dtype} b{bits} G{group} nearest", flush=True)
        _sweep(H, dtype, bits, group, W.NEAREST, gps)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 3, 4, 6, 8])
def test_sweep_group_sizes_stochastic(H, dtype, bits):
    for group in [8, 64, 128, 1600, 4096, 8200]:
        gps = 37 if group <= 2048 else 5
        print(f"sweep {dtype} b{bits} G{group} stochastic", flush=True)
        _sweep(H, dtype, bits, group, W.STOCHASTIC, gps)


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_sweep_any_shape_fallback(H, dtype):
    for bits, groups in ODD_GROUPS.items():
        for group in groups:
            for rounding in (W.NEAREST, W.STOCHASTIC):
                print(f"fallback {dtype} b{bits} G{group} r{rounding}", flush=True)
                _sweep(H, dtype, bits, group, rounding, 8 * 131)
    for group in HUGE_GROUPS:
        print(f"fallback {dtype} b4 G{group}", flush=True)
        _sweep(H, dtype, 4, group, W.NEAREST, 3)


def test_long_samples_cross_block_strides(H):
    """Many groups per sample so the grid-stride loops and gridDim.y both turn over."""
    cfg = _case_cfg("f16", 4, 64, W.NEAREST, groups_per_sample=5000, batch=5, n_samples=11)
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=2, log=lambda *a, **k: None)
    cfg = _case_cfg("bf16", 3, 1600, W.STOCHASTIC, groups_per_sample=1030, batch=2, n_samples=5)
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=2, log=lambda *a, **k: None)


def test_more_samples_in_a_call_than_grid_rows(H):
    """70001 samples in one call: the launch has at most 65535 rows of workgroups, so
    the kernels' loop over samples must come round a second time."""
    quiet = lambda *a, **k: None
    cfg = _case_cfg("f16", 4, 64, W.NEAREST, groups_per_sample=2, batch=70001, n_samples=70010)
    H.replay_and_compare(cfg, calls_per_epoch=1, epochs=2, log=quiet)
    cfg = _case_cfg("f32", 8, 12, W.STOCHASTIC, groups_per_sample=1, batch=66000, n_samples=66000)   # any-shape kernels
    H.replay_and_compare(cfg, calls_per_epoch=1, epochs=2, log=quiet)


# ---------------------------------------------------------------------------
# edge cases
# ---------------------------------------------------------------------------
def test_empty_call_touches_nothing(H):
    d = H.dev()
    m = torch.ones((4, 256), dtype=torch.float16, device=d)
    desc = B.make_desc(batch=0, n_per=256, n_samples=4, bits=4, group=64, dtype="f16")
    e = torch.empty(0, dtype=torch.uint8, device=d)
    B.encode(desc, torch.empty((0, 256), dtype=torch.float16, device=d),
             torch.empty(0, dtype=torch.int64, device=d), m, e, torch.empty(0, device=d))
    torch.cuda.synchronize()
    assert bool((m == 1).all())


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_unchanged_activation_sends_zero_scale(H, dtype):
    import oracle
    d = H.dev()
    rng = np.random.default_rng(3)
    m_np = W.to_storage(rng.standard_normal((6, 1024)).astype(np.float32), dtype)
    ids_np = np.array([5, 0, 3], dtype=np.int64)
    act_np = np.ascontiguousarray(m_np[ids_np])
    # one group of the second sample does change, its neighbours do not
    tweak = W.storage_to_f32(act_np, dtype)
    tweak[1, 128:192] += 0.25
    act_np = W.to_storage(tweak, dtype)
    for bits in (2, 3, 4, 6, 8):
        m = W.to_torch(m_np.copy(), dtype, d)
        desc = B.make_desc(batch=3, n_per=1024, n_samples=6, bits=bits, group=64, dtype=dtype)
        codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
        scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
        B.encode(desc, W.to_torch(act_np, dtype, d), torch.from_numpy(ids_np).to(d), m, codes, scales)
        m_host = m_np.copy()
        wc, ws = oracle.encode(act_np, ids_np, m_host, dtype=dtype, bits=bits, group=64)
        torch.cuda.synchronize()
        assert H.same_bytes(codes.cpu().numpy(), wc) and H.same_bytes(scales.cpu().numpy(), ws)
        assert H.same_bytes(W.from_torch(m, dtype), m_host)
        assert int((scales == 0).sum()) == 3 * 16 - 1


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_tiny_magnitudes_keep_binary32_subnormals(H, bits):
    """Groups whose max-abs sits around the 2^-120 floor: some are sent as zero,
    the others have a level spacing that is a binary32 subnormal.  Nothing may be
    flushed to zero on the way."""
    import oracle
    d = H.dev()
    rng = np.random.default_rng(40 + bits)
    n_per, G, N = 64 * 96, 64, 5
    mag = np.repeat(10.0 ** rng.uniform(-37.5, -35.0, size=(3, n_per // G)), G, axis=1)
    act_np = (rng.standard_normal((3, n_per)) * mag).astype(np.float32)
    m_np = np.zeros((N, n_per), dtype=np.float32)
    ids_np = np.array([4, 1, 2], dtype=np.int64)
    m_send = torch.zeros((N, n_per), device=d)
    m_recv = torch.zeros((N, n_per), device=d)
    desc = B.make_desc(batch=3, n_per=n_per, n_samples=N, bits=bits, group=G, dtype="f32")
    codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
    scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
    out = torch.empty((3, n_per), device=d)
    ids = torch.from_numpy(ids_np).to(d)
    for visit in range(2):
        a = (act_np * np.float32(1.0 + 0.25 * visit)).astype(np.float32)
        B.encode(desc, torch.from_numpy(a).to(d), ids, m_send, codes, scales)
        B.decode(desc, codes, scales, ids, m_recv, out)
        wc, ws = oracle.encode(a, ids_np, m_np, dtype="f32", bits=bits, group=G)
        torch.cuda.synchronize()
        assert H.same_bytes(scales.cpu().numpy(), ws), H.first_diff(scales.cpu().numpy(), ws)
        assert H.same_bytes(codes.cpu().numpy(), wc), H.first_diff(codes.cpu().numpy(), wc)
        assert H.same_bytes(m_send.cpu().numpy(), m_np)
        assert H.same_bytes(m_recv.cpu().numpy(), m_np)
        assert H.same_bytes(out.cpu().numpy(), m_np[ids_np])
        if visit == 0:
            live = ws > 0
            assert (~live).any() and live.any()
            sub = (np.abs(a.reshape(-1, G)) < 2.0**-126) & (a.reshape(-1, G) != 0) & live[:, None]
            assert sub.any()                                   # subnormal inputs in live groups
            if bits == 8:                                      # and subnormal level spacings
                assert (ws[live] / 127.5 < 2.0**-126).any()


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("n_per", [4096, 1001, 24])        # 16-byte rows and ragged rows
def test_seed_then_encode_follows_algorithm_1(H, dtype, n_per):
    """Uncompressed first visit on both sides, then a compressed second visit."""
    import oracle
    d = H.dev()
    rng = np.random.default_rng(7 + n_per)
    N, Bn = 9, 4
    ids_np = np.array([8, 0, 3, 5], dtype=np.int64)
    a0 = W.to_storage(rng.standard_normal((Bn, n_per)).astype(np.float32), dtype)
    a1 = W.to_storage(W.storage_to_f32(a0, dtype) + 0.05 * rng.standard_normal((Bn, n_per)).astype(np.float32), dtype)
    m_host = W.to_storage(rng.standard_normal((N, n_per)).astype(np.float32), dtype)   # stale contents
    m_send = W.to_torch(m_host.copy(), dtype, d)
    m_recv = W.to_torch(m_host.copy(), dtype, d)
    ids = torch.from_numpy(ids_np).to(d)
    desc = B.make_desc(batch=Bn, n_per=n_per, n_samples=N, bits=8, group=1, dtype=dtype)
    B.seed(desc, W.to_torch(a0, dtype, d), ids, m_send)
    B.seed(desc, W.to_torch(a0, dtype, d), ids, m_recv)
    oracle.seed(a0, ids_np, m_host, dtype=dtype)
    torch.cuda.synchronize()
    assert H.same_bytes(W.from_torch(m_send, dtype), m_host)
    assert H.same_bytes(W.from_torch(m_recv, dtype), m_host)
    # second visit through the codec
    codes = torch.empty(B.codes_bytes(desc), dtype=torch.uint8, device=d)
    scales = torch.empty(B.scales_count(desc), dtype=torch.float32, device=d)
    out = torch.empty((Bn, n_per), dtype=B.DTYPE_NAME[dtype], device=d)
    B.encode(desc, W.to_torch(a1, dtype, d), ids, m_send, codes, scales)
    B.decode(desc, codes, scales, ids, m_recv, out)
    wc, ws = oracle.encode(a1, ids_np, m_host, dtype=dtype, bits=8, group=1)
    torch.cuda.synchronize()
    assert H.same_bytes(codes.cpu().numpy(), wc) and H.same_bytes(scales.cpu().numpy(), ws)
    assert H.same_bytes(W.from_torch(m_send, dtype), m_host)
    assert H.same_bytes(W.from_torch(m_recv, dtype), m_host)
    assert H.same_bytes(W.from_torch(out, dtype), m_host[ids_np])


def test_check_ids_flags_duplicates_and_range(H):
    d = H.dev()
    for ids, want in [([0, 1, 2, 3], 0), ([0, 9, 2, 3], 1), ([0, 2, 2, 3], 2), ([-1, 5, 5, 1], 3)]:
        flag = torch.zeros(1, dtype=torch.int32, device=d)
        B.check_ids(torch.tensor(ids, dtype=torch.int64, device=d), 8, flag)
        assert int(flag.item()) == want


def test_non_default_stream_and_reuse_of_buffers(H):
    """The call uses the stream it is given; outputs land in caller memory."""
    cfg = _case_cfg("f16", 4, 1600, W.NEAREST, groups_per_sample=64)
    s = torch.cuda.Stream()
    visited = W.parity_ids(cfg, 1)
    stream = W.ActivationStream(cfg, visited=visited)
    gpu = H.DeviceBoundary(cfg, stream=s)
    cpu = H.OracleBoundary(cfg, visited)
    ids = stream.epoch_ids(0)[0]
    act = stream.activations(ids, 0)
    got = gpu.forward(act, ids, 0)
    want = cpu.forward(act, ids, 0)
    s.synchronize()
    H.compare_call("side stream", cfg, got, want)


# ---------------------------------------------------------------------------
# the five workload configurations at their full per-call shapes, with the
# buffers allocated at full size (row offsets far beyond 2^32 elements) and a
# few dozen rows visited, first and last row included.
# ---------------------------------------------------------------------------
def test_config1_tiny_whole_stream(H):
    cfg = W.tiny()
    stats = H.replay_and_compare(cfg, calls_per_epoch=cfg.n_samples // cfg.batch)
    assert stats["calls"] == 16 * 3
    s0 = np.mean([s for t, s in stats["mean_scale"] if t == 0])
    s2 = np.mean([s for t, s in stats["mean_scale"] if t == 2])
    assert s2 < s0 / 10          # deltas, not activations, are what later epochs send


def test_config2_gpt2_4bit_full_shape(H):
    cfg = W.gpt2_4bit()
    assert cfg.n_samples * cfg.n_per > 2**32
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=2)


def test_config3_gpt2_2bit_stochastic_full_shape(H):
    cfg = W.gpt2_2bit_stochastic()
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=4)


def test_config4_deberta_3bit_full_shape(H):
    cfg = W.deberta_3bit()
    assert cfg.n_samples * cfg.n_per * 2 > 78e9
    H.replay_and_compare(cfg, calls_per_epoch=2, epochs=2)


def test_config5_stress_eight_boundaries_on_streams(H):
    """Eight independent boundaries (own buffers, own stream, 2/4/8-bit mix) run
    concurrently; each must match the oracle, which runs them one after another."""
    cfgs = [W.stress(b, i) for i, b in enumerate(W.STRESS_BITS)]
    base = cfgs[0]
    visited = W.parity_ids(base, 1)
    src = W.ActivationStream(base, visited=visited)
    streams = [torch.cuda.Stream() for _ in cfgs]
    gpus = [H.DeviceBoundary(c, stream=s) for c, s in zip(cfgs, streams)]
    cpus = [H.OracleBoundary(c, visited) for c in cfgs]
    for t in range(2):
        ids = src.epoch_ids(t)[0]
        act = src.activations(ids, t)                 # the same input feeds every boundary
        print(f"[stress] epoch {t}: launching 8 boundaries", flush=True)
        torch.cuda.synchronize()
        got = [g.forward(act, ids, 0) for g in gpus]  # enqueue all eight before any sync
        torch.cuda.synchronize()
        for i, (c, cpu) in enumerate(zip(cfgs, cpus)):
            want = cpu.forward(act, ids, 0)
            H.compare_call(f"{c.name} e{t}", c, got[i], want)
            for which, want_m in (("send", cpu.m_send), ("recv", cpu.m_recv)):
                assert H.same_bytes(gpus[i].rows(which, cpu.order), want_m)
            print(f"[stress] epoch {t} boundary {i} b{c.fwd_bits} ok", flush=True)
        got = None
    grad = src.gradients(src.epoch_ids(0)[0], 0)
    gotb = gpus[2].backward(grad, 0)
    torch.cuda.synchronize()
    H.compare_call("stress bwd", cfgs[2], gotb, cpus[2].backward(grad, 0))
