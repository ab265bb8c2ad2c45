"""GPU parity of the sparsified backward message (Appendix H.6 of the paper: the
largest fifth of the gradient entries, at 8 bits) against the CPU oracle, byte for
byte: bitmap, levels, scales and the reconstruction."""
import ctypes

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


def _gradient(n, seed, dtype, kind):
    rng = np.random.default_rng(seed)
    if kind == "heavy":                               # small noise, a few large entries
        g = rng.standard_normal(n).astype(np.float32) * 1e-3
        hot = rng.choice(n, size=max(1, n // 50), replace=False)
        g[hot] *= 40.0
    elif kind == "ties":                              # few distinct magnitudes: the threshold is always tied
        g = rng.integers(-3, 4, size=n).astype(np.float32) * 0.25
    elif kind == "sparse":                            # mostly exact zeros, some groups entirely zero
        g = rng.standard_normal(n).astype(np.float32)
        g[rng.random(n) < 0.9] = 0.0
        g[: n // 4] = 0.0
        g[::7] *= -1.0                                # some of the zeros are negative zeros
    elif kind == "edge":                              # one kind of degenerate group after the other
        big = {"f16": 65504.0, "bf16": 3.3895e38, "f32": 3.4028e38}[dtype]
        tiny = {"f16": 2.0 ** -24, "bf16": 2.0 ** -133, "f32": 2.0 ** -149}[dtype]
        g = np.zeros(n, dtype=np.float64)
        G = n // 8
        j = np.arange(G)
        g[0 * G:1 * G] = 0.75                                        # every magnitude equal
        g[1 * G:2 * G] = np.where(j % 2 == 0, 0.75, -0.75)           # ... with mixed signs
        g[2 * G + G // 3] = -1e-3                                    # a single non-zero entry
        g[3 * G:4 * G] = 1.0 + (j % 97) * 2.0 ** -7                  # one leading byte, close low bits
        g[4 * G:5 * G] = np.where(j % 3 == 0, big, -big / 2)         # the largest finite values
        g[5 * G:6 * G] = (j % 50) * tiny                             # subnormal magnitudes and zeros
        g[6 * G:7 * G] = (G - j) * 1e-2                              # descending
        g[7 * G:8 * G] = -(j + 1) * 1e-2                             # ascending magnitudes, negative
        g = g.astype(np.float32)
    else:
        raise ValueError(kind)
    return W.to_storage(g, dtype)


def _run(H, dtype, group, keep, n_groups, kind, rounding=0, seed=1, batch=1):
    import oracle
    d = H.dev()
    n = group * n_groups
    assert n % batch == 0 and (n // batch) % group == 0
    g_np = _gradient(n, seed + group, dtype, kind)
    desc = B.make_desc(batch=batch, n_per=n // batch, bits=8, group=group, dtype=dtype, rounding=rounding,
                       rng_seed=seed)
    assert B.topk_bitmap_bytes(desc) == n // 8 and B.topk_codes_bytes(desc, keep) == n_groups * keep
    grad = W.to_torch(g_np, dtype, d)
    bitmap = torch.full((n // 8,), 0xAA, dtype=torch.uint8, device=d)
    codes = torch.full((n_groups * keep,), 0xCC, dtype=torch.uint8, device=d)
    scales = torch.full((n_groups,), -1.0, dtype=torch.float32, device=d)
    out = W.to_torch(W.to_storage(np.full(n, 7.0, dtype=np.float32), dtype), dtype, d)
    B.grad_topk_quant(desc, keep, grad, bitmap, codes, scales)
    B.grad_topk_dequant(desc, keep, bitmap, codes, scales, out)
    torch.cuda.synchronize()
    wb, wc, ws = oracle.grad_topk_quant(g_np, dtype=dtype, bits=8, group=group, keep=keep, rounding=rounding,
                                        seed=seed)
    wo = oracle.grad_topk_dequant(wb, wc, ws, dtype=dtype, bits=8, group=group, keep=keep)
    tag = f"{dtype} G={group} keep={keep} groups={n_groups} {kind} rounding={rounding}"
    assert H.same_bytes(bitmap.cpu().numpy(), wb), f"{tag}: bitmap: {H.first_diff(bitmap.cpu().numpy(), wb)}"
    assert H.same_bytes(scales.cpu().numpy(), ws), f"{tag}: scales: {H.first_diff(scales.cpu().numpy(), ws)}"
    assert H.same_bytes(codes.cpu().numpy(), wc), f"{tag}: codes: {H.first_diff(codes.cpu().numpy(), wc)}"
    got = W.from_torch(out, dtype)
    assert H.same_bytes(got, wo), f"{tag}: out: {H.first_diff(got, wo)}"


SHAPES = [(8, 1), (8, 8), (64, 13), (128, 26), (512, 112), (520, 104), (1024, 208), (1600, 320), (2048, 411),
          (1600, 1), (1600, 1599), (1600, 1600), (2048, 1), (2048, 2048),    # nothing but the largest; (nearly) everything
          (1544, 7), (1560, 300), (576, 100), (1592, 1591),                  # a last round of 1, 3, 8 and 7 chunks
          (1536, 307), (1088, 217)]                                          # three rounds; two rounds and eight chunks


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
@pytest.mark.parametrize("group,keep", SHAPES)
def test_topk_matches_oracle(H, dtype, group, keep):
    for kind in ("heavy", "ties", "sparse"):
        _run(H, dtype, group, keep, n_groups=13, kind=kind)


@pytest.mark.parametrize("dtype", ["f16", "bf16", "f32"])
def test_topk_degenerate_groups(H, dtype):
    """Eight groups, each degenerate in its own way (all equal, a single entry, one leading
    byte, the largest finite values, subnormals, sorted either way)."""
    for group, keep in ((1600, 320), (64, 13), (2048, 1), (512, 511)):
        _run(H, dtype, group, keep, n_groups=8, kind="edge")


@pytest.mark.parametrize("dtype", ["f16", "f32"])
def test_topk_stochastic_rounding(H, dtype):
    _run(H, dtype, 1600, 320, n_groups=9, kind="heavy", rounding=1, seed=77)
    _run(H, dtype, 128, 32, n_groups=21, kind="ties", rounding=1, seed=78)


def test_topk_batched_call_and_many_groups(H):
    _run(H, "f16", 1600, 320, n_groups=4 * 64, kind="heavy", batch=4)        # more groups than one pass of the grid
    _run(H, "bf16", 64, 16, n_groups=4099, kind="ties")


def test_topk_gpt2_backward_shape_full_size(H):
    """The backward tensor of the GPT2-1.5B boundary (4 x 1024 x 1600 halves), a fifth kept."""
    _run(H, "f16", 1600, 320, n_groups=4096, kind="heavy", batch=4)


def test_topk_rejects_what_it_does_not_support(H):
    L = B.lib()
    p = ctypes.c_void_p(4096)
    ok = B.make_desc(batch=2, n_per=1600, bits=8, group=1600, dtype="f16")
    assert L.aqsgd_grad_topk_quant(ctypes.byref(ok), 0, p, p, p, p, None) == -5
    assert L.aqsgd_grad_topk_quant(ctypes.byref(ok), 1601, p, p, p, p, None) == -5
    four = B.make_desc(batch=2, n_per=1600, bits=4, group=1600, dtype="f16")
    assert L.aqsgd_grad_topk_quant(ctypes.byref(four), 320, p, p, p, p, None) == -2
    odd = B.make_desc(batch=2, n_per=1600, bits=8, group=100, dtype="f16")
    assert L.aqsgd_grad_topk_dequant(ctypes.byref(odd), 20, p, p, p, p, None) == -3
    big = B.make_desc(batch=2, n_per=4096, bits=8, group=4096, dtype="f16")
    assert L.aqsgd_grad_topk_dequant(ctypes.byref(big), 20, p, p, p, p, None) == -3
    assert L.aqsgd_grad_topk_quant(ctypes.byref(ok), 320, None, p, p, p, None) == -1
    assert L.aqsgd_grad_topk_quant(ctypes.byref(ok), 320, p, p, ctypes.c_void_p(4100), p, None) == -6
    assert B.topk_codes_bytes(ok, 320) == 640 and B.topk_bitmap_bytes(ok) == 400
    assert B.topk_codes_bytes(four, 320) == 0
