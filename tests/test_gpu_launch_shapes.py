"""The launch-shape settings (workgroups per launch, unroll of the dequantising kernel)
change how the work is cut and never a result bit: a few boundaries are replayed against
the oracle with grids so small that every kernel's grid-stride loops turn over many times."""
import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2206_01299_amd import binding as B
from paper_2206_01299_amd import workloads as W

CASES = [("f16", 4, 1600, W.NEAREST, 41), ("f16", 2, 128, W.STOCHASTIC, 301), ("bf16", 3, 64, W.NEAREST, 517),
         ("bf16", 6, 64, W.NEAREST, 130), ("f32", 4, 4096, W.NEAREST, 9), ("f32", 8, 256, W.STOCHASTIC, 77),
         ("f32", 3, 64, W.NEAREST, 99), ("f16", 8, 8200, W.NEAREST, 5), ("f16", 8, 50, W.NEAREST, 333)]


def _cfg(dtype, bits, group, rounding, gps, batch=3, n_samples=7):
    return W.BoundaryConfig(name=f"shape_{dtype}_b{bits}_g{group}", n_samples=n_samples, batch=batch, seq=gps,
                            hidden=group, dtype=dtype, fwd_bits=bits, fwd_group=group, fwd_rounding=rounding,
                            bwd_bits=bits, bwd_group=group, bwd_rounding=rounding, law="normal", drift=0.05,
                            epochs=2, shuffle_ids=True, seed=4242 + bits + group)


@pytest.mark.parametrize("max_blocks,unroll", [(3, 1), (7, 4), (64, 2)])
def test_results_do_not_depend_on_the_launch_shape(max_blocks, unroll):
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    B.lib()
    import oracle
    oracle.build()
    import gpu_harness as H
    B.set_launch_shape(max_blocks, unroll)
    try:
        for case in CASES:
            print("launch shape", max_blocks, unroll, "case", case, flush=True)
            H.replay_and_compare(_cfg(*case), calls_per_epoch=2, epochs=2, log=lambda *a, **k: None)
        # the extension kernels go through the same bound
        import test_gpu_lowbit
        import test_gpu_topk
        test_gpu_lowbit._replay(H, _cfg("f16", 4, 1600, W.NEAREST, 41), 8, calls_per_epoch=2, epochs=2)
        test_gpu_lowbit._replay(H, _cfg("f32", 2, 64, W.STOCHASTIC, 203), 2, calls_per_epoch=2, epochs=2)
        test_gpu_topk._run(H, "f16", 1600, 320, n_groups=67, kind="heavy")
        test_gpu_topk._run(H, "f32", 64, 13, n_groups=1031, kind="ties")
    finally:
        B.set_launch_shape(0, 0)


def test_launch_shape_rejects_bad_values():
    if not torch.cuda.is_available():
        pytest.fail("needs the MI355X")
    L = B.lib()
    assert L.aqsgd_set_launch_shape(-1, 0) == -5
    assert L.aqsgd_set_launch_shape(0, 3) == -5
    assert L.aqsgd_set_launch_shape(0, 0) == 0
