"""GPU parity of aqsgd_run_jobs against the CPU oracle: several independent messages in
one call (the sending stage's encode + grad_dequant, the receiving stage's decode +
grad_quant, the eight boundaries of the stress configuration, more jobs than one grid
holds, jobs that need the any-shape kernels).  Every job's outputs and every touched
row of its m are compared byte for byte with the oracle's result for that job alone."""
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


class Boundary:
    """One boundary's buffers on the device and on the host, and the four kinds of job on
    them.  Each kind keeps its own message buffers, so any mix of jobs is independent."""

    def __init__(self, H, rng, dtype, fb, fg, fr, bb, bg, br, batch, n_per, n_rows, seed):
        self.H, self.rng, self.dtype = H, rng, dtype
        self.fb, self.fg, self.fr, self.bb, self.bg, self.br = fb, fg, fr, bb, bg, br
        self.batch, self.n_per, self.n_rows, self.seed = batch, n_per, n_rows, seed
        d = H.dev()
        td = B.DTYPE_NAME[dtype]
        npdt = W.storage_numpy_dtype(dtype)
        self.m_s = torch.zeros((n_rows, n_per), dtype=td, device=d)
        self.m_r = torch.zeros_like(self.m_s)
        self.om_s = np.zeros((n_rows, n_per), dtype=npdt)
        self.om_r = self.om_s.copy()
        self.base = rng.standard_normal((n_rows, n_per)).astype(np.float32) * 3.0
        self.fdesc = B.make_desc(batch=batch, n_per=n_per, n_samples=n_rows, bits=fb, group=fg, dtype=dtype,
                                 rounding=fr, rng_seed=seed)
        self.bdesc = B.make_desc(batch=batch, n_per=n_per, n_samples=n_rows, bits=bb, group=bg, dtype=dtype,
                                 rounding=br, rng_seed=seed + 1)
        self.keep = []           # device tensors of jobs in flight
        self.checks = []         # (name, device tensor, expected numpy)

    def _dev(self, x):
        return W.to_torch(x, self.dtype, self.H.dev())

    def _new(self, n, dt, fill):
        t = torch.full((n,), fill, dtype=dt, device=self.H.dev())
        self.keep.append(t)
        return t

    def encode_job(self, step):
        import oracle
        ids_np = self.rng.choice(self.n_rows, size=self.batch, replace=False).astype(np.int64)
        a_np = W.to_storage(self.base[ids_np] + 0.1 * step * self.rng.standard_normal(
            (self.batch, self.n_per)).astype(np.float32), self.dtype)
        act, ids = self._dev(a_np), torch.from_numpy(ids_np).to(self.H.dev())
        codes = self._new(B.codes_bytes(self.fdesc), torch.uint8, 0x5A)
        scales = self._new(B.scales_count(self.fdesc), torch.float32, -1.0)
        self.keep += [act, ids]
        wc, ws = oracle.encode(a_np, ids_np, self.om_s, dtype=self.dtype, bits=self.fb, group=self.fg,
                               rounding=self.fr, seed=self.seed)
        self.checks += [("encode codes", codes, wc), ("encode scales", scales, ws)]
        self.wire = (codes, scales, ids, wc, ws, ids_np)
        return B.encode_job(self.fdesc, act, ids, self.m_s, codes, scales)

    def decode_job(self):
        """Decodes the message of the last encode_job (which must have run already)."""
        import oracle
        codes, scales, ids, wc, ws, ids_np = self.wire
        out = self._dev(W.to_storage(np.full((self.batch, self.n_per), 9.0, dtype=np.float32), self.dtype))
        self.keep += [out, codes, scales, ids]            # a later encode_job replaces self.wire
        wo = oracle.decode(wc, ws, ids_np, self.om_r, dtype=self.dtype, bits=self.fb, group=self.fg)
        self.checks.append(("decode out", out, wo))
        return B.decode_job(self.fdesc, codes, scales, ids, self.m_r, out)

    def grad_quant_job(self):
        import oracle
        g_np = W.to_storage(1e-3 * self.rng.standard_normal((self.batch, self.n_per)).astype(np.float32),
                            self.dtype)
        grad = self._dev(g_np)
        codes = self._new(B.codes_bytes(self.bdesc), torch.uint8, 0xA5)
        scales = self._new(B.scales_count(self.bdesc), torch.float32, -2.0)
        self.keep.append(grad)
        wc, ws = oracle.grad_quant(g_np.reshape(-1), dtype=self.dtype, bits=self.bb, group=self.bg,
                                   rounding=self.br, seed=self.seed + 1)
        self.checks += [("grad_quant codes", codes, wc), ("grad_quant scales", scales, ws)]
        self.gwire = (codes, scales, wc, ws)
        return B.grad_quant_job(self.bdesc, grad, codes, scales)

    def grad_dequant_job(self):
        """Reconstructs the message of the last grad_quant_job (which must have run already)."""
        import oracle
        codes, scales, wc, ws = self.gwire
        out = self._dev(W.to_storage(np.full((self.batch, self.n_per), 7.0, dtype=np.float32), self.dtype))
        self.keep += [out, codes, scales]                 # a later grad_quant_job replaces self.gwire
        wo = oracle.grad_dequant(wc, ws, dtype=self.dtype, bits=self.bb, group=self.bg)
        self.checks.append(("grad_dequant out", out, wo))
        return B.grad_dequant_job(self.bdesc, codes, scales, out)

    def verify(self, tag):
        H = self.H
        torch.cuda.synchronize()
        for name, got_t, want in self.checks:
            got = (W.from_torch(got_t, self.dtype) if name.endswith("out") else got_t.cpu().numpy()).reshape(-1)
            assert H.same_bytes(got, want.reshape(-1)), f"{tag}: {name}: {H.first_diff(got, want.reshape(-1))}"
        for name, dev_m, want_m in (("sender m", self.m_s, self.om_s), ("receiver m", self.m_r, self.om_r)):
            got = W.from_torch(dev_m, self.dtype)
            assert H.same_bytes(got, want_m), f"{tag}: {name}: {H.first_diff(got, want_m)}"
        self.checks.clear()
        self.keep.clear()


PAIRS = [
    # dtype, fwd bits/group/rounding, bwd bits/group/rounding, batch, n_per
    ("f16", 4, 1600, 0, 8, 1600, 0, 3, 1600 * 37),       # the GPT2 boundary's kernels, ragged rows
    ("f16", 2, 128, 1, 4, 128, 1, 2, 128 * 301),         # stochastic, half-wave teams
    ("bf16", 3, 64, 0, 6, 64, 0, 5, 64 * 517),           # 3- and 6-bit pieces, 8-lane teams
    ("f32", 4, 4096, 0, 8, 4096, 0, 2, 4096 * 9),        # float32 in 16-byte units, whole-workgroup teams
    ("f32", 3, 64, 1, 2, 256, 0, 3, 256 * 33),           # float32 one-piece layout (3 bits)
    ("f16", 8, 16384, 0, 4, 32768, 1, 2, 32768 * 3),     # 1024-lane teams host the dequantising job
    ("bf16", 6, 512, 1, 3, 2048, 0, 2, 2048 * 11),
]


@pytest.mark.parametrize("case", PAIRS, ids=[f"{c[0]}-fw{c[1]}g{c[2]}-bw{c[4]}g{c[5]}" for c in PAIRS])
def test_stage_side_pairs(H, case):
    """Three steps of a boundary driven the way a pipeline stage would: the sending stage's
    launch holds encode(k) and grad_dequant(k-1), the receiving stage's decode(k) and
    grad_quant(k)."""
    dtype, fb, fg, fr, bb, bg, br, batch, n_per = case
    rng = np.random.default_rng(1000 + PAIRS.index(case))
    b = Boundary(H, rng, dtype, fb, fg, fr, bb, bg, br, batch, n_per, n_rows=2 * batch + 1, seed=900)
    pending_grad = False
    for step in range(3):
        print("jobs", case, "step", step, flush=True)
        sender = [b.encode_job(step)] + ([b.grad_dequant_job()] if pending_grad else [])
        B.run_jobs(sender)
        B.run_jobs([b.decode_job(), b.grad_quant_job()])
        pending_grad = True
        b.verify(f"{case} step {step}")
    B.run_jobs([b.grad_dequant_job()])
    b.verify(f"{case} tail")


def test_eight_boundaries_with_mixed_bits_in_one_call(H):
    """The stress configuration's structure at a small size: eight boundaries, 2/4/8-bit
    mixed, all encodes in one call, then all decodes and gradient jobs in another."""
    rng = np.random.default_rng(5)
    bs = [Boundary(H, rng, "f32", bits, 512, 0, 8, 512, 0, 3, 512 * 21, n_rows=7, seed=40 + i)
          for i, bits in enumerate(W.STRESS_BITS)]
    for step in range(2):
        print("eight boundaries step", step, flush=True)
        B.run_jobs([b.encode_job(step) for b in bs])
        B.run_jobs([b.decode_job() for b in bs] + [b.grad_quant_job() for b in bs])
        B.run_jobs([b.grad_dequant_job() for b in bs])
        for i, b in enumerate(bs):
            b.verify(f"boundary {i} step {step}")


THREE_MIXES = [
    # dtype, group, rounding, forward bits of the boundaries, backward bits, batch, groups per sample
    ("bf16", 64, 0, (3, 4, 3), 6, 5, 517),               # the DeBERTa boundary's widths, 8-lane teams
    ("f16", 1600, 0, (3, 8), 2, 2, 37),                  # one-wave teams of four chunks per lane
    ("f32", 512, 1, (2, 3), 4, 2, 19),                   # float32: unit layout and one-piece layout side by side
    ("f16", 4096, 1, (6, 3), 8, 2, 5),                   # whole-workgroup teams
]


@pytest.mark.parametrize("case", THREE_MIXES, ids=[f"{c[0]}-g{c[1]}-fw{'_'.join(map(str, c[3]))}-bw{c[4]}"
                                                    for c in THREE_MIXES])
def test_3bit_jobs_share_a_grid_with_other_widths(H, case):
    """A whole time slot in one call (encode of step k, decode and grad_quant of step k-1,
    grad_dequant of step k-2) over boundaries whose quantising jobs have 3 bits and other
    widths at one team shape: they share a launch, the kernel variant with the 3-bit bodies."""
    dtype, group, rnd, fws, bw, batch, gps = case
    rng = np.random.default_rng(2000 + THREE_MIXES.index(case))
    bs = [Boundary(H, rng, dtype, fb, group, rnd, bw, group, rnd, batch, group * gps, n_rows=2 * batch + 1,
                   seed=300 + i) for i, fb in enumerate(fws)]
    for step in range(4):
        print("3-bit mix", case, "slot", step, flush=True)
        jobs = []
        if step >= 2:
            jobs += [b.grad_dequant_job() for b in bs]       # message quantised in the slot before
        if step >= 1:
            jobs += [b.decode_job() for b in bs]             # message encoded in the slot before
            jobs += [b.grad_quant_job() for b in bs]
        jobs += [b.encode_job(step) for b in bs]
        B.run_jobs(jobs)
        for i, b in enumerate(bs):
            b.verify(f"{case} boundary {i} slot {step}")


def test_a_time_slot_over_the_launch_budget_of_small_teams(H):
    """Small-team launches get a bounded number of workgroups, shared by the jobs in
    proportion to their sizes, and every workgroup loops over several steps: a slot of four
    messages whose grids would ask for several times that budget, with a ragged last step."""
    rng = np.random.default_rng(8)
    b = Boundary(H, rng, "f16", 2, 128, 1, 4, 128, 1, 3, 128 * 20011, n_rows=4, seed=77)
    for step in range(3):
        print("over budget, slot", step, flush=True)
        jobs = [b.grad_dequant_job()] if step >= 2 else []
        if step >= 1:
            jobs += [b.decode_job(), b.grad_quant_job()]
        jobs.append(b.encode_job(step))
        B.run_jobs(jobs)
        b.verify(f"over budget slot {step}")


def test_more_jobs_than_one_grid_holds_and_any_shape_jobs(H):
    rng = np.random.default_rng(6)
    same = [Boundary(H, rng, "f16", 4, 256, 0, 8, 256, 1, 2, 256 * 13, n_rows=5, seed=70 + i) for i in range(11)]
    odd = Boundary(H, rng, "f16", 8, 50, 0, 4, 6, 1, 3, 150, n_rows=4, seed=99)         # any-shape kernels
    everyone = same + [odd]
    print("many jobs: encode + grad_quant", flush=True)
    B.run_jobs([b.encode_job(1) for b in everyone] + [b.grad_quant_job() for b in everyone])
    print("many jobs: decode + grad_dequant", flush=True)
    B.run_jobs([b.decode_job() for b in everyone] + [b.grad_dequant_job() for b in everyone])
    for i, b in enumerate(everyone):
        b.verify(f"job set member {i}")


def test_a_bad_job_stops_the_whole_call_before_any_launch(H):
    rng = np.random.default_rng(7)
    b = Boundary(H, rng, "f16", 4, 256, 0, 8, 256, 0, 2, 256 * 5, n_rows=4, seed=1)
    good = b.encode_job(0)
    bad = b.grad_quant_job()
    bad.desc.bits = 5
    arr = (B.Job * 2)(good, bad)
    assert B.lib().aqsgd_run_jobs(arr, 2, None) == -2
    bad.desc.bits = 8
    bad.kind = 9
    arr = (B.Job * 2)(good, bad)
    assert B.lib().aqsgd_run_jobs(arr, 2, None) == -5
    assert B.lib().aqsgd_run_jobs(arr, -1, None) == -5
    assert B.lib().aqsgd_run_jobs(None, 1, None) == -1
    assert B.lib().aqsgd_run_jobs(None, 0, None) == 0
    torch.cuda.synchronize()
    assert not bool(b.m_s.any())                         # the good job did not run either
    codes = b.wire[0]
    assert bool((codes == 0x5A).all())
