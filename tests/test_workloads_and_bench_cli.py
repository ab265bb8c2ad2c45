"""CPU checks of the seeded input streams (the recipe both the oracle and the
HIP path are fed from) and of bench.py's command line."""
import subprocess
import sys
from pathlib import Path

import numpy as np

from paper_2206_01299_amd import workloads as W

ROOT = Path(__file__).resolve().parent.parent


def test_streams_are_seeded_and_stateless():
    cfg = W.gpt2_4bit().scaled(n_samples=16, seq=8)
    s1, s2 = W.ActivationStream(cfg), W.ActivationStream(cfg)
    ids = s1.epoch_ids(1)[2]
    a = s1.activations(ids, 1)
    # any (sample, epoch) on its own, in any order, from a fresh object
    b = np.stack([s2.activations(np.array([i]), 1)[0] for i in ids[::-1]])[::-1]
    assert a.dtype == np.float16 and a.shape == (cfg.batch, cfg.seq, cfg.hidden)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    assert not np.array_equal(a, s1.activations(ids, 0))
    other = W.ActivationStream(cfg.scaled(seed=99)).activations(ids, 1)
    assert not np.array_equal(a, other)


def test_drift_is_small_against_the_activation():
    """The property the method relies on: change << activation between visits."""
    cfg = W.gpt2_4bit().scaled(n_samples=8, seq=16)
    s = W.ActivationStream(cfg)
    ids = s.epoch_ids(0)[0]
    a0 = s.activations(ids, 0).astype(np.float32)
    a1 = s.activations(ids, 1).astype(np.float32)
    assert np.abs(a1 - a0).mean() < 0.08 * np.abs(a0).mean()


def test_outliers_and_laws():
    c2 = W.gpt2_4bit().scaled(n_samples=4, seq=64)
    x = W.ActivationStream(c2).sample_f32(0, 0)
    per_channel = x.std(axis=0)
    big = per_channel > 8
    assert big.sum() == 16                       # 1 % of 1600 channels carry 20x the scale
    assert 0.9 < per_channel[~big].mean() < 1.1
    c4 = W.deberta_3bit().scaled(n_samples=32, seq=32)
    t = W.ActivationStream(c4).sample_f32(1, 0)
    assert np.abs(t).max() > 8 and 0.5 < np.median(np.abs(t)) < 1.0     # heavy tails of Student-t(3)
    c5 = W.stress(4, 0).scaled(n_samples=8, seq=400, hidden=64)
    z = W.ActivationStream(c5).sample_f32(3, 0)
    row_scale = np.abs(z).mean(axis=1)
    assert (row_scale > 20).sum() == 2           # 0.5 % of 400 token rows x100
    g = W.ActivationStream(c2).gradients(np.array([0, 1, 2, 3]), 0)
    assert g.dtype == np.float16 and (np.abs(g[g != 0]) < 6.2e-5).any()   # float16 subnormals occur


def test_epoch_ids_cover_every_sample_once():
    cfg = W.gpt2_2bit_stochastic().scaled(n_samples=64, seq=4)
    s = W.ActivationStream(cfg)
    e0, e1 = s.epoch_ids(0), s.epoch_ids(1)
    assert sorted(e0.reshape(-1).tolist()) == list(range(64))
    assert sorted(e1.reshape(-1).tolist()) == list(range(64))
    assert not np.array_equal(e0, e1)            # a fresh permutation per epoch
    ids = W.parity_ids(W.deberta_3bit(), 2)
    assert len(set(ids.tolist())) == 64 and 0 in ids and 99_999 in ids


def test_call_seeds_are_distinct():
    cfg = W.gpt2_2bit_stochastic()
    seeds = {W.call_seed(cfg, t, k, b) for t in range(4) for k in range(50) for b in (False, True)}
    assert len(seeds) == 400


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, str(ROOT / "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""
