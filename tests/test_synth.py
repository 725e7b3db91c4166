"""The synthetic workloads have the shapes, sparsity and routing skew they claim."""
import numpy as np

from paper_2310_16795_amd import synth


def test_ternary_statistics_and_reproducibility():
    t = synth.ternary(7, 512, 2080, 0.90)
    assert t.dtype == np.int8 and t.shape == (512, 2080)
    assert set(np.unique(t).tolist()) == {-1, 0, 1}
    assert abs((t == 0).mean() - 0.90) < 2e-3
    assert abs((t == 1).mean() - (t == -1).mean()) < 2e-3
    assert np.array_equal(t, synth.ternary(7, 512, 2080, 0.90))
    assert not np.array_equal(t, synth.ternary(8, 512, 2080, 0.90))
    # neighbouring values are independent: P(nonzero, nonzero) ~ 0.01
    nz = t != 0
    assert abs((nz[:, :-1] & nz[:, 1:]).mean() - 0.01) < 1e-3


def test_per_row_zero_fraction_spread():
    w = synth.WORKLOADS["c2048_ragged256"]
    p = w._p0_rows(3, 1, 4096)
    assert p.min() >= 0.80 and p.max() <= 0.97 and abs(p.mean() - 0.885) < 0.01
    assert abs(np.var((p - 0.80) / 0.17) - 0.05) < 0.01  # Beta(2,2) variance = 1/20
    t = synth.ternary(9, 64, 6144, p[:64])
    assert np.all(np.abs((t == 0).mean(1) - p[:64]) < 0.03)


def test_activations_and_scales():
    x = synth.bf16_to_f64(synth.normal_bf16(10, (200000,)))
    assert abs(x.mean()) < 0.01 and abs(x.std() - 1.0) < 0.01
    s = synth.f16_to_f64(synth.uniform_f16(11, (50000,), 0.01, 0.1))
    assert s.min() >= 0.01 - 1e-5 and s.max() <= 0.1 and abs(s.mean() - 0.055) < 1e-3


def test_routing_recipes():
    w = synth.WORKLOADS["switch_base128"]
    idx = w.expert_idx()
    assert idx.shape == (128,) and idx.min() >= 0 and idx.max() < 128
    z = synth.WORKLOADS["c2048"].expert_idx()
    counts = np.bincount(z, minlength=2048)
    assert z.size == 2048 and 400 < (counts > 0).sum() < 700  # many experts get no token
    assert counts.max() > 100  # a few get dozens to hundreds
    b = synth.WORKLOADS["c2048_ragged256"].expert_idx()
    cb = np.bincount(b, minlength=256)
    assert cb.min() >= 1 and cb.max() <= 32 and 3500 < b.size < 5000
    shapes = {k: (v.d_model, v.d_ff) for k, v in synth.WORKLOADS.items()}
    assert shapes["switch_large128"] == (1024, 4096) and shapes["c2048"] == (2080, 6144)


def test_bf16_pairs_round_like_torch():
    import torch

    v = np.random.default_rng(8).normal(size=2000).astype(np.float32)
    want = torch.from_numpy(v).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(synth.f64_to_bf16(v.astype(np.float64)), want)
    mm = synth.minmax_bf16(5, 100, 0.01, 0.1)
    assert mm.shape == (100, 2) and mm.dtype == np.uint16
    assert np.all(mm[:, 0] & 0x8000) and not np.any(mm[:, 1] & 0x8000)
    assert np.array_equal(mm, synth.minmax_bf16(5, 100, 0.01, 0.1))
