"""Pins for the oracle's number formats, dense ternary product, feed-forward block and dispatch."""
import numpy as np
import torch

import oracle
from paper_2310_16795_amd import synth


def _bf16_bits(x):
    """float array -> bfloat16 bit patterns, via torch's own rounding."""
    t = torch.tensor(np.asarray(x, dtype=np.float64)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def test_number_formats_against_numpy_and_torch():
    lib = oracle._load()
    rng = np.random.default_rng(5)
    h = rng.integers(0, 1 << 16, 4000).astype(np.uint16)
    h = h[(h & 0x7C00) != 0x7C00]  # finite halves (includes subnormals)
    want = h.view(np.float16).astype(np.float64)
    got = np.array([lib.orc_f16_to_double(int(v)) for v in h])
    assert np.array_equal(got, want)
    b = rng.integers(0, 1 << 16, 4000).astype(np.uint16)
    b = b[(b & 0x7F80) != 0x7F80]
    want = torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = np.array([lib.orc_bf16_to_double(int(v)) for v in b])
    assert np.array_equal(got, want)
    # rounding to bfloat16: random doubles, exact ties, and values a hair off a tie
    xs = np.concatenate([rng.normal(size=3000) * 10.0 ** rng.integers(-6, 6, 3000),
                         np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -40,
                                   1.0 + 2.0 ** -8 - 2.0 ** -40, 0.0, 3.0, 257.0, 258.0, 259.0])])
    got = np.array([lib.orc_double_to_bf16(float(v)) for v in xs], dtype=np.uint16)
    # torch rounds double -> bf16 through float32; avoid its double rounding by pre-checking exactness
    via_f32 = _bf16_bits(xs)
    exact_in_f32 = xs.astype(np.float32).astype(np.float64) == xs
    assert np.array_equal(got[exact_in_f32], via_f32[exact_in_f32])
    # the two near-tie probes must go to different sides
    assert got[3002] == _bf16_bits([1.0 + 2.0 ** -7])[0] and got[3003] == _bf16_bits([1.0])[0]
    # every result is one of the two neighbours and the nearer one
    back = (got.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(xs), 2.0 ** -126))) - 7)  # 8 significant bits
    assert np.all(np.abs(back - xs) <= ulp * 0.5)
    # ties go to the even mantissa: 257 -> 256, 259 -> 260
    assert back[-3:].tolist() == [256.0, 258.0, 260.0]


def test_matvec_tiny_integer_brute_force():
    rng = np.random.default_rng(1)
    rows, cols, batch = 16, 28, 3
    t = rng.integers(-1, 2, (rows, cols)).astype(np.int8)
    xi = rng.integers(-2, 3, (batch, cols))
    x = _bf16_bits(xi.astype(np.float64))
    one = np.full(rows, np.float16(1.0).view(np.uint16), dtype=np.uint16)
    y, bound = oracle.matvec(t, one, x, with_bound=True)
    for b in range(batch):
        for r in range(rows):
            acc = 0
            mag = 0
            for c in range(cols):
                acc += int(t[r, c]) * int(xi[b, c])
                mag += abs(int(t[r, c]) * int(xi[b, c]))
            assert y[b, r] == acc and bound[b, r] == mag
    # x = 1, s = 1  =>  (#plus - #minus) per row
    ones = _bf16_bits(np.ones((1, cols)))
    assert np.array_equal(oracle.matvec(t, one, ones)[0], (t == 1).sum(1) - (t == -1).sum(1))
    # a single -1 weight with a positive input gives a negative output (sign convention)
    t1 = np.zeros((1, 2), dtype=np.int8)
    t1[0, 1] = -1
    assert oracle.matvec(t1, one[:1], _bf16_bits([[5.0, 3.0]]))[0, 0] == -3.0


def test_matvec_against_numpy_dense():
    rows, cols, batch = 96, 770, 5
    t = synth.ternary(81, rows, cols, 0.9)
    s = synth.uniform_f16(82, (rows,), 0.01, 0.1)
    x = synth.normal_bf16(83, (batch, cols))
    y, bound = oracle.matvec(t, s, x, with_bound=True)
    xd, sd = synth.bf16_to_f64(x), synth.f16_to_f64(s)
    want = (xd @ t.astype(np.float64).T) * sd[None, :]
    assert np.allclose(y, want, rtol=1e-12, atol=1e-15)
    want_b = (np.abs(xd) @ np.abs(t).astype(np.float64).T) * sd[None, :]
    assert np.allclose(bound, want_b, rtol=1e-12)
    # row permutation permutes outputs; transposed operands would not even have this shape
    perm = np.random.default_rng(2).permutation(rows)
    assert np.array_equal(oracle.matvec(t[perm], s[perm], x), y[:, perm])
    # scales in range and really per row
    assert sd.min() >= 0.01 - 1e-4 and sd.max() <= 0.1 and np.unique(sd).size > rows // 2


def test_matvec_linearity_in_integers():
    rng = np.random.default_rng(3)
    t = synth.ternary(91, 40, 64, 0.7)
    one = np.full(40, np.float16(1.0).view(np.uint16), dtype=np.uint16)
    a, b = rng.integers(-8, 9, (1, 64)), rng.integers(-8, 9, (1, 64))
    ya = oracle.matvec(t, one, _bf16_bits(a.astype(float)))
    yb = oracle.matvec(t, one, _bf16_bits(b.astype(float)))
    yab = oracle.matvec(t, one, _bf16_bits((a + b).astype(float)))
    assert np.array_equal(ya + yb, yab)


def test_ffn_token_reduces_to_two_products():
    d_model, d_ff = 64, 160
    wi, wo = synth.ternary(101, d_ff, d_model, 0.8), synth.ternary(102, d_model, d_ff, 0.8)
    wis, wos = synth.uniform_f16(103, (d_ff,), 0.01, 0.1), synth.uniform_f16(104, (d_model,), 0.01, 0.1)
    x = synth.normal_bf16(105, (d_model,))
    y, h, bound = oracle.ffn_token(wi, wis, wo, wos, x, gate=0.5)
    pre = (wi.astype(np.float64) @ synth.bf16_to_f64(x)) * synth.f16_to_f64(wis)
    relu = np.maximum(pre, 0.0)
    assert (pre < 0).any() and (pre > 0).any()
    # hidden vector: rounded to bfloat16; compare with torch where float32 holds the value exactly enough
    hb = (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(hb[pre <= 0] == 0.0)
    assert np.all(np.abs(hb - relu) <= np.abs(relu) * 2.0 ** -8)
    want = 0.5 * (wo.astype(np.float64) @ hb) * synth.f16_to_f64(wos)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-15)
    y1 = oracle.matvec(wo, wos, h)[0]
    assert np.allclose(y, 0.5 * y1, rtol=1e-15)
    assert np.allclose(bound, 0.5 * (np.abs(wo).astype(np.float64) @ np.abs(hb)) * synth.f16_to_f64(wos))


def test_dispatch_against_stable_argsort():
    rng = np.random.default_rng(4)
    for E, T in ((1, 5), (7, 0), (16, 100), (300, 1000)):
        idx = rng.integers(0, E, T).astype(np.int32)
        tok_off, perm = oracle.dispatch(idx, E)
        assert np.array_equal(perm, np.argsort(idx, kind="stable"))
        assert np.array_equal(tok_off, np.concatenate([[0], np.cumsum(np.bincount(idx, minlength=E))]))
    # tokens with an out-of-range expert are left out
    idx = np.array([2, -1, 0, 5, 2], dtype=np.int32)
    tok_off, perm = oracle.dispatch(idx, 3)
    assert tok_off.tolist() == [0, 1, 1, 3] and perm.tolist() == [2, 0, 4]


def test_moe_layer_routing_invariance():
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=6, d_model=32, d_ff=64, n_tokens=20)
    idx, x = w.expert_idx(), w.tokens()
    assert idx.min() >= 0 and idx.max() < 6
    full = oracle.moe_layer(w, idx, x)
    perm = np.random.default_rng(6).permutation(idx.size)
    shuffled = oracle.moe_layer(w, idx[perm], x[perm])
    for new_t, old_t in enumerate(perm):
        assert np.array_equal(shuffled[new_t][0], full[int(old_t)][0])
    # a token's output depends on its own expert only
    t0 = 3
    alone = oracle.ffn_token(w.wi_ternary(int(idx[t0])), w.wi_scale(int(idx[t0])),
                             w.wo_ternary(int(idx[t0])), w.wo_scale(int(idx[t0])), x[t0])
    assert np.array_equal(alone[0], full[t0][0])


def _f16_bits(v):
    return np.asarray(v, dtype=np.float16).view(np.uint16)


def test_asymmetric_grid_tiny_brute_force():
    """Section 4.1's per-row grid {w_min, 0, w_max}: the product with the dequantised matrix written out."""
    rng = np.random.default_rng(11)
    rows, cols, batch = 12, 21, 2
    t = rng.integers(-1, 2, (rows, cols)).astype(np.int8)
    xi = rng.integers(-3, 4, (batch, cols))
    x = _bf16_bits(xi.astype(np.float64))
    # scales exact in binary16 and small powers of two times integers, so fp64 sums are exact in any order
    pos = rng.integers(1, 8, rows) * 0.25
    neg = rng.integers(1, 8, rows) * 0.125
    y, bound = oracle.matvec(t, _f16_bits(pos), x, with_bound=True, scale_neg_f16=_f16_bits(neg))
    for b in range(batch):
        for r in range(rows):
            acc = 0.0
            mag = 0.0
            for c in range(cols):
                w = pos[r] if t[r, c] == 1 else (-neg[r] if t[r, c] == -1 else 0.0)
                acc += w * xi[b, c]
                mag += abs(w * xi[b, c])
            assert y[b, r] == acc and bound[b, r] == mag
    # sign convention: a lone -1 weight contributes -n * x, a lone +1 weight +s * x, whichever column it sits in
    t1 = np.array([[0, -1, 0], [1, 0, 0]], dtype=np.int8)
    got = oracle.matvec(t1, _f16_bits([0.5, 0.5]), _bf16_bits([[7.0, 3.0, 11.0]]), scale_neg_f16=_f16_bits([2.0, 2.0]))
    assert got.tolist() == [[-6.0, 3.5]]


def test_asymmetric_grid_special_cases():
    rows, cols, batch = 64, 300, 4
    t = synth.ternary(111, rows, cols, 0.85)
    s = synth.uniform_f16(112, (rows,), 0.01, 0.1)
    n = synth.uniform_f16(113, (rows,), 0.01, 0.1)
    x = synth.normal_bf16(114, (batch, cols))
    xd, sd, nd = synth.bf16_to_f64(x), synth.f16_to_f64(s), synth.f16_to_f64(n)
    y, bound = oracle.matvec(t, s, x, with_bound=True, scale_neg_f16=n)
    # against numpy on the dequantised matrix
    w = np.where(t > 0, sd[:, None], 0.0) - np.where(t < 0, nd[:, None], 0.0)
    assert np.allclose(y, xd @ w.T, rtol=1e-12, atol=1e-15)
    assert np.allclose(bound, np.abs(xd) @ np.abs(w).T, rtol=1e-12)
    assert not np.allclose(y, oracle.matvec(t, s, x), rtol=1e-3)  # the second scale really matters
    # equal scales: the symmetric product (one signed sum against two sums: equal up to fp64 rounding)
    sym = oracle.matvec(t, s, x)
    assert np.allclose(oracle.matvec(t, s, x, scale_neg_f16=s), sym, rtol=1e-12, atol=1e-15)
    # flipping every sign and swapping the two scales negates the output exactly
    assert np.array_equal(oracle.matvec((-t).astype(np.int8), n, x, scale_neg_f16=s), -y)
    # a row with only positive weights ignores the negative scale, and the other way round
    tp = np.abs(t).astype(np.int8)
    assert np.array_equal(oracle.matvec(tp, s, x, scale_neg_f16=n), oracle.matvec(tp, s, x, scale_neg_f16=s))
    tn = (-tp).astype(np.int8)
    assert np.array_equal(oracle.matvec(tn, s, x, scale_neg_f16=n), oracle.matvec(tn, n, x, scale_neg_f16=n))
    # split into the two symmetric products it is made of
    zero = np.zeros_like(s)
    parts = oracle.matvec(t, s, x, scale_neg_f16=zero) + oracle.matvec(t, zero, x, scale_neg_f16=n)
    assert np.allclose(parts, y, rtol=1e-15, atol=0)


def test_asymmetric_ffn_token_and_layer():
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=5, d_model=32, d_ff=96, n_tokens=12)
    idx, x = w.expert_idx(), w.tokens()
    full = oracle.moe_layer(w, idx, x, asym=True)
    sym = oracle.moe_layer(w, idx, x)
    assert any(not np.allclose(full[t][0], sym[t][0], rtol=1e-3) for t in range(idx.size))
    t0 = 4
    e = int(idx[t0])
    y, h, bound = full[t0]
    pre = oracle.matvec(w.wi_ternary(e), w.wi_scale(e), x[t0][None, :], scale_neg_f16=w.wi_scale_neg(e))[0]
    hb = (h.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    assert np.all(hb[pre <= 0] == 0.0) and np.all(np.abs(hb - np.maximum(pre, 0)) <= np.abs(pre) * 2.0 ** -8)
    y2 = oracle.matvec(w.wo_ternary(e), w.wo_scale(e), h[None, :], scale_neg_f16=w.wo_scale_neg(e))[0]
    assert np.array_equal(y, y2)
    # the negative scales are drawn apart from the positive ones
    assert not np.array_equal(w.wi_scale(e), w.wi_scale_neg(e)) and not np.array_equal(w.wo_scale(e), w.wo_scale_neg(e))
