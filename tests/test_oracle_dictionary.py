"""Pins for the oracle's dictionary (Section 4.3.2, Algorithm 1 and the entry layout).

Nothing here calls back into the oracle to obtain an expected value: expected
values come from the paper's printed numbers, from combinatorial closed forms,
or from brute-force enumeration written out in this file.
"""
import itertools
import math
from collections import Counter

import numpy as np
import pytest

import oracle


def _logp(seq, p0):
    a = sum(1 for v in seq if v == 0)
    b = len(seq) - a
    return a * math.log(p0) + b * math.log((1 - p0) / 2)


def _base3(seq):
    v = 0
    for s in seq:
        v = v * 3 + s
    return v


def test_size_and_layout_constants(oracle_dict, golden):
    d = oracle_dict
    assert d.n == int(golden["n_codewords"]) == 1 << 16
    assert d.words.dtype == np.uint32 and d.words.shape == (d.n, 2)
    assert d.words.nbytes == d.n * int(golden["entry_bytes"]) == 512 * 1024
    assert d.npairs.min() == 1 and d.npairs.max() == int(golden["max_pairs"])


def test_source_model_entropy_limit(golden):
    # 16 / H(p0) with P(0)=p0, P(1)=P(2)=(1-p0)/2 must give the printed 25.40x at p0 = 0.885.
    got = oracle.entropy_limit_ratio(golden["p0_example"])
    assert abs(got - golden["entropy_limit_ratio"]) < 0.005
    # a wrong split of the non-zero mass (e.g. P(1)=P(2)=1-p0) is far off
    p = golden["p0_example"]
    wrong = 16.0 / -(p * math.log2(p) + 2 * (1 - p) * math.log2(1 - p))
    assert abs(wrong - golden["entropy_limit_ratio"]) > 1.0


def test_dictionary_is_the_top_k_by_probability(oracle_dict):
    """Popping by decreasing probability enumerates all even-length sequences in
    probability order (an extension is strictly less probable than its parent),
    so the dictionary must be the 2^16 most probable sequences of 1..14 pairs.
    Classes (length L, k non-zeros) hold C(L,k)*2^k equiprobable sequences."""
    p0 = 0.885
    classes = []
    for L in range(2, 29, 2):
        for k in range(0, L + 1):
            lp = (L - k) * math.log(p0) + k * math.log((1 - p0) / 2)
            classes.append((lp, L, k, math.comb(L, k) * 2 ** k))
    classes.sort(key=lambda c: -c[0])
    expect = Counter()
    total = 0
    cut = None
    for lp, L, k, cnt in classes:
        take = min(cnt, (1 << 16) - total)
        if take <= 0:
            break
        expect[(L, k)] = take
        total += take
        if take < cnt:
            cut = (L, k, take, cnt)
    got = Counter()
    for s in oracle_dict.sequences():
        got[(len(s), sum(1 for v in s if v))] += 1
    assert got == expect
    # the cut falls inside one tie class; the tie rule keeps the smallest base-3 strings
    assert cut is not None
    L, k, take, cnt = cut
    assert (L, k) == (26, 3) and cnt == 20800 and take == 2490
    members = []
    for pos in itertools.combinations(range(L), k):
        for signs in itertools.product((1, 2), repeat=k):
            s = [0] * L
            for p, v in zip(pos, signs):
                s[p] = v
            members.append(tuple(s))
    members.sort(key=_base3)
    kept = sorted((s for s in oracle_dict.sequences()
                   if len(s) == L and sum(1 for v in s if v) == k), key=_base3)
    assert kept == members[:take]


def test_counts_per_length_and_nonzeros(oracle_dict):
    # closed form: all sequences with <=3 non-zeros up to 24 values, <=2 up to 28, plus 2490 of (26,3)
    per_len = Counter(int(n) for n in oracle_dict.npairs)
    for npairs in range(1, 15):
        L = 2 * npairs
        n = 1 + 2 * L + 4 * math.comb(L, 2)
        if L <= 24:
            n += 8 * math.comb(L, 3)
        if L == 26:
            n += 2490
        assert per_len[npairs] == n, (npairs, per_len[npairs], n)
    assert sum(per_len.values()) == 65536
    assert int((oracle_dict.syms != 0).sum(axis=1).max()) == 3


def test_order_is_by_decreasing_probability_then_base3(oracle_dict):
    seqs = oracle_dict.sequences()
    keys = [(-_logp(s, 0.885), _base3(s)) for s in seqs]
    for a, b in zip(keys, keys[1:]):
        assert a[0] < b[0] - 1e-12 or (abs(a[0] - b[0]) <= 1e-12 and a[1] < b[1])
    # head of the table: all-zero runs of 1..12 pairs come before any non-zero
    # (0.885^24 > 0.885*0.0575 > 0.885^26), then the four one-non-zero pairs in base-3 order
    for k in range(12):
        assert seqs[k] == (0,) * (2 * (k + 1))
    assert seqs[12:16] == [(0, 1), (0, 2), (1, 0), (2, 0)]


def test_prefix_closed_and_complete(oracle_dict):
    S = set(oracle_dict.sequences())
    assert len(S) == oracle_dict.n  # no duplicates
    for a in range(3):
        for b in range(3):
            assert (a, b) in S  # every even-length row is encodable
    for s in S:
        if len(s) > 2:
            assert s[:-2] in S


@pytest.mark.parametrize("p0,max_pairs,n", [(0.6, 2, 20), (0.8, 3, 64), (0.7, 2, 90), (0.9, 3, 300)])
def test_tiny_dictionaries_by_brute_force(p0, max_pairs, n):
    allseq = []
    for npairs in range(1, max_pairs + 1):
        allseq.extend(itertools.product(range(3), repeat=2 * npairs))
    # equal (zeros, non-zeros) give the identical float, so ties are exact and fall to base-3 order
    allseq.sort(key=lambda s: (-_logp(s, p0), _base3(s)))
    d = oracle.Dictionary(p0=p0, max_pairs=max_pairs, n_entries=n)
    assert d.n == min(n, len(allseq))
    assert d.sequences() == [tuple(s) for s in allseq[: d.n]]


def test_thirteen_pair_reading_has_no_28_value_entries():
    d = oracle.Dictionary(max_pairs=13)
    assert d.n == 65536 and d.npairs.max() == 13


def test_same_entry_set_for_nearby_p0(oracle_dict):
    base = set(oracle_dict.sequences())
    for p0 in (0.90, 0.92):
        assert set(oracle.Dictionary(p0=p0).sequences()) == base


def test_packed_words_hand_examples(oracle_dict):
    idx = {s: k for k, s in enumerate(oracle_dict.sequences())}
    # (0,1,2,0): 2 pairs; symbols at bits 4.., two bits each -> 2 | 1<<6 | 2<<8
    k = idx[(0, 1, 2, 0)]
    assert oracle_dict.words[k].tolist() == [2 + 64 + 512, 2]
    # 8 pairs, 14 zeros then (1,2): the second word starts at symbol 14
    k = idx[(0,) * 14 + (1, 2)]
    assert oracle_dict.words[k].tolist() == [8, 8 + (1 << 4) + (2 << 6)]
    # 14 pairs, all zero except the very last symbol = 2 -> bit 4+2*13 of word 1
    k = idx[(0,) * 27 + (2,)]
    assert oracle_dict.words[k].tolist() == [14, 14 + (2 << 30)]


def test_packed_words_unpack_to_symbols(oracle_dict):
    w = oracle_dict.words.astype(np.uint64)
    assert np.array_equal(w[:, 0] & 15, oracle_dict.npairs)
    assert np.array_equal(w[:, 1] & 15, oracle_dict.npairs)
    syms = np.zeros((oracle_dict.n, 28), dtype=np.uint8)
    for j in range(28):
        syms[:, j] = (w[:, j // 14] >> np.uint64(4 + 2 * (j % 14))) & np.uint64(3)
    assert np.array_equal(syms, oracle_dict.syms)
    assert syms.max() == 2  # symbol value 3 never occurs
    slot = np.arange(28)[None, :]
    assert np.all(syms[slot >= 2 * oracle_dict.npairs[:, None].astype(int)] == 0)  # padding is 0
