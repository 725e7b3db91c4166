"""CPU tests of the library's host side: exports, dictionary, encoder, validation, error paths.

The library's dictionary builder and encoder are written independently of the
oracle's; here they must reproduce the oracle's table and streams exactly.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2310_16795_amd as q
from paper_2310_16795_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib_dict():
    d = q.qmoe_dict_create()
    yield d
    q.qmoe_dict_destroy(d)


def test_library_exports_every_declared_symbol():
    header = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                     if h.endswith(".h"))
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)  # declarations only
    declared = set(re.findall(r"\b(qmoe_[a-z0-9_]+)\s*\(", header))
    declared -= {"qmoe_status"}
    assert declared == set(q.EXPORTS), declared ^ set(q.EXPORTS)
    L = q.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert ctypes.sizeof(q.qmoe_matrix) == 64 and q.qmoe_matrix.minmax_bf16.offset == 40
    assert (q.FORMAT_DEVICE_ORDER, q.FORMAT_GRID_MINMAX) == (1, 2)
    assert L.qmoe_strerror(0) == b"ok" and L.qmoe_strerror(-4) == b"corrupt codeword stream"
    # run entries, interchange words, device-order table and map, then the encoder's trie (2^17 nodes)
    assert q.qmoe_dict_device_bytes() == 65536 * 4 + 65536 * 8 + 20480 * 4 + 65536 * 2 + (9 + 1) * 4 * (1 << 17)


def test_dictionary_equals_oracle_table(lib_dict, oracle_dict):
    assert np.array_equal(q.qmoe_dict_words(lib_dict), oracle_dict.words)
    assert q.qmoe_dict_max_nonzeros(lib_dict) == 3


@pytest.mark.parametrize("p0,max_pairs,n", [(0.6, 2, 20), (0.8, 3, 64), (0.9, 13, 65536), (0.5, 3, 500), (0.7, 2, 200)])
def test_dictionary_variants_equal_oracle(p0, max_pairs, n):
    d = q.qmoe_dict_create(p0, max_pairs, n)
    od = oracle.Dictionary(p0=p0, max_pairs=max_pairs, n_entries=n)
    w = q.qmoe_dict_words(d)
    assert w.shape[0] == od.n  # (0.7, 2, 200): only 90 sequences exist
    assert np.array_equal(w, od.words)
    assert q.qmoe_dict_max_nonzeros(d) == int((od.syms != 0).sum(1).max())
    q.qmoe_dict_destroy(d)


def test_dictionary_argument_errors():
    for args in ((0.0, 14, 65536), (1.0, 14, 65536), (0.885, 0, 65536), (0.885, 15, 65536), (0.885, 14, 0),
                 (0.885, 14, 65537)):
        with pytest.raises(q.QmoeError) as ei:
            q.qmoe_dict_create(*args)
        assert ei.value.status == -1


def test_from_words_round_trip_and_validation(oracle_dict):
    d = q.qmoe_dict_from_words(oracle_dict.words)
    assert np.array_equal(q.qmoe_dict_words(d), oracle_dict.words)
    q.qmoe_dict_destroy(d)
    bad = oracle_dict.words[:100].copy()
    bad[7, 1] ^= 1  # count nibbles differ
    with pytest.raises(q.QmoeError) as ei:
        q.qmoe_dict_from_words(bad)
    assert ei.value.status == -3
    bad = oracle_dict.words[:100].copy()
    bad[0, 0] |= 3 << 4  # symbol value 3
    with pytest.raises(q.QmoeError):
        q.qmoe_dict_from_words(bad)
    bad = oracle_dict.words[:100].copy()
    bad[0, 1] |= 1 << 10  # entry 0 has one pair: a non-zero symbol in an unused slot
    with pytest.raises(q.QmoeError):
        q.qmoe_dict_from_words(bad)


def test_encoder_equals_oracle_encoder(lib_dict, oracle_dict):
    mats = [synth.ternary(201, 300, 770, 0.9), synth.ternary(202, 5, 2, 0.5), synth.ternary(203, 9, 30, 0.0),
            synth.ternary(204, 9, 58, 1.0), synth.ternary(205, 70, 6144, 0.97), synth.ternary(206, 64, 2080, 0.80),
            np.tile(np.array([1, -1], dtype=np.int8), (3, 50))]
    for t in mats:
        codes, row_off = q.qmoe_encode_host(lib_dict, t)
        oc, oro = oracle.encode(oracle_dict, t)
        assert np.array_equal(codes, oc) and np.array_equal(row_off, oro)
        q.qmoe_validate_host(lib_dict, codes, row_off, *t.shape)
        assert np.array_equal(oracle.decode(oracle_dict.words, codes, row_off, *t.shape), t)


def test_encoder_thread_count_does_not_change_the_stream(lib_dict):
    t = synth.ternary(207, 1000, 514, 0.88)
    q.qmoe_set_tuning("host_threads", 1)
    a = q.qmoe_encode_host(lib_dict, t)
    q.qmoe_set_tuning("host_threads", 7)
    b = q.qmoe_encode_host(lib_dict, t)
    q.qmoe_set_tuning("host_threads", 0)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_encoder_with_small_dictionaries_equals_oracle():
    for p0, mp, n in ((0.6, 2, 20), (0.5, 3, 500)):
        d = q.qmoe_dict_create(p0, mp, n)
        od = oracle.Dictionary(p0=p0, max_pairs=mp, n_entries=n)
        t = synth.ternary(208, 50, 64, p0)
        codes, row_off = q.qmoe_encode_host(d, t)
        oc, oro = oracle.encode(od, t)
        assert np.array_equal(codes, oc) and np.array_equal(row_off, oro)
        q.qmoe_dict_destroy(d)


def test_encode_error_paths(lib_dict):
    L = q.lib()
    n = ctypes.c_size_t(0)
    t = np.zeros((2, 8), dtype=np.int8)
    ro = np.zeros(3, dtype=np.uint32)
    codes = np.zeros(8, dtype=np.uint16)
    call = lambda tern, rows, cols, c, cap: L.qmoe_encode_host(  # noqa: E731
        lib_dict, tern.ctypes.data, rows, cols, c, cap, ro.ctypes.data, ctypes.byref(n))
    assert call(t, 2, 7, codes.ctypes.data, 8) == -1          # odd cols
    assert call(t, 0, 8, codes.ctypes.data, 8) == -1          # no rows
    assert L.qmoe_encode_host(lib_dict, None, 2, 8, None, 0, ro.ctypes.data, ctypes.byref(n)) == -1
    bad = t.copy()
    bad[1, 5] = 2
    assert call(bad, 2, 8, codes.ctypes.data, 8) == -3        # symbol outside {-1,0,1}
    assert call(t, 2, 8, None, 0) == 0 and n.value == 2       # sizing call
    assert ro.tolist() == [0, 1, 2]
    assert call(t, 2, 8, codes.ctypes.data, 1) == -2 and n.value == 2  # capacity too small
    # a dictionary without all nine pairs cannot encode everything
    d = q.qmoe_dict_create(0.9, 2, 5)
    dense = np.ones((1, 4), dtype=np.int8)
    with pytest.raises(q.QmoeError) as ei:
        q.qmoe_encode_host(d, dense)
    assert ei.value.status == -7
    q.qmoe_dict_destroy(d)


def test_validate_detects_corruption(lib_dict):
    t = synth.ternary(209, 6, 200, 0.9)
    codes, row_off = q.qmoe_encode_host(lib_dict, t)
    q.qmoe_validate_host(lib_dict, codes, row_off, 6, 200)
    for mutate in ("short", "cols", "decreasing", "start"):
        c, r, cols = codes.copy(), row_off.copy(), 200
        if mutate == "short":
            r[-1] -= 1
        elif mutate == "cols":
            cols = 198
        elif mutate == "decreasing":
            r[3] = r[2] - 1
        else:
            r[0] = 1
        with pytest.raises(q.QmoeError) as ei:
            q.qmoe_validate_host(lib_dict, c, r, 6, cols)
        assert ei.value.status == -4
    small = q.qmoe_dict_create(0.885, 14, 1000)
    big_code = codes.copy()
    big_code[0] = 60000
    with pytest.raises(q.QmoeError):
        q.qmoe_validate_host(small, big_code, row_off, 6, 200)
    q.qmoe_dict_destroy(small)


def test_layer_workspace_layout_and_limits():
    l = q.qmoe_moe_layer_ws_layout(128, 768, 3072, 128)
    offs = [l.tok_off, l.perm, l.counters, l.items_wi, l.items_wo, l.items_mm, l.hidden, l.total]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    assert l.perm - l.tok_off >= 4 * 129 and l.items_wo - l.items_wi >= 16 * 128
    assert l.hidden - l.items_mm >= 16 * 128 and l.items_wi - l.counters >= 4 * 16
    assert l.total - l.hidden >= 2 * 128 * 3072
    assert q.qmoe_moe_layer_workspace(128, 768, 3072, 128) == l.total
    assert q.qmoe_moe_layer_workspace(0, 768, 3072, 128) == 0
    assert q.qmoe_moe_layer_workspace(128, 767, 3072, 128) == 0
    with pytest.raises(q.QmoeError) as ei:
        q.qmoe_moe_layer_ws_layout(20000, 768, 3072, 128)
    assert ei.value.status == -10
    with pytest.raises(q.QmoeError):
        q.qmoe_set_tuning("no_such_key", 1)


def test_device_calls_reject_bad_arguments_before_touching_the_gpu(lib_dict):
    L = q.lib()
    W = q.qmoe_matrix(0, 0, 0, 4, 8, 0, 0)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), None, 1, None, None) == -1   # NULL pointers
    W = q.qmoe_matrix(256, 256, 256, 4, 7, 0, 0)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -1     # odd cols
    W = q.qmoe_matrix(256, 256, 256, 4, 65536, 0, 0)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -10    # too wide
    W = q.qmoe_matrix(256, 256, 256, 4, 8, 0, 0)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -9     # not uploaded
    assert L.qmoe_decode_dense(lib_dict, ctypes.byref(W), 256, 0, None) == -9
    W = q.qmoe_matrix(256, 256, None, 4, 8, 0, 0, 258)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -1     # pair array not 4-byte aligned
    W = q.qmoe_matrix(256, 256, None, 4, 8, 0, 0, None)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -1     # neither scales nor pairs
    W = q.qmoe_matrix(256, 256, None, 4, 8, 0, 0, 256)
    assert L.qmoe_decode_matvec(lib_dict, ctypes.byref(W), 256, 1, 256, None) == -9     # pairs alone are enough
    assert L.qmoe_moe_dispatch(lib_dict, 4, 256, 4, 4, 8, 16, 256, 1 << 30, None) == -1  # unknown format bit
    assert L.qmoe_decompress(lib_dict, 256, 5, 2, 8, 16, 0, 256, None) == -1
    assert L.qmoe_moe_layer_forward(lib_dict, 256, 256, 0, 4, 8, 16, 256, 256, None, 4, 256, None, 0, None, None) == -9
    assert L.qmoe_moe_layer_forward_static(lib_dict, 256, 256, 0, 4, 8, 16, 256, 256, None, 4, 256, None) == -9
    assert L.qmoe_static_workspace_bytes() == 8 << 20
    assert L.qmoe_codes_to_device_order(lib_dict, 256, 10, None) == -9
    assert L.qmoe_codes_to_device_order(lib_dict, None, 10, None) == -1
    assert L.qmoe_dict_upload(lib_dict, None, 0, None) == -1
    assert L.qmoe_dict_upload(lib_dict, 256, 10, None) == -2
    assert L.qmoe_bf16_layer_forward(256, 256, 4, 12, 16, 256, 256, None, 4, 256, 256, 1 << 30, None) == -1
    assert L.qmoe_decompress(lib_dict, 256, 1, 2, 8, 16, 0, 256, None) == -9               # not uploaded
    assert L.qmoe_encode_device(lib_dict, 256, 4, 8, 256, 100, 256, 256, None) == -9
    assert L.qmoe_encode_device(lib_dict, 256, 4, 7, 256, 100, 256, 256, None) == -1       # odd cols
    assert L.qmoe_encode_device(lib_dict, 256, 4, 8, 256, 100, 256, None, None) == -1      # no status
    assert L.qmoe_decompress(lib_dict, 256, 1, 2, 8, 12, 0, 256, None) == -1               # cols % 8
    assert L.qmoe_decompress(lib_dict, None, 1, 2, 8, 16, 0, 256, None) == -1
    assert L.qmoe_moe_dispatch(lib_dict, 0, 256, 4, 4, 8, 16, 256, 16, None) == -5
    assert L.qmoe_moe_dispatch(None, 0, 256, 4, 4, 8, 16, 256, 1 << 30, None) == -1                   # workspace too small


def _decode_device_code(code, table, n_groups):
    """Symbols of a device-order code, decoded the way include/qmoe.h describes it."""
    e = int(table[code >> 2 if code < 4 * n_groups else code - 3 * n_groups])
    if code & 1:
        e ^= 1 << 18
    if code & 2:
        e ^= 1 << 26
    # the kernels' branch-free index: the two expressions cross at 4 * n_groups
    assert max(code >> 2, max(code - 3 * n_groups, 0)) == (code >> 2 if code < 4 * n_groups else code - 3 * n_groups)
    length = (e & 0xFF) >> 3
    syms = [0] * length
    for j in range(3):
        f = (e >> (8 + 8 * j)) & 0xFF
        if f:
            assert f & 1 == 0
            w = (f >> 1) & 3
            assert w in (1, 3)
            assert syms[f >> 3] == 0
            syms[f >> 3] = 2 if w == 1 else 1
    return tuple(syms)


def test_device_order_is_a_renumbering_of_the_same_runs(lib_dict, oracle_dict):
    code_map, table, n_groups = q.qmoe_dict_device_order(lib_dict)
    assert code_map is not None and table.size <= 20480 and 4 * n_groups + (table.size - n_groups) <= 65536
    assert np.unique(code_map).size == 65536  # a bijection on the codes in use
    seqs = oracle_dict.sequences()
    for k in range(0, 65536, 7):
        assert _decode_device_code(int(code_map[k]), table, n_groups) == seqs[k]
    for k in list(range(40)) + [65535, 65534, 57401, 57402]:
        assert _decode_device_code(int(code_map[k]), table, n_groups) == seqs[k]
    # groups really are the four sign variants of the last two non-zeros
    inv = np.argsort(code_map)
    for g in (0, 1, n_groups // 2, n_groups - 1):
        variants = [seqs[int(inv[4 * g + b])] for b in range(4)]
        assert len({tuple(v != 0 for v in s) for s in variants}) == 1  # same positions
        assert len(set(variants)) == 4


def test_device_order_of_small_and_dense_dictionaries():
    d = q.qmoe_dict_create(0.5, 3, 500)   # entries with up to 6 non-zeros -> no device order
    assert q.qmoe_dict_max_nonzeros(d) > 3 and q.qmoe_dict_device_order(d)[0] is None
    q.qmoe_dict_destroy(d)
    d = q.qmoe_dict_create(0.95, 14, 3000)
    od = oracle.Dictionary(p0=0.95, max_pairs=14, n_entries=3000)
    assert q.qmoe_dict_max_nonzeros(d) <= 3
    code_map, table, n_groups = q.qmoe_dict_device_order(d)
    seqs = od.sequences()
    for k in range(3000):
        assert _decode_device_code(int(code_map[k]), table, n_groups) == seqs[k]
    # codes that name no entry all land on one empty entry
    assert len(set(code_map[3000:].tolist())) == 1
    assert _decode_device_code(int(code_map[3000]), table, n_groups) == ()
    q.qmoe_dict_destroy(d)


def test_bench_refuses_more_than_one_gpu():
    """One GPU only: bench.py --gpus N with N above 1 exits with a message that says so, before touching a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "one GPU" in r.stderr


def test_lane_layout_round_trip_and_placement(lib_dict):
    """The lane-interleaved layout is a re-packing of the same codewords: piece p of lane g sits at
    wave_off[g // 64] + 64 p + g % 64, lanes own rows by the even split, padding is zero, and
    unpacking gives the stream back."""
    rng = np.random.default_rng(3)
    for rows, cols, lanes in [(300, 280, 128), (64, 56, 64), (50, 120, 64), (777, 96, 192)]:
        tern = synth.ternary(4000 + rows, rows, cols, 0.9)
        codes, row_off = q.qmoe_encode_host(lib_dict, tern)
        pieces, wave_off = q.qmoe_lane_layout_build(codes, row_off, rows, lanes)
        assert pieces.size % 8 == 0 and wave_off[0] == 0 and 8 * int(wave_off[-1]) == pieces.size
        base, extra = divmod(rows, lanes)
        seen = np.zeros(pieces.size, dtype=bool)
        for g in range(lanes):
            ra = g * base + min(g, extra)
            rb = ra + base + (1 if g < extra else 0)
            mine = codes[row_off[ra]: row_off[rb]]
            for p in range((mine.size + 7) // 8):
                at = 8 * (int(wave_off[g // 64]) + 64 * p + g % 64)
                want = np.zeros(8, dtype=np.uint16)
                want[: min(8, mine.size - 8 * p)] = mine[8 * p: 8 * p + 8]
                assert np.array_equal(pieces[at: at + 8], want)
                seen[at: at + 8] = True
            # a group of 64 lanes is as long as its longest lane
            assert (mine.size + 7) // 8 <= (int(wave_off[g // 64 + 1]) - int(wave_off[g // 64])) // 64
        assert not pieces[~seen].any()
        assert np.array_equal(q.qmoe_lane_layout_unpack(pieces, wave_off, row_off, rows, lanes), codes)
    L = q.lib()
    n = ctypes.c_size_t()
    ro = np.array([0, 3, 5], dtype=np.uint32)
    assert L.qmoe_lane_layout_size(ro.ctypes.data, 2, 100, ctypes.byref(n)) == -1     # lanes not a multiple of 64
    assert L.qmoe_lane_layout_size(ro.ctypes.data, 2, 64, None) == -1
    assert L.qmoe_lane_layout_size(ro.ctypes.data, 2, 64, ctypes.byref(n)) == 0 and n.value == 64
    bad = np.array([0, 5, 3], dtype=np.uint32)
    assert L.qmoe_lane_layout_size(bad.ctypes.data, 2, 64, ctypes.byref(n)) == -4     # offsets that decrease
    out = np.zeros(8 * 64, dtype=np.uint16)
    wo = np.zeros(2, dtype=np.uint32)
    c = np.arange(5, dtype=np.uint16)
    assert L.qmoe_lane_layout_build(c.ctypes.data, ro.ctypes.data, 2, 64, out.ctypes.data, 63, wo.ctypes.data) == -2
    assert L.qmoe_lane_layout_build(c.ctypes.data, ro.ctypes.data, 2, 64, out.ctypes.data, 64, wo.ctypes.data) == 0
    assert out[:3].tolist() == [0, 1, 2] and out[8:10].tolist() == [3, 4]  # lane 0 owns row 0, lane 1 row 1
    assert L.qmoe_plan_lanes(None, 8, 16, 4, 4) == 0
