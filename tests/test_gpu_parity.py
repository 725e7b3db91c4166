"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Decoded weights and dispatch results must be bit-exact.  Products are
compared element by element with
    |y - y*| <= 1e-3 * s_r * sum_c |T[r][c] x[c]|
(relative error 1e-3 against the sum of absolute terms, which cancellation
cannot shrink; fp32 accumulation of n non-zeros errs by about n * 2^-24 of that
sum), and per token in the 2-norm.  The streams the kernels decode here are
produced by the oracle's encoder with the oracle's table.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_16795_amd as q
from paper_2310_16795_amd import device as dev
from paper_2310_16795_amd import synth

pytestmark = pytest.mark.gpu

REL = 1e-3


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("the GPU tests need a GPU: the HIP path has no fallback")
    return "cuda:0"


@pytest.fixture(scope="module")
def ddict(gpu, oracle_dict):
    """Device dictionary built from the oracle's table (an input to the kernels, not shared code)."""
    dd = dev.DeviceDict(q.qmoe_dict_from_words(oracle_dict.words), gpu)
    yield dd
    dd.close()


def _upload(oracle_dict, tern, scale, gpu, order_of=None, minmax=None):
    """order_of: renumber the stream to the device order of that dictionary (None: as encoded).
    minmax: bf16 (w_min, w_max) pairs [rows, 2] for the asymmetric grid (then scale is None)."""
    codes, row_off = oracle.encode(oracle_dict, tern)
    return dev.DeviceMatrix(codes, row_off, scale, *tern.shape, device=gpu, device_order_of=order_of,
                            minmax_bf16=minmax)


def _to_dev16(bits, gpu):
    return torch.from_numpy(bits.view(np.int16).copy()).to(gpu)


def _check_product(y_gpu, y_ref, bound, label=""):
    err = np.abs(y_gpu.astype(np.float64) - y_ref)
    tol = REL * bound + 1e-30
    worst = float((err / tol).max()) if err.size else 0.0
    assert worst <= 1.0, f"{label}: worst error is {worst:.3g} x the tolerance"
    for b in range(y_ref.shape[0]):
        n = np.linalg.norm(y_ref[b])
        if n > 0:
            assert np.linalg.norm(y_gpu[b] - y_ref[b]) / n <= REL, label


SHAPES = [
    (3072, 768, 0.90, 301),   # Switch-base wi: the single-matrix workload
    (96, 770, 0.90, 302),     # ragged: cols not a multiple of 28 or 32, rows not a multiple of the block
    (5, 2, 0.5, 303),         # one pair per row
    (33, 30, 0.0, 304),       # no zeros at all
    (17, 58, 1.0, 305),       # only zeros
    (70, 6144, 0.97, 306),    # long sparse rows
    (130, 2080, 0.80, 307),   # dense end of the natural-sparsity range
]


@pytest.mark.parametrize("rows,cols,p0,seed", SHAPES)
@pytest.mark.parametrize("path,order", [(0, 0), (1, 0), (0, 1)])
def test_decode_dense_bit_exact(gpu, ddict, oracle_dict, rows, cols, p0, seed, path, order):
    """path 0/1: run-entry table / interchange words; order 1: stream renumbered to the device order."""
    tern = synth.ternary(seed, rows, cols, p0)
    scale = synth.uniform_f16(seed + 1000, (rows,), 0.01, 0.1)
    M = _upload(oracle_dict, tern, scale, gpu, ddict if order else None)
    out = torch.full((rows, cols), 77, dtype=torch.int8, device=gpu)
    q.qmoe_decode_dense(ddict.handle, M.desc, out, path)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), tern)


@pytest.mark.parametrize("rows,cols,p0,seed", SHAPES)
@pytest.mark.parametrize("batch", [1, 3, 8, 19])
@pytest.mark.parametrize("order", [0, 1])
def test_decode_matvec_against_oracle(gpu, ddict, oracle_dict, rows, cols, p0, seed, batch, order):
    tern = synth.ternary(seed, rows, cols, p0)
    scale = synth.uniform_f16(seed + 1000, (rows,), 0.01, 0.1)
    x = synth.normal_bf16(seed + 2000, (batch, cols))
    M = _upload(oracle_dict, tern, scale, gpu, ddict if order else None)
    y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
    q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
    torch.cuda.synchronize()
    y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True)
    _check_product(y.cpu().numpy(), y_ref, bound, f"{rows}x{cols} batch {batch}")


def test_matvec_integer_inputs_are_exact(gpu, ddict, oracle_dict):
    # small integers and scale 1: every partial sum is exact in fp32, so the result must be too
    rows, cols = 64, 280
    tern = synth.ternary(311, rows, cols, 0.85)
    one = np.full(rows, np.float16(1.0).view(np.uint16), dtype=np.uint16)
    xi = np.random.default_rng(1).integers(-4, 5, (5, cols)).astype(np.float32)
    x = torch.from_numpy(xi).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    M = _upload(oracle_dict, tern, one, gpu, ddict)
    y = torch.empty((5, rows), dtype=torch.float32, device=gpu)
    q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
    torch.cuda.synchronize()
    assert np.array_equal(y.cpu().numpy().astype(np.float64), oracle.matvec(tern, one, x))


def test_general_dictionary_with_many_nonzeros_per_entry(gpu):
    """A table whose entries hold up to six non-zeros cannot use run entries: the
    kernels must fall back to reading the interchange words, with the same results."""
    od = oracle.Dictionary(p0=0.5, max_pairs=3, n_entries=500)
    assert int((od.syms != 0).sum(1).max()) > 3
    dd = dev.DeviceDict(q.qmoe_dict_from_words(od.words), gpu)
    rows, cols = 50, 66
    tern = synth.ternary(321, rows, cols, 0.5)
    scale = synth.uniform_f16(322, (rows,), 0.01, 0.1)
    x = synth.normal_bf16(323, (4, cols))
    M = _upload(od, tern, scale, gpu)
    out = torch.zeros((rows, cols), dtype=torch.int8, device=gpu)
    q.qmoe_decode_dense(dd.handle, M.desc, out, 0)
    y = torch.empty((4, rows), dtype=torch.float32, device=gpu)
    q.qmoe_decode_matvec(dd.handle, M.desc, _to_dev16(x, gpu), y)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), tern)
    y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True)
    _check_product(y.cpu().numpy(), y_ref, bound, "general dictionary")
    dd.close()


def test_library_encoder_feeds_the_kernels(gpu, oracle_dict):
    """End to end on the product's own dictionary and encoder."""
    dd = dev.DeviceDict(device=gpu)
    tern = synth.ternary(331, 200, 1024, 0.92)
    scale = synth.uniform_f16(332, (200,), 0.01, 0.1)
    codes, row_off = q.qmoe_encode_host(dd.handle, tern)
    M = dev.DeviceMatrix(codes, row_off, scale, 200, 1024, gpu)
    out = torch.zeros((200, 1024), dtype=torch.int8, device=gpu)
    q.qmoe_decode_dense(dd.handle, M.desc, out, 0)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), tern)
    dd.close()


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("E,T,seed", [(1, 5, 1), (7, 1, 2), (16, 100, 3), (300, 1000, 4), (2048, 2048, 5), (64, 5000, 6)])
def test_dispatch_bit_exact(gpu, E, T, seed, order):
    rng = np.random.default_rng(seed)
    idx = rng.integers(0, E, T).astype(np.int32)
    if T > 50:
        idx[rng.integers(0, T, 5)] = np.array([-1, E, E + 7, -5, 2 ** 30], dtype=np.int32)  # dropped tokens
        idx[10:40] = idx[10]  # one crowded expert
    d_model, d_ff = 64, 128
    dd = dev.DeviceDict(device=gpu)
    ws = torch.empty(q.qmoe_moe_layer_workspace(E, d_model, d_ff, T), dtype=torch.uint8, device=gpu)
    q.qmoe_moe_dispatch(dd.handle, order, torch.from_numpy(idx).to(gpu), E, d_model, d_ff, ws)
    torch.cuda.synchronize()
    got = dev.read_workspace(ws, E, d_model, d_ff, T)
    tok_off, perm = oracle.dispatch(idx, E)
    n_valid = int(tok_off[-1])
    assert np.array_equal(got["tok_off"], tok_off)
    assert np.array_equal(got["perm"][:n_valid], perm)
    counts = np.diff(tok_off)
    assert got["counters"][0] == n_valid and got["counters"][1] == T - n_valid
    assert got["counters"][2] == int((counts > 0).sum())
    n_mm = got["counters"][7]
    # crowded experts only leave the scalar kernel with device-order streams, and only in
    # calls with at least four tokens per compute unit
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    if order == 0 or T < 4 * cus:
        assert n_mm == 0
    else:
        assert n_mm == int(sum((c + 63) // 64 for c in counts if c >= 8)) and n_mm > 0
    crowded = set()
    for e, slot0, ntok, _ in got["items_mm"][:n_mm]:
        assert 1 <= ntok <= 64
        crowded.add(int(e))
    for e in crowded:  # an expert is wholly on one side, with full tiles except the last
        sizes = [int(n) for ee, _, n, _ in got["items_mm"][:n_mm] if ee == e]
        assert sum(sizes) == counts[e] and all(n == 64 for n in sizes[:-1])
    for key, n_items in (("items_wi", got["counters"][3]), ("items_wo", got["counters"][4])):
        covered = np.zeros(n_valid, dtype=np.int32)
        for limit, items in ((8, got[key][:n_items]), (64, got["items_mm"][:n_mm])):
            for e, slot0, ntok, _ in items:
                assert counts[e] > 0 and 1 <= ntok <= limit  # never an expert without tokens
                assert tok_off[e] <= slot0 and slot0 + ntok <= tok_off[e + 1]
                covered[slot0:slot0 + ntok] += 1
        assert np.all(covered == 1)
        assert not crowded & {int(e) for e, *_ in got[key][:n_items]}
    dd.close()


def _build_layer(w, oracle_dict, gpu, encoder="oracle", lib_dict=None, experts=None, order_of=None, minmax=False,
                 lanes_for_tokens=0):
    layer = dev.DeviceLayer(w.n_experts, w.d_model, w.d_ff, gpu, minmax=minmax)
    for e in (range(w.n_experts) if experts is None else experts):
        for which, tern, scale in (("wi", w.wi_ternary(e), w.wi_minmax(e) if minmax else w.wi_scale(e)),
                                   ("wo", w.wo_ternary(e), w.wo_minmax(e) if minmax else w.wo_scale(e))):
            if encoder == "oracle":
                codes, row_off = oracle.encode(oracle_dict, tern)
            else:
                codes, row_off = q.qmoe_encode_host(lib_dict, tern)
            layer.set_expert(e, which, codes, row_off, scale)
    return layer.finalize(device_order_of=order_of, lanes_for_tokens=lanes_for_tokens)


def _run_layer(layer, ddict, x_bits, idx, gpu, gate=None):
    T = idx.size
    y = torch.full((T, layer.d_model), float("nan"), dtype=torch.float32, device=gpu)
    ws = layer.workspace(T)
    g = None if gate is None else torch.from_numpy(gate.astype(np.float32)).to(gpu)
    layer.forward(ddict, _to_dev16(x_bits, gpu), torch.from_numpy(idx).to(gpu), y, ws, g)
    torch.cuda.synchronize()
    return y.cpu().numpy(), dev.read_workspace(ws, layer.n_experts, layer.d_model, layer.d_ff, T)


def _check_layer(w, idx, x_bits, y_gpu, wsout, tokens, gate=None, asym=False):
    ref = oracle.moe_layer(w, idx, x_bits, gate=gate, tokens=tokens, asym=asym)
    slot_of = {int(t): s for s, t in enumerate(wsout["perm"][: wsout["counters"][0]])}
    flips = total = 0
    for t in tokens:
        y_ref, h_ref, bound = ref[t]
        h_gpu = wsout["hidden"][slot_of[t]]
        diff = h_gpu.astype(np.int32) - h_ref.astype(np.int32)
        assert np.all(np.abs(diff) <= 1), "hidden vector differs by more than one bf16 ulp"
        flips += int((diff != 0).sum())
        total += diff.size
        if diff.any():
            # A hidden value that sat on a rounding boundary went the other way (fp32 against
            # fp64 sums): the second product is checked on the hidden vector it actually read.
            # One such value moves an output by 2^-8 of one term, more than the tolerance on a
            # sum of a few terms.
            e = int(idx[t])
            g = 1.0 if gate is None else float(gate[t])
            y2, b2 = oracle.matvec(w.wo_ternary(e), None if asym else w.wo_scale(e), h_gpu[None, :], with_bound=True,
                                   minmax_bf16=w.wo_minmax(e) if asym else None)
            y_ref, bound = g * y2[0], abs(g) * b2[0]
        _check_product(y_gpu[t][None, :], y_ref[None, :], bound[None, :], f"token {t}")
    assert flips <= max(2, total * 2e-3), f"{flips} of {total} hidden values rounded differently"


@pytest.mark.parametrize("d_model,d_ff,order",
                         [(96, 200, 0), (96, 200, 1), (260, 300, 1), (450, 228, 0), (224, 226, 1), (226, 224, 1)])
def test_small_layer_every_token(gpu, ddict, oracle_dict, d_model, d_ff, order):
    """Widths on both sides of 224 (rows longer than that hold at most one row end in eight codewords and take
    the branch-free form; 224 itself is the widest row of the general form, 226 the narrowest of the other)."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=12, d_model=d_model, d_ff=d_ff, n_tokens=70)
    idx, x = w.expert_idx(), w.tokens()
    idx[5:40] = 3      # one expert with many tokens (several tiles)
    idx[idx == 7] = 8  # at least one expert without tokens
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict if order else None)
    gate = np.random.default_rng(7).uniform(0.2, 1.0, idx.size)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
    _check_layer(w, idx, x, y, wsout, list(range(idx.size)), gate)
    # same call again: bitwise identical (fixed reduction order)
    y2, _ = _run_layer(layer, ddict, x, idx, gpu, gate)
    assert np.array_equal(y, y2)


@pytest.mark.parametrize("d_model,d_ff", [(136, 600), (520, 72)])
def test_crowded_experts_take_the_matrix_core_kernel(gpu, ddict, oracle_dict, d_model, d_ff):
    """Experts with 8..130 tokens (tiles of 64: full, one short, one over; 32-token blocks
    likewise), more than 512 rows on one side (two row blocks), widths that are no
    multiple of the 64-column step, gates, a dropped token.  Every token is checked."""
    counts = [130, 65, 64, 33, 32, 31, 8, 7, 1, 0]
    idx = np.concatenate([np.full(n, e, dtype=np.int32) for e, n in enumerate(counts)])
    np.random.default_rng(11).shuffle(idx)
    idx = np.concatenate([idx, np.array([-1], dtype=np.int32)])
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=len(counts), d_model=d_model, d_ff=d_ff,
                                                 n_tokens=idx.size)
    x = w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    gate = np.random.default_rng(12).uniform(0.2, 1.0, idx.size)
    y0, ws0 = _run_layer(layer, ddict, x, idx, gpu, gate)
    assert ws0["counters"][7] == 0  # a call this small stays on the scalar kernel by default
    q.qmoe_set_tuning("mfma_min_tokens", 8)
    try:
        y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)
    n_mm = wsout["counters"][7]
    assert n_mm == 3 + 2 + 1 + 1 + 1 + 1 + 1  # tiles of the experts with at least 8 tokens
    assert sorted(int(n) for _, _, n, _ in wsout["items_mm"][:n_mm]) == sorted([64, 64, 2, 64, 1, 64, 33, 32, 31, 8])
    good = [t for t in range(idx.size) if idx[t] >= 0]
    assert not y[-1].any()
    _check_layer(w, idx, x, y, wsout, good, gate)
    _check_layer(w, idx, x, y0, ws0, good, gate)
    # every expert with two tokens or more through the matrix cores (twice: bitwise the
    # same), then none: same answers
    try:
        q.qmoe_set_tuning("mfma_min_tokens", 2)
        y3, ws3 = _run_layer(layer, ddict, x, idx, gpu, gate)
        assert ws3["counters"][7] == n_mm + 1
        _check_layer(w, idx, x, y3, ws3, good, gate)
        y3b, _ = _run_layer(layer, ddict, x, idx, gpu, gate)
        assert np.array_equal(y3, y3b)
        q.qmoe_set_tuning("mfma_min_tokens", -1)
        y4, ws4 = _run_layer(layer, ddict, x, idx, gpu, gate)
        assert ws4["counters"][7] == 0
        _check_layer(w, idx, x, y4, ws4, good, gate)
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)


def _bf16_bits_of_f16(scale_f16_bits):
    """Round-to-nearest-even bf16 bit patterns of binary16 values (numpy only)."""
    u = scale_f16_bits.view(np.float16).astype(np.float32).view(np.uint32)
    return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)


@pytest.mark.parametrize("d_model,d_ff", [(136, 600), (1024, 72)])
def test_decompress_whole_matrices_bit_exact(gpu, ddict, oracle_dict, d_model, d_ff):
    """Every expert of a small layer to int8 and to scaled bf16 in one launch each: widths
    that are no multiple of the 64-column step, more than 512 rows on one side, a skipped
    matrix.  int8 must equal the encoder's input, bf16 must equal bf16(scale) * weight."""
    w = synth.WORKLOADS["c2048_ragged256"].scaled(n_experts=5, d_model=d_model, d_ff=d_ff, n_tokens=8)
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    for which, rows, cols in (("wi", d_ff, d_model), ("wo", d_model, d_ff)):
        tern = [w.wi_ternary(e) if which == "wi" else w.wo_ternary(e) for e in range(w.n_experts)]
        scale = [w.wi_scale(e) if which == "wi" else w.wo_scale(e) for e in range(w.n_experts)]
        skip = 3
        for kind, dt in ((0, torch.int8), (1, torch.int16)):
            outs = [torch.full((rows, cols), 77, dtype=dt, device=gpu) for _ in range(w.n_experts)]
            ptrs = torch.tensor([0 if e == skip else o.data_ptr() for e, o in enumerate(outs)], dtype=torch.int64,
                                device=gpu)
            q.qmoe_decompress(ddict.handle, layer.desc_dev[which], 1, w.n_experts, rows, cols, kind, ptrs)
            torch.cuda.synchronize()
            for e in range(w.n_experts):
                got = outs[e].cpu().numpy()
                if e == skip:
                    assert (got == 77).all()
                elif kind == 0:
                    assert np.array_equal(got, tern[e]), f"{which} expert {e}"
                else:
                    sb = _bf16_bits_of_f16(scale[e])[:, None].astype(np.uint16)
                    want = np.where(tern[e] == 0, np.uint16(0), np.where(tern[e] > 0, sb, sb | np.uint16(0x8000)))
                    assert np.array_equal(got.view(np.uint16), want.astype(np.uint16)), f"{which} expert {e}"


def test_decompress_destinations_anywhere_in_the_address_space(gpu, ddict, oracle_dict):
    """Destinations whose addresses have bit 31 set and clear (address arithmetic in 32-bit halves
    must not sign-extend the low half): carved out of one 5 GiB allocation."""
    w = synth.WORKLOADS["c2048_ragged256"].scaled(n_experts=4, d_model=72, d_ff=200, n_tokens=4)
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    rows, cols = w.d_ff, w.d_model
    pool = torch.empty(5 << 30, dtype=torch.int8, device=gpu)
    base = pool.data_ptr()
    offs = []
    for want_high in (True, False, True, False):
        off = 256 * len(offs) * 1024
        while (((base + off) >> 31) & 1) != int(want_high):
            off += 1 << 30
        assert off + rows * cols <= pool.numel()
        offs.append(off)
    pool[: 1 << 20].fill_(77)
    ptrs = torch.tensor([base + o for o in offs], dtype=torch.int64, device=gpu)
    q.qmoe_decompress(ddict.handle, layer.desc_dev["wi"], 1, w.n_experts, rows, cols, 0, ptrs)
    torch.cuda.synchronize()
    for e, o in enumerate(offs):
        got = pool[o: o + rows * cols].cpu().numpy().reshape(rows, cols)
        assert np.array_equal(got, w.wi_ternary(e)), f"expert {e} at offset {o:#x}"


@pytest.mark.parametrize("rows,cols,p0,seed", [(1, 2, 0.5, 1), (7, 58, 0.9, 2), (300, 136, 0.885, 3), (2080, 6144, 0.9, 4),
                                               (513, 770, 0.3, 5)])
def test_encode_device_equals_the_oracle_stream(gpu, ddict, oracle_dict, rows, cols, p0, seed):
    """The device encoder's codewords and row offsets against the oracle's longest-prefix coder."""
    tern = synth.ternary(seed, rows, cols, p0)
    codes_ref, off_ref = oracle.encode(oracle_dict, tern)
    d_t = torch.from_numpy(tern).to(gpu)
    d_codes = torch.full((codes_ref.size + 8,), -1, dtype=torch.int16, device=gpu)
    d_off = torch.empty(rows + 1, dtype=torch.int32, device=gpu)
    d_status = torch.full((2,), 99, dtype=torch.int32, device=gpu)
    q.qmoe_encode_device(ddict.handle, d_t, d_codes, d_off, d_status)
    torch.cuda.synchronize()
    assert d_status[0].item() == 0
    assert np.array_equal(d_off.cpu().numpy().view(np.uint32), off_ref.astype(np.uint32))
    got = d_codes.cpu().numpy().view(np.uint16)
    assert np.array_equal(got[: codes_ref.size], codes_ref) and (got[codes_ref.size:] == 0xFFFF).all()


def test_encode_device_reports_errors(gpu, ddict, oracle_dict):
    tern = synth.ternary(9, 20, 64, 0.9)
    n_ref = oracle.encode(oracle_dict, tern)[0].size
    d_off = torch.empty(21, dtype=torch.int32, device=gpu)
    d_status = torch.zeros(2, dtype=torch.int32, device=gpu)
    # capacity one codeword short
    d_codes = torch.zeros(n_ref - 1, dtype=torch.int16, device=gpu)
    q.qmoe_encode_device(ddict.handle, torch.from_numpy(tern).to(gpu), d_codes, d_off, d_status)
    torch.cuda.synchronize()
    assert d_status[0].item() == -2  # BUFFER_TOO_SMALL
    assert d_off[-1].item() == n_ref  # the size needed is still reported
    # a value that is no ternary symbol
    bad = tern.copy()
    bad[11, 5] = 2
    d_codes = torch.zeros(n_ref + 8, dtype=torch.int16, device=gpu)
    q.qmoe_encode_device(ddict.handle, torch.from_numpy(bad).to(gpu), d_codes, d_off, d_status)
    torch.cuda.synchronize()
    assert d_status[0].item() == -3 and d_status[1].item() == 11  # BAD_SYMBOL in row 11


def test_decompress_full_size_expert(gpu, ddict, oracle_dict):
    """Two c2048-sized matrices (2080 x 6144): the oracle's decode of the oracle's stream."""
    w = synth.WORKLOADS["c2048"]
    mats, want = [], []
    for e in (5, 1234):
        tern = w.wo_ternary(e)
        codes, row_off = oracle.encode(oracle_dict, tern)
        assert np.array_equal(oracle.decode(oracle_dict.words, codes, row_off, *tern.shape), tern)
        mats.append(dev.DeviceMatrix(codes, row_off, w.wo_scale(e), *tern.shape, device=gpu, device_order_of=ddict))
        want.append(tern)
    desc = (q.qmoe_matrix * 2)(mats[0].desc, mats[1].desc)
    d_desc = torch.from_numpy(np.frombuffer(bytes(desc), dtype=np.uint8).copy()).to(gpu)
    outs = [torch.empty(want[0].shape, dtype=torch.int8, device=gpu) for _ in range(2)]
    ptrs = torch.tensor([o.data_ptr() for o in outs], dtype=torch.int64, device=gpu)
    q.qmoe_decompress(ddict.handle, d_desc, 1, 2, want[0].shape[0], want[0].shape[1], 0, ptrs)
    torch.cuda.synchronize()
    for o, t in zip(outs, want):
        assert np.array_equal(o.cpu().numpy(), t)


def test_layer_forward_in_a_hip_graph(gpu, ddict, oracle_dict):
    """A layer call captured into a HIP graph (dispatch, both chains, the fork to the side
    stream and the join) and replayed with other work in between: every replay must equal
    the eager result bit for bit, also after the inputs change in place."""
    counts = [70, 9, 3, 2, 1, 1, 0, 5]
    idx = np.concatenate([np.full(n, e, dtype=np.int32) for e, n in enumerate(counts)])
    np.random.default_rng(21).shuffle(idx)
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=len(counts), d_model=136, d_ff=264, n_tokens=idx.size)
    x = w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    T = idx.size
    d_x, d_idx = _to_dev16(x, gpu), torch.from_numpy(idx).to(gpu)
    y = torch.zeros((T, w.d_model), dtype=torch.float32, device=gpu)
    ws = layer.workspace(T)
    q.qmoe_set_tuning("mfma_min_tokens", 8)  # both kinds of experts, hence both streams
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            layer.forward(ddict, d_x, d_idx, y, ws)  # warm-up outside the capture
            torch.cuda.synchronize()
            eager = y.clone()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                layer.forward(ddict, d_x, d_idx, y, ws, stream=side.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            y.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y, eager), f"replay {rep}"
            (y * 2).sum().item()  # unrelated eager work between replays
        # new activations in the same buffers: the graph must follow
        x2 = w.scaled(cfg_id=97).tokens()  # other seeds, same shape
        d_x.copy_(_to_dev16(x2, gpu))
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        layer.forward(ddict, d_x, d_idx, y, ws)
        torch.cuda.synchronize()
        assert torch.equal(got, y)
        wsout = dev.read_workspace(ws, w.n_experts, w.d_model, w.d_ff, T)
        assert wsout["counters"][7] == 3
        _check_layer(w, idx, x2, got.cpu().numpy(), wsout, list(range(T)))
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)


def test_layer_drops_tokens_with_bad_expert_index(gpu, ddict, oracle_dict):
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=4, d_model=64, d_ff=96, n_tokens=20)
    idx, x = w.expert_idx(), w.tokens()
    idx[3], idx[11] = -2, 4
    layer = _build_layer(w, oracle_dict, gpu)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    assert not y[3].any() and not y[11].any()
    good = [t for t in range(20) if t not in (3, 11)]
    _check_layer(w, idx, x, y, wsout, good)


def test_layer_with_every_token_dropped(gpu, ddict, oracle_dict):
    """No token names a valid expert: nothing to multiply, every output row is zero, and
    the poisoned descriptors of the experts are never read."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=4, d_model=64, d_ff=96, n_tokens=9)
    x = w.tokens()
    idx = np.array([-1, 4, 7, -3, 2 ** 30, -(2 ** 31), 4, 5, 99], dtype=np.int32)
    layer = dev.DeviceLayer(w.n_experts, w.d_model, w.d_ff, gpu).finalize(device_order_of=ddict)  # no expert set
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    assert not y.any()
    assert wsout["counters"][0] == 0 and wsout["counters"][1] == idx.size and wsout["counters"][2] == 0
    assert wsout["counters"][3] == 0 and wsout["counters"][4] == 0 and wsout["counters"][7] == 0


def test_layer_with_thousands_of_dropped_tokens(gpu, ddict, oracle_dict):
    """More dropped tokens than the dispatch kernel's list of them holds (2048): the rest are cleared one
    row per thread; the kept tokens, scattered among them, still come out right."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=4, d_model=72, d_ff=96, n_tokens=5000)
    x = w.tokens()
    idx = np.full(5000, -1, dtype=np.int32)
    keep = np.random.default_rng(31).choice(5000, size=40, replace=False)
    idx[keep] = np.random.default_rng(32).integers(0, 4, size=40).astype(np.int32)
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    assert wsout["counters"][0] == 40 and wsout["counters"][1] == 4960
    dropped = np.ones(5000, dtype=bool)
    dropped[keep] = False
    assert not y[dropped].any()
    _check_layer(w, idx, x, y, wsout, sorted(int(t) for t in keep))


def test_dispatch_many_tokens(gpu):
    """100 000 tokens on 2048 experts, Zipf-like crowding: the single-workgroup dispatch at scale."""
    rng = np.random.default_rng(9)
    E, T = 2048, 100_000
    idx = np.minimum((rng.pareto(1.1, T) * 3).astype(np.int64), E - 1).astype(np.int32)
    dd = dev.DeviceDict(device=gpu)
    ws = torch.empty(q.qmoe_moe_layer_workspace(E, 64, 128, T), dtype=torch.uint8, device=gpu)
    q.qmoe_moe_dispatch(dd.handle, 1, torch.from_numpy(idx).to(gpu), E, 64, 128, ws)
    torch.cuda.synchronize()
    got = dev.read_workspace(ws, E, 64, 128, T)
    tok_off, perm = oracle.dispatch(idx, E)
    assert np.array_equal(got["tok_off"], tok_off) and np.array_equal(got["perm"], perm)
    counts = np.diff(tok_off)
    n_mm = got["counters"][7]
    assert n_mm == int(sum((c + 63) // 64 for c in counts if c >= 8))
    covered = np.zeros(T, dtype=np.int32)
    for items, n in ((got["items_mm"], n_mm), (got["items_wi"], got["counters"][3])):
        for e, slot0, ntok, _ in items[:n]:
            covered[slot0:slot0 + ntok] += 1
    assert np.all(covered == 1)
    dd.close()


def test_layer_single_token(gpu, ddict, oracle_dict):
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=3, d_model=770, d_ff=130, n_tokens=1)
    idx, x = w.expert_idx(), w.tokens()
    layer = _build_layer(w, oracle_dict, gpu)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    _check_layer(w, idx, x, y, wsout, [0])


def test_switch_base128_layer_full_size(gpu, ddict, oracle_dict):
    """128 experts of 3072x768 / 768x3072, 128 tokens routed uniformly: every token checked."""
    w = synth.WORKLOADS["switch_base128"]
    idx, x = w.expert_idx(), w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, experts=sorted(set(idx.tolist())), order_of=ddict)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    assert np.isfinite(y).all()
    _check_layer(w, idx, x, y, wsout, list(range(idx.size)))


def test_switch_large128_layer_full_size(gpu, ddict, oracle_dict):
    """128 experts, d_model 1024, d_ff 4096, 512 tokens: every 8th token checked against the oracle."""
    w = synth.WORKLOADS["switch_large128"]
    idx, x = w.expert_idx(), w.tokens()
    lib_dict = q.qmoe_dict_create()
    layer = _build_layer(w, oracle_dict, gpu, encoder="library", lib_dict=lib_dict, order_of=ddict)
    q.qmoe_dict_destroy(lib_dict)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    assert np.isfinite(y).all()
    _check_layer(w, idx, x, y, wsout, list(range(0, idx.size, 8)))


def test_switch_large128_interchange_numbering(gpu, ddict, oracle_dict):
    """The same layer with the streams left as encoded (table head in LDS, the rest from L2)."""
    w = synth.WORKLOADS["switch_large128"].scaled(n_experts=16, n_tokens=64)
    idx, x = w.expert_idx(), w.tokens()
    layer = _build_layer(w, oracle_dict, gpu)
    q.qmoe_set_tuning("lds_dict_entries", 20000)  # force the LDS head even for this small layer
    try:
        y, wsout = _run_layer(layer, ddict, x, idx, gpu)
    finally:
        q.qmoe_set_tuning("lds_dict_entries", 0)
    _check_layer(w, idx, x, y, wsout, list(range(0, idx.size, 2)))


def test_bf16_comparator_close_to_the_compressed_layer(gpu, ddict, oracle_dict):
    """The uncompressed comparator multiplies bf16-rounded (scale * ternary) weights, so it can
    only agree to bf16 precision; a wrong dispatch or a wrong row would show as an O(1) error."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=6, d_model=136, d_ff=264, n_tokens=40)
    idx, x = w.expert_idx(), w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    y, _ = _run_layer(layer, ddict, x, idx, gpu)
    wi_ptr, wo_ptr, keep = np.zeros(6, dtype=np.int64), np.zeros(6, dtype=np.int64), []
    for e in range(6):
        for which, tern, scale, arr in (("wi", w.wi_ternary(e), w.wi_scale(e), wi_ptr),
                                        ("wo", w.wo_ternary(e), w.wo_scale(e), wo_ptr)):
            dense = torch.from_numpy(tern.astype(np.float32) * synth.f16_to_f64(scale).astype(np.float32)[:, None])
            dense = dense.to(torch.bfloat16).to(gpu).contiguous()
            keep.append(dense)
            arr[e] = dense.data_ptr()
    y2 = torch.full((idx.size, w.d_model), float("nan"), dtype=torch.float32, device=gpu)
    ws = layer.workspace(idx.size)
    q.qmoe_bf16_layer_forward(torch.from_numpy(wi_ptr).to(gpu), torch.from_numpy(wo_ptr).to(gpu), 6, w.d_model,
                              w.d_ff, _to_dev16(x, gpu), torch.from_numpy(idx).to(gpu), None, y2, ws)
    torch.cuda.synchronize()
    y2 = y2.cpu().numpy()
    assert np.isfinite(y2).all()
    assert np.linalg.norm(y2 - y) / np.linalg.norm(y) < 2e-2


# ---------------------------------------------------------------------------
# Full-size workloads in the launch configuration bench.py times: the library's
# own dictionary and encoder, device-order streams, sampled tokens checked one
# by one against the oracle (which regenerates and multiplies the expert densely).

def _full_layer(w, gpu, minmax=False, lanes_for_tokens=0):
    """minmax: the same streams on the asymmetric grid (bf16 pairs in place of the scales);
    lanes_for_tokens: the streams re-packed into the lane-interleaved layout."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    dd = dev.DeviceDict(device=gpu)
    layer = dev.DeviceLayer(w.n_experts, w.d_model, w.d_ff, gpu, minmax=minmax)
    q.qmoe_set_tuning("host_threads", 1)

    def one(e):
        out = []
        for which, tern, scale in (("wi", w.wi_ternary(e), w.wi_minmax(e) if minmax else w.wi_scale(e)),
                                   ("wo", w.wo_ternary(e), w.wo_minmax(e) if minmax else w.wo_scale(e))):
            codes, row_off = q.qmoe_encode_host(dd.handle, tern)
            out.append((which, codes, row_off, scale))
        return e, out

    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
        for e, parts in pool.map(one, range(w.n_experts)):
            for which, codes, row_off, scale in parts:
                layer.set_expert(e, which, codes, row_off, scale)
    q.qmoe_set_tuning("host_threads", 0)
    return dd, layer.finalize(device_order_of=dd, lanes_for_tokens=lanes_for_tokens)


def _sample_tokens(idx, n_experts, per_class=4):
    """Tokens from experts with 1 token, a few tokens, and the most tokens."""
    counts = np.bincount(idx, minlength=n_experts)
    order = np.argsort(-counts, kind="stable")
    picks = []
    busiest = [int(e) for e in order[:2]]
    singles = [int(e) for e in np.nonzero(counts == 1)[0][:per_class]]
    middle = [int(e) for e in np.nonzero((counts >= 3) & (counts <= 12))[0][:per_class]]
    for e in busiest + singles + middle:
        toks = np.nonzero(idx == e)[0]
        picks.extend(int(t) for t in toks[:: max(1, toks.size // 3)][:3])
    return sorted(set(picks))


def test_c2048_layer_full_size_sampled(gpu, oracle_dict):
    """2048 experts 2080 x 6144, 2048 tokens, Zipf routing: the benchmark's workload."""
    w = synth.WORKLOADS["c2048"]
    idx, x = w.expert_idx(), w.tokens()
    dd, layer = _full_layer(w, gpu)
    # the library's encoder must have produced the oracle's stream (checked on two experts)
    for e in (int(idx[0]), int(idx[-1])):
        oc, oro = oracle.encode(oracle_dict, w.wo_ternary(e))
        assert layer.n_codes["wo"][e] == oc.size
    y, wsout = _run_layer(layer, dd, x, idx, gpu)
    assert np.isfinite(y).all()
    counts = np.bincount(idx, minlength=w.n_experts)
    assert wsout["counters"][2] == int((counts > 0).sum()) and wsout["counters"][0] == idx.size
    _check_layer(w, idx, x, y, wsout, _sample_tokens(idx, w.n_experts))
    y2, _ = _run_layer(layer, dd, x, idx, gpu)
    assert np.array_equal(y, y2)  # run-to-run bitwise identical
    dd.close()


# ---------------------------------------------------------------- the lane-interleaved layout
#
# Same codewords, re-packed when the layer is loaded so that the 64 loads of a wavefront of the
# scalar kernel are one run of memory; every kernel of a layer call and the decompression read it.

@pytest.mark.parametrize("d_model,d_ff,tokens", [(96, 200, 70), (260, 300, 70), (450, 228, 9), (136, 600, 40)])
def test_small_layer_lane_interleaved_every_token(gpu, ddict, oracle_dict, d_model, d_ff, tokens):
    """Rows on both sides of 224 columns, fewer rows than lanes, lanes with unequal row counts; tiles of one to
    four tokens and (second call) the matrix-core kernel; the answers equal those of the plain layout bit for bit."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=12, d_model=d_model, d_ff=d_ff, n_tokens=tokens)
    idx, x = w.expert_idx(), w.tokens()
    idx[5: 5 + tokens // 2] = 3  # one expert with many tokens
    idx[idx == 7] = 8            # at least one expert without tokens
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict, lanes_for_tokens=tokens)
    plain = _build_layer(w, oracle_dict, gpu, order_of=ddict)
    assert layer.lanes["wi"] % 64 == 0 and layer.lanes["wo"] % 64 == 0 and layer.format >> 8
    gate = np.random.default_rng(7).uniform(0.2, 1.0, idx.size)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
    _check_layer(w, idx, x, y, wsout, list(range(idx.size)), gate)
    y_plain, _ = _run_layer(plain, ddict, x, idx, gpu, gate)
    assert np.array_equal(y, y_plain)
    q.qmoe_set_tuning("mfma_min_tokens", 8)
    try:
        y2, ws2 = _run_layer(layer, ddict, x, idx, gpu, gate)
        assert (ws2["counters"][7] >= 1) == (d_model % 8 == 0 and d_ff % 8 == 0 and tokens >= 16)
        _check_layer(w, idx, x, y2, ws2, list(range(idx.size)), gate)
        y2_plain, _ = _run_layer(plain, ddict, x, idx, gpu, gate)
        assert np.array_equal(y2, y2_plain)
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)
    # decompression reads the layout too
    out = torch.zeros((w.n_experts, w.d_ff, w.d_model), dtype=torch.int8, device=gpu) if d_model % 8 == 0 else None
    if out is not None:
        ptrs = torch.tensor([out[e].data_ptr() for e in range(w.n_experts)], dtype=torch.int64, device=gpu)
        q.qmoe_decompress(ddict.handle, layer.desc_dev["wi"], layer.format, w.n_experts, w.d_ff, w.d_model, 0, ptrs)
        torch.cuda.synchronize()
        for e in range(w.n_experts):
            assert np.array_equal(out[e].cpu().numpy(), w.wi_ternary(e))
    # a single-matrix call refuses the layout; a layer call refuses lane counts its launch cannot take
    with pytest.raises(q.QmoeError):
        q.qmoe_decode_matvec(ddict.handle, layer.desc_host["wi"][0], _to_dev16(x[:1], gpu),
                             torch.empty((1, d_ff), dtype=torch.float32, device=gpu))
    with pytest.raises(q.QmoeError):
        q.qmoe_moe_layer_forward(ddict.handle, layer.desc_dev["wi"], layer.desc_dev["wo"], 1 | q.format_lanes(64, 0),
                                 w.n_experts, d_model, d_ff, _to_dev16(x, gpu), torch.from_numpy(idx).to(gpu), None,
                                 torch.empty((idx.size, d_model), dtype=torch.float32, device=gpu),
                                 layer.workspace(idx.size))
    torch.cuda.synchronize()


def test_c2048_lane_interleaved_full_size_sampled(gpu, oracle_dict):
    """The benchmark's layer in the lane-interleaved layout: sampled tokens against the oracle, and the
    padding of the layout stays small."""
    w = synth.WORKLOADS["c2048"]
    idx, x = w.expert_idx(), w.tokens()
    dd, layer = _full_layer(w, gpu, lanes_for_tokens=idx.size)
    y, wsout = _run_layer(layer, dd, x, idx, gpu)
    assert np.isfinite(y).all()
    _check_layer(w, idx, x, y, wsout, _sample_tokens(idx, w.n_experts))
    # every token of the busiest expert (several tiles of the matrix-core kernel, the last one partial)
    counts = np.bincount(idx, minlength=w.n_experts)
    busiest = int(np.argmax(counts))
    assert counts[busiest] > 128
    _check_layer(w, idx, x, y, wsout, [int(t) for t in np.nonzero(idx == busiest)[0]])
    e = int(idx[0])
    oc, _ = oracle.encode(oracle_dict, w.wo_ternary(e))
    assert oc.size <= layer.n_codes["wo"][e] <= 1.06 * oc.size  # padding of the layout: a few per cent
    dd.close()


def test_c2048_ragged_layer_full_size_sampled(gpu, oracle_dict):
    """256 experts, 1-32 tokens each, per-row zero fraction 0.80-0.97."""
    w = synth.WORKLOADS["c2048_ragged256"]
    idx, x = w.expert_idx(), w.tokens()
    dd, layer = _full_layer(w, gpu)
    y, wsout = _run_layer(layer, dd, x, idx, gpu)
    assert np.isfinite(y).all()
    _check_layer(w, idx, x, y, wsout, _sample_tokens(idx, w.n_experts, per_class=3))
    dd.close()


# ---------------------------------------------------------------- the asymmetric grid {w_min, 0, w_max}
#
# Same streams, one bf16 (w_min, w_max) pair per row in place of the scale; the oracle multiplies
# with the dequantised matrix.  The bound is |w_max| * sum |x under +1| + |w_min| * sum |x under -1|.

@pytest.mark.parametrize("rows,cols,p0,seed", [SHAPES[0], SHAPES[1], SHAPES[2], SHAPES[3], SHAPES[5], SHAPES[6]])
@pytest.mark.parametrize("batch", [1, 3, 8, 19])
@pytest.mark.parametrize("order", [0, 1])
def test_decode_matvec_minmax_against_oracle(gpu, ddict, oracle_dict, rows, cols, p0, seed, batch, order):
    tern = synth.ternary(seed, rows, cols, p0)
    mm = synth.minmax_bf16(seed + 3000, rows, 0.01, 0.1)
    x = synth.normal_bf16(seed + 2000, (batch, cols))
    M = _upload(oracle_dict, tern, None, gpu, ddict if order else None, minmax=mm)
    y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
    q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
    torch.cuda.synchronize()
    y_ref, bound = oracle.matvec(tern, None, x, with_bound=True, minmax_bf16=mm)
    _check_product(y.cpu().numpy(), y_ref, bound, f"{rows}x{cols} batch {batch}")


def test_matvec_minmax_integer_inputs_are_exact(gpu, ddict, oracle_dict):
    """Small integers and grid points that are small multiples of 1/4, of either sign: every partial
    sum is exact in fp32, so a swapped pair, a wrong sign or a dropped term shows as a wrong integer."""
    rows, cols = 64, 280
    tern = synth.ternary(312, rows, cols, 0.85)
    rng = np.random.default_rng(2)
    w_min = rng.integers(-6, 3, rows) * 0.25
    w_max = rng.integers(-1, 7, rows) * 0.25
    mm = np.stack([synth.f64_to_bf16(w_min), synth.f64_to_bf16(w_max)], axis=1)
    xi = rng.integers(-4, 5, (5, cols)).astype(np.float32)
    x = torch.from_numpy(xi).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    for order in (None, ddict):
        M = _upload(oracle_dict, tern, None, gpu, order, minmax=mm)
        y = torch.empty((5, rows), dtype=torch.float32, device=gpu)
        q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
        torch.cuda.synchronize()
        assert np.array_equal(y.cpu().numpy().astype(np.float64), oracle.matvec(tern, None, x, minmax_bf16=mm))


@pytest.mark.parametrize("d_model,d_ff,order", [(96, 200, 0), (96, 200, 1), (260, 300, 1), (450, 228, 0)])
def test_small_layer_minmax_every_token(gpu, ddict, oracle_dict, d_model, d_ff, order):
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=12, d_model=d_model, d_ff=d_ff, n_tokens=70)
    idx, x = w.expert_idx(), w.tokens()
    idx[5:40] = 3      # one expert with many tokens (several tiles)
    idx[idx == 7] = 8  # at least one expert without tokens
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict if order else None, minmax=True)
    gate = np.random.default_rng(7).uniform(0.2, 1.0, idx.size)
    y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
    _check_layer(w, idx, x, y, wsout, list(range(idx.size)), gate, asym=True)
    y2, _ = _run_layer(layer, ddict, x, idx, gpu, gate)
    assert np.array_equal(y, y2)
    # the pairs really are in use: the symmetric layer gives other numbers
    sym = oracle.moe_layer(w, idx, x, gate=gate, tokens=[0])[0][0]
    assert not np.allclose(y[0], sym, rtol=1e-2)
    # tiles of one, two and eight tokens as well
    for tile in (1, 2, 8):
        q.qmoe_set_tuning("token_tile", tile)
        try:
            yt, wst = _run_layer(layer, ddict, x, idx, gpu, gate)
        finally:
            q.qmoe_set_tuning("token_tile", 0)
        _check_layer(w, idx, x, yt, wst, list(range(idx.size)), gate, asym=True)


@pytest.mark.parametrize("d_model,d_ff", [(136, 600), (520, 72)])
def test_crowded_experts_minmax_on_the_matrix_cores(gpu, ddict, oracle_dict, d_model, d_ff):
    counts = [130, 65, 64, 33, 32, 31, 8, 7, 1, 0]
    idx = np.concatenate([np.full(n, e, dtype=np.int32) for e, n in enumerate(counts)])
    np.random.default_rng(11).shuffle(idx)
    idx = np.concatenate([idx, np.array([-1], dtype=np.int32)])
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=len(counts), d_model=d_model, d_ff=d_ff,
                                                 n_tokens=idx.size)
    x = w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict, minmax=True)
    gate = np.random.default_rng(12).uniform(0.2, 1.0, idx.size)
    good = [t for t in range(idx.size) if idx[t] >= 0]
    for min_tokens, n_mm in ((8, 10), (2, 11), (-1, 0)):
        q.qmoe_set_tuning("mfma_min_tokens", min_tokens)
        try:
            y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
            y_again, _ = _run_layer(layer, ddict, x, idx, gpu, gate)
        finally:
            q.qmoe_set_tuning("mfma_min_tokens", 0)
        assert wsout["counters"][7] == n_mm
        assert not y[-1].any() and np.array_equal(y, y_again)
        _check_layer(w, idx, x, y, wsout, good, gate, asym=True)


@pytest.mark.parametrize("d_model,d_ff", [(136, 600), (1024, 72)])
def test_decompress_minmax_bit_exact(gpu, ddict, oracle_dict, d_model, d_ff):
    """bf16 output on the asymmetric grid is the row's own w_max / w_min / 0, bit for bit; int8 output
    does not depend on the grid."""
    w = synth.WORKLOADS["c2048_ragged256"].scaled(n_experts=4, d_model=d_model, d_ff=d_ff, n_tokens=8)
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict, minmax=True)
    for which, rows, cols in (("wi", d_ff, d_model), ("wo", d_model, d_ff)):
        for kind, dt in ((0, torch.int8), (1, torch.int16)):
            outs = [torch.full((rows, cols), 77, dtype=dt, device=gpu) for _ in range(w.n_experts)]
            ptrs = torch.tensor([o.data_ptr() for o in outs], dtype=torch.int64, device=gpu)
            q.qmoe_decompress(ddict.handle, layer.desc_dev[which], layer.format, w.n_experts, rows, cols, kind, ptrs)
            torch.cuda.synchronize()
            for e in range(w.n_experts):
                tern = w.wi_ternary(e) if which == "wi" else w.wo_ternary(e)
                mm = w.wi_minmax(e) if which == "wi" else w.wo_minmax(e)
                got = outs[e].cpu().numpy()
                if kind == 0:
                    assert np.array_equal(got, tern), f"{which} expert {e}"
                else:
                    want = np.where(tern == 0, np.uint16(0), np.where(tern > 0, mm[:, 1:2], mm[:, 0:1]))
                    assert np.array_equal(got.view(np.uint16), want.astype(np.uint16)), f"{which} expert {e}"


def test_minmax_format_errors(gpu, ddict, oracle_dict):
    tern = synth.ternary(5, 8, 30, 0.8)
    mm = synth.minmax_bf16(6, 8, 0.01, 0.1)
    M = _upload(oracle_dict, tern, None, gpu, None, minmax=mm)
    x = _to_dev16(synth.normal_bf16(7, (1, 30)), gpu)
    y = torch.empty((1, 8), dtype=torch.float32, device=gpu)
    bad = q.qmoe_matrix(M.desc.codes, M.desc.row_off, None, 8, 30, M.desc.n_codes, 0, M.desc.minmax_bf16 + 2)
    with pytest.raises(q.QmoeError):  # pairs are read as one 32-bit word
        q.qmoe_decode_matvec(ddict.handle, bad, x, y)
    neither = q.qmoe_matrix(M.desc.codes, M.desc.row_off, None, 8, 30, M.desc.n_codes, 0, None)
    with pytest.raises(q.QmoeError):
        q.qmoe_decode_matvec(ddict.handle, neither, x, y)
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=2, d_model=32, d_ff=64, n_tokens=4)
    layer = _build_layer(w, oracle_dict, gpu, minmax=True)
    yl = torch.empty((4, 32), dtype=torch.float32, device=gpu)
    with pytest.raises(q.QmoeError):  # unknown format bit
        q.qmoe_moe_layer_forward(ddict.handle, layer.desc_dev["wi"], layer.desc_dev["wo"], 4, 2, 32, 64,
                                 _to_dev16(w.tokens(), gpu), torch.from_numpy(w.expert_idx()).to(gpu), None, yl,
                                 layer.workspace(4))
    torch.cuda.synchronize()


def test_c2048_ragged_minmax_full_size_sampled(gpu, oracle_dict):
    """The ragged full-size layer on the asymmetric grid: scalar and matrix-core kernels side by side."""
    w = synth.WORKLOADS["c2048_ragged256"]
    idx, x = w.expert_idx(), w.tokens()
    dd, layer = _full_layer(w, gpu, minmax=True)
    y, wsout = _run_layer(layer, dd, x, idx, gpu)
    assert np.isfinite(y).all()
    assert wsout["counters"][7] > 0  # crowded experts went to the matrix cores
    _check_layer(w, idx, x, y, wsout, _sample_tokens(idx, w.n_experts, per_class=3), asym=True)
    dd.close()


@pytest.mark.parametrize("minmax", [False, True])
def test_layer_at_the_densest_natural_sparsity(gpu, ddict, oracle_dict, minmax):
    """76.5 % zeros (the paper's natural sparsity of its 2-bit c2048 model): more than twice the codewords
    per row of the 90 % workloads, most entries with two or three non-zeros.  Scalar kernel, then the
    matrix-core kernel for every expert with two tokens or more."""
    counts = [70, 33, 9, 4, 2, 1, 1, 0]
    idx = np.concatenate([np.full(n, e, dtype=np.int32) for e, n in enumerate(counts)])
    np.random.default_rng(21).shuffle(idx)
    w = synth.WORKLOADS["c2048_sparsity765"].scaled(n_experts=len(counts), d_model=264, d_ff=520, n_tokens=idx.size)
    assert abs((w.wi_ternary(0) == 0).mean() - 0.765) < 0.01
    x = w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict, minmax=minmax)
    for min_tokens in (-1, 2):
        q.qmoe_set_tuning("mfma_min_tokens", min_tokens)
        try:
            y, wsout = _run_layer(layer, ddict, x, idx, gpu)
        finally:
            q.qmoe_set_tuning("mfma_min_tokens", 0)
        assert (wsout["counters"][7] > 0) == (min_tokens == 2)
        _check_layer(w, idx, x, y, wsout, list(range(idx.size)), asym=minmax)


@pytest.mark.parametrize("rows,cols,p0,seed", [(3072, 768, 0.90, 401), (200, 2080, 0.885, 402), (70, 6144, 0.97, 403),
                                               (1000, 136, 0.80, 404)])
@pytest.mark.parametrize("batch", [64, 65, 200])
@pytest.mark.parametrize("minmax", [False, True])
def test_decode_matvec_large_batch_on_the_matrix_cores(gpu, ddict, oracle_dict, rows, cols, p0, seed, batch, minmax):
    """A device-order matrix with many tokens goes through the matrix-core kernel (tiles of 64 tokens
    made up by the kernel itself, row blocks as small as fit the GPU in one round; forced here from 64
    tokens on, by default a cost estimate decides); with the matrix cores switched off the
    16-lanes-per-row kernel must give the same numbers to the tolerance."""
    tern = synth.ternary(seed, rows, cols, p0)
    scale = None if minmax else synth.uniform_f16(seed + 1000, (rows,), 0.01, 0.1)
    mm = synth.minmax_bf16(seed + 3000, rows, 0.01, 0.1) if minmax else None
    x = synth.normal_bf16(seed + 2000, (batch, cols))
    M = _upload(oracle_dict, tern, scale, gpu, ddict, minmax=mm)
    y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True, minmax_bf16=mm)
    xd = _to_dev16(x, gpu)
    for setting in (64, -1):
        q.qmoe_set_tuning("mfma_min_tokens", setting)
        try:
            y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
            q.qmoe_decode_matvec(ddict.handle, M.desc, xd, y)
            torch.cuda.synchronize()
        finally:
            q.qmoe_set_tuning("mfma_min_tokens", 0)
        _check_product(y.cpu().numpy(), y_ref, bound, f"{rows}x{cols} batch {batch} setting {setting}")
    # a small batch forced onto the matrix cores, and an activation pointer that is not 16-byte
    # aligned (falls back to the other kernel): same answers
    q.qmoe_set_tuning("mfma_min_tokens", 2)
    try:
        y = torch.full((5, rows), float("nan"), dtype=torch.float32, device=gpu)
        q.qmoe_decode_matvec(ddict.handle, M.desc, xd[:5], y)
        shifted = torch.empty(batch * cols + 1, dtype=torch.int16, device=gpu)
        shifted[1:] = xd.reshape(-1)
        y_un = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
        q.qmoe_decode_matvec(ddict.handle, M.desc, shifted[1:].view(batch, cols), y_un)
        torch.cuda.synchronize()
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)
    _check_product(y.cpu().numpy(), y_ref[:5], bound[:5], "forced small batch")
    _check_product(y_un.cpu().numpy(), y_ref, bound, "unaligned activations")


# ---------------------------------------------------------------- widest inputs the kernels take
#
# The activations of a tile sit in LDS (160 KB), 8 bytes per column for up to four tokens, next to
# the table when the stream uses the device numbering; beyond that the calls refuse (LIMIT).

@pytest.mark.parametrize("order", [0, 1])
def test_decode_matvec_at_the_widest_row(gpu, ddict, oracle_dict, order):
    rows, cols = 24, 20448
    tern = synth.ternary(501, rows, cols, 0.93)
    scale = synth.uniform_f16(502, (rows,), 0.01, 0.1)
    M = _upload(oracle_dict, tern, scale, gpu, ddict if order else None)
    for batch in (1, 6):  # six tokens: a tile of eight does not fit, tiles of four do
        x = synth.normal_bf16(503 + batch, (batch, cols))
        y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
        q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
        torch.cuda.synchronize()
        y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True)
        _check_product(y.cpu().numpy(), y_ref, bound, f"batch {batch}")
    # two columns more: refused, nothing launched
    wide = q.qmoe_matrix(M.desc.codes, M.desc.row_off, M.desc.scale_f16, rows, cols + 2, M.desc.n_codes, order, None)
    xw = torch.zeros((1, cols + 2), dtype=torch.int16, device=gpu)
    yw = torch.zeros((1, rows), dtype=torch.float32, device=gpu)
    with pytest.raises(q.QmoeError) as ei:
        q.qmoe_decode_matvec(ddict.handle, wide, xw, yw)
    assert ei.value.status == -10


@pytest.mark.parametrize("order,d_ff,ok", [(1, 10016, True), (1, 10080, True), (1, 20400, True), (1, 20480, False),
                                           (0, 20400, True), (0, 20480, False)])
def test_layer_at_the_widest_hidden_size(gpu, ddict, oracle_dict, order, d_ff, ok):
    """The second product stages d_ff activations per token; with the device numbering the whole table
    shares the LDS with them up to 10022 columns, beyond that it is read from L2."""
    w = synth.WORKLOADS["switch_base128"].scaled(n_experts=3, d_model=64, d_ff=d_ff, n_tokens=7)
    idx, x = w.expert_idx(), w.tokens()
    layer = _build_layer(w, oracle_dict, gpu, order_of=ddict if order else None)
    if ok:
        y, wsout = _run_layer(layer, ddict, x, idx, gpu)
        _check_layer(w, idx, x, y, wsout, list(range(idx.size)))
    else:
        with pytest.raises(q.QmoeError) as ei:
            _run_layer(layer, ddict, x, idx, gpu)
        assert ei.value.status == -10


def test_decode_matvec_in_a_hip_graph(gpu, ddict, oracle_dict):
    """Both kernels of the single-matrix call (a few tokens; many tokens on the matrix cores) captured into
    one HIP graph and replayed: neither needs anything that a capture forbids."""
    rows, cols = 300, 520
    tern = synth.ternary(601, rows, cols, 0.9)
    scale = synth.uniform_f16(602, (rows,), 0.01, 0.1)
    M = _upload(oracle_dict, tern, scale, gpu, ddict)
    x_few, x_many = synth.normal_bf16(603, (3, cols)), synth.normal_bf16(604, (80, cols))
    d_few, d_many = _to_dev16(x_few, gpu), _to_dev16(x_many, gpu)
    y_few = torch.zeros((3, rows), dtype=torch.float32, device=gpu)
    y_many = torch.zeros((80, rows), dtype=torch.float32, device=gpu)
    q.qmoe_set_tuning("mfma_min_tokens", 64)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            q.qmoe_decode_matvec(ddict.handle, M.desc, d_few, y_few, stream=side.cuda_stream)
            q.qmoe_decode_matvec(ddict.handle, M.desc, d_many, y_many, stream=side.cuda_stream)
            torch.cuda.synchronize()
            eager = (y_few.clone(), y_many.clone())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                q.qmoe_decode_matvec(ddict.handle, M.desc, d_few, y_few, stream=side.cuda_stream)
                q.qmoe_decode_matvec(ddict.handle, M.desc, d_many, y_many, stream=side.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            y_few.fill_(float("nan"))
            y_many.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y_few, eager[0]) and torch.equal(y_many, eager[1]), f"replay {rep}"
            (y_many * 2).sum().item()
    finally:
        q.qmoe_set_tuning("mfma_min_tokens", 0)
    for y, x in ((y_few, x_few), (y_many, x_many)):
        y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True)
        _check_product(y.cpu().numpy(), y_ref, bound, f"batch {x.shape[0]}")


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_layer_shapes(gpu, ddict, oracle_dict, seed):
    """Seeded random layer calls inside the documented limits: expert counts, widths (multiples of 2, 8 and 64),
    token counts on both sides of every tile size and of the call size that switches the matrix-core kernel on,
    both numberings, both stream layouts, both grids, skewed routing, a token without an expert.  Outputs of up
    to 24 tokens a case against the oracle; the same layer decompressed (when its format allows) bit for bit,
    destinations at different 16-byte offsets, nothing written outside them."""
    rng = np.random.default_rng(seed)
    for case in range(14):
        E = int(rng.choice([1, 2, 5, 12, 33, 130]))
        mult = int(rng.choice([2, 8, 8, 8, 64]))
        big = rng.integers(0, 8) == 0
        d_model = mult * int(rng.integers(max(1, 40 // mult), (2200 if big else 600) // mult))
        d_ff = mult * int(rng.integers(max(1, 40 // mult), (3300 if big else 900) // mult))
        T = int(rng.choice([1, 2, 3, 8, 17, 64, 65, 70, 129, 300, 1024, 1030, 1300, 2100]))
        order = int(rng.integers(0, 2))
        lanes = bool(order and rng.integers(0, 2))
        minmax = bool(rng.integers(0, 3) == 0)
        skew = bool(rng.integers(0, 2))
        label = f"seed {seed} case {case}: E={E} d_model={d_model} d_ff={d_ff} T={T} order={order} lanes={lanes} minmax={minmax}"
        print(label, flush=True)
        w = synth.WORKLOADS["switch_base128"].scaled(n_experts=E, d_model=d_model, d_ff=d_ff, n_tokens=T)
        idx, x = w.expert_idx(), w.tokens()
        if skew and E > 1:
            idx[: T // 2] = int(rng.integers(0, E))
        if T > 5:
            idx[int(rng.integers(0, T))] = -1 if rng.integers(0, 2) else E + 3
        if lanes and min(q.qmoe_plan_lanes(ddict.handle, d_ff, d_model, E, T),
                         q.qmoe_plan_lanes(ddict.handle, d_model, d_ff, E, T)) <= 0:
            lanes = False
        layer = _build_layer(w, oracle_dict, gpu, order_of=ddict if order else None, minmax=minmax,
                             lanes_for_tokens=T if lanes else 0)
        gate = rng.uniform(0.2, 1.0, idx.size)
        y, wsout = _run_layer(layer, ddict, x, idx, gpu, gate)
        valid = [t for t in range(T) if 0 <= idx[t] < E]
        pick = valid if len(valid) <= 24 else [int(v) for v in rng.choice(valid, 24, replace=False)]
        _check_layer(w, idx, x, y, wsout, pick, gate, asym=minmax)
        for t in range(T):
            if not 0 <= idx[t] < E:
                assert np.all(y[t] == 0.0), f"{label}: dropped token {t} not zeroed"
        if not (order and not minmax and d_model % 8 == 0 and d_ff % 8 == 0 and E <= 33 and d_model * d_ff <= 600000):
            continue
        for which, rows, cols in (("wi", d_ff, d_model), ("wo", d_model, d_ff)):
            kind = int(rng.integers(0, 2))
            skip = int(rng.integers(0, E + 1))  # E: none skipped
            span = rows * cols + 256
            pool = torch.full((E * span,), 77, dtype=torch.int8 if kind == 0 else torch.int16, device=gpu)
            offs = [e * span + 8 * int(rng.integers(0, 8)) * (2 if kind == 0 else 1) for e in range(E)]
            ptrs = torch.tensor([0 if e == skip else pool.data_ptr() + offs[e] * pool.element_size() for e in range(E)],
                                dtype=torch.int64, device=gpu)
            q.qmoe_decompress(ddict.handle, layer.desc_dev[which], 1, E, rows, cols, kind, ptrs)
            torch.cuda.synchronize()
            host = pool.cpu().numpy()
            outside = np.ones(host.size, dtype=bool)
            for e in range(E):
                if e == skip:
                    continue
                got = host[offs[e]: offs[e] + rows * cols].reshape(rows, cols)
                outside[offs[e]: offs[e] + rows * cols] = False
                tern = w.wi_ternary(e) if which == "wi" else w.wo_ternary(e)
                if kind == 0:
                    assert np.array_equal(got, tern), f"{label}: {which} expert {e}"
                else:
                    sb = _bf16_bits_of_f16(w.wi_scale(e) if which == "wi" else w.wo_scale(e))[:, None].astype(np.uint16)
                    want = np.where(tern == 0, np.uint16(0), np.where(tern > 0, sb, sb | np.uint16(0x8000)))
                    assert np.array_equal(got.view(np.uint16), want.astype(np.uint16)), f"{label}: {which} expert {e}"
            assert (host[outside] == 77).all(), f"{label}: {which} written outside the destinations"


@pytest.mark.parametrize("seed", [21, 22])
def test_random_single_matrix_shapes(gpu, ddict, oracle_dict, seed):
    """Seeded random single-matrix calls: 1..2200 rows, 2..6200 columns, zero fractions from 0 to 1, batches on
    both sides of the tile sizes and of the switch to the matrix-core kernel, both numberings, both grids: the
    product against the oracle and the decoded matrix bit for bit."""
    rng = np.random.default_rng(seed)
    for case in range(40):
        mult = int(rng.choice([2, 8, 8, 64]))
        big = rng.integers(0, 6) == 0
        rows = int(rng.integers(1, 2200 if big else 400))
        cols = mult * int(rng.integers(1, (6200 if big else 900) // mult))
        p0 = float(rng.choice([0.0, 0.5, 0.8, 0.885, 0.9, 0.97, 1.0]))
        batch = int(rng.choice([1, 2, 3, 4, 5, 8, 9, 33, 64, 65, 200, 513]))
        order = int(rng.integers(0, 2))
        minmax = bool(rng.integers(0, 3) == 0)
        label = f"seed {seed} case {case}: {rows}x{cols} p0={p0} batch={batch} order={order} minmax={minmax}"
        print(label, flush=True)
        s = 1000 * seed + case
        tern = synth.ternary(s, rows, cols, p0)
        scale = None if minmax else synth.uniform_f16(s + 1, (rows,), 0.01, 0.1)
        pairs = synth.minmax_bf16(s + 2, rows, 0.01, 0.1) if minmax else None
        M = _upload(oracle_dict, tern, scale, gpu, order_of=ddict if order else None, minmax=pairs)
        x = synth.normal_bf16(s + 3, (batch, cols))
        y = torch.full((batch, rows), float("nan"), dtype=torch.float32, device=gpu)
        q.qmoe_decode_matvec(ddict.handle, M.desc, _to_dev16(x, gpu), y)
        torch.cuda.synchronize()
        y_ref, bound = oracle.matvec(tern, scale, x, with_bound=True, minmax_bf16=pairs)
        _check_product(y.cpu().numpy(), y_ref, bound, label)
        out = torch.full((rows, cols), 7, dtype=torch.int8, device=gpu)
        q.qmoe_decode_dense(ddict.handle, M.desc, out, 0)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), tern), label
