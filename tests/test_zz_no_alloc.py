"""The layer entry point that brings no workspace (`qmoe_moe_layer_forward_static`): its
output must equal that of `qmoe_moe_layer_forward` on a caller's workspace, bit for bit (the
same kernels run on the same inputs, only the scratch memory lives elsewhere), on two calls in
a row that share the library's scratch array, the second smaller than the first.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2310_16795_amd as q
from paper_2310_16795_amd import device as dev
from paper_2310_16795_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    if not torch.cuda.is_available():
        pytest.fail("the GPU tests need a GPU: the HIP path has no fallback")
    return "cuda:0"


def _layer(w, od, dd, gpu):
    layer = dev.DeviceLayer(w.n_experts, w.d_model, w.d_ff, gpu)
    for e in range(w.n_experts):
        for which, tern, scale in (("wi", w.wi_ternary(e), w.wi_scale(e)), ("wo", w.wo_ternary(e), w.wo_scale(e))):
            codes, row_off = oracle.encode(od, tern)
            layer.set_expert(e, which, codes, row_off, scale)
    return layer.finalize(device_order_of=dd)


def _both(layer, dd, w, idx, x_bits, gpu, gate=None):
    """-> (y of the static entry point, y of the workspace entry point)"""
    T = idx.size
    x = torch.from_numpy(x_bits.view(np.int16).copy()).to(gpu)
    d_idx = torch.from_numpy(idx).to(gpu)
    g = None if gate is None else torch.from_numpy(gate.astype(np.float32)).to(gpu)
    y_static = torch.full((T, w.d_model), float("nan"), dtype=torch.float32, device=gpu)
    y_ws = torch.full((T, w.d_model), float("nan"), dtype=torch.float32, device=gpu)
    print(f"static layer call: {T} tokens, {w.n_experts} experts {w.d_model}x{w.d_ff}", flush=True)
    layer.forward_static(dd, x, d_idx, y_static, g)
    torch.cuda.synchronize()
    layer.forward(dd, x, d_idx, y_ws, layer.workspace(T), g)
    torch.cuda.synchronize()
    return y_static.cpu().numpy(), y_ws.cpu().numpy()


def test_static_workspace_entry_point_equals_the_workspace_one(gpu, oracle_dict):
    dd = dev.DeviceDict(q.qmoe_dict_from_words(oracle_dict.words), gpu)
    # first call: 300 tokens, one crowded expert (matrix-core kernel) next to experts with few tokens
    w1 = synth.WORKLOADS["switch_base128"].scaled(n_experts=12, d_model=264, d_ff=520, n_tokens=300)
    idx1, x1 = w1.expert_idx(), w1.tokens()
    idx1[20:120] = 3
    idx1[idx1 == 7] = 8  # an expert without tokens
    idx1[5] = -1         # a dropped token: zero row
    layer1 = _layer(w1, oracle_dict, dd, gpu)
    gate = np.random.default_rng(3).uniform(0.2, 1.0, idx1.size)
    a1, b1 = _both(layer1, dd, w1, idx1, x1, gpu, gate)
    assert np.isfinite(b1).all() and np.array_equal(a1, b1)
    assert not a1[5].any()
    # against the oracle as well, on a few tokens
    ref = oracle.moe_layer(w1, idx1, x1, gate=gate, tokens=[0, 21, 299])
    for t in (0, 21, 299):
        y_ref = ref[t][0]
        assert np.linalg.norm(a1[t] - y_ref) <= 1e-3 * np.linalg.norm(y_ref)
    # second call, smaller in every size: it finds the first call's contents in the scratch array
    w2 = synth.WORKLOADS["switch_base128"].scaled(n_experts=5, d_model=96, d_ff=200, n_tokens=23)
    idx2, x2 = w2.expert_idx(), w2.tokens()
    layer2 = _layer(w2, oracle_dict, dd, gpu)
    a2, b2 = _both(layer2, dd, w2, idx2, x2, gpu)
    assert np.isfinite(b2).all() and np.array_equal(a2, b2)
    # and the first one again, after the smaller one
    a3, _ = _both(layer1, dd, w1, idx1, x1, gpu, gate)
    assert np.array_equal(a3, b1)
    # a layer whose workspace would not fit the scratch array is refused before anything is enqueued
    big = q.qmoe_moe_layer_workspace(2048, 2080, 6144, 2048)
    assert big > q.qmoe_static_workspace_bytes()
    assert q.lib().qmoe_moe_layer_forward_static(dd.handle, 256, 256, 1, 2048, 2080, 6144, 256, 256, None, 2048, 256,
                                                 None) == -10
    torch.cuda.synchronize()
    dd.close()
