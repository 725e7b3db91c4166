"""ctypes binding of libqmoe.so: the same entry points as include/qmoe.h.

Argument marshalling only.  Device buffers are torch tensors (PyTorch is used
for device memory and streams, nothing else); every step of the hot path runs
inside the library's kernels.  There is no CPU fallback: if the library is
missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_int, c_int32, c_size_t, c_uint32, c_void_p

import numpy as np

from . import build as _build

_lib = None


class QmoeError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().qmoe_strerror(status).decode()
        if status == -6:
            msg += f" (hipError {lib().qmoe_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{status}]")


class qmoe_matrix(Structure):
    _fields_ = [("codes", c_void_p), ("row_off", c_void_p), ("scale_f16", c_void_p),
                ("rows", c_int32), ("cols", c_int32), ("n_codes", c_uint32), ("code_order", c_uint32),
                ("minmax_bf16", c_void_p), ("wave_off", c_void_p), ("lanes", c_uint32), ("reserved", c_uint32)]


FORMAT_DEVICE_ORDER = 1
FORMAT_GRID_MINMAX = 2


def format_lanes(lanes_wi: int, lanes_wo: int) -> int:
    """QMOE_FORMAT_LANES: the lane counts the lane-interleaved layouts of the two projections were built for."""
    return ((lanes_wi // 64) << 8) | ((lanes_wo // 64) << 16)


class qmoe_ws_layout(Structure):
    _fields_ = [(n, c_size_t) for n in ("tok_off", "perm", "counters", "items_wi", "items_wo", "items_mm", "hidden", "total")]


EXPORTS = [
    "qmoe_strerror", "qmoe_last_hip_error", "qmoe_dict_create", "qmoe_dict_from_words", "qmoe_dict_words",
    "qmoe_dict_max_nonzeros", "qmoe_dict_device_bytes", "qmoe_dict_upload", "qmoe_dict_destroy",
    "qmoe_encode_host", "qmoe_validate_host", "qmoe_decode_matvec", "qmoe_decode_dense",
    "qmoe_moe_layer_ws_layout", "qmoe_moe_layer_workspace", "qmoe_moe_layer_forward", "qmoe_moe_dispatch",
    "qmoe_bf16_layer_forward", "qmoe_set_tuning", "qmoe_stream_copy", "qmoe_dict_device_order",
    "qmoe_codes_to_device_order", "qmoe_decompress", "qmoe_encode_device", "qmoe_hook_set", "qmoe_static_workspace_bytes", "qmoe_moe_layer_forward_static",
    "qmoe_lane_layout_size", "qmoe_lane_layout_build", "qmoe_lane_layout_unpack", "qmoe_plan_lanes",
]


def lib():
    """Load the library.  It is built first when no built copy exists; a copy older than any of
    its sources or headers is refused (run `python paper_2310_16795_amd/build.py`, or
    __graft_entry__.build(), after editing them): figures from a stale binary describe old code."""
    global _lib
    if _lib is None:
        path = os.environ.get("QMOE_LIBRARY")  # another build of the same sources, e.g. one with host sanitizers
        if not path:
            path = _build.LIB
            if not os.path.exists(path):
                _build.build_library()
            elif _build.stale():
                raise RuntimeError(f"{path} was built from other sources than the ones present: rebuild it "
                                   "(python paper_2310_16795_amd/build.py)")
        L = ctypes.CDLL(path)
        vp, sz, i = c_void_p, c_size_t, c_int
        L.qmoe_strerror.argtypes, L.qmoe_strerror.restype = [i], c_char_p
        L.qmoe_last_hip_error.argtypes, L.qmoe_last_hip_error.restype = [], i
        L.qmoe_dict_create.argtypes = [c_double, i, i, POINTER(vp)]
        L.qmoe_dict_from_words.argtypes = [vp, i, POINTER(vp)]
        L.qmoe_dict_words.argtypes = [vp, POINTER(vp), POINTER(i)]
        L.qmoe_dict_max_nonzeros.argtypes = [vp]
        L.qmoe_dict_device_bytes.argtypes, L.qmoe_dict_device_bytes.restype = [], sz
        L.qmoe_dict_upload.argtypes = [vp, vp, sz, vp]
        L.qmoe_dict_destroy.argtypes, L.qmoe_dict_destroy.restype = [vp], None
        L.qmoe_encode_host.argtypes = [vp, vp, i, i, vp, sz, vp, POINTER(sz)]
        L.qmoe_validate_host.argtypes = [vp, vp, vp, i, i]
        L.qmoe_decode_matvec.argtypes = [vp, POINTER(qmoe_matrix), vp, i, vp, vp]
        L.qmoe_decode_dense.argtypes = [vp, POINTER(qmoe_matrix), vp, i, vp]
        L.qmoe_moe_layer_ws_layout.argtypes = [i, i, i, i, POINTER(qmoe_ws_layout)]
        L.qmoe_moe_layer_workspace.argtypes, L.qmoe_moe_layer_workspace.restype = [i, i, i, i], sz
        L.qmoe_moe_layer_forward.argtypes = [vp, vp, vp, i, i, i, i, vp, vp, vp, i, vp, vp, sz, vp, vp]
        L.qmoe_moe_layer_forward_static.argtypes = [vp, vp, vp, i, i, i, i, vp, vp, vp, i, vp, vp]
        L.qmoe_static_workspace_bytes.argtypes, L.qmoe_static_workspace_bytes.restype = [], sz
        L.qmoe_dict_device_order.argtypes = [vp, POINTER(vp), POINTER(vp), POINTER(i), POINTER(i)]
        L.qmoe_codes_to_device_order.argtypes = [vp, vp, sz, vp]
        L.qmoe_moe_dispatch.argtypes = [vp, i, vp, i, i, i, i, vp, sz, vp]
        L.qmoe_decompress.argtypes = [vp, vp, i, i, i, i, i, vp, vp]
        L.qmoe_encode_device.argtypes = [vp, vp, i, i, vp, sz, vp, vp, vp]
        L.qmoe_bf16_layer_forward.argtypes = [vp, vp, i, i, i, vp, vp, vp, i, vp, vp, sz, vp]
        L.qmoe_set_tuning.argtypes = [c_char_p, i]
        L.qmoe_lane_layout_size.argtypes = [vp, i, i, POINTER(sz)]
        L.qmoe_lane_layout_build.argtypes = [vp, vp, i, i, vp, sz, vp]
        L.qmoe_lane_layout_unpack.argtypes = [vp, vp, vp, i, i, vp, sz]
        L.qmoe_plan_lanes.argtypes = [vp, i, i, i, i]
        L.qmoe_hook_set.argtypes = [c_char_p, i]
        L.qmoe_stream_copy.argtypes = [vp, vp, sz, vp]
        _lib = L
    return _lib


def _check(status: int, where: str):
    if status != 0:
        raise QmoeError(status, where)


def _host_ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


def _dev_ptr(t) -> int:
    """Address of a contiguous CUDA/HIP torch tensor (None -> NULL)."""
    if t is None:
        return 0
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


# ------------------------------------------------------------------ dictionary

def qmoe_dict_create(p0: float = 0.885, max_pairs: int = 14, n_entries: int = 65536) -> int:
    h = c_void_p()
    _check(lib().qmoe_dict_create(p0, max_pairs, n_entries, byref(h)), "qmoe_dict_create")
    return h.value


def qmoe_dict_from_words(words: np.ndarray) -> int:
    w = np.ascontiguousarray(words, dtype=np.uint32)
    assert w.ndim == 2 and w.shape[1] == 2
    h = c_void_p()
    _check(lib().qmoe_dict_from_words(_host_ptr(w), w.shape[0], byref(h)), "qmoe_dict_from_words")
    return h.value


def qmoe_dict_words(d: int) -> np.ndarray:
    p, n = c_void_p(), c_int()
    _check(lib().qmoe_dict_words(d, byref(p), byref(n)), "qmoe_dict_words")
    buf = (c_uint32 * (2 * n.value)).from_address(p.value)
    return np.frombuffer(buf, dtype=np.uint32).reshape(n.value, 2).copy()


def qmoe_dict_max_nonzeros(d: int) -> int:
    return lib().qmoe_dict_max_nonzeros(d)


def qmoe_dict_device_bytes() -> int:
    return lib().qmoe_dict_device_bytes()


def qmoe_dict_device_order(d: int):
    """-> (code_map uint16 [65536], table uint32 [n_table], n_groups), or (None, None, 0)"""
    m, t, g, n = c_void_p(), c_void_p(), c_int(), c_int()
    _check(lib().qmoe_dict_device_order(d, byref(m), byref(t), byref(g), byref(n)), "qmoe_dict_device_order")
    if not n.value:
        return None, None, 0
    cm = np.frombuffer((ctypes.c_uint16 * 65536).from_address(m.value), dtype=np.uint16).copy()
    tb = np.frombuffer((c_uint32 * n.value).from_address(t.value), dtype=np.uint32).copy()
    return cm, tb, g.value


def qmoe_codes_to_device_order(d: int, codes_dev, stream=None) -> None:
    """Renumber a device tensor of 16-bit codewords in place."""
    if codes_dev.element_size() != 2:
        raise ValueError("16-bit codewords expected")
    _check(lib().qmoe_codes_to_device_order(d, _dev_ptr(codes_dev), codes_dev.numel(), _stream_ptr(stream)),
           "qmoe_codes_to_device_order")


def qmoe_dict_upload(d: int, dev_buf, stream=None) -> None:
    _check(lib().qmoe_dict_upload(d, _dev_ptr(dev_buf), dev_buf.numel() * dev_buf.element_size(),
                                  _stream_ptr(stream)), "qmoe_dict_upload")


def qmoe_dict_destroy(d: int) -> None:
    lib().qmoe_dict_destroy(d)


# ------------------------------------------------------------------ host codec

def qmoe_encode_host(d: int, tern: np.ndarray):
    """-> (codes uint16 [n_codes], row_off uint32 [rows+1])"""
    t = np.ascontiguousarray(tern, dtype=np.int8)
    if t.ndim != 2:
        raise ValueError("2-D ternary matrix expected")
    rows, cols = t.shape
    row_off = np.zeros(rows + 1, dtype=np.uint32)
    n = c_size_t(0)
    cap = rows * (cols // 2)
    codes = np.empty(max(cap, 1), dtype=np.uint16)
    _check(lib().qmoe_encode_host(d, _host_ptr(t), rows, cols, _host_ptr(codes), cap, _host_ptr(row_off),
                                  byref(n)), "qmoe_encode_host")
    return codes[: n.value].copy(), row_off


def qmoe_validate_host(d: int, codes: np.ndarray, row_off: np.ndarray, rows: int, cols: int) -> None:
    c = np.ascontiguousarray(codes, dtype=np.uint16)
    r = np.ascontiguousarray(row_off, dtype=np.uint32)
    if r.shape != (rows + 1,):
        raise ValueError("row_off must hold rows+1 offsets")
    _check(lib().qmoe_validate_host(d, _host_ptr(c), _host_ptr(r), rows, cols), "qmoe_validate_host")


# ------------------------------------------------------------------ device calls

def qmoe_decode_matvec(d: int, W: qmoe_matrix, x_bf16, y, stream=None) -> None:
    """x_bf16: device int16/uint16/bfloat16 [batch, cols]; y: device float32 [batch, rows]."""
    batch = x_bf16.shape[0]
    if x_bf16.shape[1] != W.cols or tuple(y.shape) != (batch, W.rows):
        raise ValueError("shape mismatch")
    if x_bf16.element_size() != 2 or y.element_size() != 4:
        raise ValueError("x must be 16-bit, y 32-bit")
    _check(lib().qmoe_decode_matvec(d, byref(W), _dev_ptr(x_bf16), batch, _dev_ptr(y), _stream_ptr(stream)),
           "qmoe_decode_matvec")


def qmoe_decode_dense(d: int, W: qmoe_matrix, out, path: int = 0, stream=None) -> None:
    if tuple(out.shape) != (W.rows, W.cols) or out.element_size() != 1:
        raise ValueError("out must be int8 [rows, cols]")
    _check(lib().qmoe_decode_dense(d, byref(W), _dev_ptr(out), path, _stream_ptr(stream)), "qmoe_decode_dense")


def qmoe_moe_layer_ws_layout(n_experts: int, d_model: int, d_ff: int, n_tokens: int) -> qmoe_ws_layout:
    l = qmoe_ws_layout()
    _check(lib().qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens, byref(l)), "qmoe_moe_layer_ws_layout")
    return l


def qmoe_moe_layer_workspace(n_experts: int, d_model: int, d_ff: int, n_tokens: int) -> int:
    return lib().qmoe_moe_layer_workspace(n_experts, d_model, d_ff, n_tokens)


def _layer_shapes(wi_dev, wo_dev, n_experts, d_model, x_bf16, expert_idx, y) -> int:
    n_tokens = x_bf16.shape[0]
    if x_bf16.shape[1] != d_model or tuple(y.shape) != (n_tokens, d_model) or expert_idx.numel() != n_tokens:
        raise ValueError("shape mismatch")
    need = ctypes.sizeof(qmoe_matrix) * n_experts
    if wi_dev.numel() * wi_dev.element_size() < need or wo_dev.numel() * wo_dev.element_size() < need:
        raise ValueError("expert descriptor arrays too small")
    return n_tokens


def qmoe_static_workspace_bytes() -> int:
    return lib().qmoe_static_workspace_bytes()


def qmoe_moe_layer_forward_static(d: int, wi_dev, wo_dev, code_order: int, n_experts: int, d_model: int, d_ff: int,
                                  x_bf16, expert_idx, gate, y, stream=None) -> None:
    """The layer call that brings no workspace (the library's bounded scratch array is used)."""
    n_tokens = _layer_shapes(wi_dev, wo_dev, n_experts, d_model, x_bf16, expert_idx, y)
    _check(lib().qmoe_moe_layer_forward_static(d, _dev_ptr(wi_dev), _dev_ptr(wo_dev), code_order, n_experts, d_model,
                                               d_ff, _dev_ptr(x_bf16), _dev_ptr(expert_idx), _dev_ptr(gate), n_tokens,
                                               _dev_ptr(y), _stream_ptr(stream)), "qmoe_moe_layer_forward_static")


def qmoe_moe_layer_forward(d: int, wi_dev, wo_dev, code_order: int, n_experts: int, d_model: int, d_ff: int,
                           x_bf16, expert_idx, gate, y, workspace, stream=None, side_stream=None) -> None:
    """wi_dev / wo_dev: device byte tensors holding n_experts qmoe_matrix structs.
    side_stream: a second stream of the caller's for the scalar kernels (None: the library's own)."""
    n_tokens = x_bf16.shape[0]
    if x_bf16.shape[1] != d_model or tuple(y.shape) != (n_tokens, d_model) or expert_idx.numel() != n_tokens:
        raise ValueError("shape mismatch")
    need = ctypes.sizeof(qmoe_matrix) * n_experts
    if wi_dev.numel() * wi_dev.element_size() < need or wo_dev.numel() * wo_dev.element_size() < need:
        raise ValueError("expert descriptor arrays too small")
    _check(lib().qmoe_moe_layer_forward(d, _dev_ptr(wi_dev), _dev_ptr(wo_dev), code_order, n_experts, d_model, d_ff,
                                        _dev_ptr(x_bf16), _dev_ptr(expert_idx), _dev_ptr(gate), n_tokens,
                                        _dev_ptr(y), _dev_ptr(workspace),
                                        workspace.numel() * workspace.element_size(), _stream_ptr(stream),
                                        0 if side_stream is None else _stream_ptr(side_stream)),
           "qmoe_moe_layer_forward")


def qmoe_moe_dispatch(d, code_order: int, expert_idx, n_experts: int, d_model: int, d_ff: int, workspace,
                      stream=None) -> None:
    _check(lib().qmoe_moe_dispatch(d, code_order, _dev_ptr(expert_idx), expert_idx.numel(), n_experts, d_model, d_ff,
                                   _dev_ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream_ptr(stream)), "qmoe_moe_dispatch")


def qmoe_encode_device(d, ternary, codes, row_off, status, stream=None) -> None:
    """ternary: device int8 [rows, cols]; codes: device 16-bit [capacity]; row_off: device 32-bit [rows + 1];
    status: device int32 [2].  Asynchronous: check status[0] == 0 after synchronising."""
    rows, cols = ternary.shape
    if row_off.numel() != rows + 1 or status.numel() < 2:
        raise ValueError("shape mismatch")
    _check(lib().qmoe_encode_device(d, _dev_ptr(ternary), rows, cols, _dev_ptr(codes), codes.numel(),
                                    _dev_ptr(row_off), _dev_ptr(status), _stream_ptr(stream)), "qmoe_encode_device")


def qmoe_decompress(d, mats, code_order: int, n_mats: int, rows: int, cols: int, out_kind: int, out_ptrs,
                    stream=None) -> None:
    """mats: device uint8 tensor holding n_mats qmoe_matrix descriptors; out_ptrs: device int64 tensor
    [n_mats] of destination addresses (0 = skip)."""
    _check(lib().qmoe_decompress(d, _dev_ptr(mats), code_order, n_mats, rows, cols, out_kind, _dev_ptr(out_ptrs),
                                 _stream_ptr(stream)), "qmoe_decompress")


def qmoe_bf16_layer_forward(wi_ptrs, wo_ptrs, n_experts: int, d_model: int, d_ff: int, x_bf16, expert_idx,
                            gate, y, workspace, stream=None) -> None:
    """wi_ptrs / wo_ptrs: device int64 tensors [n_experts] of addresses of dense bf16 matrices (0 = none)."""
    n_tokens = x_bf16.shape[0]
    _check(lib().qmoe_bf16_layer_forward(_dev_ptr(wi_ptrs), _dev_ptr(wo_ptrs), n_experts, d_model, d_ff,
                                         _dev_ptr(x_bf16), _dev_ptr(expert_idx), _dev_ptr(gate), n_tokens,
                                         _dev_ptr(y), _dev_ptr(workspace),
                                         workspace.numel() * workspace.element_size(), _stream_ptr(stream)),
           "qmoe_bf16_layer_forward")


def qmoe_set_tuning(key: str, value: int) -> None:
    _check(lib().qmoe_set_tuning(key.encode(), int(value)), "qmoe_set_tuning")


def qmoe_plan_lanes(d: int, rows: int, cols: int, n_experts: int, n_tokens: int) -> int:
    n = lib().qmoe_plan_lanes(d, rows, cols, n_experts, n_tokens)
    if n <= 0:
        raise QmoeError(-1, "qmoe_plan_lanes")
    return n


def qmoe_lane_layout_build(codes: np.ndarray, row_off: np.ndarray, rows: int, lanes: int):
    """-> (pieces uint16 [8 * n_pieces], wave_off uint32 [lanes / 64 + 1])"""
    c = np.ascontiguousarray(codes, dtype=np.uint16)
    r = np.ascontiguousarray(row_off, dtype=np.uint32)
    n = c_size_t(0)
    _check(lib().qmoe_lane_layout_size(_host_ptr(r), rows, lanes, byref(n)), "qmoe_lane_layout_size")
    out = np.empty(8 * max(n.value, 1), dtype=np.uint16)
    wave_off = np.zeros(lanes // 64 + 1, dtype=np.uint32)
    _check(lib().qmoe_lane_layout_build(_host_ptr(c), _host_ptr(r), rows, lanes, _host_ptr(out), n.value,
                                        _host_ptr(wave_off)), "qmoe_lane_layout_build")
    return out[: 8 * n.value], wave_off


def qmoe_lane_layout_unpack(pieces: np.ndarray, wave_off: np.ndarray, row_off: np.ndarray, rows: int, lanes: int):
    p = np.ascontiguousarray(pieces, dtype=np.uint16)
    w = np.ascontiguousarray(wave_off, dtype=np.uint32)
    r = np.ascontiguousarray(row_off, dtype=np.uint32)
    codes = np.empty(max(int(r[rows]), 1), dtype=np.uint16)
    _check(lib().qmoe_lane_layout_unpack(_host_ptr(p), _host_ptr(w), _host_ptr(r), rows, lanes, _host_ptr(codes),
                                         codes.size), "qmoe_lane_layout_unpack")
    return codes[: int(r[rows])]


def qmoe_hook_set(key: str, value: int) -> None:
    """Measurement hooks (include/qmoe_hooks.h): not part of the product ABI."""
    _check(lib().qmoe_hook_set(key.encode(), int(value)), "qmoe_hook_set")


def qmoe_stream_copy(dst, src, stream=None) -> None:
    n = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() < n:
        raise ValueError("destination too small")
    _check(lib().qmoe_stream_copy(_dev_ptr(dst), _dev_ptr(src), n, _stream_ptr(stream)), "qmoe_stream_copy")
