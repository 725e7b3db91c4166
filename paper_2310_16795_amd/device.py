"""Plumbing between host arrays and device memory (torch tensors).  No arithmetic."""
from __future__ import annotations

import ctypes

import numpy as np
import torch

from . import _binding as B


class DeviceDict:
    """A dictionary handle together with the device buffer it is bound to."""

    def __init__(self, handle: int | None = None, device="cuda:0"):
        self.handle = B.qmoe_dict_create() if handle is None else handle
        self.buf = torch.empty(B.qmoe_dict_device_bytes(), dtype=torch.uint8, device=device)
        B.qmoe_dict_upload(self.handle, self.buf)
        torch.cuda.current_stream().synchronize()

    def close(self):
        if self.handle:
            B.qmoe_dict_destroy(self.handle)
            self.handle = 0


def _pad_to(a: np.ndarray, multiple: int) -> np.ndarray:
    extra = (-a.size) % multiple
    return a if extra == 0 else np.concatenate([a, np.zeros(extra, dtype=a.dtype)])


class DeviceMatrix:
    """One compressed matrix in device memory and its qmoe_matrix descriptor."""

    def __init__(self, codes: np.ndarray, row_off: np.ndarray, scale_f16: "np.ndarray | None", rows: int, cols: int,
                 device="cuda:0", device_order_of: "DeviceDict | None" = None,
                 minmax_bf16: "np.ndarray | None" = None):
        """scale_f16 [rows] for the symmetric grid, or minmax_bf16 [rows, 2] = (w_min, w_max) for the asymmetric one."""
        assert row_off.shape == (rows + 1,)
        assert (scale_f16 is None) != (minmax_bf16 is None)
        self.codes = torch.from_numpy(_pad_to(codes.view(np.int16), 8).copy()).to(device)
        self.row_off = torch.from_numpy(row_off.astype(np.uint32).view(np.int32).copy()).to(device)
        self.scale = self.minmax = None
        if scale_f16 is not None:
            assert scale_f16.shape == (rows,)
            self.scale = torch.from_numpy(scale_f16.view(np.int16).copy()).to(device)
        else:
            assert minmax_bf16.shape == (rows, 2)
            self.minmax = torch.from_numpy(np.ascontiguousarray(minmax_bf16).view(np.int16).copy()).to(device)
        order = 0
        if device_order_of is not None:  # renumber the stream for this dictionary, once
            B.qmoe_codes_to_device_order(device_order_of.handle, self.codes)
            order = 1
        self.desc = B.qmoe_matrix(self.codes.data_ptr(), self.row_off.data_ptr(),
                                  self.scale.data_ptr() if self.scale is not None else None, rows,
                                  cols, int(codes.size), order,
                                  self.minmax.data_ptr() if self.minmax is not None else None)


class DeviceLayer:
    """All experts of one MoE layer: three big device buffers per projection and
    a device array of qmoe_matrix descriptors pointing into them."""

    def __init__(self, n_experts: int, d_model: int, d_ff: int, device="cuda:0", minmax: bool = False):
        """minmax: the experts are on the asymmetric grid; set_expert then takes bf16 (w_min, w_max)
        pairs [rows, 2] in place of the binary16 scales [rows]."""
        self.n_experts, self.d_model, self.d_ff, self.device = n_experts, d_model, d_ff, device
        self.minmax = minmax
        self._host = {"wi": [None] * n_experts, "wo": [None] * n_experts}
        self.compressed_bytes = 0
        self.n_codes = {"wi": np.zeros(n_experts, dtype=np.int64), "wo": np.zeros(n_experts, dtype=np.int64)}

    def set_expert(self, e: int, which: str, codes: np.ndarray, row_off: np.ndarray, scale: np.ndarray):
        rows = self.d_ff if which == "wi" else self.d_model
        assert row_off.shape == (rows + 1,) and row_off[-1] == codes.size
        assert scale.shape == ((rows, 2) if self.minmax else (rows,))
        self._host[which][e] = (codes, row_off.astype(np.uint32), scale)
        self.n_codes[which][e] = codes.size

    def finalize(self, device_order_of: "DeviceDict | None" = None, lanes_for_tokens: int = 0):
        """Upload everything; with device_order_of, renumber the streams for that dictionary; with
        lanes_for_tokens (a typical token count of the calls to come; needs device_order_of), re-pack
        every stream into the lane-interleaved layout for the lane count the planner picks."""
        self.code_order = 0 if device_order_of is None else 1
        self.format = self.code_order | (B.FORMAT_GRID_MINMAX if self.minmax else 0)
        per_row = 2 if self.minmax else 1  # 16-bit values of scale data per row
        self.bufs, self.desc_dev, self.desc_host = {}, {}, {}
        self.lanes = {"wi": 0, "wo": 0}
        for which in ("wi", "wo"):
            rows = self.d_ff if which == "wi" else self.d_model
            cols = self.d_model if which == "wi" else self.d_ff
            parts = self._host[which]
            lanes = 0
            wave_off = None
            if lanes_for_tokens > 0:
                assert device_order_of is not None
                lanes = B.qmoe_plan_lanes(device_order_of.handle, rows, cols, self.n_experts, lanes_for_tokens)
                self.lanes[which] = lanes
                wave_off = np.zeros((self.n_experts, lanes // 64 + 1), dtype=np.uint32)
                for e, p in enumerate(parts):
                    if p is not None:
                        pieces, wave_off[e] = B.qmoe_lane_layout_build(p[0], p[1], rows, lanes)
                        parts[e] = (pieces, p[1], p[2])  # the stream as the device holds it (padding included)
                        self.n_codes[which][e] = pieces.size
            code_off, total = [], 0
            for p in parts:
                code_off.append(total)
                if p is not None:
                    total += (p[0].size + 7) // 8 * 8  # 16-byte aligned start for every matrix
            codes = np.zeros(max(total, 8), dtype=np.uint16)
            row_off = np.zeros((self.n_experts, rows + 1), dtype=np.uint32)
            scale = np.zeros((self.n_experts, rows * per_row), dtype=np.uint16)
            for e, p in enumerate(parts):
                if p is None:
                    continue
                codes[code_off[e]: code_off[e] + p[0].size] = p[0]
                row_off[e] = p[1]
                scale[e] = p[2].reshape(-1)
            d_codes = torch.from_numpy(codes.view(np.int16)).to(self.device)
            if device_order_of is not None:
                B.qmoe_codes_to_device_order(device_order_of.handle, d_codes)
            d_row = torch.from_numpy(row_off.view(np.int32)).to(self.device)
            d_scale = torch.from_numpy(scale.view(np.int16)).to(self.device)
            d_wave = None if wave_off is None else torch.from_numpy(wave_off.view(np.int32)).to(self.device)
            descs = (B.qmoe_matrix * self.n_experts)()
            for e, p in enumerate(parts):
                if p is None:
                    continue  # stays all-zero: never touched unless a token is routed there
                at = d_scale.data_ptr() + 2 * e * rows * per_row
                descs[e] = B.qmoe_matrix(d_codes.data_ptr() + 2 * code_off[e],
                                         d_row.data_ptr() + 4 * e * (rows + 1),
                                         None if self.minmax else at, rows, cols, int(p[0].size), self.code_order,
                                         at if self.minmax else None,
                                         None if d_wave is None else d_wave.data_ptr() + 4 * e * (lanes // 64 + 1), lanes, 0)
            raw = np.frombuffer(bytes(descs), dtype=np.uint8).copy()
            self.bufs[which] = (d_codes, d_row, d_scale, d_wave)
            self.desc_host[which] = descs
            self.desc_dev[which] = torch.from_numpy(raw).to(self.device)
            # bytes of a matrix as the device holds it: codewords (lane-interleaved: padding included),
            # per row a 4-byte offset and the scale (pair), per group of 64 lanes a 4-byte piece offset
            self.row_meta = 4 + 2 * per_row
            self.matrix_meta = {**getattr(self, "matrix_meta", {}), which: self.row_meta * rows + (4 * (lanes // 64 + 1) if lanes else 0)}
            self.compressed_bytes += sum(2 * p[0].size + self.matrix_meta[which] for p in parts if p is not None)
        if self.lanes["wi"]:
            self.format |= B.format_lanes(self.lanes["wi"], self.lanes["wo"])
        self._host = None
        return self

    def workspace(self, n_tokens: int) -> torch.Tensor:
        n = B.qmoe_moe_layer_workspace(self.n_experts, self.d_model, self.d_ff, n_tokens)
        return torch.empty(n, dtype=torch.uint8, device=self.device)

    def forward(self, dd: DeviceDict, x_bf16: torch.Tensor, expert_idx: torch.Tensor, y: torch.Tensor,
                workspace: torch.Tensor, gate: torch.Tensor | None = None, stream=None, side_stream=None):
        B.qmoe_moe_layer_forward(dd.handle, self.desc_dev["wi"], self.desc_dev["wo"], self.format, self.n_experts,
                                 self.d_model, self.d_ff, x_bf16, expert_idx, gate, y, workspace, stream, side_stream)

    def forward_static(self, dd: DeviceDict, x_bf16: torch.Tensor, expert_idx: torch.Tensor, y: torch.Tensor,
                       gate: torch.Tensor | None = None, stream=None):
        """The same layer on the library's own bounded scratch array (no workspace, nothing allocated)."""
        B.qmoe_moe_layer_forward_static(dd.handle, self.desc_dev["wi"], self.desc_dev["wo"], self.format,
                                        self.n_experts, self.d_model, self.d_ff, x_bf16, expert_idx, gate, y, stream)


def read_workspace(workspace: torch.Tensor, n_experts: int, d_model: int, d_ff: int, n_tokens: int):
    """Copy the dispatch results out of a layer workspace (synchronises)."""
    l = B.qmoe_moe_layer_ws_layout(n_experts, d_model, d_ff, n_tokens)
    host = workspace.cpu().numpy()
    def view(off, n, dt):
        return host[off: off + n * np.dtype(dt).itemsize].view(dt).copy()
    return {
        "tok_off": view(l.tok_off, n_experts + 1, np.int32),
        "perm": view(l.perm, n_tokens, np.int32),
        "counters": view(l.counters, 16, np.int32),
        "items_wi": view(l.items_wi, 4 * n_tokens, np.int32).reshape(n_tokens, 4),
        "items_wo": view(l.items_wo, 4 * n_tokens, np.int32).reshape(n_tokens, 4),
        "items_mm": view(l.items_mm, 4 * n_tokens, np.int32).reshape(n_tokens, 4),
        "hidden": _untile_hidden(view(l.hidden, n_tokens * d_ff, np.uint16).reshape(n_tokens, d_ff),
                                 view(l.items_mm, 4 * n_tokens, np.int32).reshape(n_tokens, 4),
                                 int(view(l.counters, 16, np.int32)[7]), d_ff),
    }


def _untile_hidden(hidden: np.ndarray, items_mm: np.ndarray, n_mm: int, d_ff: int) -> np.ndarray:
    """The hidden vectors by slot.  The matrix-core kernels keep those of their tiles in blocks of up to
    16 tokens, [8-column group][token of the block][8 columns], in the bytes of the same slots: put
    them back into [slot][column] order (a permutation of the buffer, no arithmetic)."""
    out = hidden.copy()
    for _, slot0, ntok, _ in items_mm[:n_mm]:
        for b0 in range(0, int(ntok), 16):
            tb = min(16, int(ntok) - b0)
            blk = hidden[slot0 + b0: slot0 + b0 + tb].reshape(-1)          # the block's bytes, as stored
            out[slot0 + b0: slot0 + b0 + tb] = blk.reshape(d_ff // 8, tb, 8).transpose(1, 0, 2).reshape(tb, d_ff)
    return out
