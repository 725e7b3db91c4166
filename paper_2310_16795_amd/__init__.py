"""MI355X-native inference hot path of QMoE (arxiv 2310.16795, Section 4.3).

The product is the C-ABI library ``csrc/libqmoe.so`` (see ``include/qmoe.h``);
this package is its thin Python binding plus the plumbing that puts compressed
experts into device memory.  ``synth`` holds the seeded workload generators.
"""
from ._binding import (  # noqa: F401
    EXPORTS, FORMAT_DEVICE_ORDER, FORMAT_GRID_MINMAX, QmoeError, qmoe_matrix, qmoe_ws_layout, lib,
    qmoe_bf16_layer_forward, qmoe_decode_dense, qmoe_decode_matvec, qmoe_dict_create, qmoe_dict_destroy,
    qmoe_codes_to_device_order, qmoe_decompress, qmoe_encode_device, qmoe_dict_device_bytes, qmoe_dict_device_order, qmoe_dict_from_words, qmoe_dict_max_nonzeros, qmoe_dict_upload, qmoe_dict_words,
    qmoe_encode_host, qmoe_moe_dispatch, qmoe_moe_layer_forward, qmoe_moe_layer_workspace,
    qmoe_moe_layer_ws_layout, qmoe_set_tuning, qmoe_stream_copy, qmoe_validate_host, qmoe_hook_set,
    qmoe_moe_layer_forward_static, qmoe_static_workspace_bytes, qmoe_lane_layout_build, qmoe_lane_layout_unpack,
    qmoe_plan_lanes, format_lanes,
)
