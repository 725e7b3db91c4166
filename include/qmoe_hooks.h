/*
 * qmoe_hooks.h -- measurement hooks of libqmoe.so.  NOT part of the product ABI (qmoe.h):
 * they exist so that a benchmark or a profiler run can time one kernel of a layer call on a
 * workspace that a full call has filled, or switch one staging decision off.  Process-wide,
 * not thread-safe against running calls; nothing in the product path sets them.
 */
#ifndef QMOE_HOOKS_H
#define QMOE_HOOKS_H

#include "qmoe.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Keys:
 *  "phases"    bit mask of the kernels qmoe_moe_layer_forward / qmoe_bf16_layer_forward enqueue:
 *              1 dispatch, 2 / 4 scalar kernel of the first / second product, 8 / 16
 *              matrix-core kernel of the first / second product; 0 = all (the default)
 *  "stage_out" -1 = the products write their results straight to global memory instead of
 *              staging a block's results in LDS; 0 = default
 * Unknown key: QMOE_E_INVALID_ARG.
 */
qmoe_status qmoe_hook_set(const char *key, int value);

#ifdef __cplusplus
}
#endif
#endif /* QMOE_HOOKS_H */
