// Internal interface of the selection stage (see ks_select.hip).
#pragma once
#include "ks_common.h"

size_t ks_select_ws_bytes(int64_t C, int B, int K);
// Enqueues the selection kernels on `st`.  Arguments must already be validated.
int ks_select_launch(const int32_t *labels, const int32_t *graph, int64_t C, int B, int K, int M,
                     int32_t *active_idx, int32_t *n_active, int32_t *target_pos, void *ws,
                     int32_t *dev_status, hipStream_t st);
