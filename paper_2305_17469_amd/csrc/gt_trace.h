// Internal hooks of the optional kernel timing (see gt_trace.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

enum { GT_TRACE_AGG_FWD = 0, GT_TRACE_AGG_BWD = 1, GT_TRACE_COMBINE = 2 };

bool gt_trace_on();
// returns a record id (or -1 when tracing is off); `work` is edges (aggregation) or M*N*K (combine)
int gt_trace_open(int kind, int64_t width, int64_t rows, int64_t work, hipStream_t st);
void gt_trace_close(int id, hipStream_t st);
