// Internal hooks of the optional kernel timing (see gt_trace.hip).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

enum { GT_TRACE_AGG_FWD = 0, GT_TRACE_AGG_BWD = 1, GT_TRACE_COMBINE = 2, GT_TRACE_FUSED = 3 };

bool gt_trace_on();
// returns a record id (or -1 when tracing is off); `work` is edges (aggregation) or M*N*K (combine)
int gt_trace_open(int kind, int64_t width, int64_t rows, int64_t work, hipStream_t st);
void gt_trace_close(int id, hipStream_t st);
// template parameters of the aggregation kernel instance a record belongs to (V elements per lane,
// G lanes per item, NP column passes per lane, U row loads in flight, output mask present)
void gt_trace_variant(int id, int V, int G, int NP, int U, int masked);
