// Internal GEMM entry point shared by gt_combine and the layer calls.
#pragma once
#include "gt_internal.h"

size_t gt_gemm_ws_bytes(int transA, int64_t M, int64_t N, int64_t K);

// C = act(rowscale .* (op(A) op(B)) + C_in + bias); C_in (same type and shape as C) may be null.
gt_status gt_gemm_run(const char *fn, gt_dtype dtype, int transA, int transB, int64_t M, int64_t N, int64_t K,
                      const void *A, int64_t lda, const void *B, int64_t ldb, const float *bias, const float *rowscale,
                      gt_act act, const void *Cin, int64_t ldcin, void *C, int64_t ldc, gt_dtype c_dtype, void *ws,
                      size_t ws_bytes, hipStream_t st);
