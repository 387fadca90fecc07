/*
 * Exports of libhbitlinear.so that exist for the test suite only.  They are not part of the public
 * interface (include/hbitlinear.h) and may change with the kernels they look into.
 */
#ifndef HBL_TEST_EXPORTS_H
#define HBL_TEST_EXPORTS_H

#include "hbitlinear.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Host only (no launch, no device access): the plan the small-batch GEMM launch of a grouped call would
 * use for these problems (every T in 1..64, n_problems <= 8; only T, K, N and hadamard are read).
 *   ksplit[i]              K slices per 32-row weight tile of problem i (inside a workgroup when every
 *                          T <= 16, over workgroups otherwise - the last of them to finish adds the slices)
 *   gemm_workgroups        grid size of the GEMM launch
 *   arrival_counters       groups of four row tiles whose K range is split over workgroups (0 = none)
 *   single_call_streams[i] 1 if a single forward call on problem i uses the weight-streaming kernel
 */
int hbl_test_grouped_plan(const hbl_problem* problems, int n_problems, int* ksplit, int* gemm_workgroups,
                          int* arrival_counters, int* single_call_streams);

/*
 * The integer contraction of Eq. 7 through one named workgroup tile of a prefill GEMM kernel (T > 64):
 * acc[t][o] = sum_k q[t][k] c[o][k] as int32 [T, N], on a shape of the caller's choice - the forward
 * calls pick the tile from the shape, so most tiles would otherwise be reachable at benchmark sizes only.
 *   code_form  HBL_CODES_INT8 (int8 matrix-core kernel, codes [T, K] bytes) or HBL_CODES_BF6 (fp6 x fp4
 *              kernel, code records; K >= 512)
 *   tile       0: 256 x 256   1: 128 x 128   2: 512 features x 128 tokens
 *              3: 128 x 128 with K cut over workgroups + reduction launch (HBL_CODES_BF6 only; the cut is
 *                 the forward's own for the shape when it has one, else 4, else 2 slices)
 *   partial    device scratch for tile 3: slices * T * N * 4 bytes (8 slices at most); else may be NULL
 */
int hbl_test_gemm_i32_tile(const void* codes, int code_form, int64_t T, int64_t K, const void* Wq_packed,
                           int64_t N, int32_t* acc, int tile, void* partial, size_t partial_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* HBL_TEST_EXPORTS_H */
