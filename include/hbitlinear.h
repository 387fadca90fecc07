/*
 * libhbitlinear - the H-BitLinear forward pass of BitNet v2 (Section 2.1) for
 * AMD MI355X (gfx950), as a C-ABI library of hand-written HIP kernels.
 *
 *   Y = Qw(W) . Q_INT8/4(X_r),   X_r = Hadamard(X)                     (Eq. 7)
 *
 * Conventions shared by every call
 *   - All tensor pointers are DEVICE pointers owned by the caller (the library
 *     never allocates, frees or keeps them); scalars and sizes are by value.
 *   - X is [T, K] row-major (token-major, K features contiguous).  W is
 *     [N, K] row-major (out x in), so Y[T, N] = Xq . Wq^T - the row form of
 *     Eq. 7 - and the Hadamard transform (Eq. 3-4) runs along K, n = K = 2^m.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work on it and return without synchronising.
 *   - Every call returns a status: HBL_OK or a negative HBL_E_* code.  On an
 *     error nothing has been launched.  No exception crosses this boundary.
 *   - bf16 tensors are 16-bit patterns (the upper half of an IEEE fp32).
 *   - `eps` is the epsilon of Eq. 1, 5 and 6 (the paper gives no value; the
 *     tests and the benchmark use 1e-5).  It is added exactly as printed:
 *     inside the quantiser gain, not in the outer dequantisation factor.
 *   - round() of Eq. 2 is round-half-to-even.
 *   - Inputs containing NaN or Inf are not checked and give undefined output.
 *
 * Shape limits (HBL_E_SHAPE otherwise): T >= 0 (T == 0 is a no-op);
 * K a multiple of 128, 128 <= K <= 16384, and a power of two when the
 * Hadamard transform is applied; N a positive multiple of 32.
 */
#ifndef HBITLINEAR_H
#define HBITLINEAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define HBL_OK 0
#define HBL_E_NULL (-1)      /* a required pointer is NULL                              */
#define HBL_E_SHAPE (-2)     /* a size violates the limits above                        */
#define HBL_E_BITS (-3)      /* bits is neither 4 nor 8                                 */
#define HBL_E_DTYPE (-4)     /* x_dtype is neither HBL_F32 nor HBL_BF16                 */
#define HBL_E_WORKSPACE (-5) /* workspace smaller than the matching *_workspace_bytes() */
#define HBL_E_HIP (-6)       /* a HIP call failed; see hbl_last_hip_error()             */
#define HBL_E_ALIGN (-7)     /* a pointer is not aligned to 16 bytes                    */
#define HBL_E_SCRATCH (-8)   /* problem exceeds the static scratch of hbl_bitlinear_forward_small */

/* activation storage types */
#define HBL_F32 0
#define HBL_BF16 1

/* forms in which the quantised activation codes travel between the two launches (stage-level calls) */
#define HBL_CODES_INT8 0        /* one signed byte per code, [T, K] in natural feature order             */
#define HBL_CODES_UINT4_PLUS8 8 /* INT4 only: byte = code + 8 in 0..15, [T, K]                           */
#define HBL_CODES_BF6 6         /* INT4 only, K >= 512: 6 bits per code.  Per 32 features a 24-byte record
                                   of 6-bit floats (e3m2, feature i at bits [6i, 6i+6); every integer in
                                   [-8, 7] is exact), the records laid out as the GEMM holds them in LDS:
                                   tokens in panels of 128, features in blocks of 128, a block = 128 token
                                   rows of 96 bytes.  hbl_code_bytes() gives the buffer size (whole panels:
                                   ceil(T/128) * 128 * 0.75 K); the layout is the library's own              */

/* Human-readable text for a status code (static storage, never NULL). */
const char* hbl_strerror(int status);
/* The hipError_t value behind the most recent HBL_E_HIP on this thread (0 if none). */
int hbl_last_hip_error(void);

/* ---------------------------------------------------------------------------
 * Weight set-up (offline, once per weight tensor)
 * ------------------------------------------------------------------------- */

/* Scratch needed by hbl_ternarize_weights_absmean for an [N, K] tensor. */
size_t hbl_ternarize_workspace_bytes(int64_t N, int64_t K);

/*
 * Per-tensor absmean ternary weight quantiser (Eq. 1-2):
 *   alpha = mean(|W|),  codes = RoundClip(W / (alpha + eps), -1, 1).
 *   W      [N, K] fp32, read only
 *   codes  [N, K] int8 out, each -1, 0 or +1; dequantised weight = alpha * codes
 *   alpha  1 fp32 out (device).  The mean is accumulated in fp64 in a fixed
 *          order (deterministic) and rounded to fp32 once.
 *   workspace  device scratch of at least hbl_ternarize_workspace_bytes(N, K)
 * Any N >= 1, K >= 1 is accepted here (the GEMM limits apply at pack time).
 */
int hbl_ternarize_weights_absmean(const float* W, int64_t N, int64_t K, float eps, int8_t* codes,
                                  float* alpha, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of the packed form of an [N, K] ternary tensor: N*K/4 (2 bits per weight) + 4*N (row sums). */
size_t hbl_packed_bytes(int64_t N, int64_t K);

/*
 * Pack ternary codes 4 per byte into the library's streaming layout (not in
 * the paper, which describes no storage format).  The layout is opaque to the
 * caller: 1 KiB tiles of 32 output rows x 128 input features, ordered so that
 * one 16-byte load per lane yields matrix-core operands; each weight is a
 * (sign, magnitude) bit pair that every GEMM kernel of the library reads (as an
 * fp4 value or, after a byte look-up, as an int8); the tiles are followed by the
 * N int32 row sums sum_k c[o][k] that the int8 epilogue uses for offset codes.
 * hbl_unpack_ternary_2bit is the exact inverse.
 *   codes  [N, K] int8 in {-1,0,1};   packed  hbl_packed_bytes(N, K) bytes, 16-byte aligned
 */
int hbl_pack_ternary_2bit(const int8_t* codes, int64_t N, int64_t K, void* packed, void* stream);
int hbl_unpack_ternary_2bit(const void* packed, int64_t N, int64_t K, int8_t* codes, void* stream);

/* ---------------------------------------------------------------------------
 * Forward pass (the hot path)
 * ------------------------------------------------------------------------- */

/* Device scratch needed by the two forward calls (activation codes, per-token
 * dequantisation scale, int32 partial tiles where a K range is split). */
size_t hbl_workspace_bytes(int64_t T, int64_t K, int64_t N, int bits);

/*
 * H-BitLinear forward (Eq. 7 with Eq. 3-6): for every token row
 *   x_r = H_m x                       fast Walsh-Hadamard transform, fp32,
 *                                     butterflies with ascending stride then
 *                                     one multiply by (float)(1/sqrt(K))
 *   bits == 8:  gamma = max|x_r|,  q = RoundClip(127/(gamma+eps) x_r, -128, 127), s = gamma/127
 *   bits == 4:  beta  = mean|x_r|, q = RoundClip(sqrt7/(beta+eps) x_r, -8, 7),    s = beta/sqrt7
 *   y[o] = bf16( (float)(sum_k q[k] c[o][k]) * s * alpha_g(o) )
 * with int32 accumulation (exact) and round-to-nearest-even to bf16.
 *   x          [T, K] x_dtype (HBL_F32 or HBL_BF16), read only, 16-byte aligned
 *   Wq_packed  from hbl_pack_ternary_2bit for an [N, K] tensor
 *   w_scales   [n_scale_groups] fp32 (device): alpha of each group of
 *              N/n_scale_groups consecutive output rows (1 = the paper's
 *              per-tensor scale; 3 for a fused QKV, 2 for up|gate).
 *              N/n_scale_groups must be a multiple of 32.
 *   y          [T, N] bf16 out; must not overlap x or the workspace
 *   workspace  at least hbl_workspace_bytes(T, K, N, bits), 256-byte aligned
 */
int hbl_hbitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed,
                           int64_t N, const float* w_scales, int64_t n_scale_groups, int bits,
                           float eps, void* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Plain BitLinear forward for the projections that keep their input
 * distribution (W_qkv, W_up/gate; Section 2, first paragraph): identical to
 * the call above with x_r = x (no Hadamard transform).  K need not be a power
 * of two.
 */
int hbl_plain_bitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K,
                                const void* Wq_packed, int64_t N, const float* w_scales,
                                int64_t n_scale_groups, int bits, float eps, void* y,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The forward call for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation and the same
 * kernels as hbl_hbitlinear_forward (hadamard != 0) / hbl_plain_bitlinear_forward (hadamard == 0), with
 * bit-identical output; the intermediates (activation codes, per-token scales) live in a 2 MiB array in the
 * library's own device image, one copy per GPU, held until the process ends.  There is no room for partial
 * tiles, so a K range is never split over workgroups (integer sums: same result, possibly a slower launch on
 * long-K, few-row shapes).  The call allocates nothing and frees nothing.
 *   Limit: T <= 64 (decode batches; every K and N the library accepts fits); beyond it HBL_E_SCRATCH and
 *   nothing is launched.
 *   Every call on a GPU shares that GPU's array, on whatever stream: two calls that may run at the same
 *   time on one GPU race (calls on one stream are ordered and safe).  Nothing in the array has to start
 *   at zero: a call writes every byte it later reads.
 * Other arguments, layouts and errors as hbl_hbitlinear_forward.
 */
int hbl_bitlinear_forward_small(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed,
                                int64_t N, const float* w_scales, int64_t n_scale_groups, int bits, float eps,
                                int hadamard, void* y, void* stream);

/*
 * Eq. 7 including its LN: y = Q_w(W) . Q_INT8/4(X_r), X_r = Hadamard(LN(X)) (hadamard != 0), or
 * X_r = LN(X) for the plain BitLinear (hadamard == 0).  LN is the model's RMS normalisation
 * (Section 2, first paragraph), fused into the quantiser launch so that the normalised row never
 * touches HBM:
 *     x_n[k] = (x[k] * r) * ln_gain[k],   r = (float)(1 / sqrt(mean_k x[k]^2 + ln_eps))
 * with the mean of squares accumulated in fp64 and two fp32 multiplies per element.
 *   ln_gain  device [K] fp32, 16-byte aligned;  ln_eps added to the mean of squares
 * All other arguments, layouts and errors as hbl_hbitlinear_forward / hbl_plain_bitlinear_forward.
 */
int hbl_ln_bitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const float* ln_gain,
                             float ln_eps, int hadamard, const void* Wq_packed, int64_t N,
                             const float* w_scales, int64_t n_scale_groups, int bits, float eps,
                             void* y, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Several independent projections in one call (Eq. 7 applied to each): the result in every y is
 * bit-identical to hbl_hbitlinear_forward / hbl_plain_bitlinear_forward on that problem alone.
 * Meant for small batches (decode), where one projection's launches are too short to keep HBM
 * busy: when every T <= 64, n_problems <= 8 and all problems share bits and x_dtype, the rows of
 * all problems are quantised by one launch and all packed weights are streamed by one launch
 * (for 16 < T <= 64 a K range may be split over workgroups; the last of them to finish adds the
 * slices, counted in a small static device array of which overlapping calls on one GPU take
 * different slots, 128 in all); otherwise the problems run one after the other through the calls above.
 *   problems   host array, read during the call only; fields as the arguments of the forward
 *              calls above (hadamard != 0 selects H-BitLinear, eps is shared)
 *   workspace  device, >= hbl_grouped_workspace_bytes(problems, n_problems), 256-byte aligned
 * The problems must not overlap: no y may alias another problem's x or y.
 * Returns the first error of any problem (nothing is launched then) or of a launch.
 */
typedef struct hbl_problem {
    const void* x;          /* device [T, K], row-major, x_dtype                       */
    int x_dtype;            /* HBL_F32 or HBL_BF16                                     */
    int bits;               /* 4 or 8                                                  */
    int hadamard;           /* 0: plain BitLinear, else H-BitLinear (K a power of two) */
    int reserved;           /* set to 0                                                */
    int64_t T, K, N;
    const void* Wq_packed;  /* device, from hbl_pack_ternary_2bit                      */
    const float* w_scales;  /* device [n_scale_groups]                                 */
    int64_t n_scale_groups;
    void* y;                /* device [T, N] bf16 out                                  */
    const float* ln_gain;   /* device [K] fp32: RMS-normalise x first (see hbl_ln_bitlinear_forward), or NULL */
    float ln_eps;
} hbl_problem;
size_t hbl_grouped_workspace_bytes(const hbl_problem* problems, int n_problems);
int hbl_bitlinear_forward_grouped(const hbl_problem* problems, int n_problems, float eps,
                                  void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------
 * Stage-level entry points (parity checks and profiling; same kernels)
 * ------------------------------------------------------------------------- */

/* Bytes of the code buffer hbl_fwht_quant writes for [T, K] activations in the given form (0 for a form
 * the shape does not allow). */
size_t hbl_code_bytes(int64_t T, int64_t K, int code_form);

/*
 * Activation front end only (Eq. 3-6): transform (if hadamard != 0) and quantise.
 *   code_offset  one of HBL_CODES_*: HBL_CODES_INT8 stores the codes as such; HBL_CODES_UINT4_PLUS8
 *              stores code + 8 - the form the forward calls use for INT4 on the int8 matrix-core
 *              path, because unsigned nibbles toggle far fewer multiplier input bits than
 *              sign-extended bytes and the matrix cores are power-limited (the GEMM epilogue removes
 *              the offset exactly in int32); HBL_CODES_BF6 writes the records the fp6 x fp4
 *              matrix-core path reads - the form the forward calls use for INT4 whenever K >= 512.
 *   codes      out, hbl_code_bytes(T, K, code_offset) bytes: [T, K] bytes in natural feature order, or the
 *              record image
 *   s_dequant  [T] fp32 out: gamma/127 or beta/sqrt7
 *   code_sum   [T] int32 out or NULL: sum_k code[t][k] of the true codes (without the offset)
 */
int hbl_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, int bits, float eps,
                   int hadamard, int code_offset, int8_t* codes, float* s_dequant, int32_t* code_sum,
                   void* stream);

/* hbl_fwht_quant with the RMS normalisation of hbl_ln_bitlinear_forward ahead of the transform. */
int hbl_ln_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, const float* ln_gain, float ln_eps,
                      int bits, float eps, int hadamard, int code_offset, int8_t* codes,
                      float* s_dequant, int32_t* code_sum, void* stream);

/*
 * The transform by itself: out[t] = H_m x[t] (Eq. 3-4, same butterfly order and 1/sqrt(K) factor as
 * the forward calls).  H_m is symmetric and orthogonal, so this is also the backward pass through
 * the transform (Section 2.2, Eq. 8): with the straight-through estimator passing the gradient
 * across the quantiser unchanged, dL/dx[t] = H_m (dL/dx_r[t]) - call it on the gradient rows.
 *   x    [T, K] x_dtype, K a power of two in [128, 16384]
 *   out  [T, K] out_dtype (HBL_F32, or HBL_BF16 rounded to nearest even); must not overlap x
 */
int hbl_fwht(const void* x, int x_dtype, int64_t T, int64_t K, void* out, int out_dtype, void* stream);

/*
 * Integer contraction only: acc[t][o] = sum_k codes[t][k] * c[o][k] (int32, exact).
 *   codes [T, K] int8 (any values in [-128,127]);  acc [T, N] int32 out
 */
int hbl_gemm_i32(const int8_t* codes, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                 int32_t* acc, void* stream);

/*
 * The same contraction on the fp6 x fp4 prefill kernel, the one every INT4 forward call with T > 64 and
 * K >= 512 runs: acc[t][o] = sum_k q[t][k] * c[o][k] as int32 [T, N], read out of that kernel's fp32
 * accumulators (exact integers) with no dequantisation, in the launch configuration (workgroup tile,
 * K split over workgroups at mid-size batches) hbl_hbitlinear_forward takes for the same T, K, N.
 *   code_records  [T, K] bytes of HBL_CODES_BF6 records as written by hbl_fwht_quant (K >= 512)
 *   workspace     device, >= hbl_workspace_bytes(T, K, N, 4), 256-byte aligned (holds the int32 partial
 *                 tiles when the K range is split; the code region of it is not touched)
 */
int hbl_gemm_i32_bf6(const void* code_records, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                     int32_t* acc, void* workspace, size_t workspace_bytes, void* stream);

/*
 * GEMM + dequantising epilogue only (Eq. 7 given the quantised activations): the second of the
 * two launches the forward calls make, on caller-held intermediates.
 *   codes [T, K] int8, s_dequant [T] fp32, code_sum [T] int32: as written by hbl_fwht_quant with
 *   the same code_offset;  y [T, N] bf16 out
 * A forward call with T > 64 is hbl_fwht_quant(x, ..., hadamard, code_offset) into the workspace followed by
 * this call, with code_offset = HBL_CODES_BF6 for INT4 activations with K >= 512 (fp6 x fp4 matrix cores),
 * HBL_CODES_UINT4_PLUS8 for INT4 on shorter rows, HBL_CODES_INT8 for INT8 activations (smaller batches run the
 * weight-streaming kernel on the same code forms).  code_sum is not read (the packed weights are signed) and
 * may be NULL.
 */
int hbl_gemm_dequant_bf16(const int8_t* codes, int code_offset, const float* s_dequant,
                          const int32_t* code_sum, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                          const float* w_scales, int64_t n_scale_groups, void* y, void* stream);

/* ---------------------------------------------------------------------------
 * Low-bit attention states (Section 3.1, Main Results: 8-, 4- and 3-bit Q/K/V heads and KV cache).
 * The head states after RoPE are quantised per head row; the paper names the method (absmax, to unsigned
 * codes, no calibration) and prints no formula, and this library takes Eq. 5 at b bits with an offset:
 *   gamma = max|h|, qmax = 2^(b-1) - 1,
 *   u[i] = RoundClip(qmax/(gamma+eps) * h[i], -2^(b-1), qmax) + 2^(b-1)  in [0, 2^b - 1],
 *   scale = gamma / qmax,  h^[i] = (u[i] - 2^(b-1)) * scale
 * (round half to even; at b = 8 this is Eq. 5 plus 128).  The [BOS] token's K/V rows, which the
 * paper keeps at 8 bits, are the caller's to route: quantise them in a call of their own with bits = 8.
 *   x       [rows, d] device, x_dtype; one row = one head of one token; d in {32, 64, 128, 256, 512}
 *   bits    8, 4 or 3
 *   packed  device, hbl_kv_packed_bytes(rows, d, bits) = rows*d*bits/8 bytes, 16-byte aligned: one
 *           little-endian bit string, row r from byte r*d*bits/8, code i of a row at bits
 *           [bits*i, bits*i + bits) of its row (bytes; low nibble first; 8 codes per 3 bytes)
 *   scales  [rows] fp32 device
 * Errors as above (HBL_E_SHAPE for another d, HBL_E_BITS, HBL_E_DTYPE, HBL_E_NULL, HBL_E_ALIGN);
 * rows = 0 is a no-op.  Nothing is allocated; the calls enqueue on `stream` and return.
 */
size_t hbl_kv_packed_bytes(int64_t rows, int64_t d, int bits);
int hbl_kv_quant_absmax(const void* x, int x_dtype, int64_t rows, int64_t d, int bits, float eps,
                        void* packed, float* scales, void* stream);
/* The inverse map: out [rows, d] out_dtype (HBL_F32, or HBL_BF16 rounded to nearest even), 16-byte aligned. */
int hbl_kv_dequant(const void* packed, const float* scales, int64_t rows, int64_t d, int bits,
                   void* out, int out_dtype, void* stream);

/* ---------------------------------------------------------------------------
 * Kernel timing (benchmarks and profiling; not part of the forward path)
 * ---------------------------------------------------------------------------
 * Between hbl_trace_begin and hbl_trace_end every kernel this library launches from the calling thread
 * goes out with a start / stop event pair of its own, filled by the runtime with that dispatch's device
 * timestamps: the durations are the kernels' own (what a kernel trace of a profiler reports), with no
 * marker packets between the launches.  The events are host objects created at hbl_trace_begin (no device
 * memory); hbl_trace_end waits for the traced launches to finish.  Do not trace calls that are being
 * captured into a HIP graph.
 *   max_launches   launches to time (later ones are launched untimed but still counted)
 *   ms             [capacity] out: duration of launch i in milliseconds, in launch order
 *   kernel_names   [capacity] out: static strings naming the kernel family of launch i (or NULL)
 *   n_launches     out: launches seen since hbl_trace_begin
 * Errors: HBL_E_SHAPE for a bad count, for begin inside an open trace or end without one; HBL_E_HIP.
 */
int hbl_trace_begin(int max_launches);
int hbl_trace_end(float* ms, const char** kernel_names, int capacity, int* n_launches);

#ifdef __cplusplus
}
#endif
#endif /* HBITLINEAR_H */
