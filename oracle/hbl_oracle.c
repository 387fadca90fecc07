/*
 * CPU oracle for the H-BitLinear forward pass of BitNet v2 (Section 2.1, Eq. 1-7).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow reference that the
 * GPU library is checked against.  It shares no code, header, table or helper
 * with the HIP path and must never be called from the product path.  Only the
 * tests, the smoke check and the benchmark's "cpu_baseline" leg may use it.
 *
 * Every function takes the steps of the paper's definition in the paper's
 * order, in fp32 where the paper's operands are fp32 (each operation rounded
 * once, no fused multiply-add: build with -ffp-contract=off, no -ffast-math)
 * and in exact integer arithmetic for the matrix product.  There is no
 * blocking, fusion or reordering beyond an OpenMP "parallel for" over
 * independent tokens / output rows.
 *
 * Readings of the paper taken here (the paper is silent on each):
 *   - epsilon is added exactly as written (alpha+eps, gamma+eps, beta+eps) and
 *     is an argument; the outer dequantisation factors use alpha, gamma/127,
 *     beta/sqrt(7) WITHOUT eps, as printed in Eq. 1, 5, 6.
 *   - round() is round-half-to-even (rintf under the default rounding mode).
 *   - "per-token": one gamma / beta per activation row of length n.
 *   - H_m carries 1/sqrt(2) per recursion level (Eq. 4), i.e. 1/sqrt(n) in
 *     total; it is applied as one multiply after the unnormalised butterflies.
 *     Output order is the natural (Sylvester) order of the recursion.
 *   - butterfly stages run with ascending stride 1,2,4,...,n/2; means are
 *     accumulated in fp64 and rounded to fp32 once.
 *   - LN of Eq. 7 is a separate routine (hblo_rmsnorm, the model's RMS
 *     normalisation); the forward routines take X as already normalised.
 *   - Eq. 8 (backward through the transform) is the same transform applied
 *     to the gradient rows, in the same fp32 butterfly order.
 *   - X is a row vector per token, W is [N out x K in]: Y[T x N] = Xq * Wq^T.
 *   - low-bit Q/K/V head states (Section 3.1, Main Results, low-bit attention):
 *     the paper names the method for the post-RoPE head states (absmax, to
 *     unsigned codes) and prints no formula.  Taken here as Eq. 5 at b bits per head row,
 *     stored with an offset: u = RoundClip(qmax/(gamma+eps) * h, -2^(b-1),
 *     2^(b-1)-1) + 2^(b-1), qmax = 2^(b-1)-1, dequantised (u - 2^(b-1)) *
 *     gamma/qmax.  At b = 8 this is Eq. 5 itself plus 128.
 *
 * Pins (tests/test_oracle_*.py): H*H^T = I and the popcount closed form for
 * hblo_hadamard_dense; dense H*x (n <= 64), exact integer inputs at full n,
 * involution, Parseval, unit vectors for hblo_fwht_rows; a hand-derived n=4
 * example, range / boundary invariants and Gaussian closed forms for the
 * quantisers; int64 brute force for hblo_gemm_i32; an fp64 float reference
 * and a hand identity-weight case for the epilogue; for
 * hblo_hadamard_backward the adjoint identity <H x, y> = <x, H y> on exact
 * integers, the gradient of a linear functional through the dense matrix
 * (n <= 64) and an independent bf16 rounding; for hblo_rmsnorm hand cases
 * with power-of-two factors, unit mean square, scale invariance, the
 * placement of ln_eps and an fp64 reference; for hblo_kv_quant_absmax
 * equality with the pinned Eq. 5 quantiser at 8 bits, hand rows at 4 and 3
 * bits, the half-step reconstruction bound, code range and extremes, and a
 * bit-by-bit unpacking of the packed stream written out in the test.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define HBLO_OK 0
#define HBLO_E_ARG (-1)
#define HBLO_F32 0
#define HBLO_BF16 1

int hblo_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* bf16 <-> fp32.  Widening is exact; narrowing rounds to nearest, ties to even. */
static float bf16_to_f32(uint16_t b) {
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return f;
}

static uint16_t f32_to_bf16_rne(float f) {
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x0040u); /* NaN stays NaN */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return (uint16_t)(u >> 16);
}

/* Eq. 2: RoundClip(x, a, b) = min(max(round(x), a), b). */
static float round_clip(float x, float a, float b) {
    float r = rintf(x);
    r = r < a ? a : r; /* max(round(x), a) */
    r = r > b ? b : r; /* min(.., b)       */
    return r;
}

static int is_pow2(int64_t n) { return n > 0 && (n & (n - 1)) == 0; }

/* ------------------------------------------------------------------------
 * Eq. 1: per-tensor absmean ternary weight quantiser.
 *   alpha = mean(|W|);  codes = RoundClip(W / (alpha + eps), -1, 1).
 * The dequantised weight is alpha * codes.
 * ---------------------------------------------------------------------- */
int hblo_ternarize_weights_absmean(const float* W, int64_t N, int64_t K, float eps,
                                   int8_t* codes, float* alpha_out) {
    if (!W || !codes || !alpha_out || N <= 0 || K <= 0) return HBLO_E_ARG;
    const int64_t count = N * K;
    double sum = 0.0;
    for (int64_t i = 0; i < count; ++i) sum += fabs((double)W[i]);
    const float alpha = (float)(sum / (double)count);
    const float denom = alpha + eps;
    for (int64_t i = 0; i < count; ++i) codes[i] = (int8_t)round_clip(W[i] / denom, -1.0f, 1.0f);
    *alpha_out = alpha;
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Eq. 4: the dense Hadamard matrix by its recursion, H_0 = (1),
 *   H_m = 1/sqrt(2) [[H_{m-1}, H_{m-1}], [H_{m-1}, -H_{m-1}]],
 * written row-major into H[n*n], n = 2^m, in fp64.  For tests only.
 * ---------------------------------------------------------------------- */
int hblo_hadamard_dense(int m, double* H) {
    if (m < 0 || m > 12 || !H) return HBLO_E_ARG;
    const int64_t n = (int64_t)1 << m;
    H[0] = 1.0;
    for (int level = 1; level <= m; ++level) {
        const int64_t h = (int64_t)1 << (level - 1); /* size of H_{level-1} */
        const double r = 1.0 / sqrt(2.0);
        /* fill the three new blocks from the top-left block, then scale all four */
        for (int64_t i = 0; i < h; ++i)
            for (int64_t j = 0; j < h; ++j) {
                const double v = H[i * n + j] * r;
                H[i * n + j] = v;
                H[i * n + (j + h)] = v;
                H[(i + h) * n + j] = v;
                H[(i + h) * n + (j + h)] = -v;
            }
    }
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Eq. 3-4 by the fast transform: u <- H_m u for one row of n = 2^m fp32
 * values.  Unnormalised butterflies with ascending stride, then one multiply
 * by c_n = (float)(1/sqrt(n)).
 * ---------------------------------------------------------------------- */
static void fwht_row(float* u, int64_t n) {
    for (int64_t h = 1; h < n; h <<= 1) {
        for (int64_t i = 0; i < n; ++i) {
            if ((i & h) == 0) {
                const float a = u[i];
                const float b = u[i + h];
                u[i] = a + b;
                u[i + h] = a - b;
            }
        }
    }
    const float c_n = (float)(1.0 / sqrt((double)n));
    for (int64_t i = 0; i < n; ++i) u[i] = u[i] * c_n;
}

/* In-place transform of T rows of length n (fp32). */
int hblo_fwht_rows(float* x, int64_t T, int64_t n) {
    if (!x || T < 0 || !is_pow2(n)) return HBLO_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) fwht_row(x + t * n, n);
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Eq. 5 / Eq. 6 for one row x_r of length n.
 *   INT8: gamma = max|x|,  q = RoundClip(127/(gamma+eps) * x, -128, 127),  s_d = gamma/127
 *   INT4: beta  = mean|x|, q = RoundClip(sqrt7/(beta+eps) * x, -8, 7),     s_d = beta/sqrt7
 * ---------------------------------------------------------------------- */
static void quant_row(const float* xr, int64_t n, int bits, float eps, int8_t* q, float* s_dequant) {
    float s_q, s_d, lo, hi;
    if (bits == 8) {
        float gamma = 0.0f;
        for (int64_t i = 0; i < n; ++i) {
            const float a = fabsf(xr[i]);
            if (a > gamma) gamma = a;
        }
        s_q = 127.0f / (gamma + eps);
        s_d = gamma / 127.0f;
        lo = -128.0f;
        hi = 127.0f;
    } else {
        double sum = 0.0;
        for (int64_t i = 0; i < n; ++i) sum += fabs((double)xr[i]);
        const float beta = (float)(sum / (double)n);
        const float root7 = (float)sqrt(7.0);
        s_q = root7 / (beta + eps);
        s_d = beta / root7;
        lo = -8.0f;
        hi = 7.0f;
    }
    for (int64_t i = 0; i < n; ++i) q[i] = (int8_t)round_clip(s_q * xr[i], lo, hi);
    *s_dequant = s_d;
}

static void load_row_f32(const void* x, int x_dtype, int64_t t, int64_t K, float* dst) {
    if (x_dtype == HBLO_F32) {
        memcpy(dst, (const float*)x + t * K, (size_t)K * sizeof(float));
    } else {
        const uint16_t* p = (const uint16_t*)x + t * K;
        for (int64_t k = 0; k < K; ++k) dst[k] = bf16_to_f32(p[k]);
    }
}

/* ------------------------------------------------------------------------
 * LN of Eq. 7, read as the model's RMS normalisation (Section 2, first
 * paragraph: LLaMA-like components, RMS normalisation, no bias):
 *   x_n[k] = x[k] / sqrt( mean_k x[k]^2 + ln_eps ) * g[k]
 * Evaluation order taken here (the paper is silent): the mean of squares in
 * fp64, r = (float)(1 / sqrt(ms + ln_eps)) rounded to fp32 once, then
 * x_n[k] = (x[k] * r) * g[k] as two fp32 multiplies.
 *   x    [T,K] fp32 or bf16 bit patterns;  g [K] fp32;  out [T,K] fp32
 * ---------------------------------------------------------------------- */
int hblo_rmsnorm(const void* x, int x_dtype, int64_t T, int64_t K, const float* g, float ln_eps, float* out) {
    if (!x || !g || !out || T < 0 || K <= 0) return HBLO_E_ARG;
    if (x_dtype != HBLO_F32 && x_dtype != HBLO_BF16) return HBLO_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float* u = out + t * K;
        load_row_f32(x, x_dtype, t, K, u);
        double ss = 0.0;
        for (int64_t k = 0; k < K; ++k) ss += (double)u[k] * (double)u[k];
        const float r = (float)(1.0 / sqrt(ss / (double)K + (double)ln_eps));
        for (int64_t k = 0; k < K; ++k) {
            const float scaled = u[k] * r;
            u[k] = scaled * g[k];
        }
    }
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Backward pass through the transform (Section 2.2, Eq. 8): the gradient with
 * respect to X is Hadamard() of the gradient with respect to Hadamard(X) -
 * H_m is symmetric and orthogonal, so its transpose is itself.  The quantiser
 * is bypassed (straight-through estimator), so this is the whole backward of
 * the activation front end.  The same routine on X gives X_r of Eq. 3.
 *   g    [T,n] fp32 or bf16 bit patterns (upstream gradient rows)
 *   out  [T,n] fp32, or bf16 bit patterns rounded to nearest even
 * ---------------------------------------------------------------------- */
int hblo_hadamard_backward(const void* g, int g_dtype, int64_t T, int64_t n, void* out, int out_dtype) {
    if (!g || !out || T < 0 || !is_pow2(n)) return HBLO_E_ARG;
    if ((g_dtype != HBLO_F32 && g_dtype != HBLO_BF16) || (out_dtype != HBLO_F32 && out_dtype != HBLO_BF16))
        return HBLO_E_ARG;
    int bad = 0;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        float* u = (float*)malloc((size_t)n * sizeof(float));
        if (!u) {
            bad = 1;
            continue;
        }
        load_row_f32(g, g_dtype, t, n, u);
        fwht_row(u, n);
        if (out_dtype == HBLO_F32) {
            memcpy((float*)out + t * n, u, (size_t)n * sizeof(float));
        } else {
            uint16_t* o = (uint16_t*)out + t * n;
            for (int64_t i = 0; i < n; ++i) o[i] = f32_to_bf16_rne(u[i]);
        }
        free(u);
    }
    return bad ? HBLO_E_ARG : HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Activation front end of Eq. 7: X_r = Hadamard(X) (skipped for the plain
 * BitLinear of the other projections), then the per-token quantiser.
 *   x        [T,K] fp32 or bf16 bit patterns
 *   codes    [T,K] int8 out, natural feature order
 *   s_deq    [T]   fp32 out, gamma/127 or beta/sqrt7
 *   xr_out   [T,K] fp32 out or NULL: the transformed activations
 * ---------------------------------------------------------------------- */
int hblo_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, int bits, float eps,
                    int hadamard, int8_t* codes, float* s_deq, float* xr_out) {
    if (!x || !codes || !s_deq || T < 0 || K <= 0) return HBLO_E_ARG;
    if (bits != 4 && bits != 8) return HBLO_E_ARG;
    if (x_dtype != HBLO_F32 && x_dtype != HBLO_BF16) return HBLO_E_ARG;
    if (hadamard && !is_pow2(K)) return HBLO_E_ARG;
    int failed = 0;
#pragma omp parallel
    {
        float* u = (float*)malloc((size_t)K * sizeof(float));
        if (!u) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(static)
        for (int64_t t = 0; t < T; ++t) {
            if (!u) continue;
            load_row_f32(x, x_dtype, t, K, u);
            if (hadamard) fwht_row(u, K);
            if (xr_out) memcpy(xr_out + t * K, u, (size_t)K * sizeof(float));
            quant_row(u, K, bits, eps, codes + t * K, s_deq + t);
        }
        free(u);
    }
    return failed ? HBLO_E_ARG : HBLO_OK;
}

/* ------------------------------------------------------------------------
 * The integer contraction of Eq. 7: acc[t][o] = sum_k q[t][k] * c[o][k].
 * Exact: |acc| <= 128 * K.
 * ---------------------------------------------------------------------- */
int hblo_gemm_i32(const int8_t* q, int64_t T, int64_t K, const int8_t* c, int64_t N, int32_t* acc) {
    if (!q || !c || !acc || T < 0 || K <= 0 || N <= 0) return HBLO_E_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        const int8_t* qr = q + t * K;
        for (int64_t o = 0; o < N; ++o) {
            const int8_t* cr = c + o * K;
            int32_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += (int32_t)qr[k] * (int32_t)cr[k];
            acc[t * N + o] = s;
        }
    }
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Outer factors of Eq. 1 and Eq. 5/6 applied to the integer product:
 *   y[t][o] = bf16( ((float)acc * s_d[t]) * alpha_g(o) ),
 * alpha_g(o) = w_scales[o / (N / groups)] (one absmean scale per row group of
 * W; groups = 1 is the paper's per-tensor scale).
 * ---------------------------------------------------------------------- */
int hblo_dequant_bf16(const int32_t* acc, int64_t T, int64_t N, const float* s_deq,
                      const float* w_scales, int64_t groups, uint16_t* y) {
    if (!acc || !s_deq || !w_scales || !y || groups <= 0 || N % groups != 0) return HBLO_E_ARG;
    const int64_t rows_per_group = N / groups;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int64_t o = 0; o < N; ++o) {
            const float a = (float)acc[t * N + o];
            const float v = (a * s_deq[t]) * w_scales[o / rows_per_group];
            y[t * N + o] = f32_to_bf16_rne(v);
        }
    return HBLO_OK;
}

/* ------------------------------------------------------------------------
 * Eq. 7 end to end (hadamard = 1: H-BitLinear; 0: plain BitLinear).
 *   wcodes [N,K] int8 ternary codes from hblo_ternarize_weights_absmean
 *   y      [T,N] bf16 bit patterns out
 *   codes_out / sdeq_out / acc_out: optional intermediates (NULL to skip)
 * ---------------------------------------------------------------------- */
int hblo_bitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const int8_t* wcodes,
                           int64_t N, const float* w_scales, int64_t groups, int bits, float eps,
                           int hadamard, uint16_t* y, int8_t* codes_out, float* sdeq_out,
                           int32_t* acc_out) {
    if (!x || !wcodes || !w_scales || !y) return HBLO_E_ARG;
    if (T == 0) return HBLO_OK;
    int8_t* codes = codes_out ? codes_out : (int8_t*)malloc((size_t)(T * K));
    float* sdeq = sdeq_out ? sdeq_out : (float*)malloc((size_t)T * sizeof(float));
    int32_t* acc = acc_out ? acc_out : (int32_t*)malloc((size_t)(T * N) * sizeof(int32_t));
    int rc = (codes && sdeq && acc) ? HBLO_OK : HBLO_E_ARG;
    if (rc == HBLO_OK) rc = hblo_fwht_quant(x, x_dtype, T, K, bits, eps, hadamard, codes, sdeq, NULL);
    if (rc == HBLO_OK) rc = hblo_gemm_i32(codes, T, K, wcodes, N, acc);
    if (rc == HBLO_OK) rc = hblo_dequant_bf16(acc, T, N, sdeq, w_scales, groups, y);
    if (!codes_out) free(codes);
    if (!sdeq_out) free(sdeq);
    if (!acc_out) free(acc);
    return rc;
}

/* ------------------------------------------------------------------------
 * Low-bit Q/K/V head states (Section 3.1, Main Results, low-bit attention; reading in the
 * header).  One row = one head of one token after RoPE, d values.
 *   gamma = max|h|,  qmax = 2^(b-1) - 1,  s_q = qmax / (gamma + eps)  (fp32 division)
 *   u[i]  = RoundClip(s_q * h[i], -2^(b-1), qmax) + 2^(b-1)           in [0, 2^b - 1]
 *   scale = gamma / qmax                                             (fp32 division)
 *   x      [rows, d] fp32 or bf16 bit patterns
 *   codes  [rows, d] unsigned codes, one per byte (unpacked)
 *   packed [rows, d*bits/8] or NULL: code i of a row at bits [bits*i, bits*i + bits) of the row's
 *          little-endian bit string (8 bits: bytes; 4 bits: low nibble first; 3 bits: 8 codes in 3 bytes)
 *   scales [rows] fp32
 * bits is 8, 4 or 3; d must make d*bits a multiple of 8.
 * ---------------------------------------------------------------------- */
int hblo_kv_quant_absmax(const void* x, int x_dtype, int64_t rows, int64_t d, int bits, float eps,
                         uint8_t* codes, uint8_t* packed, float* scales) {
    if (!x || !codes || !scales || rows < 0 || d <= 0) return HBLO_E_ARG;
    if (x_dtype != HBLO_F32 && x_dtype != HBLO_BF16) return HBLO_E_ARG;
    if (bits != 8 && bits != 4 && bits != 3) return HBLO_E_ARG;
    if ((d * bits) % 8 != 0) return HBLO_E_ARG;
    const int half = 1 << (bits - 1);
    const float qmax = (float)(half - 1);
    const int64_t row_bytes = d * bits / 8;
#pragma omp parallel
    {
        float* h = (float*)malloc((size_t)d * sizeof(float));
#pragma omp for schedule(static)
        for (int64_t r = 0; r < rows; ++r) {
            load_row_f32(x, x_dtype, r, d, h);
            float gamma = 0.0f;
            for (int64_t i = 0; i < d; ++i) {
                const float a = fabsf(h[i]);
                if (a > gamma) gamma = a;
            }
            const float s_q = qmax / (gamma + eps);
            scales[r] = gamma / qmax;
            for (int64_t i = 0; i < d; ++i)
                codes[r * d + i] = (uint8_t)((int)round_clip(s_q * h[i], -(float)half, qmax) + half);
            if (packed) {
                uint8_t* out = packed + r * row_bytes;
                memset(out, 0, (size_t)row_bytes);
                for (int64_t i = 0; i < d; ++i)
                    for (int b = 0; b < bits; ++b) {
                        const int64_t pos = i * bits + b;
                        if ((codes[r * d + i] >> b) & 1) out[pos >> 3] |= (uint8_t)(1u << (pos & 7));
                    }
            }
        }
        free(h);
    }
    return HBLO_OK;
}

/* Inverse map of the above: h^[i] = ((float)u[i] - 2^(b-1)) * scale, as fp32 (out_dtype F32) or rounded to
 * nearest even to bf16.  codes are the unpacked unsigned codes. */
int hblo_kv_dequant(const uint8_t* codes, const float* scales, int64_t rows, int64_t d, int bits, void* out,
                    int out_dtype) {
    if (!codes || !scales || !out || rows < 0 || d <= 0) return HBLO_E_ARG;
    if (bits != 8 && bits != 4 && bits != 3) return HBLO_E_ARG;
    if (out_dtype != HBLO_F32 && out_dtype != HBLO_BF16) return HBLO_E_ARG;
    const float half = (float)(1 << (bits - 1));
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t i = 0; i < d; ++i) {
            const float v = ((float)codes[r * d + i] - half) * scales[r];
            if (out_dtype == HBLO_F32) ((float*)out)[r * d + i] = v;
            else ((uint16_t*)out)[r * d + i] = f32_to_bf16_rne(v);
        }
    return HBLO_OK;
}
