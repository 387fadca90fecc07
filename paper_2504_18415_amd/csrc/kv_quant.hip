// Low-bit Q/K/V head states (Section 3.1, Main Results: the 8/4/3-bit attention results): per head row of d values
//   gamma = max|h|,  qmax = 2^(b-1) - 1,
//   u[i]  = RoundClip(qmax/(gamma+eps) * h[i], -2^(b-1), qmax) + 2^(b-1)   (unsigned, in [0, 2^b - 1])
//   scale = gamma / qmax,   h^[i] = (u[i] - 2^(b-1)) * scale.
// The paper names the method (absmax, to unsigned codes) and prints no formula; this is Eq. 5 at b bits with an
// offset (Eq. 5 itself plus 128 at b = 8).  Round-half-to-even, IEEE fp32 divisions, eps added as in Eq. 5.
//
// Memory-bound streaming kernels.  A thread owns 8 consecutive values (one 16-byte load of bf16, two of
// fp32); the d/8 threads of a row are neighbouring lanes of one wave, so the row maximum is a handful of
// xor-shuffles.  The packed output is one flat little-endian bit string (row r starts at byte r*d*b/8, code i
// of a row at bits [b*i, b*i+b)): a thread's 8 codes are 8, 4 or 3 bytes; at 3 bits the four lanes of a quad
// merge their 24-bit pieces into three dwords so that every store is an aligned dword.
#include "hbl_internal.h"

namespace hbl {
namespace {

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

constexpr float kMagic = 12582912.0f;   // 1.5 * 2^23: adding it rounds to an integer (nearest-even)

template <int CTRL>
__device__ __forceinline__ uint32_t quad_lane(uint32_t v) {   // value of one fixed lane of the quad
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, false);
}

constexpr int kItems = 1;   // 16-byte pieces per thread, all loaded before any arithmetic (2 measured no faster:
                            // the kernel already runs at the rate a plain copy reaches on this chip)

template <int BITS, bool BF16>
__global__ __launch_bounds__(256) void kv_quant_kernel(const void* __restrict__ x, int64_t threads, int lanes_per_row,
                                                       float eps, uint8_t* __restrict__ packed,
                                                       float* __restrict__ scales) {
    const int64_t t0 = (int64_t)blockIdx.x * (256 * kItems) + threadIdx.x;
    uint4 raw[kItems][BF16 ? 1 : 2];
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t t = t0 + 256 * k;
#pragma unroll
        for (int q = 0; q < (BF16 ? 1 : 2); ++q) raw[k][q] = make_uint4(0, 0, 0, 0);
        if (t < threads) {   // whole rows (and whole quads) are live or not: lanes_per_row divides 64
            if constexpr (BF16) {
                raw[k][0] = reinterpret_cast<const uint4*>(x)[t];
            } else {
                raw[k][0] = reinterpret_cast<const uint4*>(x)[2 * t];
                raw[k][1] = reinterpret_cast<const uint4*>(x)[2 * t + 1];
            }
        }
    }
#pragma unroll
    for (int k = 0; k < kItems; ++k) {
        const int64_t t = t0 + 256 * k;
        const bool live = t < threads;
        float h[8];
        if constexpr (BF16) {
            const uint32_t w[4] = {raw[k][0].x, raw[k][0].y, raw[k][0].z, raw[k][0].w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                h[2 * i] = as_f(w[i] << 16);
                h[2 * i + 1] = as_f(w[i] & 0xFFFF0000u);
            }
        } else {
            h[0] = as_f(raw[k][0].x); h[1] = as_f(raw[k][0].y); h[2] = as_f(raw[k][0].z); h[3] = as_f(raw[k][0].w);
            h[4] = as_f(raw[k][1].x); h[5] = as_f(raw[k][1].y); h[6] = as_f(raw[k][1].z); h[7] = as_f(raw[k][1].w);
        }
        float gamma = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) gamma = fmaxf(gamma, fabsf(h[i]));
        for (int m = 1; m < lanes_per_row; m <<= 1) gamma = fmaxf(gamma, __shfl_xor(gamma, m, 64));

        constexpr int half = 1 << (BITS - 1);
        constexpr float qmax = (float)(half - 1);
        const float s_q = qmax / (gamma + eps);
        if (live && (t % lanes_per_row) == 0) scales[t / lanes_per_row] = gamma / qmax;

        // t + (1.5*2^23 + half): the fp32 adder rounds to nearest even and leaves code + half in the low mantissa bits
        uint32_t u[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            u[i] = as_u(__builtin_amdgcn_fmed3f(h[i] * s_q, -(float)half, qmax) + (kMagic + (float)half)) & 0xFFu;

        if constexpr (BITS == 8) {
            if (live)
                reinterpret_cast<uint2*>(packed)[t] = make_uint2(u[0] | (u[1] << 8) | (u[2] << 16) | (u[3] << 24),
                                                                 u[4] | (u[5] << 8) | (u[6] << 16) | (u[7] << 24));
        } else if constexpr (BITS == 4) {
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) w |= u[i] << (4 * i);
            if (live) reinterpret_cast<uint32_t*>(packed)[t] = w;
        } else {
            uint32_t w = 0;
#pragma unroll
            for (int i = 0; i < 8; ++i) w |= u[i] << (3 * i);   // 24 bits
            // quad_perm [k,k,k,k]: every lane of the quad reads lane k's piece
            const uint32_t v0 = quad_lane<0x00>(w), v1 = quad_lane<0x55>(w), v2 = quad_lane<0xAA>(w), v3 = quad_lane<0xFF>(w);
            const int q = (int)(t & 3);
            const uint32_t dword = q == 0 ? (v0 | (v1 << 24)) : q == 1 ? ((v1 >> 8) | (v2 << 16)) : ((v2 >> 16) | (v3 << 8));
            if (live && q < 3) reinterpret_cast<uint32_t*>(packed)[3 * (t >> 2) + q] = dword;
        }
    }
}

template <int BITS, bool BF16OUT>
__global__ __launch_bounds__(256) void kv_dequant_kernel(const uint8_t* __restrict__ packed,
                                                         const float* __restrict__ scales, int64_t threads,
                                                         int lanes_per_row, void* __restrict__ out) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= threads) return;
    uint32_t u[8];
    if constexpr (BITS == 8) {
        const uint2 w = reinterpret_cast<const uint2*>(packed)[t];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            u[i] = (w.x >> (8 * i)) & 0xFFu;
            u[4 + i] = (w.y >> (8 * i)) & 0xFFu;
        }
    } else if constexpr (BITS == 4) {
        const uint32_t w = reinterpret_cast<const uint32_t*>(packed)[t];
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = (w >> (4 * i)) & 0xFu;
    } else {
        // three bytes at byte 3t: from the aligned dword that holds the first one and, if they straddle, the next
        // (the thread count is a multiple of 4, so the stream is a whole number of dwords and 3t + 2 is inside it)
        const int64_t byte = 3 * t;
        const uint32_t* p = reinterpret_cast<const uint32_t*>(packed) + (byte >> 2);
        const int sh = (int)(byte & 3);
        const uint32_t lo = p[0];
        const uint32_t hi = sh >= 2 ? p[1] : 0u;
        const uint32_t w = __builtin_amdgcn_alignbyte(hi, lo, sh);
#pragma unroll
        for (int i = 0; i < 8; ++i) u[i] = (w >> (3 * i)) & 0x7u;
    }
    const float scale = scales[t / lanes_per_row];
    constexpr float half = (float)(1 << (BITS - 1));
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = ((float)u[i] - half) * scale;
    if constexpr (BF16OUT) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){v[2 * i], v[2 * i + 1]}, bf16x2));
        reinterpret_cast<uint4*>(out)[t] = make_uint4(w[0], w[1], w[2], w[3]);
    } else {
        reinterpret_cast<float4*>(out)[2 * t] = make_float4(v[0], v[1], v[2], v[3]);
        reinterpret_cast<float4*>(out)[2 * t + 1] = make_float4(v[4], v[5], v[6], v[7]);
    }
}

}  // namespace

bool kv_shape_ok(int64_t rows, int64_t d, int bits) {
    if (rows < 0 || rows > 0x7FFFFFFF || (bits != 8 && bits != 4 && bits != 3)) return false;   // grid fits 32 bits
    return d == 32 || d == 64 || d == 128 || d == 256 || d == 512;   // d/8 lanes per row, a power of two in 4..64
}

int launch_kv_quant(const void* x, int x_dtype, int64_t rows, int64_t d, int bits, float eps, void* packed,
                    float* scales, hipStream_t stream) {
    const int64_t threads = rows * (d / 8);
    if (threads == 0) return HBL_OK;
    const dim3 grid((unsigned)((threads + 256 * kItems - 1) / (256 * kItems))), block(256);
    const int lpr = (int)(d / 8);
    uint8_t* out = static_cast<uint8_t*>(packed);
    const bool bf = x_dtype == HBL_BF16;
#define HBL_KVQ(B)                                                                                               \
    if (bf) launch_kernel("kv_quant_kernel", (kv_quant_kernel<B, true>), grid, block, 0, stream, x, threads, lpr, eps, out, scales); \
    else launch_kernel("kv_quant_kernel", (kv_quant_kernel<B, false>), grid, block, 0, stream, x, threads, lpr, eps, out, scales);
    if (bits == 8) { HBL_KVQ(8) } else if (bits == 4) { HBL_KVQ(4) } else { HBL_KVQ(3) }
#undef HBL_KVQ
    return after_launch();
}

int launch_kv_dequant(const void* packed, const float* scales, int64_t rows, int64_t d, int bits, void* out,
                      int out_dtype, hipStream_t stream) {
    const int64_t threads = rows * (d / 8);
    if (threads == 0) return HBL_OK;
    const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    const int lpr = (int)(d / 8);
    const uint8_t* in = static_cast<const uint8_t*>(packed);
    const bool bf = out_dtype == HBL_BF16;
#define HBL_KVD(B)                                                                                              \
    if (bf) launch_kernel("kv_dequant_kernel", (kv_dequant_kernel<B, true>), grid, block, 0, stream, in, scales, threads, lpr, out);  \
    else launch_kernel("kv_dequant_kernel", (kv_dequant_kernel<B, false>), grid, block, 0, stream, in, scales, threads, lpr, out);
    if (bits == 8) { HBL_KVD(8) } else if (bits == 4) { HBL_KVD(4) } else { HBL_KVD(3) }
#undef HBL_KVD
    return after_launch();
}

}  // namespace hbl
