// Weight set-up kernels: the per-tensor absmean ternary quantiser (Eq. 1-2) and the
// 2-bit packing of its codes into the streaming layout the GEMM kernels read.
//
// Packed layout (one form, 2 bits per weight, read by every GEMM kernel).  The [N, K] code matrix is cut into
// tiles of 32 output rows x 128 input features, stored K-block-major (all row tiles of features 0..127, then
// all of 128..255, ...):
//   tile(nt, kb) at byte ((kb * (N/32) + nt) * 1024), nt = o / 32, kb = k / 128,
// so that a prefill workgroup's stage (16 row tiles of one K-block) is one contiguous 16 KiB piece and the waves
// of a small-batch launch, each walking the K range of its own row tile, together sweep memory linearly.
// A tile is 64 lanes x 4 dwords (lane-major, 16 bytes per lane).  Lane l, dword j holds the 16 weights of
// row 32*nt + (l & 31) at features
//   k = 128*kb + 64*(j >> 1) + 32*(l >> 5) + 16*(j & 1) + i,  i = 0..15,
// i.e. dwords 2s, 2s+1 are one lane's share of the A operand of a 32x32x64 fp6/fp4 MFMA for K-step s, and
// dword j one lane's share of a 32x32x32 int8 MFMA operand.  A weight is a (sign, magnitude) bit pair:
// weight i < 8 has its magnitude at bit 4*i + 1 and its sign at bit 4*i + 3, weight i >= 8 its magnitude at
// bit 4*(i-8) and its sign at bit 4*(i-8) + 2.  Then
//   p & 0xAAAAAAAA  and  (p << 1) & 0xAAAAAAAA
// are eight fp4 (e2m1) values each (+-1.0 = s010, 0 = 0000), and (p >> {0,1,4,5}) & 0x05050505 are four
// weights each as byte values {0, 1, 5} that one byte-permute look-up turns into int8 {0, +1, -1}.
// After the N*K/4 bytes of tiles come N int32 row sums sum_k c[o][k] (the epilogue of the int8 path needs
// them when activation codes are stored with an offset).
#include "hbl_internal.h"

namespace hbl {
namespace {

constexpr int kSumBlock = 256;
constexpr int kSumItems = 16;  // floats per thread per block

// Eq. 1: partial sums of |W| in fp64, one per workgroup, fixed order inside the workgroup.
__global__ __launch_bounds__(kSumBlock) void abs_sum_partial_kernel(const float* __restrict__ W, int64_t count,
                                                                    double* __restrict__ partial) {
    __shared__ double red[kSumBlock / 64];
    const int64_t base = (int64_t)blockIdx.x * (kSumBlock * kSumItems);
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < kSumItems; ++i) {
        const int64_t idx = base + (int64_t)i * kSumBlock + threadIdx.x;
        if (idx < count) s += (double)fabsf(W[idx]);
    }
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) s += __shfl_xor(s, sft, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = red[0];
        for (int w = 1; w < kSumBlock / 64; ++w) t += red[w];
        partial[blockIdx.x] = t;
    }
}

// Final reduction by one workgroup (fixed order), alpha = (float)(sum / count).
__global__ __launch_bounds__(256) void abs_mean_final_kernel(const double* __restrict__ partial, int64_t nparts,
                                                             int64_t count, float* __restrict__ alpha) {
    __shared__ double red[4];
    double s = 0.0;
    for (int64_t i = threadIdx.x; i < nparts; i += 256) s += partial[i];
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) s += __shfl_xor(s, sft, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        const double t = ((red[0] + red[1]) + red[2]) + red[3];
        *alpha = (float)(t / (double)count);
    }
}

// Eq. 1-2: codes = RoundClip(W / (alpha + eps), -1, 1).
__global__ __launch_bounds__(256) void ternarize_kernel(const float* __restrict__ W, int64_t count,
                                                        const float* __restrict__ alpha, float eps,
                                                        int8_t* __restrict__ codes) {
    const float denom = *alpha + eps;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += stride) {
        float r = rintf(W[i] / denom);
        r = fminf(fmaxf(r, -1.0f), 1.0f);
        codes[i] = (int8_t)(int)r;
    }
}

// dword d of the packed stream -> (row, first feature) of its 16 weights
__device__ __forceinline__ void packed_dword_origin(int64_t d, int64_t N, int64_t* row, int64_t* k0) {
    const int64_t ntiles = N / 32;
    const int dd = (int)(d & 3);
    const int lane = (int)((d >> 2) & 63);
    const int64_t tile = d >> 8;
    const int64_t kb = tile / ntiles, nt = tile % ntiles;
    *row = nt * 32 + (lane & 31);
    *k0 = kb * 128 + (dd >> 1) * 64 + (lane >> 5) * 32 + (dd & 1) * 16;
}

__global__ __launch_bounds__(256) void unpack_kernel(const uint32_t* __restrict__ packed, int64_t N, int64_t K,
                                                     int8_t* __restrict__ codes) {
    const int64_t total = (N / 32) * (K / 128) * 256;
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d >= total) return;
    int64_t row, k0;
    packed_dword_origin(d, N, &row, &k0);
    const uint32_t p = packed[d];
    uint4 raw;
    int8_t* c = reinterpret_cast<int8_t*>(&raw);
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        const int ma = (p >> (4 * n + 1)) & 1, sa = (p >> (4 * n + 3)) & 1;
        const int mb = (p >> (4 * n)) & 1, sb = (p >> (4 * n + 2)) & 1;
        c[n] = (int8_t)(sa ? -ma : ma);
        c[8 + n] = (int8_t)(sb ? -mb : mb);
    }
    *reinterpret_cast<uint4*>(codes + row * K + k0) = raw;
}

__global__ __launch_bounds__(256) void pack_kernel(const int8_t* __restrict__ codes, int64_t N, int64_t K,
                                                      uint32_t* __restrict__ packed) {
    const int64_t total = (N / 32) * (K / 128) * 256;  // dwords
    const int64_t d = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (d >= total) return;
    int64_t row, k0;
    packed_dword_origin(d, N, &row, &k0);
    const uint4 raw = *reinterpret_cast<const uint4*>(codes + row * K + k0);
    const int8_t* c = reinterpret_cast<const int8_t*>(&raw);
    uint32_t out = 0;
#pragma unroll
    for (int n = 0; n < 8; ++n) {
        const int a = c[n], b = c[8 + n];
        out |= (uint32_t)(a != 0) << (4 * n + 1);
        out |= (uint32_t)(a < 0) << (4 * n + 3);
        out |= (uint32_t)(b != 0) << (4 * n);
        out |= (uint32_t)(b < 0) << (4 * n + 2);
    }
    packed[d] = out;
}

// Row sums of the ternary codes, sum_k c[o][k], one wave per output row.
__global__ __launch_bounds__(256) void row_sum_kernel(const int8_t* __restrict__ codes, int64_t N, int64_t K,
                                                      int32_t* __restrict__ row_sum) {
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= N) return;
    const int lane = threadIdx.x & 63;
    int s = 0;
    for (int64_t k = lane * 16; k < K; k += 64 * 16) {
        const uint4 raw = *reinterpret_cast<const uint4*>(codes + row * K + k);
        const int8_t* c = reinterpret_cast<const int8_t*>(&raw);
#pragma unroll
        for (int i = 0; i < 16; ++i) s += c[i];
    }
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) s += __shfl_xor(s, sft, 64);
    if (lane == 0) row_sum[row] = s;
}

int64_t sum_blocks(int64_t count) { return (count + kSumBlock * kSumItems - 1) / (kSumBlock * kSumItems); }

}  // namespace

size_t ternarize_workspace_bytes(int64_t count) { return round_up((size_t)sum_blocks(count) * sizeof(double), 256); }

int launch_ternarize(const float* W, int64_t count, float eps, int8_t* codes, float* alpha, void* workspace,
                     hipStream_t stream) {
    double* partial = static_cast<double*>(workspace);
    const int64_t nb = sum_blocks(count);
    launch_kernel("abs_sum_partial_kernel", abs_sum_partial_kernel, dim3((unsigned)nb), dim3(kSumBlock), 0, stream, W, count, partial);
    int rc = after_launch();
    if (rc != HBL_OK) return rc;
    launch_kernel("abs_mean_final_kernel", abs_mean_final_kernel, dim3(1), dim3(256), 0, stream, partial, nb, count, alpha);
    rc = after_launch();
    if (rc != HBL_OK) return rc;
    int64_t blocks = (count + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    launch_kernel("ternarize_kernel", ternarize_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, W, count, alpha, eps, codes);
    return after_launch();
}

int launch_pack(const int8_t* codes, int64_t N, int64_t K, void* packed, hipStream_t stream) {
    const int64_t total = (N / 32) * (K / 128) * 256;
    launch_kernel("pack_kernel", pack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, codes, N, K,
                  static_cast<uint32_t*>(packed));
    int rc = after_launch();
    if (rc != HBL_OK) return rc;
    int32_t* row_sum = reinterpret_cast<int32_t*>(static_cast<char*>(packed) + packed_tile_bytes(N, K));
    launch_kernel("row_sum_kernel", row_sum_kernel, dim3((unsigned)((N + 3) / 4)), dim3(256), 0, stream, codes, N, K, row_sum);
    return after_launch();
}

int launch_unpack(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream) {
    const int64_t total = (N / 32) * (K / 128) * 256;
    launch_kernel("unpack_kernel", unpack_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream,
                       static_cast<const uint32_t*>(packed), N, K, codes);
    return after_launch();
}

}  // namespace hbl
