// Stand-alone micro-benchmarks of what one MI355X sustains, used to put the library's kernels in
// context: matrix-core rate with register-resident operands for the
// two MFMA forms the GEMM kernels use, by operand bit pattern, and HBM read / copy bandwidth.
// Build and run:  python -m paper_2504_18415_amd.microbench
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

#define CHECK(x)                                                                  \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));        \
            exit(1);                                                              \
        }                                                                         \
    } while (0)

__device__ unsigned lcg(unsigned& h) { return h = h * 1664525u + 1013904223u; }

// 16 independent 32x32x32 int8 MFMAs per iteration and wave, operands fixed in registers
__global__ __launch_bounds__(256) void mfma_i8_kernel(int* out, int iters, unsigned mask_a, unsigned mask_b) {
    unsigned h = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
    v4i a[4], b[4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j) {
            a[i][j] = (int)(lcg(h) & mask_a);
            b[i][j] = (int)(lcg(h) & mask_b);
        }
    v16i acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i & 3], b[i >> 2], acc[i], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

// 16 independent 32x32x64 f8f6f4 MFMAs per iteration and wave: A = fp4 (e2m1), B = bf6 (e3m2)
__global__ __launch_bounds__(256) void mfma_f6f4_kernel(float* out, int iters, unsigned mask_a, unsigned mask_b) {
    unsigned h = (threadIdx.x * 2654435761u) ^ (blockIdx.x * 40503u);
    v8i a[4], b[4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 8; ++j) {
            a[i][j] = (int)(lcg(h) & mask_a);
            b[i][j] = (int)(lcg(h) & mask_b);
        }
    v16f acc[16];
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i)
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i & 3], b[i >> 2], acc[i], 4, 3, 0, 0, 0, 0);
    }
    float s = 0;
    for (int i = 0; i < 16; ++i)
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void read_kernel(const uint4* __restrict__ src, size_t n, uint4* sink) {
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const uint4 v = src[i];
        acc.x ^= v.x; acc.y ^= v.y; acc.z ^= v.z; acc.w ^= v.w;
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u) *sink = acc;   // never true in practice: keeps the loads
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Skeleton of the small-batch weight-streaming kernel: 512 workgroups of 4 waves, every wave walking its own run
// of 1 KiB tiles through a ring of D global->LDS copies (16 bytes per lane), optionally with a second, 768-byte
// copy per stage from a small cache-resident buffer (the activation codes) and with the LDS operand reads and two
// 16x16x128 fp6 x fp4 MFMAs per tile that the real kernel issues.  What a launch of one decode layer's size can
// reach at all with this structure, before any of the library's own bookkeeping.
__device__ __forceinline__ void lds_dma16(unsigned lds_addr, const void* base, unsigned voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}
__device__ __forceinline__ void lds_dma16_first48(unsigned lds_addr, const void* base, unsigned voff) {
    unsigned long long saved;
    asm volatile(
        "s_mov_b64 %0, exec\n\ts_bfm_b64 exec, 48, 0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(voff), "s"(base)
        : "memory", "m0");
}
template <int D, bool CODES, bool WORK>
__global__ __launch_bounds__(256, 2) void stream_skeleton_kernel(const char* __restrict__ src, const char* __restrict__ codes,
                                                                 int tiles_per_wave, uint4* sink) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds + wave * D * 2048;
    const size_t wid = (size_t)blockIdx.x * 4 + wave;
    auto issue = [&](int it, int slot) {
        if (CODES) lds_dma16_first48(lds0 + slot * 2048 + 1024, codes + (size_t)it * 12288, lane * 16);
        lds_dma16(lds0 + slot * 2048, src + (wid * tiles_per_wave + it) * 1024, lane * 16);
    };
    constexpr int PER = CODES ? 2 : 1;
    for (int s = 0; s < D - 1; ++s)
        if (s < tiles_per_wave) issue(s, s);
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f acc[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    unsigned x = 0;
    int slot = 0;
    for (int it = 0; it < tiles_per_wave; ++it) {
        if (tiles_per_wave - 1 - it >= D - 2) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((D - 2) * PER) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        if (it + D - 1 < tiles_per_wave) issue(it + D - 1, slot == 0 ? D - 1 : slot - 1);
        const char* st = lds + wave * D * 2048 + slot * 2048;
        if (WORK) {
            const uint4 lo = *reinterpret_cast<const uint4*>(st + 1024 + (lane & 15) * 48);
            const uint2 hi = *reinterpret_cast<const uint2*>(st + 1024 + (lane & 15) * 48 + 16);
            const v8i b = {(int)lo.x, (int)lo.y, (int)lo.z, (int)lo.w, (int)hi.x, (int)hi.y, 0, 0};
            for (int hf = 0; hf < 2; ++hf) {
                const uint2 wp = *reinterpret_cast<const uint2*>(st + hf * 512 + lane * 8);
                const v8i a = {(int)(wp.x & 0xAAAAAAAAu), (int)((wp.x << 1) & 0xAAAAAAAAu), (int)(wp.y & 0xAAAAAAAAu),
                               (int)((wp.y << 1) & 0xAAAAAAAAu), 0, 0, 0, 0};
                acc[hf] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, acc[hf], 4, 3, 0, 0, 0, 0);
            }
        } else {
            x ^= *reinterpret_cast<const unsigned*>(st + lane * 16);
        }
        slot = slot + 1 == D ? 0 : slot + 1;
    }
    if (x == 0x12345678u || acc[0][0] + acc[1][1] == 1.2345f) sink[0] = make_uint4(x, 0, 0, 0);
}

// Skeleton of the small-batch kernel's shared form (17-64 tokens): per stage the four waves of a workgroup copy 4 x 1 KiB
// of weights and XC x 4 x 768 bytes of codes (XC = 1: 32 token rows, 2: 64) into one stage buffer, meet at a barrier (every
// stage, or every second one with PAIRB = 2), and with WORK read two weight tiles and one token tile and issue 4 MFMAs.
template <int D, int XC, bool WORK, int PAIRB>
__global__ __launch_bounds__(256, 2) void shared_skeleton_kernel(const char* __restrict__ src, const char* __restrict__ codes,
                                                                 int tiles_per_wave, uint4* sink) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    constexpr int XB = XC * 4 * 768, STAGE = XB + 4096;
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) char*)lds;
    const size_t wid = (size_t)blockIdx.x * 4 + wave;
    auto issue = [&](int it, int slot) {
        for (int m = 0; m < XC; ++m)
            lds_dma16_first48(lds0 + slot * STAGE + (wave + 4 * m) * 768, codes + (size_t)it * 12288 + (wave + 4 * m) * 768, lane * 16);
        lds_dma16(lds0 + slot * STAGE + XB + wave * 1024, src + (wid * tiles_per_wave + it) * 1024, lane * 16);
    };
    constexpr int PER = XC + 1;
    constexpr int AHEAD = PAIRB == 2 ? D - 2 : D - 1;
    for (int s = 0; s < AHEAD; ++s)
        if (s < tiles_per_wave) issue(s, s);
    v16f acc[2];
    for (int i = 0; i < 2; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.0f;
    unsigned x = 0;
    int slot = 0;
    for (int it = 0; it < tiles_per_wave; it += PAIRB) {
        // steady state only (tiles_per_wave is a multiple of PAIRB and much larger than D): the tail waits for everything
        if (tiles_per_wave - it > AHEAD) asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((AHEAD - PAIRB) * PER) : "memory");
        else asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        asm volatile("s_barrier" ::: "memory");
        for (int u = 0; u < PAIRB; ++u) {
            const char* st = lds + slot * STAGE;
            uint4 w0, w1, lo0, lo1; uint2 hi0, hi1;
            if (WORK) {
                w0 = *reinterpret_cast<const uint4*>(st + XB + (2 * (wave >> 1)) * 1024 + lane * 16);
                w1 = *reinterpret_cast<const uint4*>(st + XB + (2 * (wave >> 1) + 1) * 1024 + lane * 16);
                const char* rows = st + (XC == 2 ? (wave & 1) * 32 * 96 : 0) + (lane & 31) * 96;
                lo0 = *reinterpret_cast<const uint4*>(rows + (lane >> 5) * 32);
                hi0 = *reinterpret_cast<const uint2*>(rows + 16 + (lane >> 5) * 8);
                lo1 = *reinterpret_cast<const uint4*>(rows + 48 + (lane >> 5) * 32 - (lane >> 5) * 16);
                hi1 = *reinterpret_cast<const uint2*>(rows + 64 + (lane >> 5) * 8);
            } else {
                x ^= *reinterpret_cast<const unsigned*>(st + XB + wave * 1024 + lane * 16);
            }
            const int ahead = it + u + AHEAD;
            if (ahead < tiles_per_wave) { int as = slot + AHEAD; as = as >= D ? as - D : as; issue(ahead, as); }
            if (WORK) {
                const v8i b0 = {(int)lo0.x, (int)lo0.y, (int)lo0.z, (int)lo0.w, (int)hi0.x, (int)hi0.y, 0, 0};
                const v8i b1 = {(int)lo1.x, (int)lo1.y, (int)lo1.z, (int)lo1.w, (int)hi1.x, (int)hi1.y, 0, 0};
                const uint4 ws[2] = {w0, w1};
                for (int i = 0; i < 2; ++i) {
                    const v8i a0 = {(int)(ws[i].x & 0xAAAAAAAAu), (int)((ws[i].x << 1) & 0xAAAAAAAAu), (int)(ws[i].y & 0xAAAAAAAAu), (int)((ws[i].y << 1) & 0xAAAAAAAAu), 0, 0, 0, 0};
                    const v8i a1 = {(int)(ws[i].z & 0xAAAAAAAAu), (int)((ws[i].z << 1) & 0xAAAAAAAAu), (int)(ws[i].w & 0xAAAAAAAAu), (int)((ws[i].w << 1) & 0xAAAAAAAAu), 0, 0, 0, 0};
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a0, b0, acc[i], 4, 3, 0, 0, 0, 0);
                    acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a1, b1, acc[i], 4, 3, 0, 0, 0, 0);
                }
            }
            slot = slot + 1 == D ? 0 : slot + 1;
        }
    }
    if (x == 0x12345678u || acc[0][0] + acc[1][1] == 1.2345f) sink[0] = make_uint4(x, 0, 0, 0);
}

template <class F>
float time_ms(F launch, int reps) {
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0));
    for (int i = 0; i < reps; ++i) launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return ms / reps;
}

int main() {
    const int blocks = 512, iters = 4096;
    void* out;
    CHECK(hipMalloc(&out, (size_t)blocks * 256 * 4));
    struct { const char* name; unsigned ma, mb; } i8[] = {
        {"int8 32x32x32  zeros", 0u, 0u},
        {"int8 32x32x32  4-bit unsigned x {0,1,2}", 0x0F0F0F0Fu, 0x03030303u},
        {"int8 32x32x32  random int8 x {0,1,2}", 0xFFFFFFFFu, 0x03030303u},
        {"int8 32x32x32  random int8 x int8", 0xFFFFFFFFu, 0xFFFFFFFFu}};
    for (auto& p : i8) {
        const float ms = time_ms([&] { mfma_i8_kernel<<<blocks, 256>>>((int*)out, iters, p.ma, p.mb); }, 1);
        printf("%-48s %8.1f TOP/s\n", p.name, (double)blocks * 4 * iters * 16 * 65536.0 / ms / 1e9);
    }
    struct { const char* name; unsigned ma, mb; } f6[] = {
        {"f8f6f4 32x32x64  fp4 x bf6 zeros", 0u, 0u},
        {"f8f6f4 32x32x64  fp4 {0,+-1} x bf6 random", 0xAAAAAAAAu, 0xFFFFFFFFu},
        {"f8f6f4 32x32x64  fp4 x bf6 random bits", 0xFFFFFFFFu, 0xFFFFFFFFu}};
    for (auto& p : f6) {
        const float ms = time_ms([&] { mfma_f6f4_kernel<<<blocks, 256>>>((float*)out, iters, p.ma, p.mb); }, 1);
        printf("%-48s %8.1f TOP/s\n", p.name, (double)blocks * 4 * iters * 16 * 131072.0 / ms / 1e9);
    }
    const size_t bytes = (size_t)2 << 30;   // 2 GiB: far larger than the 256 MB memory-side cache
    uint4 *src, *dst;
    CHECK(hipMalloc(&src, bytes));
    CHECK(hipMalloc(&dst, bytes));
    CHECK(hipMemset(src, 1, bytes));
    CHECK(hipMemset(dst, 0, bytes));
    const float r = time_ms([&] { read_kernel<<<4096, 256>>>(src, bytes / 16, dst); }, 5);
    printf("%-48s %8.1f GB/s\n", "HBM read stream, 2 GiB", bytes / r / 1e6);
    // the same read stream cut into launches of one decode layer's size (64 MiB each, 24 distinct chunks per
    // pass so that nothing is served from cache): what launch ramp and drain leave of the stream rate
    for (int wgs : {512, 1024, 2048, 4096}) {
        const size_t chunk = (size_t)64 << 20;
        const float t = time_ms([&] {
            for (int i = 0; i < 24; ++i)
                read_kernel<<<wgs, 256>>>(src + i * (chunk / 16), chunk / 16, dst);
        }, 3) / 24;
        printf("HBM read, 64 MiB per launch, %4d workgroups      %8.1f GB/s (%.1f us per launch)\n", wgs,
               chunk / t / 1e6, t * 1e3);
    }
    // and one 64 MiB chunk read again and again: every launch after the first is served by the 256 MB
    // memory-side cache, so what remains is the launch's ramp and drain and the fabric, not HBM
    for (int wgs : {1024, 2048}) {
        const size_t chunk = (size_t)64 << 20;
        const float t = time_ms([&] {
            for (int i = 0; i < 24; ++i) read_kernel<<<wgs, 256>>>(src, chunk / 16, dst);
        }, 3) / 24;
        printf("cached read, one 64 MiB chunk, %4d workgroups     %8.1f GB/s (%.1f us per launch)\n", wgs,
               chunk / t / 1e6, t * 1e3);
    }
    {   // the weight-streaming skeleton on the same 64 MiB chunks
        const int wgs = 512, tpw = (int)(((size_t)64 << 20) / 1024 / (wgs * 4));
        char* codes;
        CHECK(hipMalloc(&codes, 12288 * 64));
        CHECK(hipMemset(codes, 0, 12288 * 64));
        const size_t chunk = (size_t)64 << 20;
        const char* base = reinterpret_cast<const char*>(src);
        auto run = [&](const char* name, auto launch_one) {
            const float t = time_ms([&] { for (int i = 0; i < 24; ++i) launch_one(base + i * chunk); }, 3) / 24;
            printf("%-64s %6.2f us per 64 MiB launch, %7.1f GB/s\n", name, t * 1e3, chunk / t / 1e6);
        };
        run("stream skeleton: LDS copy ring D=4, 512 wgs", [&](const char* p) {
            stream_skeleton_kernel<4, false, false><<<wgs, 256, 4 * 4 * 2048>>>(p, codes, tpw, dst); });
        run("stream skeleton: + 768 B code copy per tile", [&](const char* p) {
            stream_skeleton_kernel<4, true, false><<<wgs, 256, 4 * 4 * 2048>>>(p, codes, tpw, dst); });
        run("stream skeleton: + code copy, LDS operand reads, 2 MFMA per tile", [&](const char* p) {
            stream_skeleton_kernel<4, true, true><<<wgs, 256, 4 * 4 * 2048>>>(p, codes, tpw, dst); });
        run("stream skeleton: ring D=8, + code copy, reads, MFMA", [&](const char* p) {
            stream_skeleton_kernel<8, true, true><<<wgs, 256, 4 * 8 * 2048>>>(p, codes, tpw, dst); });
        auto shared_case = [&](const char* name, auto kern, int ldsb) {
            CHECK(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, ldsb));
            run(name, [&](const char* p) { kern<<<wgs, 256, ldsb>>>(p, codes, tpw, dst); });
        };
        shared_case("shared skeleton: 32 token rows, barrier per stage, reads + 4 MFMA", shared_skeleton_kernel<4, 1, true, 1>,
                    4 * (1 * 4 * 768 + 4096));
        shared_case("shared skeleton: 64 token rows, barrier per stage, reads + 4 MFMA", shared_skeleton_kernel<4, 2, true, 1>,
                    4 * (2 * 4 * 768 + 4096));
        shared_case("shared skeleton: 64 token rows, barrier per 2 stages, ring of 6", shared_skeleton_kernel<6, 2, true, 2>,
                    6 * (2 * 4 * 768 + 4096));
    }
    const float c = time_ms([&] { copy_kernel<<<4096, 256>>>(src, dst, bytes / 16); }, 5);
    printf("%-48s %8.1f GB/s (read + write)\n", "HBM copy, 2 GiB -> 2 GiB", 2.0 * bytes / c / 1e6);
    return 0;
}
