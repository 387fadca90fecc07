// Ternary GEMM of H-BitLinear / BitLinear (Eq. 7): acc[t][o] = sum_k q[t][k] * c[o][k] on the int8
// matrix cores with int32 accumulation, and the fused dequantising epilogue
//   y[t][o] = bf16( (float)acc * s_d[t] * alpha_g(o) )           (outer factors of Eq. 1, 5, 6).
//
// Operand roles: the 32x32x32 int8 MFMA computes D[i][j] += sum_k A[i][k] B[k][j].  A is a 32-row
// tile of W (i = output feature), B a 32-token tile of activation codes (j = token), so a lane of D
// holds 4 consecutive output features of one token per register quad and can store 8 bytes of bf16.
//
// Weights arrive 2-bit packed, 16 weights per dword, already in per-lane operand order (see
// ternary_setup.hip); a 1 KiB tile (32 features x 128 inputs) is one 16-byte read per lane, and
// shift+and expands it into bytes {0,1,2} = code+1.  The matrix cores therefore compute sum_k q*(c+1); the exact correction
// sum_k q[t][k] (the per-token code sum written by the quantiser kernel) is subtracted in the
// epilogue, all in int32.  Both operands are staged through LDS with direct global->LDS 16-byte
// loads, NSTAGE deep: codes into an XOR-swizzled [token][128 B] layout, weights tile by tile.
#include "hbl_internal.h"

namespace hbl {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 128;  // features per pipeline stage = one packed weight tile

__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Wait until at most N of this wave's vector-memory loads are still in flight, then workgroup barrier.
// Written as one asm block: __syncthreads() carries a release fence that the compiler lowers to
// vmcnt(0), which would drain the whole global->LDS pipeline at every stage.  The "memory" clobber
// keeps every load / store on its side of the barrier.
template <int N>
__device__ __forceinline__ void wait_loads_then_barrier() {
    asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(N) : "memory");
}

__device__ __forceinline__ uint32_t f32_to_bf16_rne(float v) {
    uint32_t u = as_u(v);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return u >> 16;
}

// Expand one packed dword into the four operand registers of a lane.
template <bool SUBTRACT_ONE>
__device__ __forceinline__ v4i expand(uint32_t p) {
    v4i r;
    r[0] = (int)(p & 0x03030303u);
    r[1] = (int)((p >> 2) & 0x03030303u);
    r[2] = (int)((p >> 4) & 0x03030303u);
    r[3] = (int)((p >> 6) & 0x03030303u);
    if constexpr (SUBTRACT_ONE) {
        // bytes {0,1,2} -> {-1,0,1}: set bit 7 so the per-byte decrement cannot borrow, then clear it
#pragma unroll
        for (int j = 0; j < 4; ++j)
            r[j] = (int)((((uint32_t)r[j] | 0x80808080u) - 0x01010101u) ^ 0x80808080u);
    }
    return r;
}

struct GemmArgs {
    const int8_t* codes;      // [T, K]
    const uint32_t* packed;   // tiles [N/32][K/128][64 lanes][4 dwords]
    const float* s_dequant;   // [T]
    const int32_t* code_sum;  // [T]
    const float* w_scales;    // [groups]
    uint16_t* y;              // [T, N] bf16
    int32_t* acc_out;         // [T, N] (RAW only)
    int T, K, N;
    int rows_per_group;
    int tiles_n, tiles_t;
};

// WAVES_N x WAVES_T waves; each wave owns TN x TT MFMA tiles (32 features x 32 tokens each).
// LDS stage = [BT tokens x 128 B codes, XOR-swizzled][BN/32 packed weight tiles x 1 KiB].
template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool RAW>
__global__ __launch_bounds__(64 * WAVES_N * WAVES_T) void ternary_gemm_kernel(const GemmArgs a) {
    constexpr int NW = WAVES_N * WAVES_T;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int BT = WAVES_T * TT * 32;
    constexpr int XBYTES = BT * kBK;               // codes per stage
    constexpr int WBYTES = (BN / 32) * 1024;       // packed weights per stage
    constexpr int STAGE = XBYTES + WBYTES;
    constexpr int XL = (BT / 8) / NW;              // global->LDS instructions per wave per stage: codes
    constexpr int WL = (BN / 32 + NW - 1) / NW;    // ... and weights (waves beyond BN/32 tiles issue none)
    static_assert((BT / 8) % NW == 0, "code loads must divide evenly over the waves");
    static_assert((BN / 32) % NW == 0 || (BN / 32) < NW, "weight loads must divide evenly over the waves");
    static_assert(NSTAGE >= 2, "need at least double buffering");
    // loads of later stages that may stay in flight while stage kb is consumed (waves that issue fewer
    // weight loads than WL simply wait for a little more than they must)
    constexpr int WL_MIN = (BN / 32) >= NW ? WL : 0;
    constexpr int PENDING = (NSTAGE - 2) * (XL + WL_MIN);

    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % WAVES_N;
    const int wt = wave / WAVES_N;

    // Workgroups are dealt round-robin over the 8 XCDs; give each XCD a contiguous run of tiles
    // (feature tile fastest) so that the workgroups sharing an activation panel share an L2.
    int wg = blockIdx.x;
    const int nwg = a.tiles_n * a.tiles_t;
    if ((nwg & 7) == 0) wg = (wg & 7) * (nwg >> 3) + (wg >> 3);
    const int tile_n = wg % a.tiles_n;
    const int tile_t = wg / a.tiles_n;
    const int n0 = tile_n * BN;
    const int t0 = tile_t * BT;
    const int nkb = a.K / kBK;

    // weight tiles this wave copies into LDS (tile index inside the workgroup tile: wave + NW*m);
    // tiles past N are clamped (their results are dropped in the epilogue)
    const uint32_t* wptr[WL];
#pragma unroll
    for (int m = 0; m < WL; ++m) {
        int nt = n0 / 32 + wave + NW * m;
        const int nt_max = a.N / 32 - 1;
        nt = nt < nt_max ? nt : nt_max;
        wptr[m] = a.packed + ((size_t)nt * nkb) * 256 + lane * 4;
    }
    // activation codes: instruction q covers tokens 8q..8q+7, lane l -> token 8q + l/8, LDS slot l%8,
    // global 16-byte chunk (l%8) ^ (token % 8)
    const int8_t* xptr[XL];
#pragma unroll
    for (int m = 0; m < XL; ++m) {
        const int q = wave + NW * m;
        const int row = 8 * q + (lane >> 3);
        int t = t0 + row;
        t = t < a.T ? t : a.T - 1;
        const int c = (lane & 7) ^ (row & 7);
        xptr[m] = a.codes + (size_t)t * a.K + c * 16;
    }

    // stage kb -> LDS buffer `slot`; past the end of K the last block is re-read so that every
    // iteration issues the same number of loads (the in-flight count above relies on it)
    auto issue = [&](int kb, int slot) {
        const int kbc = kb < nkb ? kb : nkb - 1;
        char* base = lds + slot * STAGE;
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int q = wave + NW * m;
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(xptr[m] + (size_t)kbc * kBK),
                (__attribute__((address_space(3))) void*)(base + q * 1024), 16, 0, 0);
        }
#pragma unroll
        for (int m = 0; m < WL; ++m) {
            const int wtile = wave + NW * m;
            if ((BN / 32) % NW == 0 || wtile < BN / 32)
                __builtin_amdgcn_global_load_lds(
                    (const __attribute__((address_space(1))) void*)(wptr[m] + (size_t)kbc * 256),
                    (__attribute__((address_space(3))) void*)(base + XBYTES + wtile * 1024), 16, 0, 0);
        }
    };

    v16i acc[TN][TT];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // LDS read offsets: token row = tile*32 + (lane & 31), chunk = 2*ks + (lane >> 5), swizzled by row % 8
    int xoff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        xoff[ks] = (wt * TT * 32 + (lane & 31)) * kBK + (((2 * ks + (lane >> 5)) ^ (lane & 7)) << 4);
    const int woff = XBYTES + wn * TN * 1024 + lane * 16;

    auto compute = [&](int slot) {
        const char* sbase = lds + slot * STAGE;
        v4i wpk[TN];
#pragma unroll
        for (int i = 0; i < TN; ++i) wpk[i] = *reinterpret_cast<const v4i*>(sbase + woff + i * 1024);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            v4i xop[TT];
#pragma unroll
            for (int j = 0; j < TT; ++j) xop[j] = *reinterpret_cast<const v4i*>(sbase + xoff[ks] + j * 32 * kBK);
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const v4i wop = expand<RAW>((uint32_t)wpk[i][ks]);
#pragma unroll
                for (int j = 0; j < TT; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop, xop[j], acc[i][j], 0, 0, 0);
            }
        }
    };

    // prologue: stages 0 .. NSTAGE-2 in flight
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) issue(s, s);

    // One iteration: this wave's loads for stage kb have landed; after the barrier so have everyone's,
    // and every wave is done reading the buffer that stage kb+NSTAGE-1 is about to overwrite.
    int kb0 = 0;
    for (; kb0 + NSTAGE <= nkb; kb0 += NSTAGE) {
#pragma unroll
        for (int u = 0; u < NSTAGE; ++u) {
            wait_loads_then_barrier<PENDING>();
            issue(kb0 + u + NSTAGE - 1, (u + NSTAGE - 1) % NSTAGE);
            compute(u);
        }
    }
#pragma unroll
    for (int u = 0; u < NSTAGE - 1; ++u) {
        if (kb0 + u < nkb) {
            wait_loads_then_barrier<PENDING>();
            issue(kb0 + u + NSTAGE - 1, (u + NSTAGE - 1) % NSTAGE);
            compute(u);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // drain the clamped tail loads before the LDS is released

    // epilogue: lane holds token t = ..+(lane&31); register quad g holds features 8g + 4*(lane>>5) + 0..3
#pragma unroll
    for (int j = 0; j < TT; ++j) {
        const int t = t0 + (wt * TT + j) * 32 + (lane & 31);
        if (t >= a.T) continue;
        float sd = 0.0f;
        int sx = 0;
        if constexpr (!RAW) {
            sd = a.s_dequant[t];
            sx = a.code_sum[t];
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int nb = n0 + (wn * TN + i) * 32;
            if (nb >= a.N) continue;
            if constexpr (RAW) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = nb + 8 * g + 4 * (lane >> 5);
                    v4i o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = acc[i][j][4 * g + r];
                    *reinterpret_cast<v4i*>(a.acc_out + (size_t)t * a.N + n) = o;
                }
            } else {
                const float alpha = a.w_scales[nb / a.rows_per_group];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = nb + 8 * g + 4 * (lane >> 5);
                    uint32_t h[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float v = ((float)(acc[i][j][4 * g + r] - sx) * sd) * alpha;
                        h[r] = f32_to_bf16_rne(v);
                    }
                    *reinterpret_cast<uint2*>(a.y + (size_t)t * a.N + n) = make_uint2(h[0] | (h[1] << 16), h[2] | (h[3] << 16));
                }
            }
        }
    }
}

template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool RAW>
int launch_cfg(GemmArgs a, hipStream_t stream) {
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int BT = WAVES_T * TT * 32;
    constexpr size_t lds = (size_t)NSTAGE * (BT * kBK + (BN / 32) * 1024);
    a.tiles_n = (a.N + BN - 1) / BN;
    a.tiles_t = (a.T + BT - 1) / BT;
    auto kern = ternary_gemm_kernel<WAVES_N, WAVES_T, TN, TT, NSTAGE, RAW>;
    if (lds > 48 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return note_hip_error(e);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)(a.tiles_n * a.tiles_t)), dim3(64 * WAVES_N * WAVES_T), lds, stream, a);
    return after_launch();
}

template <bool RAW>
int choose(const GemmArgs& a, hipStream_t stream) {
    const int64_t big_tiles = (int64_t)((a.N + 255) / 256) * ((a.T + 255) / 256);
    if (a.T <= 32) return launch_cfg<4, 1, 2, 1, 4, RAW>(a, stream);        // 256 features x 32 tokens
    if (a.T <= 64) return launch_cfg<4, 1, 2, 2, 4, RAW>(a, stream);        // 256 x 64
    if (big_tiles >= 200) return launch_cfg<2, 2, 4, 4, 3, RAW>(a, stream);  // 256 x 256, 4 waves
    return launch_cfg<2, 2, 2, 2, 4, RAW>(a, stream);                        // 128 x 128
}

}  // namespace

int launch_ternary_gemm(const int8_t* codes, int64_t T, int64_t K, const void* packed, int64_t N,
                        const float* s_dequant, const int32_t* code_sum, const float* w_scales,
                        int64_t n_scale_groups, void* y_bf16, int32_t* acc_out, hipStream_t stream) {
    if (T == 0) return HBL_OK;
    GemmArgs a;
    a.codes = codes;
    a.packed = static_cast<const uint32_t*>(packed);
    a.s_dequant = s_dequant;
    a.code_sum = code_sum;
    a.w_scales = w_scales;
    a.y = static_cast<uint16_t*>(y_bf16);
    a.acc_out = acc_out;
    a.T = (int)T;
    a.K = (int)K;
    a.N = (int)N;
    a.rows_per_group = n_scale_groups > 0 ? (int)(N / n_scale_groups) : (int)N;
    a.tiles_n = a.tiles_t = 0;
    return acc_out ? choose<true>(a, stream) : choose<false>(a, stream);
}

}  // namespace hbl
