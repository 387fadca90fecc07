// Small-batch (decode) form of the ternary GEMM of Eq. 7: T <= 64 tokens, so the packed weights are
// read once from HBM and dominate the traffic, and the job is to keep as many weight tiles in flight as
// the memory system needs.  One launch serves up to kMaxGroup independent projections.
//
// A wave owns one 32-row weight tile at a time and walks its K range tile by tile (1 KiB of packed
// weights = 32 rows x 128 features).  Weights and activation codes both arrive by direct global->LDS
// copies, D = 4 stages deep per wave.  Per problem one of two operand paths:
//  - fp6 x fp4 (INT4 activations, K >= 512): codes from the record image (96 bytes per token and stage),
//    weights to fp4 with 3 vector-ALU instructions per 16; two 16x16x128 MFMAs per tile for up to 16 tokens,
//    two 32x32x64 per tile and 32 tokens above that.  fp32 accumulators hold exact integers.
//  - int8 (INT8 activations, short rows): codes as bytes (128 per token and stage), weights to signed bytes
//    (15 instructions per 16), four 32x32x32 MFMAs per tile and 32 tokens.
//
// Two forms:
//  - streaming (T <= 16): a wave's code stage is private (8 or 16 rows), so the waves never meet at a
//    barrier.  The K range of one row tile may be split over the 2 or 4 waves of a workgroup; their
//    accumulators are added through LDS at the end (exact).
//  - shared (T <= 64): the four waves take four row tiles over one K range and share the code stage
//    (32 or 64 rows): one barrier per stage.  A K range split over workgroups leaves int32 slices in the
//    workspace; the workgroup of a K range that finishes last (an arrival counter) adds the others' slices to
//    its own accumulators and dequantises.  (A group with more split row groups than a slot has counters runs
//    without the split.)
#include <atomic>

#include "gemm_common.h"

namespace hbl {
namespace {

using namespace gemm;
typedef int v16i __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

// The 16-byte-per-lane global -> LDS copy of gemm_common.h by the first 48 lanes only: 768 contiguous bytes, eight
// 96-byte rows of the record image.  (The 12-byte-per-lane form of the instruction strides the LDS side by 16
// bytes per lane - measured - so it cannot lay down contiguous rows.)  The execution mask is narrowed around
// the copy inside one asm block and put back.
__device__ __forceinline__ void lds_dma16_first48(uint32_t lds_addr, const void* base, uint32_t voff) {
    uint64_t saved;
    asm volatile(
        "s_mov_b64 %0, exec\n\ts_bfm_b64 exec, 48, 0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\t"
        "global_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
        : "=&s"(saved)
        : "s"(lds_addr), "v"(voff), "s"(base)
        : "memory", "m0");
}

// Two packed dwords (32 weights) -> the four fp4 operand registers of a lane.
__device__ __forceinline__ v8i fp4_operand(uint32_t p0, uint32_t p1) {
    return v8i{(int)(p0 & 0xAAAAAAAAu), (int)((p0 << 1) & 0xAAAAAAAAu), (int)(p1 & 0xAAAAAAAAu),
               (int)((p1 << 1) & 0xAAAAAAAAu), 0, 0, 0, 0};
}

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
// y = bf16((acc * s_d) * alpha) for four consecutive features; acc holds exact integers.
__device__ __forceinline__ uint2 dequant_quad_f32(float a0, float a1, float a2, float a3, float sd, float alpha) {
    const bf16x2 lo = __builtin_convertvector((f32x2){(a0 * sd) * alpha, (a1 * sd) * alpha}, bf16x2);
    const bf16x2 hi = __builtin_convertvector((f32x2){(a2 * sd) * alpha, (a3 * sd) * alpha}, bf16x2);
    return make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
}

// NW = waves per workgroup.  Four everywhere except the streaming form on a single long-K problem with few row
// tiles (W_down alone): there 8 waves share a row tile's K range, which shortens each wave's serial chain of
// tiles (128 workgroups cannot be made more without narrower row tiles).
// F6: the problem's codes are bf6 records and the fp6 x fp4 matrix cores do the work.
template <bool SHARE, int TT, int RQ, int D, int NW, bool F6>
__device__ __forceinline__ void decode_body(const DecodeProblem& p, const int w, char* lds, unsigned int* p_arrive) {
    constexpr int ROWS = SHARE ? TT * 32 : RQ * 8;    // token rows of one code stage
    constexpr int ROWB = F6 ? kRecordRowBytes : kBK;  // bytes of one token row of a stage
    constexpr int XB = ROWS * ROWB;                   // bytes of one code stage
    constexpr int XW = SHARE ? XB : NW * XB;          // code bytes per stage in the workgroup
    constexpr int STAGE = XW + NW * 1024;             // + one packed weight tile per wave
    constexpr int XL = SHARE ? TT : RQ;               // code copies per wave per stage (8 rows each)
    constexpr int NACC = TT == 1 ? 2 : TT;
    // PAIR (shared form, two token tiles, fp6 x fp4): a wave multiplies two weight tiles by one token tile instead of
    // one weight tile by two token tiles - waves 2p and 2p + 1 share the weight tiles 2p, 2p + 1 of the stage and take
    // token tile 0 and 1.  Same MFMAs, but 5 KiB of LDS operand reads per wave and stage instead of 7: at 33-64
    // tokens the eight waves of a CU are bound by the LDS read rate (56 KiB per stage at 128 bytes per clock).
    constexpr bool PAIR = SHARE && F6 && TT == 2;
    constexpr bool PAIRED = SHARE && TT == 2;   // two stages per wait and barrier (below)
    static_assert(D >= 3 && (ROWS & (ROWS - 1)) == 0, "pipeline depth / row count");
    static_assert(!SHARE || NW == 4, "the shared form is written for four waves");
    static_assert(NW * 4096 <= D * STAGE, "the in-workgroup reduction reuses the stage buffers");

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kl = __builtin_ctz((unsigned)p.ksplit);   // p.ksplit is a power of two, at most NW
    const int nkb_total = p.K / kBK;
    const int nkb = nkb_total >> kl;
    int nt, ks;
    if constexpr (SHARE) {
        nt = 4 * (w >> kl) + wave;
        ks = w & (p.ksplit - 1);
    } else {
        nt = w * (NW >> kl) + (wave >> kl);
        ks = wave & (p.ksplit - 1);
    }
    const int nt_max = p.N / 32 - 1;
    const bool live = nt <= nt_max;          // a wave past the last row tile streams that tile again, writes nothing
    const int ntc = live ? nt : nt_max;
    // accumulator a of this wave: weight tile and token tile
    auto tile_of = [&](int a) { return PAIR ? 4 * (w >> kl) + 2 * (wave >> 1) + a : nt; };
    auto tok_tile_of = [&](int a) { return PAIR ? (wave & 1) : a; };
    const int kb0 = ks * nkb;

    // packed tiles are stored K-block-major (tile (nt, kb) at (kb * N/32 + nt) KiB): at any moment the waves
    // of a launch, all at about the same kb, read one window of consecutive addresses
    const size_t wstride = (size_t)(p.N / 32) * 1024;
    const char* wbase = reinterpret_cast<const char*>(p.packed) + (size_t)kb0 * wstride + (size_t)ntc * 1024;
    const uint32_t wlane = lane * 16;
    // Code copy m of a stage covers rows 8q..8q+7.
    //  bytes: lane l -> row 8q + l/8, LDS slot l%8 of that row, global 16-byte chunk (l%8) ^ ((row/2) % 8); rows
    //         past T re-read the last token;
    //  records: the rows are 768 contiguous bytes of the stage's block of the record image (rows past T exist
    //         there and hold finite garbage that is never stored).
    const char* xbase = reinterpret_cast<const char*>(p.codes) + (size_t)kb0 * (F6 ? kRecordBlockBytes : kBK);
    uint32_t xlane[XL];
#pragma unroll
    for (int m = 0; m < XL; ++m) {
        const int q = SHARE ? wave + 4 * m : m;
        if constexpr (F6) {
            xlane[m] = q * 768 + lane * 16;   // 8 rows of 96 bytes: the first 48 lanes of a 16-byte-per-lane copy
        } else {
            const int row = 8 * q + (lane >> 3);
            const int t = row < p.T ? row : p.T - 1;
            const int c = (lane & 7) ^ ((row >> 1) & 7);
            xlane[m] = (uint32_t)t * (uint32_t)p.K + c * 16;
        }
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const uint32_t xarea = SHARE ? 0 : wave * XB;

    // Copies of stage kb into buffer `slot`.
    auto issue = [&](int kb, int slot) {
#pragma unroll
        for (int m = 0; m < XL; ++m) {
            const int q = SHARE ? wave + 4 * m : m;
            if constexpr (F6) lds_dma16_first48(lds0 + slot * STAGE + xarea + q * 768, xbase + (size_t)kb * kRecordBlockBytes, xlane[m]);
            else lds_dma16(lds0 + slot * STAGE + xarea + q * 1024, xbase + (size_t)kb * kBK, xlane[m]);
        }
        lds_dma16(lds0 + slot * STAGE + XW + wave * 1024, wbase + (size_t)kb * wstride, wlane);
    };

    // Operand read offsets inside a stage.
    //  int8: token row (lane & 31) of tile j (rows beyond the stage wrap onto loaded rows; their results are
    //        never written), the 16-byte chunk that matches packed dword k4, swizzled like the copy.
    //  fp6 x fp4, streaming: 16x16x128 MFMA - lane = (token lane & 15, feature group g = lane >> 4 of 32);
    //        the weights of row 16 hf + (lane & 15), features 32 g + 0..31, are dwords 2 (g >> 1), +1 of tile
    //        lane row + 32 (g & 1).
    //  fp6 x fp4, shared: 32x32x64 MFMA as in the prefill kernel - lane = (token lane & 31, half lane >> 5).
    int xoff[4];
    int xo_lo[2], xo_hi[2], wo[2];
    if constexpr (!F6) {
        const int r0 = (lane & 31) & (ROWS - 1);
#pragma unroll
        for (int k4 = 0; k4 < 4; ++k4) xoff[k4] = r0 * kBK + ((code_chunk_of_dword(k4, lane >> 5) ^ ((r0 >> 1) & 7)) << 4);
    } else if constexpr (!SHARE) {
        const int r0 = (lane & 15) & (ROWS - 1), g = lane >> 4;
        xo_lo[0] = r0 * kRecordRowBytes + record_lo_offset(r0, g >> 1, g & 1);
        xo_hi[0] = r0 * kRecordRowBytes + record_hi_offset(r0, g >> 1, g & 1);
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) wo[hf] = (16 * hf + (lane & 15) + 32 * (g & 1)) * 16 + 8 * (g >> 1);
    } else {
        const int r0 = lane & 31;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            xo_lo[s] = r0 * kRecordRowBytes + record_lo_offset(r0, s, lane >> 5);
            xo_hi[s] = r0 * kRecordRowBytes + record_hi_offset(r0, s, lane >> 5);
        }
    }

    v16i acc[NACC];          // int8 path
    v4f facc[2];             // fp6 x fp4, streaming: row halves 0..15, 16..31 of the tile
    v16f wacc[TT];           // fp6 x fp4, shared: one 32 x 32 tile per token tile
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0;
#pragma unroll
    for (int i = 0; i < 2; ++i) facc[i] = v4f{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int i = 0; i < TT; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) wacc[i][r] = 0.0f;

    // Stage kb may be consumed once at most min(D - 2, nkb - 1 - kb) later stages are still in flight
    // (copies return in order).  Nothing is requested past the end of the K range, so the count
    // shrinks over the last D - 2 stages: those take the switch.
    auto wait_stage = [&](int later) {
        if (later >= D - 2) {
            asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"((D - 2) * (XL + 1)) : "memory");
            return;
        }
        switch (later) {
            case 0: asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory"); break;
            case 1: asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(1 * (XL + 1)) : "memory"); break;
            case 2: asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(2 * (XL + 1)) : "memory"); break;
            case 3: asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(3 * (XL + 1)) : "memory"); break;
            case 4: asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(4 * (XL + 1)) : "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(5 * (XL + 1)) : "memory"); break;
        }
    };
    static_assert(D - 2 <= 6, "wait_stage covers up to 5 later stages below the steady state");

#pragma unroll
    for (int s = 0; s < (PAIRED ? D - 2 : D - 1); ++s)
        if (s < nkb) issue(s, s);

    // Epilogue operands, requested right behind the first stages: under a saturated memory system a load
    // issued after the loop would add its whole latency to the workgroup's run time, and ahead of the first
    // copies they would delay the stream.  (They return in order behind the D - 1 stages in flight, which
    // only makes the first waits below stricter than they need to be.)
    const bool write_partial = SHARE && p.ksplit > 1;
    const bool writer = (PAIR ? tile_of(0) <= nt_max : live) && (SHARE || ks == 0);
    constexpr bool TOK16 = F6 && !SHARE;     // the 16x16 accumulator layout: token = lane & 15
    float alpha[TT], sd[TT];
    v4i wsum[4];
#pragma unroll
    for (int j = 0; j < TT; ++j) sd[j] = alpha[j] = 0.0f;
#pragma unroll
    for (int g = 0; g < 4; ++g) wsum[g] = v4i{0, 0, 0, 0};
    if (writer) {   // (with a K range split over workgroups any of them may turn out to be the one that dequantises)
#pragma unroll
        for (int j = 0; j < TT; ++j) {
            const int tile = tile_of(j) <= nt_max ? tile_of(j) : nt_max;
            alpha[j] = p.w_scales[(tile * 32) / p.rows_per_group];
            const int t = TOK16 ? (lane & 15) : tok_tile_of(j) * 32 + (lane & 31);
            if (t < p.T) sd[j] = p.s_dequant[t];
        }
        if (!F6 && p.code_offset != 0) {
#pragma unroll
            for (int g = 0; g < 4; ++g)
                wsum[g] = *reinterpret_cast<const v4i*>(p.w_row_sum + nt * 32 + 8 * g + 4 * (lane >> 5));
        }
    }

    // One stage: its operand reads go out first, then `copies()` (the copies of a later stage), then the MFMAs, so
    // that the LDS latency passes while the copies are being accepted (worth 0.1-0.2 us per launch in the streaming
    // form: the stream itself already runs at what HBM delivers, a shorter stage only lengthens the wait).
    auto stage_work = [&](const char* st, auto&& copies) {
        if constexpr (!F6) {
            const v4i wpk = *reinterpret_cast<const v4i*>(st + XW + wave * 1024 + lane * 16);
            v4i xop[4][TT];
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
                for (int j = 0; j < TT; ++j) xop[k4][j] = *reinterpret_cast<const v4i*>(st + xarea + xoff[k4] + j * 32 * kBK);
            copies();
#pragma unroll
            for (int k4 = 0; k4 < 4; ++k4) {
                const v4i wop = expand_weights_i8((uint32_t)wpk[k4]);
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    // TT == 1: two accumulators take turns so that consecutive MFMAs do not depend on each other
                    const int ai = TT == 1 ? (k4 & 1) : j;
                    acc[ai] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop, xop[k4][j], acc[ai], 0, 0, 0);
                }
            }
        } else if constexpr (!SHARE) {
            const v4i lo = *reinterpret_cast<const v4i*>(st + xarea + xo_lo[0]);
            const int2 hi = *reinterpret_cast<const int2*>(st + xarea + xo_hi[0]);
            uint2 wp[2];
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) wp[hf] = *reinterpret_cast<const uint2*>(st + XW + wave * 1024 + wo[hf]);
            copies();
            const v8i xop = {lo[0], lo[1], lo[2], lo[3], hi.x, hi.y, 0, 0};
#pragma unroll
            for (int hf = 0; hf < 2; ++hf)
                facc[hf] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fp4_operand(wp[hf].x, wp[hf].y), xop, facc[hf],
                                                                            4 /*A: fp4*/, 3 /*B: bf6*/, 0, 0, 0, 0);
        } else if constexpr (PAIR) {
            v4i wpk[2];
#pragma unroll
            for (int i = 0; i < 2; ++i)
                wpk[i] = *reinterpret_cast<const v4i*>(st + XW + (2 * (wave >> 1) + i) * 1024 + lane * 16);
            v8i xop[2];
            const char* rows = st + (wave & 1) * 32 * kRecordRowBytes;
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const v4i lo = *reinterpret_cast<const v4i*>(rows + xo_lo[s]);
                const int2 hi = *reinterpret_cast<const int2*>(rows + xo_hi[s]);
                xop[s] = v8i{lo[0], lo[1], lo[2], lo[3], hi.x, hi.y, 0, 0};
            }
            copies();
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int i = 0; i < 2; ++i)
                    wacc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                        fp4_operand((uint32_t)wpk[i][2 * s], (uint32_t)wpk[i][2 * s + 1]), xop[s], wacc[i], 4, 3, 0, 0, 0, 0);
        } else {
            const v4i wpk = *reinterpret_cast<const v4i*>(st + XW + wave * 1024 + lane * 16);
            v8i xop[2][TT];
#pragma unroll
            for (int s = 0; s < 2; ++s)
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    const char* rows = st + j * 32 * kRecordRowBytes;
                    const v4i lo = *reinterpret_cast<const v4i*>(rows + xo_lo[s]);
                    const int2 hi = *reinterpret_cast<const int2*>(rows + xo_hi[s]);
                    xop[s][j] = v8i{lo[0], lo[1], lo[2], lo[3], hi.x, hi.y, 0, 0};
                }
            copies();
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                const v8i wop = fp4_operand((uint32_t)wpk[2 * s], (uint32_t)wpk[2 * s + 1]);
#pragma unroll
                for (int j = 0; j < TT; ++j)
                    wacc[j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wop, xop[s][j], wacc[j], 4, 3, 0, 0, 0, 0);
            }
        }
    };
    if constexpr (PAIRED) {
        // Shared form with two token tiles: one wait and one barrier per two stages (with one token tile the deeper
        // ring this needs costs more than the barriers: 25.3 against 24.7 us per layer at batch 32).  The prologue
        // has requested stages 0 .. D - 3; at the barrier of a pair every wave is done reading the previous pair,
        // whose two buffers take stages kb + D - 2 and kb + D - 1.
        static_assert(D >= 6 && D % 2 == 0, "the paired loop keeps two pairs of stages in flight");
        int slot = 0;
        for (int kb = 0; kb < nkb; kb += 2) {
            const int n2 = nkb - kb < 2 ? nkb - kb : 2;
            const int issued = kb + D - 2 < nkb ? kb + D - 2 : nkb;
            wait_stage(issued - kb - n2);
            asm volatile("s_barrier" ::: "memory");
            for (int u = 0; u < n2; ++u) {
                const int ahead = kb + u + D - 2;
                const int aslot = slot >= 2 ? slot - 2 : slot + D - 2;
                stage_work(lds + slot * STAGE, [&]() {
                    if (ahead < nkb) issue(ahead, aslot);
                });
                slot = slot + 1 == D ? 0 : slot + 1;
            }
        }
    } else {
        int slot = 0;
        for (int kb = 0; kb < nkb; ++kb) {
            // stage kb has landed (for every wave, if the code stage is shared); the buffer read in the previous
            // iteration is free for stage kb + D - 1
            wait_stage(nkb - 1 - kb);
            if constexpr (SHARE) asm volatile("s_barrier" ::: "memory");
            stage_work(lds + slot * STAGE, [&]() {
                if (kb + D - 1 < nkb) issue(kb + D - 1, slot == 0 ? D - 1 : slot - 1);
            });
            slot = slot + 1 == D ? 0 : slot + 1;
        }
    }
    if constexpr (!F6 && TT == 1) acc[0] += acc[1];

    if constexpr (!SHARE) {
        if (p.ksplit > 1) {   // uniform over the workgroup
            __syncthreads();  // every wave is done with the stage buffers
            int* red = reinterpret_cast<int*>(lds);
            float* fred = reinterpret_cast<float*>(lds);
            if (ks != 0) {
                if constexpr (F6) {
#pragma unroll
                    for (int r = 0; r < 8; ++r) fred[(wave * 8 + r) * 64 + lane] = facc[r >> 2][r & 3];
                } else {
#pragma unroll
                    for (int r = 0; r < 16; ++r) red[(wave * 16 + r) * 64 + lane] = acc[0][r];
                }
            }
            __syncthreads();
            if (ks == 0) {
                for (int kk = 1; kk < p.ksplit; ++kk) {
                    if constexpr (F6) {
#pragma unroll
                        for (int r = 0; r < 8; ++r) facc[r >> 2][r & 3] += fred[((wave + kk) * 8 + r) * 64 + lane];
                    } else {
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[0][r] += red[((wave + kk) * 16 + r) * 64 + lane];
                    }
                }
            }
        }
        if (ks != 0) return;
    }
    if constexpr (!SHARE) {
        if (!writer) return;
    }

    if constexpr (TOK16) {
        // lane holds token lane & 15; facc[hf] holds features 16 hf + 4 (lane >> 4) + 0..3 of the row tile
        const int t = lane & 15;
        if (t >= p.T) return;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const int n = nt * 32 + 16 * hf + 4 * (lane >> 4);
            *reinterpret_cast<uint2*>(p.y + (size_t)t * p.N + n) =
                dequant_quad_f32(facc[hf][0], facc[hf][1], facc[hf][2], facc[hf][3], sd[0], alpha[0]);
        }
        return;
    }
    // accumulator j (token tile j, or weight tile j of the wave's two in the pair form): lane holds token (lane & 31)
    // of its token tile; register quad g holds features 8g + 4*(lane >> 5) + 0..3 of its weight tile
    v4i tot[TT][4];
#pragma unroll
    for (int j = 0; j < TT; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if constexpr (F6) {
#pragma unroll
                for (int r = 0; r < 4; ++r) tot[j][g][r] = (int)wacc[j][4 * g + r];
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r) tot[j][g][r] = acc[TT == 1 ? 0 : j][4 * g + r];
            }
        }
    if constexpr (SHARE) {
        if (write_partial) {   // uniform over the workgroup
            // This workgroup's slice of the K range, as int32 tiles (exact).  A slice is only ever read by a workgroup
            // of the same shape, so it is kept as the lanes hold it - quad (j, g) of wave `wave` of slice k at v4i index (((k * groups + group) * 4 + wave) *
            // 4 TT + 4 j + g) * 64 + lane: every store and load instruction moves 1 KiB of consecutive bytes.  The
            // stores are device-scope (write-through): readable from the other XCDs without a write-back of this L2.
            const int groups = (p.N / 32 + 3) / 4;
            v4i* const frag = reinterpret_cast<v4i*>(p.partial);
            auto frag_index = [&](int k, int q) { return ((((size_t)k * groups + (w >> kl)) * 4 + wave) * (4 * TT) + q) * 64 + lane; };
#pragma unroll
            for (int q = 0; q < 4 * TT; ++q)
                asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(frag + frag_index(ks, q)), "v"(tot[q >> 2][q & 3]) : "memory");
            // Arrival: once a workgroup's stores have completed it counts itself in; the counter wraps at ksplit, so
            // the workgroup that brings it back to zero is the last of its K range and every slice is in memory.
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();   // (every wave of the workgroup is here: the stage buffers are free)
            unsigned int* arrived = reinterpret_cast<unsigned int*>(lds);
            if (tid == 0) *arrived = atomicInc(p_arrive + p.arrive_begin + (w >> kl), (unsigned)p.ksplit - 1u);
            __syncthreads();
            if (*arrived != (unsigned)p.ksplit - 1u || !writer) return;
            // (device-scope loads, 8 bytes each: they do not stop at this XCD's L2)
            for (int k = 0; k < p.ksplit; ++k) {
                if (k == ks) continue;   // (uniform)
#pragma unroll
                for (int q = 0; q < 4 * TT; ++q) {
                    const uint64_t* src = reinterpret_cast<const uint64_t*>(frag + frag_index(k, q));
                    const uint64_t lo = __hip_atomic_load(src, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    const uint64_t hi = __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    tot[q >> 2][q & 3] += v4i{(int)(uint32_t)lo, (int)(uint32_t)(lo >> 32), (int)(uint32_t)hi, (int)(uint32_t)(hi >> 32)};
                }
            }
        } else if (!writer) {
            return;
        }
    }
#pragma unroll
    for (int j = 0; j < TT; ++j) {
        const int t = tok_tile_of(j) * 32 + (lane & 31);
        if (t >= p.T || tile_of(j) > nt_max) continue;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = tile_of(j) * 32 + 8 * g + 4 * (lane >> 5);
            if constexpr (F6) {
                *reinterpret_cast<uint2*>(p.y + (size_t)t * p.N + n) =
                    dequant_quad_f32((float)tot[j][g][0], (float)tot[j][g][1], (float)tot[j][g][2], (float)tot[j][g][3], sd[j], alpha[j]);
            } else {
                *reinterpret_cast<uint2*>(p.y + (size_t)t * p.N + n) = dequant_quad_sums(tot[j][g], sd[j], alpha[j], p.code_offset, wsum[g]);
            }
        }
    }
}

template <bool SHARE, int TT, int RQ, int D, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void decode_gemm_kernel(const DecodeArgs args) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const DecodeProblem p = args.p[group_index_of(args.wg_begin, args.n, (int)blockIdx.x)];
    const int w = (int)blockIdx.x - p.wg_begin;
    if (p.f6) decode_body<SHARE, TT, RQ, D, NW, true>(p, w, lds, args.arrive);      // uniform over the workgroup
    else decode_body<SHARE, TT, RQ, D, NW, false>(p, w, lds, args.arrive);
}

// Arrival counters of the shared form's in-kernel reduction: one per group of four row tiles whose K range is split
// over workgroups.  A counter wraps at the number of slices, so it is back at zero when its launch is over and needs
// no initialisation beyond the zeros the array is loaded with.  The host hands the kArriveSlots slots out round-robin:
// launches that overlap on one GPU (other streams) count in different words unless more than that many are in flight.
constexpr int kArriveWords = 2048;
constexpr int kArriveSlots = 128;
__device__ __attribute__((aligned(256))) unsigned int g_arrive[kArriveSlots * kArriveWords];

// This device's copy of the array (each GPU holds its own, at its own address), advanced to the next slot.
int next_arrive_slot(unsigned int** out) {
    static std::atomic<unsigned int*> base[64];
    static std::atomic<unsigned int> next{0};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error(e);
    unsigned int* ptr = base[dev & 63].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(g_arrive));
        if (e != hipSuccess) return note_hip_error(e);
        base[dev & 63].store(ptr, std::memory_order_release);
    }
    *out = ptr + (size_t)(next.fetch_add(1, std::memory_order_relaxed) % kArriveSlots) * kArriveWords;
    return HBL_OK;
}

template <bool SHARE, int TT, int RQ, int D, int NW = 4>
int launch_form(const DecodeArgs& planned, int wgs, int counters, hipStream_t stream) {
    DecodeArgs a = planned;
    a.arrive = nullptr;
    if (counters != 0) {   // some K range is split over workgroups
        if (const int rc = next_arrive_slot(&a.arrive); rc != HBL_OK) return rc;
    }
    constexpr int ROWS = SHARE ? TT * 32 : RQ * 8;
    constexpr size_t lds = (size_t)D * ((SHARE ? 1 : NW) * ROWS * kBK + NW * 1024);
    auto kern = decode_gemm_kernel<SHARE, TT, RQ, D, NW>;
    static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
    if (const int rc = allow_dynamic_lds(kern, lds, lds_allowed); rc != HBL_OK) return rc;
    launch_kernel("decode_gemm_kernel", kern, dim3((unsigned)wgs), dim3(64 * NW), lds, stream, a);
    return after_launch();
}

// Workgroups a problem occupies in the GEMM grid for a given K split.
int problem_wgs(const DecodeProblem& p, bool share) {
    const int tiles = p.N / 32;
    return share ? ((tiles + 3) / 4) * p.ksplit : (tiles * p.ksplit + 3) / 4;
}


// K split of every problem, then each problem's first workgroup in the grid and its first arrival counter.
// About 32 weight tiles (32 KiB) per wave; while the grid is too small to occupy the chip (256 CUs x
// 2 workgroups) split further, down to 8 tiles per wave.  The streaming form adds the slices inside a
// workgroup, so a split is free; the shared form needs the partial buffer and ends with the last workgroup of a
// K range adding the others' slices, so it splits further only when less than three quarters of the CUs would get
// a workgroup.
void plan(DecodeArgs& a, bool share, int* wgs_out, int* counters_out) {
    const int enough = share ? 192 : 384;
    int total = 0;
    for (int i = 0; i < a.n; ++i) {
        DecodeProblem& p = a.p[i];
        const int nkb = p.K / 128;
        const bool may_split = !share || p.partial != nullptr;
        p.ksplit = 1;
        while (may_split && p.ksplit < kMaxDecodeSplit && nkb % (2 * p.ksplit) == 0 && nkb / (2 * p.ksplit) >= 32)
            p.ksplit *= 2;
        total += problem_wgs(p, share);
    }
    for (int pass = 0; pass < 2 && total < enough; ++pass) {
        total = 0;
        for (int i = 0; i < a.n; ++i) {
            DecodeProblem& p = a.p[i];
            const int nkb = p.K / 128;
            const bool may_split = !share || p.partial != nullptr;
            if (may_split && p.ksplit < kMaxDecodeSplit && nkb % (2 * p.ksplit) == 0 && nkb / (2 * p.ksplit) >= 8)
                p.ksplit *= 2;
            total += problem_wgs(p, share);
        }
    }
    // a K range split over workgroups (shared form) needs one arrival counter per group of four row tiles; a group
    // with more of them than a slot holds runs without that split
    int counters = 0;
    for (int i = 0; i < a.n; ++i)
        if (share && a.p[i].ksplit > 1) counters += (a.p[i].N / 32 + 3) / 4;
    if (counters > kArriveWords) {
        for (int i = 0; i < a.n; ++i) a.p[i].ksplit = 1;
        counters = 0;
    }
    int wgs = 0, next_counter = 0;
    for (int i = 0; i < a.n; ++i) {
        DecodeProblem& p = a.p[i];
        p.wg_begin = a.wg_begin[i] = wgs;
        wgs += problem_wgs(p, share);
        p.arrive_begin = next_counter;
        if (share && p.ksplit > 1) next_counter += (p.N / 32 + 3) / 4;
    }
    *wgs_out = wgs;
    *counters_out = counters;
}

// A single streaming-form problem whose four-wave plan would leave long serial chains of tiles on few
// workgroups (W_down alone: 128 row tiles, 128 K blocks): waves per workgroup for the wide form, or 0.
int wide_waves(const DecodeArgs& a, int max_t) {
    if (a.n != 1 || max_t > 16) return 0;
    const DecodeProblem& p = a.p[0];
    const int nkb = p.K / 128, tiles = p.N / 32;
    if (nkb < 64 || tiles > 192) return 0;
    const int nw = 8;   // 16 waves measured equal at batch 1 and 5 % slower at batch 8 and 16
    return nkb % nw == 0 ? nw : 0;
}
void plan_wide(DecodeArgs& a, int nw, int* wgs_out) {
    DecodeProblem& p = a.p[0];
    p.ksplit = nw;   // one row tile per workgroup, its K range over all waves: 8 tiles or more per wave (nkb >= 64)
    p.wg_begin = a.wg_begin[0] = 0;
    p.arrive_begin = 0;
    *wgs_out = (p.N / 32 * p.ksplit + nw - 1) / nw;
}

}  // namespace

bool decode_stream_preferred(int64_t T, int64_t K, int64_t N) {
    if (T <= 0 || T > 16) return false;
    DecodeArgs a = {};
    a.n = 1;
    a.p[0].T = (int)T;
    a.p[0].K = (int)K;
    a.p[0].N = (int)N;
    if (wide_waves(a, (int)T) != 0) return true;
    int wgs, counters;
    plan(a, false, &wgs, &counters);
    // a wave's tiles are a serial chain: few workgroups with long chains leave most of the chip idle
    return (K / 128) / a.p[0].ksplit <= 16 || wgs >= 256;
}

int decode_plan_for_tests(DecodeArgs& a, int* wgs, int* counters) {
    int max_t = 0;
    for (int i = 0; i < a.n; ++i) max_t = a.p[i].T > max_t ? a.p[i].T : max_t;
    if (a.n <= 0 || max_t > 64) return HBL_E_SHAPE;
    if (const int nw = wide_waves(a, max_t); nw != 0) {
        plan_wide(a, nw, wgs);
        *counters = 0;
        return HBL_OK;
    }
    plan(a, max_t > 16, wgs, counters);
    return HBL_OK;
}

int launch_decode_gemm(DecodeArgs& a, hipStream_t stream) {
    if (a.n <= 0) return HBL_OK;
    int max_t = 0;
    for (int i = 0; i < a.n; ++i) max_t = a.p[i].T > max_t ? a.p[i].T : max_t;
    if (max_t > 64) return HBL_E_SHAPE;
    int wgs, counters;
    if (const int nw = wide_waves(a, max_t); nw != 0) {
        plan_wide(a, nw, &wgs);
        return max_t <= 8 ? launch_form<false, 1, 1, 4, 8>(a, wgs, 0, stream)
                          : launch_form<false, 1, 2, 4, 8>(a, wgs, 0, stream);
    }
    plan(a, max_t > 16, &wgs, &counters);
    // Stages in flight per wave: 4.  Shallow is best (3 to 8 measured): the memory-level parallelism comes from
    // the 2048 waves of a full grid, and deeper rings only cost LDS and queueing.
    if (max_t <= 8) return launch_form<false, 1, 1, 4>(a, wgs, 0, stream);
    if (max_t <= 16) return launch_form<false, 1, 2, 4>(a, wgs, 0, stream);
    if (max_t <= 32) return launch_form<true, 1, 1, 4>(a, wgs, counters, stream);
    return launch_form<true, 2, 1, 6>(a, wgs, counters, stream);
}

}  // namespace hbl
