// Ternary GEMM of H-BitLinear / BitLinear (Eq. 7): acc[t][o] = sum_k q[t][k] * c[o][k] on the int8
// matrix cores with int32 accumulation, and the fused dequantising epilogue
//   y[t][o] = bf16( (float)acc * s_d[t] * alpha_g(o) )           (outer factors of Eq. 1, 5, 6).
//
// Operand roles: the 32x32x32 int8 MFMA computes D[i][j] += sum_k A[i][k] B[k][j].  A is a 32-row
// tile of W (i = output feature), B a 32-token tile of activation codes (j = token), so a lane of D
// holds 4 consecutive output features of one token per register quad and can store 8 bytes of bf16.
//
// Weights arrive 2-bit packed (sign / magnitude pairs, 16 weights per dword, per-lane operand order: see
// ternary_setup.hip); a 1 KiB tile (32 features x 128 inputs) is one 16-byte read per lane, and 15 vector-ALU
// instructions expand a dword into four registers of signed bytes {-1, 0, +1} (gemm_common.h).  The only
// correction left is for an offset on the stored codes (INT4 codes travel as q + 8): offset * sum_k c[o][k],
// removed in the epilogue in int32.  Both operands are staged through LDS with direct global->LDS 16-byte
// loads, NSTAGE deep: codes into an XOR-swizzled [token][128 B] layout, weights tile by tile.
#include <atomic>
#include <type_traits>

#include "gemm_common.h"

namespace hbl {
namespace {

using namespace gemm;
typedef int v16i __attribute__((ext_vector_type(16)));

// OCC = waves per SIMD the register budget must allow (2: two workgroups of 4 waves share a CU).
template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool RAW, bool SPLIT, int OCC>
__global__ __launch_bounds__(64 * WAVES_N * WAVES_T, OCC) void ternary_gemm_kernel(const GemmArgs a) {
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
    int ks = 0;
    const int nwg = a.tiles_n * a.tiles_t;
    if constexpr (SPLIT) {
        ks = wg % a.split_k;
        wg = wg / a.split_k;
    } else {
        if ((nwg & 7) == 0) wg = (wg & 7) * (nwg >> 3) + (wg >> 3);
    }
    const int tile_n = wg % a.tiles_n;
    const int tile_t = wg / a.tiles_n;
    const int n0 = tile_n * BN;
    const int t0 = tile_t * BT;
    const int nkb_total = a.K / kBK;
    const int nkb = SPLIT ? nkb_total / a.split_k : nkb_total;   // K-blocks of this workgroup
    const int kb_first = ks * nkb;

    // Global -> LDS copies: wave-uniform 64-bit base (SGPR pair) + 32-bit per-lane offset, so that
    // advancing along K is scalar arithmetic only.
    // weights: this wave copies tiles wave + NW*m of the workgroup tile; tiles past N are clamped (their
    // results are dropped in the epilogue)
    // (K-block-major tiles: a stage's BN/32 tiles of this workgroup are consecutive KiB)
    const size_t wstride = (size_t)(a.N / 32) * 1024;
    const char* wbase[WL];
#pragma unroll
    for (int m = 0; m < WL; ++m) {
        int nt = n0 / 32 + wave + NW * m;
        const int nt_max = a.N / 32 - 1;
        nt = nt < nt_max ? nt : nt_max;
        wbase[m] = reinterpret_cast<const char*>(a.packed) + (size_t)kb_first * wstride + (size_t)nt * 1024;
    }
    const uint32_t wlane = lane * 16;
    // activation codes: instruction q covers tokens 8q..8q+7, lane l -> token 8q + l/8, LDS slot l%8,
    // global 16-byte chunk (l%8) ^ ((token/2) % 8); rows past T are clamped to the last row.
    // (rows are 128 B = half of the 64 LDS banks: 16 consecutive rows then cover every bank group once)
    const char* xbase = reinterpret_cast<const char*>(a.codes) + (size_t)t0 * a.K + (size_t)kb_first * kBK;
    uint32_t xlane[XL];
#pragma unroll
    for (int m = 0; m < XL; ++m) {
        const int q = wave + NW * m;
        const int row = 8 * q + (lane >> 3);
        int t = t0 + row;
        t = t < a.T ? t : a.T - 1;
        const int c = (lane & 7) ^ ((row >> 1) & 7);
        xlane[m] = (uint32_t)(t - t0) * (uint32_t)a.K + c * 16;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

    // Copy number m (0 .. XL+WL-1) of stage kb into LDS buffer `slot`.  Past the end of K the last
    // block is re-read so that every stage issues the same number of copies (the in-flight count
    // PENDING relies on it).
    auto issue_one = [&](int m, int kb, int slot) {
        const int kbc = kb < nkb ? kb : nkb - 1;
        if (m < XL) {
            const int q = wave + NW * m;
            lds_dma16(lds0 + slot * STAGE + q * 1024, xbase + (size_t)kbc * kBK, xlane[m]);
        } else {
            const int wtile = wave + NW * (m - XL);
            if ((BN / 32) % NW == 0 || wtile < BN / 32)
                lds_dma16(lds0 + slot * STAGE + XBYTES + wtile * 1024, wbase[m - XL] + (size_t)kbc * wstride, wlane);
        }
    };
    auto issue = [&](int kb, int slot) {
#pragma unroll
        for (int m = 0; m < XL + WL; ++m) issue_one(m, kb, slot);
    };

    v16i acc[TN][TT];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // LDS read offsets: token row = tile*32 + (lane & 31), the 16-byte chunk that matches packed dword ks of the
    // weight tile for this lane half, swizzled by (row/2) % 8
    int xoff[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
        xoff[ks] = (wt * TT * 32 + (lane & 31)) * kBK + ((code_chunk_of_dword(ks, lane >> 5) ^ ((lane >> 1) & 7)) << 4);
    const int woff = XBYTES + wn * TN * 1024 + lane * 16;

    // Register pipeline.  With one or two waves per SIMD, whatever a wave issues between two MFMAs is
    // time the matrix core idles unless it fits under the previous MFMA (8 passes = 32 cycles), so the
    // work for K-step s+1 - LDS operand reads, weight expansion, and once per stage the barrier and the
    // global->LDS copies - is dealt out in small pieces, one piece after each MFMA of K-step s.
    // sched_barrier(0) after every piece pins that order.
    v4i wpk[TN];      // packed weights of the current stage (reloaded for the next one in its last K-step)
    v4i xop[2][TT];   // code operands of the current / next K-step
    v4i wop[2][TN];   // expanded weight operands of the current / next K-step
    uint32_t wtmp[TN][4];   // the four groups of weight bytes of the dword being expanded (gemm_common.h)
    constexpr int NMF = TN * TT;                 // MFMAs per K-step
    constexpr int EOPS = 15;                     // VALU instructions to expand one packed dword
    // one VALU instruction of the expansion of wpk[i][ks] into wop[obuf][i]: 7 to separate the four groups of
    // (magnitude, sign) pairs, 4 look-ups to signed bytes, 4 interleaves into natural feature order
    auto expand_op = [&](int ks, int obuf, int i, int op) {
        const uint32_t p = (uint32_t)wpk[i][ks];
        if (op == 0) wtmp[i][0] = p & 0x05050505u;
        else if (op <= 6) {
            const int g = (op + 1) / 2;               // groups 1..3: shift, then mask
            if (op & 1) wtmp[i][g] = p >> (g == 1 ? 1 : g == 2 ? 4 : 5);
            else wtmp[i][g] &= 0x05050505u;
        } else if (op <= 10) {
            wtmp[i][op - 7] = weight_bytes(wtmp[i][op - 7]);
        } else {
            // groups: 0 = b even, 1 = a even, 2 = b odd, 3 = a odd; a = features 0..7, b = features 8..15
            const int r = op - 11;
            wop[obuf][i][r] = (int)weight_interleave(wtmp[i][r < 2 ? 3 : 2], wtmp[i][r < 2 ? 1 : 0], r & 1);
        }
    };
    auto expand_all = [&](int ks, int obuf) {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int op = 0; op < EOPS; ++op) expand_op(ks, obuf, i, op);
    };
    auto load_w_one = [&](int slot, int i) {
        wpk[i] = *reinterpret_cast<const v4i*>(lds + slot * STAGE + woff + i * 1024);
    };
    auto load_x_one = [&](int slot, int ks, int buf, int j) {
        xop[buf][j] = *reinterpret_cast<const v4i*>(lds + slot * STAGE + xoff[ks] + j * 32 * kBK);
    };

    // K-step with operands (wop[CUR], xop[CUR]); meanwhile fetch / expand K-step ks_next of the same
    // stage into (wop[CUR^1], xop[CUR^1]).
    auto kstep_inner = [&](auto cur_tag, int slot, int ks_next) {
        constexpr int CUR = decltype(cur_tag)::value;
        constexpr int TOTAL = EOPS * TN;
        constexpr int VPER = (TOTAL + NMF - 1) / NMF;
#pragma unroll
        for (int g = 0; g < NMF; ++g) {
            const int i = g / TT, j = g % TT;
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop[CUR][i], xop[CUR][j], acc[i][j], 0, 0, 0);
            if (g < TT) load_x_one(slot, ks_next, CUR ^ 1, g);
#pragma unroll
            for (int v = g * VPER; v < (g + 1) * VPER && v < TOTAL; ++v)
                expand_op(ks_next, CUR ^ 1, v / EOPS, v % EOPS);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // Last K-step of a stage (operands in [1]; the packed weights in wpk are dead by now): the copies of
    // stage kb+NSTAGE and the next stage's LDS reads go out under the first MFMAs, the expansion of the
    // next stage's first K-step (which needs those reads) under the last ones.
    auto kstep_last = [&](int kb, int slot) {
        constexpr int TOTAL = EOPS * TN;
        constexpr int SIDE = XL + WL > TN + TT ? XL + WL : TN + TT;   // MFMAs that carry a copy / read
        constexpr int FIRSTV = SIDE < NMF ? SIDE : 0;                  // first MFMA that carries expansion
        constexpr int VPER = (TOTAL + (NMF - FIRSTV) - 1) / (NMF - FIRSTV);
        const int nslot = slot + 1 == NSTAGE ? 0 : slot + 1;
        if (SIDE >= NMF) {   // small tiles: not enough MFMAs to hide the side work under, issue it up front
            issue(kb + NSTAGE, slot);
#pragma unroll
            for (int i = 0; i < TN; ++i) load_w_one(nslot, i);
#pragma unroll
            for (int j = 0; j < TT; ++j) load_x_one(nslot, 0, 0, j);
        }
#pragma unroll
        for (int g = 0; g < NMF; ++g) {
            const int i = g / TT, j = g % TT;
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wop[1][i], xop[1][j], acc[i][j], 0, 0, 0);
            if (SIDE < NMF) {
                if (g < XL + WL) issue_one(g, kb + NSTAGE, slot);
                if (g < TN) load_w_one(nslot, g);
                else if (g < TN + TT) load_x_one(nslot, 0, 0, g - TN);
            }
            if (g >= FIRSTV) {
#pragma unroll
                for (int v = (g - FIRSTV) * VPER; v < (g - FIRSTV + 1) * VPER && v < TOTAL; ++v)
                    expand_op(0, 0, v / EOPS, v % EOPS);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // prologue: stages 0 .. NSTAGE-2 in flight, then stage 0 visible and NSTAGE-1 issued
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) issue(s, s);
    wait_loads_then_barrier<PENDING>();
    issue(NSTAGE - 1, NSTAGE - 1);
#pragma unroll
    for (int i = 0; i < TN; ++i) load_w_one(0, i);
#pragma unroll
    for (int j = 0; j < TT; ++j) load_x_one(0, 0, 0, j);
    expand_all(0, 0);
    __builtin_amdgcn_sched_barrier(0);

    // Stage kb sits in LDS buffer `slot`; on entry wpk holds its packed weights and (wop[0], xop[0])
    // the operands of its K-step 0.  Before the last K-step the next stage is made visible (barrier)
    // and this stage's buffer is handed to the copies of stage kb+NSTAGE.  The last stage runs the same
    // code (one code path keeps the 256 accumulators in place): its "next stage" work re-reads stale
    // data that nothing consumes.
    using std::integral_constant;
    int slot = 0;
    for (int kb = 0; kb < nkb; ++kb) {
        kstep_inner(integral_constant<int, 0>{}, slot, 1);
        kstep_inner(integral_constant<int, 1>{}, slot, 2);
        kstep_inner(integral_constant<int, 0>{}, slot, 3);
        wait_loads_then_barrier<PENDING>();
        kstep_last(kb, slot);
        slot = slot + 1 == NSTAGE ? 0 : slot + 1;
    }
    // (the epilogue's scales are requested first, so that their latency passes under the drain: behind the
    // scheduling fences of the epilogue every one of them would cost its whole round trip)
    float sd_of[TT], alpha_of[TN];
    if (!RAW && !(SPLIT && a.split_k > 1)) {   // (the int32 forms have no scales: the pointers may be null)
#pragma unroll
        for (int j = 0; j < TT; ++j) {
            const int t = t0 + (wt * TT + j) * 32 + (lane & 31);
            sd_of[j] = t < a.T ? a.s_dequant[t] : 0.0f;
        }
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int nb = n0 + (wn * TN + i) * 32;
            alpha_of[i] = nb < a.N ? a.w_scales[a.rows_per_group == a.N ? 0 : nb / a.rows_per_group] : 0.0f;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    // drain the clamped tail loads, and wait until every wave is done with the stage buffers: the bf16
    // epilogue reuses them
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // epilogue: lane holds token t = ..+(lane&31); register quad g holds features 8g + 4*(lane>>5) + 0..3
    const bool write_partial = SPLIT && a.split_k > 1;
    if (RAW || write_partial) {   // int32 tiles (debug export / split-K partials): stored from where they are
#pragma unroll
        for (int j = 0; j < TT; ++j) {
            const int t = t0 + (wt * TT + j) * 32 + (lane & 31);
            if (t >= a.T) continue;
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                // one accumulator tile at a time: without this fence the compiler reads all TN*TT*16
                // accumulators out of the AGPRs up front and spills
                __builtin_amdgcn_sched_barrier(0);
                const int nb = n0 + (wn * TN + i) * 32;
                if (nb >= a.N) continue;
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = nb + 8 * g + 4 * (lane >> 5);
                    v4i o;
#pragma unroll
                    for (int r = 0; r < 4; ++r) o[r] = acc[i][j][4 * g + r];
                    if constexpr (RAW) *reinterpret_cast<v4i*>(a.acc_out + (size_t)t * a.N + n) = o;
                    else *reinterpret_cast<v4i*>(a.partial + ((size_t)ks * a.T + t) * a.N + n) = o;
                }
            }
        }
        return;
    }
    if constexpr (!RAW) {
        // bf16 output.  Stored from the accumulator layout, every instruction would touch 32 token rows
        // with 16 bytes each, and the output burst at the end of each round of workgroups is bound by the
        // number of such partial-line writes.  So the dequantised tiles go through the wave's share of the
        // LDS and leave as whole rows: TN*64 contiguous bytes per token, 16 bytes per lane.
        constexpr int ROWB = TN * 64 + 16;       // padded LDS row: 16-byte chunks stay aligned, rows shift by 4 banks
        constexpr int JG = TT < 2 ? TT : 2;      // token tiles per pass through the LDS
        constexpr int CPR = TN * 4;              // 16-byte chunks per row
        constexpr int RPI = 64 / CPR;            // rows per read instruction
        static_assert(NW * JG * 32 * ROWB <= NSTAGE * STAGE && 64 % CPR == 0 && TT % JG == 0, "epilogue staging");
        char* obuf = lds + wave * (JG * 32 * ROWB);
#pragma unroll
        for (int jg = 0; jg < TT; jg += JG) {
#pragma unroll
            for (int jj = 0; jj < JG; ++jj) {
                const int j = jg + jj;
                const float sd = sd_of[j];
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    __builtin_amdgcn_sched_barrier(0);   // one accumulator tile at a time (register pressure)
                    const int nb = n0 + (wn * TN + i) * 32;
                    const bool in_n = nb < a.N;
                    const float alpha = alpha_of[i];
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = nb + 8 * g + 4 * (lane >> 5);
                        v4i o;
#pragma unroll
                        for (int r = 0; r < 4; ++r) o[r] = acc[i][j][4 * g + r];
                        v4i ws = {0, 0, 0, 0};
                        if (a.code_offset != 0 && in_n) ws = *reinterpret_cast<const v4i*>(a.w_row_sum + n);
                        *reinterpret_cast<uint2*>(obuf + (jj * 32 + (lane & 31)) * ROWB +
                                                  (i * 32 + 8 * g + 4 * (lane >> 5)) * 2) =
                            dequant_quad_sums(o, sd, alpha, a.code_offset, ws);
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // a wave's LDS accesses execute in order: no barrier between its own writes and reads
#pragma unroll
            for (int r = 0; r < JG * 32; r += RPI) {
                const int row = r + lane / CPR;
                const int c = lane % CPR;
                const uint4 val = *reinterpret_cast<const uint4*>(obuf + row * ROWB + c * 16);
                const int t = t0 + (wt * TT + jg + row / 32) * 32 + (row & 31);
                const int n = n0 + wn * TN * 32 + c * 8;
                if (t < a.T && n < a.N) store_y16(a.y + (size_t)t * a.N + n, val);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Second half of the split-K path: y[t][n..n+3] from the split_k int32 partial tiles, summed in fixed
// order (integer, so exact) and passed through the same dequantising epilogue.  A separate launch: the
// kernel boundary is what makes the partials of workgroups on other XCDs visible.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const GemmArgs a) {
    const int quads = a.N / 4;
    const int64_t total = (int64_t)a.T * quads;
    for (int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x; idx < total; idx += (int64_t)gridDim.x * 256) {
        const int t = (int)(idx / quads);
        const int n = (int)(idx % quads) * 4;
        v4i sum = {0, 0, 0, 0};
        for (int k = 0; k < a.split_k; ++k)
            sum += *reinterpret_cast<const v4i*>(a.partial + ((size_t)k * a.T + t) * a.N + n);
        if (a.acc_out) {   // raw export: the integer sum itself
            *reinterpret_cast<v4i*>(a.acc_out + (size_t)t * a.N + n) = sum;
            continue;
        }
        *reinterpret_cast<uint2*>(a.y + (size_t)t * a.N + n) =
            dequant_quad(sum, a.s_dequant[t], a.w_scales[n / a.rows_per_group], a.code_offset, a.w_row_sum + n);
    }
}

}  // namespace
namespace gemm {
int launch_splitk_reduce(const GemmArgs& a, hipStream_t stream) {
    const int64_t quads = (int64_t)a.T * (a.N / 4);
    int64_t blocks = (quads + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    launch_kernel("splitk_reduce_kernel", splitk_reduce_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, a);
    return after_launch();
}
}  // namespace gemm
namespace {

template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool RAW, bool SPLIT = false, int OCC = 1>
int launch_cfg(GemmArgs a, hipStream_t stream) {
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int BT = WAVES_T * TT * 32;
    constexpr size_t lds = (size_t)NSTAGE * (BT * kBK + (BN / 32) * 1024);
    a.tiles_n = (a.N + BN - 1) / BN;
    a.tiles_t = (a.T + BT - 1) / BT;
    if (!SPLIT) a.split_k = 1;
    auto kern = ternary_gemm_kernel<WAVES_N, WAVES_T, TN, TT, NSTAGE, RAW, SPLIT, OCC>;
    static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
    if (const int rc = allow_dynamic_lds(kern, lds, lds_allowed); rc != HBL_OK) return rc;
    launch_kernel("ternary_gemm_kernel", kern, dim3((unsigned)(a.tiles_n * a.tiles_t * a.split_k)), dim3(64 * WAVES_N * WAVES_T), lds,
                       stream, a);
    int rc = after_launch();
    if (rc != HBL_OK || !SPLIT || a.split_k == 1) return rc;
    return launch_splitk_reduce(a, stream);
}

template <bool RAW>
int choose(const GemmArgs& a, hipStream_t stream, int tile) {
    const int64_t big_tiles = (int64_t)((a.N + 255) / 256) * ((a.T + 255) / 256);
    int cfg;
    if (a.T <= 64 && a.partial != nullptr && !RAW) cfg = a.T <= 32 ? 6 : 7;
    else if (a.T > 64 && a.partial != nullptr && a.split_k > 1 && !RAW) cfg = 8;   // mid-size batch, long K
    else if (a.T <= 32) cfg = 0;
    else if (a.T <= 64) cfg = 1;
    else if (big_tiles >= 200) {
        // 512 features x 128 tokens moves 32 KB per stage (16 codes + 16 weights) against 40 KB for 256 x 256:
        // 1-3 % faster here (4 % on the fp6 x fp4 kernel); the square tile stays where the wide one pads more
        const int64_t wide_tiles = (int64_t)((a.N + 511) / 512) * ((a.T + 127) / 128);
        cfg = wide_tiles <= big_tiles ? 4 : 3;
    } else cfg = 2;
    if (tile != kTileAuto && cfg < 6) {   // parity tests name the tile of the unsplit kernel themselves
        if (tile == kTileSquare) cfg = 3;
        else if (tile == kTileSmall) cfg = 2;
        else if (tile == kTileWide) cfg = 4;
        else return HBL_E_SHAPE;
    }
    switch (cfg) {
        case 0: return launch_cfg<4, 1, 2, 1, 4, RAW>(a, stream);   // 256 features x 32 tokens, 4 waves
        case 1: return launch_cfg<4, 1, 2, 2, 4, RAW>(a, stream);   // 256 x 64, 4 waves
        case 2: return launch_cfg<2, 2, 2, 2, 4, RAW>(a, stream);   // 128 x 128, 4 waves
        case 3: return launch_cfg<2, 2, 4, 4, 3, RAW>(a, stream);   // 256 x 256, 4 waves of 128 x 128
        case 4: return launch_cfg<4, 1, 4, 4, 3, RAW>(a, stream);   // 512 features x 128 tokens, 4 waves of 128 x 128
        case 6: if constexpr (!RAW) return launch_cfg<4, 1, 1, 1, 4, false, true>(a, stream);   // 128 x 32, split-K
        case 7: if constexpr (!RAW) return launch_cfg<4, 1, 1, 2, 4, false, true>(a, stream);   // 128 x 64, split-K
        case 8: if constexpr (!RAW) return launch_cfg<2, 2, 2, 2, 4, false, true>(a, stream);   // 128 x 128, split-K
        default: return HBL_E_SHAPE;
    }
}

}  // namespace

int launch_ternary_gemm(const int8_t* codes, int code_offset, int64_t T, int64_t K, const void* packed, int64_t N,
                        const float* s_dequant, const float* w_scales,
                        int64_t n_scale_groups, void* y_bf16, int32_t* acc_out, int32_t* splitk_partial,
                        hipStream_t stream, int tile) {
    if (T == 0) return HBL_OK;
    GemmArgs a;
    a.codes = codes;
    a.packed = static_cast<const uint32_t*>(packed);
    a.s_dequant = s_dequant;
    a.w_row_sum = reinterpret_cast<const int32_t*>(static_cast<const char*>(packed) + packed_tile_bytes(N, K));
    a.code_offset = code_offset;
    a.w_scales = w_scales;
    a.y = static_cast<uint16_t*>(y_bf16);
    a.acc_out = acc_out;
    a.T = (int)T;
    a.K = (int)K;
    a.N = (int)N;
    a.rows_per_group = n_scale_groups > 0 ? (int)(N / n_scale_groups) : (int)N;
    a.tiles_n = a.tiles_t = 0;
    a.split_k = splitk_partial ? (T <= 64 ? decode_split_k(T, K, N) : prefill_split_k(T, K, N)) : 1;
    a.partial = splitk_partial;
    return acc_out ? choose<true>(a, stream, tile) : choose<false>(a, stream, tile);
}

}  // namespace hbl
