// Ternary GEMM of H-BitLinear for INT4 activations on the fp6 x fp4 matrix-core path (Eq. 7):
//   acc[t][o] = sum_k q[t][k] * c[o][k],  q in [-8, 7] carried as bf6 (e3m2), c in {-1, 0, 1} as fp4 (e2m1).
// Every code and weight is exactly representable, every product is an integer of magnitude <= 8 and
// every partial sum stays below 2^24, so the fp32 accumulators of v_mfma_f32_32x32x64_f8f6f4 hold the
// same integers the int8 path produces (checked bit for bit by the parity tests) - at twice the int8
// MFMA rate per instruction and with far fewer toggling multiplier bits, which matters because the
// matrix cores are power-limited.  No offset trick is needed here: the operands are signed.
//
// Same skeleton as ternary_gemm.hip (256 x 256 tiles, 4 waves of 128 x 128, direct global->LDS copies,
// one small piece of side work after every MFMA).  Differences:
//   - a pipeline stage is still 128 features but only two MFMA K-steps of 64;
//   - activation codes arrive as the record image of code_records.h: 6 bits per code, a token row of a
//     stage is 96 bytes, a 128-token panel of a stage one contiguous 12 KiB block that is copied to LDS
//     as it is (twelve 1 KiB pieces), and an operand is one 16-byte + one 8-byte LDS read;
//   - the packed weights (sign / magnitude bit pairs) become fp4 operands with two AND and one shift per
//     dword: two operand registers of eight fp4 values each.
#include <atomic>
#include <type_traits>

#include "gemm_common.h"

namespace hbl {
namespace {

using namespace gemm;
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

// SPLIT: workgroup (tile, ks) covers K-blocks [ks * nkb/split_k, (ks+1) * nkb/split_k) and leaves its accumulators,
// converted to int32 (they are exact integers), in partial[ks][T][N] for the reduction launch.
// RAW: the accumulators themselves leave the kernel, as int32 [T, N] (acc_out), with no dequantisation: the
// export the parity tests compare with the integer contraction of Eq. 7 bit for bit.  With SPLIT the partial
// tiles are int32 either way and the reduction launch writes their sum undequantised.
template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool SPLIT = false, bool RAW = false>
__global__ __launch_bounds__(64 * WAVES_N * WAVES_T) void ternary_gemm_f6f4_kernel(const GemmArgs a) {
    constexpr int NW = WAVES_N * WAVES_T;
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int BT = WAVES_T * TT * 32;
    constexpr int XBYTES = BT * kRecordRowBytes;   // code records per stage (0.75 byte per feature)
    constexpr int WBYTES = (BN / 32) * 1024;       // packed weights per stage
    constexpr int STAGE = XBYTES + WBYTES;
    constexpr int XPIECES = XBYTES / 1024;         // 1 KiB pieces of the code panels of a stage
    constexpr int XL = XPIECES / NW;               // global->LDS copies per wave per stage: codes
    constexpr int WL = (BN / 32) / NW;             // ... and weights
    static_assert(BT % kPanelTokens == 0 && XPIECES % NW == 0 && (BN / 32) % NW == 0,
                  "stage copies must divide evenly over the waves");
    static_assert(NSTAGE >= 2, "need at least double buffering");
    constexpr int PENDING = (NSTAGE - 2) * (XL + WL);

    extern __shared__ __attribute__((aligned(1024))) char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % WAVES_N;
    const int wt = wave / WAVES_N;

    // each XCD gets a contiguous run of tiles, feature tile fastest (workgroups are dealt round-robin)
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
    const int kb0 = ks * nkb;

    // (K-block-major tiles: a stage's BN/32 tiles of this workgroup are consecutive KiB)
    const size_t wstride = (size_t)(a.N / 32) * 1024;
    const char* wbase[WL];
#pragma unroll
    for (int m = 0; m < WL; ++m) {
        int nt = n0 / 32 + wave + NW * m;
        const int nt_max = a.N / 32 - 1;
        nt = nt < nt_max ? nt : nt_max;
        wbase[m] = reinterpret_cast<const char*>(a.packed) + (size_t)kb0 * wstride + (size_t)nt * 1024;
    }
    const uint32_t wlane = lane * 16;
    // codes: the stage's panel blocks (one per 128 tokens of the tile, 12 KiB each, contiguous in the record
    // image) are copied as they are, piece q = 1 KiB; piece q of this wave belongs to panel q / 12
    const char* xbase = reinterpret_cast<const char*>(a.codes) +
                        ((size_t)(t0 / kPanelTokens) * nkb_total + kb0) * kRecordBlockBytes;
    const size_t panel_stride = (size_t)nkb_total * kRecordBlockBytes;
    const char* xpiece[XL];
#pragma unroll
    for (int m = 0; m < XL; ++m) {
        const int q = wave + NW * m;
        int panel = q / 12;
        const int panel_max = (a.T - 1) / kPanelTokens - t0 / kPanelTokens;   // panels past T do not exist: re-read the last one
        panel = panel < panel_max ? panel : panel_max;
        xpiece[m] = xbase + panel * panel_stride + (q % 12) * 1024;
    }
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;

    auto issue_one = [&](int m, int kb, int slot) {
        const int kbc = kb < nkb ? kb : nkb - 1;   // past the end: re-read the last block (keeps PENDING valid)
        if (m < XL) {
            const int q = wave + NW * m;
            lds_dma16(lds0 + slot * STAGE + q * 1024, xpiece[m] + (size_t)kbc * kRecordBlockBytes, wlane);
        } else {
            const int wtile = wave + NW * (m - XL);
            lds_dma16(lds0 + slot * STAGE + XBYTES + wtile * 1024, wbase[m - XL] + (size_t)kbc * wstride, wlane);
        }
    };
    auto issue = [&](int kb, int slot) {
#pragma unroll
        for (int m = 0; m < XL + WL; ++m) issue_one(m, kb, slot);
    };

    v16f acc[TN][TT];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TT; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

    // record of K-step s (64 features) for lane half h = lane >> 5: 16 bytes + 8 bytes of the token's 96-byte
    // row (code_records.h; the tile's rows are whole panels, so row mod 128 and lane agree in bits 3 and 4)
    int xoff_lo[2], xoff_hi[2];
    {
        const int r = lane & 31;
        const int rowoff = (wt * TT * 32 + r) * kRecordRowBytes;
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            xoff_lo[s] = rowoff + record_lo_offset(r, s, lane >> 5);
            xoff_hi[s] = rowoff + record_hi_offset(r, s, lane >> 5);
        }
    }
    const int woff = XBYTES + wn * TN * 1024 + lane * 16;

    v4i wpk[TN];      // packed weights of the current stage: dword 2s + d
    v8i xop[2][TT];   // code operands (6 registers used) of the current / next K-step
    v8i wop[2][TN];   // weight operands (4 registers used)
#pragma unroll
    for (int b = 0; b < 2; ++b) {
#pragma unroll
        for (int j = 0; j < TT; ++j) xop[b][j][6] = xop[b][j][7] = 0;
#pragma unroll
        for (int i = 0; i < TN; ++i) wop[b][i][4] = wop[b][i][5] = wop[b][i][6] = wop[b][i][7] = 0;
    }
    constexpr int NMF = TN * TT;
    constexpr int EOPS = 6;   // VALU instructions to expand the two packed dwords of one K-step
    auto expand_op = [&](int s, int obuf, int i, int op) {
        const uint32_t p = (uint32_t)wpk[i][2 * s + op / 3];
        const int r = 2 * (op / 3);
        const int st = op % 3;
        if (st == 0) wop[obuf][i][r] = (int)(p & 0xAAAAAAAAu);
        else if (st == 1) wop[obuf][i][r + 1] = (int)(p << 1);
        else wop[obuf][i][r + 1] = (int)((uint32_t)wop[obuf][i][r + 1] & 0xAAAAAAAAu);
    };
    auto load_w_one = [&](int slot, int i) {
        wpk[i] = *reinterpret_cast<const v4i*>(lds + slot * STAGE + woff + i * 1024);
    };
    // half an operand per call: part 0 = the 16-byte piece, part 1 = the 8-byte piece
    auto load_x_part = [&](int slot, int s, int buf, int j, int part) {
        const char* base = lds + slot * STAGE + j * 32 * kRecordRowBytes;
        if (part == 0) {
            const v4i lo = *reinterpret_cast<const v4i*>(base + xoff_lo[s]);
            xop[buf][j][0] = lo[0]; xop[buf][j][1] = lo[1]; xop[buf][j][2] = lo[2]; xop[buf][j][3] = lo[3];
        } else {
            const int2 hi = *reinterpret_cast<const int2*>(base + xoff_hi[s]);
            xop[buf][j][4] = hi.x; xop[buf][j][5] = hi.y;
        }
    };
    auto mfma = [&](int cur, int g) {
        const int i = g / TT, j = g % TT;
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(wop[cur][i], xop[cur][j], acc[i][j], 4 /*A: fp4*/,
                                                                    3 /*B: bf6*/, 0, 0, 0, 0);
    };

    // K-step 0 of a stage (operands in [0]); meanwhile fetch / expand K-step 1 into [1]
    auto kstep_first = [&](int slot) {
        constexpr int TOTAL = EOPS * TN;
        constexpr int VPER = (TOTAL + NMF - 1) / NMF;
        if (2 * TT > NMF) {
#pragma unroll
            for (int x = 0; x < 2 * TT; ++x) load_x_part(slot, 1, 1, x / 2, x % 2);
        }
#pragma unroll
        for (int g = 0; g < NMF; ++g) {
            mfma(0, g);
            if (2 * TT <= NMF && g < 2 * TT) load_x_part(slot, 1, 1, g / 2, g % 2);
#pragma unroll
            for (int v = g * VPER; v < (g + 1) * VPER && v < TOTAL; ++v) expand_op(1, 1, v / EOPS, v % EOPS);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // K-step 1 (operands in [1]; wpk is dead): copies of stage kb+NSTAGE and the next stage's LDS reads go
    // out under the first MFMAs, the expansion of the next stage's K-step 0 under the last ones
    auto kstep_last = [&](int kb, int slot) {
        constexpr int TOTAL = EOPS * TN;
        constexpr int READS = TN + 2 * TT;
        constexpr int SIDE = XL + WL > READS ? XL + WL : READS;
        constexpr bool FITS = SIDE <= NMF - 2;
        constexpr int FIRSTV = FITS ? (TN + 2 < NMF - 2 ? TN + 2 : NMF - 2) : 0;
        constexpr int VPER = (TOTAL + (NMF - FIRSTV) - 1) / (NMF - FIRSTV);
        const int nslot = slot + 1 == NSTAGE ? 0 : slot + 1;
        if (!FITS) {
            issue(kb + NSTAGE, slot);
#pragma unroll
            for (int i = 0; i < TN; ++i) load_w_one(nslot, i);
#pragma unroll
            for (int x = 0; x < 2 * TT; ++x) load_x_part(nslot, 0, 0, x / 2, x % 2);
        }
#pragma unroll
        for (int g = 0; g < NMF; ++g) {
            mfma(1, g);
            if (FITS) {
                if (g < XL + WL) issue_one(g, kb + NSTAGE, slot);
                if (g < TN) load_w_one(nslot, g);
                else if (g < READS) load_x_part(nslot, 0, 0, (g - TN) / 2, (g - TN) % 2);
            }
            if (g >= FIRSTV) {
#pragma unroll
                for (int v = (g - FIRSTV) * VPER; v < (g - FIRSTV + 1) * VPER && v < TOTAL; ++v)
                    expand_op(0, 0, v / EOPS, v % EOPS);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // prologue
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) issue(s, s);
    wait_loads_then_barrier<PENDING>();
    issue(NSTAGE - 1, NSTAGE - 1);
#pragma unroll
    for (int i = 0; i < TN; ++i) load_w_one(0, i);
#pragma unroll
    for (int x = 0; x < 2 * TT; ++x) load_x_part(0, 0, 0, x / 2, x % 2);
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int op = 0; op < EOPS; ++op) expand_op(0, 0, i, op);
    __builtin_amdgcn_sched_barrier(0);

    // One code path for every stage (the last one's "next stage" work re-reads stale data nobody uses).
    int slot = 0;
    for (int kb = 0; kb < nkb; ++kb) {
        kstep_first(slot);
        wait_loads_then_barrier<PENDING>();
        kstep_last(kb, slot);
        slot = slot + 1 == NSTAGE ? 0 : slot + 1;
    }
    // drain the clamped tail copies, and wait until every wave is done with the stage buffers: the
    // epilogue reuses them
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
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");

    if constexpr (SPLIT || RAW) {
        if (RAW || a.split_k > 1) {   // int32 tiles, stored from where the accumulators are
            int32_t* const out = (SPLIT && a.split_k > 1) ? a.partial + (size_t)ks * a.T * a.N : a.acc_out;
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TT; ++j) {
                    __builtin_amdgcn_sched_barrier(0);   // one accumulator tile at a time (register pressure)
                    const int t = t0 + (wt * TT + j) * 32 + (lane & 31);
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int n = n0 + (wn * TN + i) * 32 + 8 * g + 4 * (lane >> 5);
                        const v4i o = {(int)acc[i][j][4 * g], (int)acc[i][j][4 * g + 1], (int)acc[i][j][4 * g + 2],
                                       (int)acc[i][j][4 * g + 3]};
                        if (t < a.T && n < a.N) *reinterpret_cast<v4i*>(out + (size_t)t * a.N + n) = o;
                    }
                }
            return;
        }
    }

    // Epilogue.  A lane holds token (lane & 31) of a 32 x 32 tile, register quad g holding features
    // 8g + 4*(lane >> 5) + 0..3: stored from there, every instruction would touch 32 token rows with
    // 16 bytes each, and the output burst at the end of each round of workgroups (all of them finish
    // together) is bound by the number of such partial-line writes, not by bytes (measured: a third of
    // the run time at K = 4096).  So the dequantised bf16 tiles go through the wave's share of the LDS
    // and leave as whole rows: TN*64 contiguous bytes per token, 16 bytes per lane.
    // The accumulators are integers held in fp32: y = bf16((acc * s_d) * alpha) as on the int8 path.
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
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
                const float alpha = alpha_of[i];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    float v[4];
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = (acc[i][j][4 * g + r] * sd) * alpha;
                    const bf16x2 lo = __builtin_convertvector((f32x2){v[0], v[1]}, bf16x2);
                    const bf16x2 hi = __builtin_convertvector((f32x2){v[2], v[3]}, bf16x2);
                    *reinterpret_cast<uint2*>(obuf + (jj * 32 + (lane & 31)) * ROWB +
                                              (i * 32 + 8 * g + 4 * (lane >> 5)) * 2) =
                        make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
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

template <int WAVES_N, int WAVES_T, int TN, int TT, int NSTAGE, bool SPLIT = false, bool RAW = false>
int launch_cfg(GemmArgs a, hipStream_t stream) {
    constexpr int BN = WAVES_N * TN * 32;
    constexpr int BT = WAVES_T * TT * 32;
    constexpr size_t lds = (size_t)NSTAGE * (BT * kRecordRowBytes + (BN / 32) * 1024);
    a.tiles_n = (a.N + BN - 1) / BN;
    a.tiles_t = (a.T + BT - 1) / BT;
    if (!SPLIT) a.split_k = 1;
    auto kern = ternary_gemm_f6f4_kernel<WAVES_N, WAVES_T, TN, TT, NSTAGE, SPLIT, RAW>;
    static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
    if (const int rc = allow_dynamic_lds(kern, lds, lds_allowed); rc != HBL_OK) return rc;
    launch_kernel("ternary_gemm_f6f4_kernel", kern, dim3((unsigned)(a.tiles_n * a.tiles_t * a.split_k)), dim3(64 * WAVES_N * WAVES_T), lds,
                       stream, a);
    const int rc = after_launch();
    if (rc != HBL_OK || a.split_k == 1) return rc;
    return launch_splitk_reduce(a, stream);
}

}  // namespace

int launch_ternary_gemm_f6f4(const int8_t* code_records, int64_t T, int64_t K, const void* packed, int64_t N,
                             const float* s_dequant, const float* w_scales, int64_t n_scale_groups, void* y_bf16,
                             hipStream_t stream, int32_t* splitk_partial, int32_t* acc_out, int tile) {
    if (T == 0) return HBL_OK;
    GemmArgs a = {};
    a.codes = code_records;
    a.packed = static_cast<const uint32_t*>(packed);
    a.s_dequant = s_dequant;
    a.w_scales = w_scales;
    a.y = static_cast<uint16_t*>(y_bf16);
    a.acc_out = acc_out;
    a.T = (int)T;
    a.K = (int)K;
    a.N = (int)N;
    a.rows_per_group = n_scale_groups > 0 ? (int)(N / n_scale_groups) : (int)N;
    a.split_k = splitk_partial ? prefill_split_k(T, K, N) : 1;
    a.partial = splitk_partial;
    a.code_offset = 0;      // signed operands: no correction terms
    // Workgroup tile: 64 K outputs either way (the 256 accumulator registers of four waves).  512 features x 128
    // tokens moves 32 KB per 128-feature stage through L2 and LDS (16 KB of codes + 16 KB of packed weights) against
    // 40 KB for 256 x 256 (32 + 8): measured 4 % faster on the GEMM at N = 4096 and 12288, equal at N = 32768.  The
    // square tile stays for shapes the wide one pads more; below ~180 tiles (256 CUs) the small tile takes over
    // (192 big tiles measured 8 % faster than 768 tiles of 128 x 128).
    const int64_t tiles_sq = (int64_t)((N + 255) / 256) * ((T + 255) / 256);
    const int64_t tiles_wide = (int64_t)((N + 511) / 512) * ((T + 127) / 128);
    int cfg = tiles_sq >= 180 ? (tiles_wide <= tiles_sq ? kTileWide : kTileSquare) : kTileSmall;
    if (a.split_k > 1) cfg = kTileSplitK;   // mid-size batch, long K
    if (tile != kTileAuto) {                // parity tests name the tile themselves
        cfg = tile;
        if (cfg == kTileSplitK) {
            if (!splitk_partial) return HBL_E_WORKSPACE;
            // any power-of-two cut that leaves whole K-blocks; the forward's own choice when it has one
            if (a.split_k == 1) a.split_k = (K / 128) % 4 == 0 ? 4 : ((K / 128) % 2 == 0 ? 2 : 1);
        }
    }
    if (cfg == kTileSplitK && a.split_k <= 1) cfg = kTileSmall;   // nothing to cut: the same tile, unsplit
    if (cfg != kTileSplitK) a.split_k = 1;
    const bool raw = acc_out != nullptr;
    switch (cfg) {
        case kTileSquare:   // 256 x 256, 2 x 2 waves of 128 x 128
            return raw ? launch_cfg<2, 2, 4, 4, 3, false, true>(a, stream) : launch_cfg<2, 2, 4, 4, 3>(a, stream);
        case kTileSmall:    // 128 x 128
            return raw ? launch_cfg<2, 2, 2, 2, 4, false, true>(a, stream) : launch_cfg<2, 2, 2, 2, 4>(a, stream);
        case kTileWide:     // 512 features x 128 tokens, 4 x 1 waves of 128 x 128
            return raw ? launch_cfg<4, 1, 4, 4, 3, false, true>(a, stream) : launch_cfg<4, 1, 4, 4, 3>(a, stream);
        case kTileSplitK:   // 128 x 128, K cut over workgroups, int32 partial tiles + reduction launch
            return launch_cfg<2, 2, 2, 2, 4, true>(a, stream);
        default: return HBL_E_SHAPE;
    }
}

}  // namespace hbl
