// Activation front end of H-BitLinear (Section 2.1): online Hadamard transform
// (Eq. 3-4) fused with the per-token INT8 absmax / INT4 absmean quantiser
// (Eq. 5-6).  One workgroup owns one token row; the row never leaves registers
// / LDS between the load of x and the store of the int8 codes.
//
// Arithmetic contract (what makes the codes reproducible bit for bit):
//   - butterflies are single fp32 adds / subtracts, stages in ascending stride
//     order 1,2,4,...,K/2 - which stage runs in registers, across lanes or
//     through LDS does not change any value;
//   - one multiply by c_n = (float)(1/sqrt(K)) after the last stage;
//   - gamma = max|x_r| (exact); beta = (float)(sum|x_r| in fp64 / K);
//   - gain = 127/(gamma+eps) or sqrt7/(beta+eps) with IEEE fp32 division,
//     code = RoundClip(gain * x_r) with round-half-to-even.
//
// Index bits of a row of K = CH*64*R*W elements, low to high:
//   [e: log2 CH in-thread][lane: 6][r: log2 R in-thread chunks][wave: log2 W]
// so that every global access is one contiguous CH-element piece per lane and
// the stage order e -> lane -> r -> wave is ascending.  The wave stages swap
// the wave bits with the low r bits through LDS once, then run in registers.
#include <atomic>
#include <type_traits>

#include "hbl_internal.h"

namespace hbl {
namespace {

constexpr float kRoot7 = 2.6457513110645907f;  // (float)sqrt(7.0), bit pattern 0x402953FD
constexpr float kMagic = 12582912.0f;          // 1.5 * 2^23: adding it rounds to an integer (nearest-even)

__device__ __forceinline__ float as_f(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Value held by lane (lane ^ MASK).
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
    const int iv = (int)as_u(v);
    if constexpr (MASK == 1) {
        return as_f((uint32_t)__builtin_amdgcn_mov_dpp(iv, 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
    } else if constexpr (MASK == 2) {
        return as_f((uint32_t)__builtin_amdgcn_mov_dpp(iv, 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
    } else if constexpr (MASK == 8) {
        return as_f((uint32_t)__builtin_amdgcn_mov_dpp(iv, 0x128, 0xF, 0xF, false));  // row_ror:8
    } else if constexpr (MASK == 4) {
        return as_f((uint32_t)__builtin_amdgcn_ds_swizzle(iv, 0x101F));  // xor 4 inside 32 lanes
    } else if constexpr (MASK == 16) {
        return as_f((uint32_t)__builtin_amdgcn_ds_swizzle(iv, 0x401F));  // xor 16 inside 32 lanes
    } else {
        return __shfl_xor(v, MASK, 64);
    }
}

// Whole-wave reductions whose result every lane receives; all 64 lanes must be active.
// Form 1, data-parallel moves: inside a row of 16 lanes two quad permutes, then the half-row and row mirrors
// (each step adds the same two partial results in both lanes of a pair, so all lanes of the row agree); the
// four row results are then read lane by lane and combined in a fixed order.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move(uint32_t v) {
    return (uint32_t)__builtin_amdgcn_mov_dpp((int)v, CTRL, 0xF, 0xF, false);
}
// v <- v(partner lane) * c + v for the four registers of a chunk, the partner reached by DPP permutation CTRL:
// v_fmac_f32 with a DPP source, which the compiler does not form by itself (it emits a DPP move and a separate
// multiply-add).  A DPP operand must not be read within two wait states of a vector-ALU write to the same
// register, and the compiler does not look inside an asm statement: the leading s_nop covers whatever
// precedes the block, and inside it the four instructions touch four different registers.  (Blocks of 16
// with one s_nop measured slower: the compiler can no longer place other work between the chunks.)
template <int CTRL>
__device__ __forceinline__ void lane_butterfly4(float (&a)[4], float c) {
    static_assert(CTRL == 0xB1 || CTRL == 0x4E || CTRL == 0x141 || CTRL == 0x128, "lane xor 1, 2, 7 or 8");
#define HBL_F(N, SEL) "v_fmac_f32_dpp %" #N ", %" #N ", %4 " SEL " row_mask:0xf bank_mask:0xf\n\t"
#define HBL_LANE_FMAC4(SEL) asm("s_nop 1\n\t" HBL_F(0, SEL) HBL_F(1, SEL) HBL_F(2, SEL) HBL_F(3, SEL) : "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) : "v"(c))
    if constexpr (CTRL == 0xB1) HBL_LANE_FMAC4("quad_perm:[1,0,3,2]");
    else if constexpr (CTRL == 0x4E) HBL_LANE_FMAC4("quad_perm:[2,3,0,1]");
    else if constexpr (CTRL == 0x141) HBL_LANE_FMAC4("row_half_mirror");
    else HBL_LANE_FMAC4("row_ror:8");
#undef HBL_LANE_FMAC4
#undef HBL_F
}
template <int CTRL>
__device__ __forceinline__ void lane_butterfly2(float (&a)[2], float c) {
#define HBL_F(N, SEL) "v_fmac_f32_dpp %" #N ", %" #N ", %2 " SEL " row_mask:0xf bank_mask:0xf\n\t"
#define HBL_LANE_FMAC2(SEL) asm("s_nop 1\n\t" HBL_F(0, SEL) HBL_F(1, SEL) : "+v"(a[0]), "+v"(a[1]) : "v"(c))
    if constexpr (CTRL == 0xB1) HBL_LANE_FMAC2("quad_perm:[1,0,3,2]");
    else if constexpr (CTRL == 0x4E) HBL_LANE_FMAC2("quad_perm:[2,3,0,1]");
    else if constexpr (CTRL == 0x141) HBL_LANE_FMAC2("row_half_mirror");
    else HBL_LANE_FMAC2("row_ror:8");
#undef HBL_LANE_FMAC2
#undef HBL_F
}
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint64_t r = (uint64_t)dpp_move<CTRL>((uint32_t)u) | ((uint64_t)dpp_move<CTRL>((uint32_t)(u >> 32)) << 32);
    return __builtin_bit_cast(double, r);
}
__device__ __forceinline__ uint32_t read_lane(uint32_t v, int lane) {
    return (uint32_t)__builtin_amdgcn_readlane((int)v, lane);
}
__device__ __forceinline__ double read_lane(double v, int lane) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint64_t r = (uint64_t)read_lane((uint32_t)u, lane) | ((uint64_t)read_lane((uint32_t)(u >> 32), lane) << 32);
    return __builtin_bit_cast(double, r);
}
__device__ __forceinline__ double wave_sum_dpp(double s) {
    s += dpp_move<0xB1>(s);    // quad_perm [1,0,3,2]
    s += dpp_move<0x4E>(s);    // quad_perm [2,3,0,1]
    s += dpp_move<0x141>(s);   // row_half_mirror
    s += dpp_move<0x140>(s);   // row_mirror
    return ((read_lane(s, 0) + read_lane(s, 16)) + read_lane(s, 32)) + read_lane(s, 48);
}
__device__ __forceinline__ int wave_sum_dpp(int value) {   // modulo 2^32
    uint32_t s = (uint32_t)value;
    s += dpp_move<0xB1>(s);
    s += dpp_move<0x4E>(s);
    s += dpp_move<0x141>(s);
    s += dpp_move<0x140>(s);
    return (int)(read_lane(s, 0) + read_lane(s, 16) + read_lane(s, 32) + read_lane(s, 48));
}
__device__ __forceinline__ float wave_max_dpp(float m) {
    m = fmaxf(m, as_f(dpp_move<0xB1>(as_u(m))));
    m = fmaxf(m, as_f(dpp_move<0x4E>(as_u(m))));
    m = fmaxf(m, as_f(dpp_move<0x141>(as_u(m))));
    m = fmaxf(m, as_f(dpp_move<0x140>(as_u(m))));
    return fmaxf(fmaxf(as_f(read_lane(as_u(m), 0)), as_f(read_lane(as_u(m), 16))),
                 fmaxf(as_f(read_lane(as_u(m), 32)), as_f(read_lane(as_u(m), 48))));
}
// Form 2, six xor-shuffle rounds through the LDS crossbar: long dependent latency but no vector-ALU work.
// A launch that keeps every SIMD busy with other waves runs faster with these (5 % on 8192 rows of 16384); a
// launch of a few rows runs faster with form 1 (1.5 us per decode layer).  `few_rows` is uniform.
__device__ __forceinline__ double wave_sum(double s, int few_rows) {
    if (few_rows) return wave_sum_dpp(s);
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) s += __shfl_xor(s, sft, 64);
    return s;
}
__device__ __forceinline__ int wave_sum(int s, int few_rows) {
    if (few_rows) return wave_sum_dpp(s);
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) s += __shfl_xor(s, sft, 64);
    return s;
}
__device__ __forceinline__ float wave_max(float m, int few_rows) {
    if (few_rows) return wave_max_dpp(m);
#pragma unroll
    for (int sft = 1; sft < 64; sft <<= 1) m = fmaxf(m, __shfl_xor(m, sft, 64));
    return m;
}

// Butterfly between lanes in one multiply-add per element (lane_butterfly4): v <- partner * c + v, c = -1 on the
// lane whose index bit is set.  That lane then holds the negative of the reference's a - b; see the large-row body
// for why a lane may simply carry that sign until the values meet their 1/sqrt(K) factor.
template <int CTRL, int R, int CH>
__device__ __forceinline__ void lane_stage_fma(float (&v)[R][CH], bool upper) {
    const float c = upper ? -1.0f : 1.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if constexpr (CH == 2) {
            lane_butterfly2<CTRL>(v[r], c);
        } else {
#pragma unroll
            for (int e = 0; e < CH; e += 4) {
                float (&q)[4] = *reinterpret_cast<float (*)[4]>(&v[r][e]);
                lane_butterfly4<CTRL>(q, c);
            }
        }
    }
}

template <int MASK, int R, int CH>
__device__ __forceinline__ void lane_stage(float (&v)[R][CH], int lane) {
    // lanes with the bit clear compute a + b, lanes with it set compute a - b = partner - own
    const uint32_t sign = (lane & MASK) ? 0x80000000u : 0u;
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            const float own = v[r][e];
            const float partner = lane_xor<MASK>(own);
            v[r][e] = partner + as_f(as_u(own) ^ sign);
        }
}

template <int BYTES>
struct Raw;
template <>
struct Raw<2> { using type = uint16_t; };
template <>
struct Raw<4> { using type = uint32_t; };
template <>
struct Raw<8> { using type = uint2; };
template <>
struct Raw<16> { using type = uint4; };
template <>
struct Raw<32> { struct type { uint4 a, b; }; };

// Load CH consecutive elements starting at element offset `off` and widen to fp32.
template <int CH, bool BF16>
__device__ __forceinline__ void load_chunk(const void* x, int64_t off, float (&dst)[CH]) {
    if constexpr (BF16) {
        using V = typename Raw<CH * 2>::type;
        V raw = *reinterpret_cast<const V*>(static_cast<const uint16_t*>(x) + off);
        const uint16_t* h = reinterpret_cast<const uint16_t*>(&raw);
#pragma unroll
        for (int e = 0; e < CH; ++e) dst[e] = as_f((uint32_t)h[e] << 16);
    } else {
        using V = typename Raw<CH * 4>::type;
        V raw = *reinterpret_cast<const V*>(static_cast<const float*>(x) + off);
        const float* f = reinterpret_cast<const float*>(&raw);
#pragma unroll
        for (int e = 0; e < CH; ++e) dst[e] = f[e];
    }
}

// Four stored bytes code + 8 (0..15) -> their bf6 (e3m2) bit patterns, 6 bits each, as 24 contiguous
// bits.  Two 8-entry byte-permute look-ups and a select:
//   -8..-5 = 38 37 36 35, -4..-1 = 34 32 30 2c, 0..3 = 00 0c 10 12, 4..7 = 14 15 16 17 (hex)
__device__ __forceinline__ uint32_t bf6_pack4(uint32_t packed) {
    const uint32_t sel = packed & 0x07070707u;
    const uint32_t neg = __builtin_amdgcn_perm(0x2C303234u, 0x35363738u, sel);
    const uint32_t pos = __builtin_amdgcn_perm(0x17161514u, 0x12100C00u, sel);
    // byte i of the result: byte i of `pos` if bit 3 of the index is set, else byte i of `neg`
    const uint32_t pick = ((packed >> 1) & 0x04040404u) | 0x03020100u;
    const uint32_t r = __builtin_amdgcn_perm(pos, neg, pick);
    // four 6-bit fields, one per byte -> 24 contiguous bits
    const uint32_t t2 = (r & 0x003F003Fu) | ((r & 0x3F003F00u) >> 2);
    return (t2 & 0xFFFu) | ((t2 >> 4) & 0xFFF000u);
}

// bf6 record output for a lane that holds the 8 features of chunk `chunk8` of token `row` as two 24-bit
// halves, where neighbouring lanes hold neighbouring chunks: the even lane of each pair fetches its
// partner's halves and stores the pair's 16 features (96 bits) into the record image (code_records.h).
// Every lane of a quad must call this.
__device__ __forceinline__ void bf6_store_pair(int8_t* codes, int64_t row, int K, int chunk8, uint32_t lo, uint32_t hi) {
    const uint32_t p_lo = (uint32_t)__builtin_amdgcn_mov_dpp((int)lo, 0xB1, 0xF, 0xF, false);   // lane ^ 1
    const uint32_t p_hi = (uint32_t)__builtin_amdgcn_mov_dpp((int)hi, 0xB1, 0xF, 0xF, false);
    if ((chunk8 & 1) == 0)
        store_code_quad(codes, row, K, chunk8 >> 1, lo | (hi << 24), (hi >> 8) | (p_lo << 16), (p_lo >> 16) | (p_hi << 8));
}

// Per-row scalars of the front end: the quantiser's epsilon and, if ln_gain != nullptr, the RMS
// normalisation that precedes the transform in Eq. 7 (LN; the model's norm is RMSNorm, Section 2):
//   x_n[k] = (x[k] * r) * ln_gain[k],  r = (float)(1 / sqrt(mean_k x[k]^2 + ln_eps)),
// mean of squares accumulated in fp64 (each square is exact there), r rounded to fp32 once, two fp32
// multiplies per element.
struct RowParams {
    float eps;
    const float* ln_gain;   // [K] fp32 or nullptr
    float ln_eps;
    int few_rows;           // a launch of at most 64 rows: latency matters, not throughput (reduction form)
};

// r of the row from this thread's partial sum of squares `ss`: wave butterfly, then a fixed-order
// combine of the NW per-wave sums through `red` (NW doubles of LDS; one barrier).
template <int NW>
__device__ __forceinline__ float rms_factor(double ss, double* red, int lane, int wave, int K, float ln_eps,
                                            int few_rows) {
    ss = wave_sum(ss, few_rows);
    if constexpr (NW > 1) {
        if (lane == 0) red[wave] = ss;
        __syncthreads();
        ss = red[0];
#pragma unroll
        for (int w = 1; w < NW; ++w) ss += red[w];
    }
    return (float)(1.0 / sqrt(ss / (double)K + (double)ln_eps));
}

// Transform-only output (BITS == 0 in the bodies below): N consecutive values of x_r as fp32 or, rounded
// to nearest even, as bf16.
template <int N>
__device__ __forceinline__ void store_xr(void* out, int out_dtype, int64_t elem, const float* v) {
    static_assert(N % 2 == 0, "pairs");
    if (out_dtype == HBL_BF16) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        typedef float f32x2 __attribute__((ext_vector_type(2)));
        uint32_t h[N / 2];
#pragma unroll
        for (int i = 0; i < N / 2; ++i)
            h[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2){v[2 * i], v[2 * i + 1]}, bf16x2));
        uint32_t* dst = reinterpret_cast<uint32_t*>(static_cast<uint16_t*>(out) + elem);
        if constexpr (N == 2) dst[0] = h[0];
        else if constexpr (N == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(h[0], h[1]);
        else {
#pragma unroll
            for (int i = 0; i < N / 8; ++i)
                reinterpret_cast<uint4*>(dst)[i] = make_uint4(h[4 * i], h[4 * i + 1], h[4 * i + 2], h[4 * i + 3]);
        }
    } else {
        float* dst = static_cast<float*>(out) + elem;
        if constexpr (N == 2) *reinterpret_cast<float2*>(dst) = make_float2(v[0], v[1]);
        else {
#pragma unroll
            for (int i = 0; i < N / 4; ++i)
                reinterpret_cast<float4*>(dst)[i] = make_float4(v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]);
        }
    }
}

// One token row per workgroup of 64*W threads; `row` and `tid` come from the caller so that the grouped
// launch (several projections' rows in one grid) can run the same body.
template <int LOG2K, int W, int BITS, bool BF16, bool HADAMARD>
__device__ __forceinline__ void fwht_quant_body(int64_t row, int tid, const void* __restrict__ x,
                                                int8_t* __restrict__ codes, float* __restrict__ s_dequant,
                                                int32_t* __restrict__ code_sum, RowParams rp, int code_offset) {
    const int few_rows = rp.few_rows;
    constexpr int K = 1 << LOG2K;
    constexpr int NT = 64 * W;
    constexpr int E = K / NT;            // elements per thread
    constexpr int CH = E < 8 ? E : 8;    // contiguous elements per chunk
    constexpr int R = E / CH;            // chunks per thread
    static_assert(E >= 1 && R >= 1 && (W == 1 || R >= W), "unsupported split");

    __shared__ double red_d[W];
    __shared__ float red_f[W];
    __shared__ int red_i[W];
    extern __shared__ float exch[];      // K floats when HADAMARD && W > 1

    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t row_off = row * (int64_t)K;
    // Position of this lane's chunks inside a group of 64.  With the transform, lane ^ (3 if bit 2 is set): flipping
    // position bit 2 then flips lane bits 0-2 together, which is the one xor-4-like permutation DPP offers inside a
    // row of 16 lanes (the half-row mirror, lane ^ 7); bits 0, 1 and 3 flip by quad permutes and a row rotation.
    const int pos = HADAMARD ? lane ^ (((lane >> 2) & 1) * 3) : lane;

    float v[R][CH];
#pragma unroll
    for (int r = 0; r < R; ++r) load_chunk<CH, BF16>(x, row_off + (int64_t)((wave * R + r) * 64 + pos) * CH, v[r]);

    if (rp.ln_gain) {   // uniform: RMS normalisation ahead of the transform
        __shared__ double red_n[W];
        double ss = 0.0;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < CH; ++e) ss += (double)v[r][e] * (double)v[r][e];
        const float rn = rms_factor<W>(ss, red_n, lane, wave, K, rp.ln_eps, few_rows);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float gv[CH];
            load_chunk<CH, false>(rp.ln_gain, (int64_t)((wave * R + r) * 64 + pos) * CH, gv);
#pragma unroll
            for (int e = 0; e < CH; ++e) v[r][e] = (v[r][e] * rn) * gv[e];
        }
    }

    bool exchanged = false;  // register slot r holds chunk g = wave*R + r until the LDS exchange

    if constexpr (HADAMARD) {
        // e bits
#pragma unroll
        for (int h = 1; h < CH; h <<= 1)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int e = 0; e < CH; ++e)
                    if ((e & h) == 0) {
                        const float a = v[r][e], b = v[r][e + h];
                        v[r][e] = a + b;
                        v[r][e + h] = a - b;
                    }
        // lane bits
        lane_stage_fma<0xB1>(v, pos & 1);    // lane ^ 1 (quad_perm [1,0,3,2])
        lane_stage_fma<0x4E>(v, pos & 2);    // lane ^ 2 (quad_perm [2,3,0,1])
        lane_stage_fma<0x141>(v, pos & 4);   // lane ^ 7 (row_half_mirror)
        lane_stage_fma<0x128>(v, pos & 8);   // lane ^ 8 (row_ror:8)
        lane_stage<16>(v, lane);             // (partners share position bits 0-3, hence the sign they carry)
        lane_stage<32>(v, lane);
        // r bits
#pragma unroll
        for (int h = 1; h < R; h <<= 1)
#pragma unroll
            for (int r = 0; r < R; ++r)
                if ((r & h) == 0) {
#pragma unroll
                    for (int e = 0; e < CH; ++e) {
                        const float a = v[r][e], b = v[r + h][e];
                        v[r][e] = a + b;
                        v[r + h][e] = a - b;
                    }
                }
        // wave bits: trade them for the low log2(W) bits of r through LDS
        if constexpr (W > 1) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                float* dst = exch + ((wave * R + r) * 64 + lane) * CH;
#pragma unroll
                for (int e = 0; e < CH; e += 4)
                    *reinterpret_cast<float4*>(dst + e) = make_float4(v[r][e], v[r][e + 1], v[r][e + 2], v[r][e + 3]);
            }
            __syncthreads();
            // slot j = r_hi*W + w2 now holds chunk g = w2*R + r_hi*W + wave
#pragma unroll
            for (int j = 0; j < R; ++j) {
                const int w2 = j % W, r_hi = j / W;
                const float* src = exch + ((w2 * R + r_hi * W + wave) * 64 + lane) * CH;
#pragma unroll
                for (int e = 0; e < CH; e += 4) {
                    const float4 t = *reinterpret_cast<const float4*>(src + e);
                    v[j][e] = t.x; v[j][e + 1] = t.y; v[j][e + 2] = t.z; v[j][e + 3] = t.w;
                }
            }
            exchanged = true;
#pragma unroll
            for (int h = 1; h < W; h <<= 1)
#pragma unroll
                for (int j = 0; j < R; ++j)
                    if ((j & h) == 0) {
#pragma unroll
                        for (int e = 0; e < CH; ++e) {
                            const float a = v[j][e], b = v[j + h][e];
                            v[j][e] = a + b;
                            v[j + h][e] = a - b;
                        }
                    }
        }
        // 1/sqrt(K), with the sign the lane stages left on this lane's values: (-1)^(set bits among position bits 0-3)
        const float c_n = (__builtin_popcount(pos & 15) & 1) ? -(float)(1.0 / sqrt((double)K)) : (float)(1.0 / sqrt((double)K));
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < CH; ++e) v[r][e] = v[r][e] * c_n;
    }

    if constexpr (BITS == 0) {
        // transform only (Eq. 3-4 by themselves, and the backward pass of Eq. 8): `codes` is the output
        // array and `code_offset` its element type
        static_assert(CH >= 2, "transform-only rows hold at least two elements per lane");
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int g = exchanged ? (r % W) * R + (r / W) * W + wave : wave * R + r;
            store_xr<CH>(codes, code_offset, row_off + (int64_t)(g * 64 + pos) * CH, v[r]);
        }
        return;
    }

    // per-token scale
    float gain, s_d;
    if constexpr (BITS == 8) {
        float m = 0.0f;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < CH; ++e) m = fmaxf(m, fabsf(v[r][e]));
        m = wave_max(m, few_rows);
        if constexpr (W > 1) {
            if (lane == 0) red_f[wave] = m;
            __syncthreads();
            m = red_f[0];
#pragma unroll
            for (int w = 1; w < W; ++w) m = fmaxf(m, red_f[w]);
        }
        gain = 127.0f / (m + rp.eps);
        s_d = m / 127.0f;
    } else {
        double s = 0.0;
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < CH; ++e) s += (double)fabsf(v[r][e]);
        s = wave_sum(s, few_rows);
        if constexpr (W > 1) {
            if (lane == 0) red_d[wave] = s;
            __syncthreads();
            s = red_d[0];
#pragma unroll
            for (int w = 1; w < W; ++w) s += red_d[w];
        }
        const float beta = (float)(s / (double)K);
        gain = kRoot7 / (beta + rp.eps);
        s_d = beta / kRoot7;
    }

    // codes: clamp, then add 1.5*2^23 so that the fp32 adder rounds to the nearest (even) integer and
    // leaves its two's complement in the low mantissa bits
    constexpr float lo = BITS == 8 ? -128.0f : -8.0f;
    constexpr float hi = BITS == 8 ? 127.0f : 7.0f;
    // bf6 records (INT4, 8-element chunks only; the launcher rejects the rest) are built from code + 8
    const bool bf6 = BITS == 4 && CH == 8 && code_offset == kCodesBf6;
    if (bf6) code_offset = 8;
    // stored byte = code + code_offset: folding the offset into the rounding constant costs nothing
    const float magic = kMagic + (float)code_offset;
    int isum = 0;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        uint32_t packed[(CH + 3) / 4];
#pragma unroll
        for (int p = 0; p < (CH + 3) / 4; ++p) packed[p] = 0;
#pragma unroll
        for (int e = 0; e < CH; ++e) {
            const float y = v[r][e] * gain;
            const float t = __builtin_amdgcn_fmed3f(y, lo, hi);
            const uint32_t bits = as_u(t + magic);
            isum += (int)bits;
            packed[e / 4] |= (bits & 0xFFu) << (8 * (e % 4));
        }
        int g;
        if (exchanged) {
            const int w2 = r % W, r_hi = r / W;
            g = w2 * R + r_hi * W + wave;
        } else {
            g = wave * R + r;
        }
        int8_t* dst = codes + row_off + (int64_t)(g * 64 + pos) * CH;
        if constexpr (CH == 8) {
            if (bf6) bf6_store_pair(codes, row, K, g * 64 + pos, bf6_pack4(packed[0]), bf6_pack4(packed[1]));
            else *reinterpret_cast<uint2*>(dst) = make_uint2(packed[0], packed[1]);
        } else if constexpr (CH == 4) {
            *reinterpret_cast<uint32_t*>(dst) = packed[0];
        } else if constexpr (CH == 2) {
            *reinterpret_cast<uint16_t*>(dst) = (uint16_t)packed[0];
        } else {
            *reinterpret_cast<uint8_t*>(dst) = (uint8_t)packed[0];
        }
    }
    isum = (int)((uint32_t)isum - (uint32_t)E * as_u(magic));  // remove the constant's bit pattern (mod 2^32)
    isum = wave_sum(isum, few_rows);
    if constexpr (W > 1) {
        if (lane == 0) red_i[wave] = isum;
        __syncthreads();
        isum = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) isum += red_i[w];
    }
    if (tid == 0) {
        s_dequant[row] = s_d;
        if (code_sum) code_sum[row] = isum;
    }
}

template <int LOG2K, int W, int BITS, bool BF16, bool HADAMARD>
__global__ __launch_bounds__(64 * W) void fwht_quant_kernel(const void* __restrict__ x, int8_t* __restrict__ codes,
                                                            float* __restrict__ s_dequant,
                                                            int32_t* __restrict__ code_sum, RowParams rp, int code_offset) {
    fwht_quant_body<LOG2K, W, BITS, BF16, HADAMARD>(blockIdx.x, threadIdx.x, x, codes, s_dequant, code_sum, rp,
                                                    code_offset);
}

template <int LOG2K, int W, int BITS, bool BF16, bool HADAMARD>
int launch_one(const void* x, int64_t T, int8_t* codes, float* s_dequant, int32_t* code_sum, RowParams rp,
               int code_offset, hipStream_t stream) {
    constexpr int K = 1 << LOG2K;
    const size_t lds = (HADAMARD && W > 1) ? sizeof(float) * K : 0;
    auto kern = fwht_quant_kernel<LOG2K, W, BITS, BF16, HADAMARD>;
    static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
    if (const int rc = allow_dynamic_lds(kern, lds, lds_allowed); rc != HBL_OK) return rc;
    launch_kernel("fwht_quant_kernel", kern, dim3((unsigned)T), dim3(64 * W), lds, stream, x, codes, s_dequant, code_sum, rp, code_offset);
    return after_launch();
}


// Plain BitLinear front end for K that is not a power of two (K % 128 == 0, K <= 16384): the same
// quantiser with the row held as up to 8 chunks of 8 elements per thread of a 256-thread workgroup.
// MAXC = chunk slots per thread (K <= 2048 * MAXC): the launcher picks the smallest that covers the row, so
// that short rows do not walk empty slots; every MAXC performs the same arithmetic in the same order.
template <int BITS, bool BF16, int MAXC = 8>
__device__ __forceinline__ void quant_generic_body(int64_t row, int tid, const void* __restrict__ x, int K,
                                                   int8_t* __restrict__ codes, float* __restrict__ s_dequant,
                                                   int32_t* __restrict__ code_sum, RowParams rp, int code_offset) {
    const int few_rows = rp.few_rows;
    __shared__ double red_d[4];
    __shared__ float red_f[4];
    __shared__ int red_i[4];
    const int lane = tid & 63, wave = tid >> 6;
    const int64_t row_off = row * K;
    const int nchunks = K / 8;
    float v[MAXC][8];
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = c * 256 + tid;
        if (ch < nchunks) {
            load_chunk<8, BF16>(x, row_off + (int64_t)ch * 8, v[c]);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[c][e] = 0.0f;
        }
    }
    if (rp.ln_gain) {   // uniform: RMS normalisation of the row (chunks past the row hold zeros)
        __shared__ double red_n[4];
        double ss = 0.0;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += (double)v[c][e] * (double)v[c][e];
        const float rn = rms_factor<4>(ss, red_n, lane, wave, K, rp.ln_eps, few_rows);
#pragma unroll
        for (int c = 0; c < MAXC; ++c) {
            const int ch = c * 256 + tid;
            if (ch < nchunks) {
                float gv[8];
                load_chunk<8, false>(rp.ln_gain, (int64_t)ch * 8, gv);
#pragma unroll
                for (int e = 0; e < 8; ++e) v[c][e] = (v[c][e] * rn) * gv[e];
            }
        }
    }
    float gain, s_d;
    if constexpr (BITS == 8) {
        float m = 0.0f;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) m = fmaxf(m, fabsf(v[c][e]));
        m = wave_max(m, few_rows);
        if (lane == 0) red_f[wave] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red_f[0], red_f[1]), fmaxf(red_f[2], red_f[3]));
        gain = 127.0f / (m + rp.eps);
        s_d = m / 127.0f;
    } else {
        double s = 0.0;
#pragma unroll
        for (int c = 0; c < MAXC; ++c)
#pragma unroll
            for (int e = 0; e < 8; ++e) s += (double)fabsf(v[c][e]);
        s = wave_sum(s, few_rows);
        if (lane == 0) red_d[wave] = s;
        __syncthreads();
        s = ((red_d[0] + red_d[1]) + red_d[2]) + red_d[3];
        const float beta = (float)(s / (double)K);
        gain = kRoot7 / (beta + rp.eps);
        s_d = beta / kRoot7;
    }
    constexpr float lo = BITS == 8 ? -128.0f : -8.0f;
    constexpr float hi = BITS == 8 ? 127.0f : 7.0f;
    const bool bf6 = BITS == 4 && code_offset == kCodesBf6;   // bf6 records are built from code + 8
    if (bf6) code_offset = 8;
    // stored byte = code + code_offset: folding the offset into the rounding constant costs nothing
    const float magic = kMagic + (float)code_offset;
    int isum = 0;
#pragma unroll
    for (int c = 0; c < MAXC; ++c) {
        const int ch = c * 256 + tid;
        if (ch < nchunks) {
            uint32_t packed[2] = {0u, 0u};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float t = __builtin_amdgcn_fmed3f(v[c][e] * gain, lo, hi);
                const uint32_t bits = as_u(t + magic);
                isum += (int)(bits - as_u(magic));
                packed[e / 4] |= (bits & 0xFFu) << (8 * (e % 4));
            }
            // K / 8 is a multiple of 16: the lanes of a quad are in or out of this branch together
            if (bf6) bf6_store_pair(codes, row, K, ch, bf6_pack4(packed[0]), bf6_pack4(packed[1]));
            else *reinterpret_cast<uint2*>(codes + row_off + (int64_t)ch * 8) = make_uint2(packed[0], packed[1]);
        }
    }
    isum = wave_sum(isum, few_rows);
    if (lane == 0) red_i[wave] = isum;
    __syncthreads();
    if (tid == 0) {
        s_dequant[row] = s_d;
        if (code_sum) code_sum[row] = red_i[0] + red_i[1] + red_i[2] + red_i[3];
    }
}

template <int BITS, bool BF16, int MAXC>
__global__ __launch_bounds__(256) void quant_generic_kernel(const void* __restrict__ x, int K,
                                                            int8_t* __restrict__ codes,
                                                            float* __restrict__ s_dequant,
                                                            int32_t* __restrict__ code_sum, RowParams rp, int code_offset) {
    quant_generic_body<BITS, BF16, MAXC>(blockIdx.x, threadIdx.x, x, K, codes, s_dequant, code_sum, rp, code_offset);
}

template <int BITS, bool BF16>
void launch_generic_slots(const void* x, int64_t T, int64_t K, RowParams rp, int8_t* codes, float* s_dequant,
                          int32_t* code_sum, int code_offset, hipStream_t stream) {
    const dim3 grid((unsigned)T), block(256);
    const int64_t per_thread = (K / 8 + 255) / 256;   // 8-element chunks per thread
#define HBL_GENERIC(MAXC)                                                                                     \
    launch_kernel("quant_generic_kernel", (quant_generic_kernel<BITS, BF16, MAXC>), grid, block, 0, stream, x, (int)K, codes, s_dequant, \
                       code_sum, rp, code_offset)
    if (per_thread <= 1) HBL_GENERIC(1);
    else if (per_thread <= 2) HBL_GENERIC(2);
    else if (per_thread <= 4) HBL_GENERIC(4);
    else HBL_GENERIC(8);
#undef HBL_GENERIC
}

int launch_generic(const void* x, int x_dtype, int64_t T, int64_t K, int bits, RowParams rp, int8_t* codes,
                   float* s_dequant, int32_t* code_sum, int code_offset, hipStream_t stream) {
    const bool bf = x_dtype == HBL_BF16;
    if (bits == 8) {
        if (bf) launch_generic_slots<8, true>(x, T, K, rp, codes, s_dequant, code_sum, code_offset, stream);
        else    launch_generic_slots<8, false>(x, T, K, rp, codes, s_dequant, code_sum, code_offset, stream);
    } else {
        if (bf) launch_generic_slots<4, true>(x, T, K, rp, codes, s_dequant, code_sum, code_offset, stream);
        else    launch_generic_slots<4, false>(x, T, K, rp, codes, s_dequant, code_sum, code_offset, stream);
    }
    return after_launch();
}


// ---------------------------------------------------------------------------------------------
// Large rows (K = 4096, 8192, 16384): every butterfly stage runs in registers.
//
// A thread holds 64 values = 16 float4 "chunks"; a chunk is 4 consecutive elements (index bits 0-1)
// and the chunk number j carries four more index bits.  Two or three register layouts, with the row exchanged through
// LDS between them (one float per element, 16-byte accesses, XOR-swizzled so that both sides are conflict
// free), and four stages between lanes in the middle:
//   layout A: j = index bits 2-5,   thread = bits 6..m-1   stages 0-5   (64 contiguous elements / thread)
//   K = 16384: index bits 6-9 are the low four bits of A's thread number: stages 6-9 run lane to lane (below)
//   K < 16384: layout B: j = index bits 6-9, thread = bits 2-5, 10.. stages 6-9, after an exchange of its own
//   layout C: j = index bits 10..   (+ finished low bits when m < 14)   stages 10..m-1
// Stage order stays ascending, so every value equals the one the reference order produces.
// In float4 units (q = index >> 2) every layout is q = q_t(thread) ^ q_j(j) with disjoint bit sets,
// and the swizzle q ^ ((q >> 4) & 15) is linear over xor: an LDS address is one xor of a per-thread
// base with a compile-time constant.
//
// Lane stages.  The butterfly on a lane bit is one instruction per element: v <- partner * c + v with the
// partner read through a DPP lane permutation and c = +1 where the bit is 0 (a + b) and -1 where it is 1
// (b - a): the product is exact and the sum rounds once, so the lower lane holds the reference's a + b and
// the upper lane the negative of its a - b.  Negation commutes with every later rounding, so a lane simply
// carries the sign (-1)^(number of its index bits 6-9 that are set); in layout C those bits belong to the
// thread number, all 64 values of a thread share the sign, the butterflies among them keep it, and it
// leaves through the factor the values are multiplied with anyway (1/sqrt(K) or the quantiser's gain).
// DPP offers xor 1, xor 2 (quad permutes), xor 7 (half-row mirror) and xor 8 (row rotation by 8) inside a row
// of 16 lanes, so the thread that takes segment t of layout A is lane t ^ (3 if bit 2 of t is set): flipping
// index bit 8 (bit 2 of t) then flips lane bits 0-2 together.
template <int LOG2K, int LAYOUT>
struct BigRowLayout {
    static constexpr int M = LOG2K;
    __host__ __device__ static constexpr uint32_t qj(int j) {
        if (LAYOUT == 0) return (uint32_t)j;
        if (LAYOUT == 1) return (uint32_t)j << 4;
        if (M == 14) return (uint32_t)j << 8;
        if (M == 13) return ((uint32_t)(j & 7) << 8) | (uint32_t)(j >> 3);
        return ((uint32_t)(j & 3) << 8) | (uint32_t)(j >> 2);   // M == 12
    }
    __device__ static uint32_t qt(uint32_t tid) {
        if (LAYOUT == 0) return tid << 4;
        if (LAYOUT == 1) return (tid & 15u) | ((tid >> 4) << 8);
        if (M == 14) return tid;
        if (M == 13) return tid << 1;
        return tid << 2;
    }
    // number of chunk bits that are unfinished index bits in this layout (stages to run on j)
    static constexpr int stages() { return LAYOUT < 2 ? 4 : M - 10; }
};
__host__ __device__ constexpr uint32_t swz16(uint32_t q) { return q ^ ((q >> 4) & 15u); }

// BF6OUT (INT4 only): instead of one byte per code, write the form the fp6 x fp4 GEMM reads - per 32
// consecutive features a 24-byte record of bf6 (e3m2) values, feature i at bits [6i, 6i+6), placed in the
// record image of code_records.h; every integer in [-8, 7] is exact in that format.
// NORM: compiled with the RMS-normalisation prologue (taken when rp.ln_gain is set).  A template switch
// rather than the run-time test alone: the prologue's presence changes the register allocation of the
// whole body, and the plain prefill path should not pay for it.
// One row's input as loaded, layout A: 64 contiguous elements per thread (8 or 16 16-byte loads).
template <bool BF16>
struct BigRowRaw {
    uint4 q[BF16 ? 8 : 16];
};
// Whether stages 6-9 run between lanes (one exchange through LDS) or in registers after an exchange of their
// own (two exchanges).  With the four waves of a K = 16384 row an exchange costs two workgroup barriers and the
// lane form is 5-6 % faster; the one or two waves of a K = 4096 / 8192 row exchange cheaply, and there the lane
// form measured 3 % / 7 % slower (a DPP multiply-add issues more slowly than an add).
template <int LOG2K>
constexpr bool kLaneStages = LOG2K >= 14;
// Segment of layout A (64 contiguous elements) that thread `tid` holds; its own inverse.
template <int LOG2K>
__device__ __forceinline__ uint32_t bigrow_segment(uint32_t tid) {
    return kLaneStages<LOG2K> ? tid ^ (((tid >> 2) & 1u) * 3u) : tid;
}
template <int LOG2K, bool BF16>
__device__ __forceinline__ void bigrow_load(const void* __restrict__ x, int64_t row, uint32_t tid, BigRowRaw<BF16>& raw) {
    constexpr int K = 1 << LOG2K;
    const int64_t first = row * (int64_t)K + bigrow_segment<LOG2K>(tid) * 64;
    const uint4* src = BF16 ? reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(x) + first)
                            : reinterpret_cast<const uint4*>(static_cast<const float*>(x) + first);
#pragma unroll
    for (int i = 0; i < (BF16 ? 8 : 16); ++i) raw.q[i] = src[i];
}

// `before_tail` is called once, by every thread, after the last exchange through LDS and ahead of the last
// butterfly stages, the row statistics and the quantiser: the place from which a caller that walks several
// rows starts the loads of its next row (few registers are live there besides the row itself).
struct NoPrefetch {
    __device__ void operator()() const {}
};
// ROWLOOP: the caller runs this body for one row after another, so the row buffer still has readers from
// the previous row until every thread has passed a barrier.
template <int LOG2K, int BITS, bool BF16, bool BF6OUT, bool NORM, bool ROWLOOP = false, typename BeforeTail = NoPrefetch>
__device__ __forceinline__ void fwht_quant_bigrow_body(int64_t row, uint32_t tid, const BigRowRaw<BF16>& raw,
                                                       int8_t* __restrict__ codes, float* __restrict__ s_dequant,
                                                       int32_t* __restrict__ code_sum, RowParams rp, int code_offset,
                                                       BeforeTail before_tail = BeforeTail{}) {
    constexpr int few_rows = ROWLOOP ? 0 : 1;   // the row loop is the throughput form
    constexpr int K = 1 << LOG2K;
    constexpr int NT = K / 64;
    constexpr int W = NT / 64;
    using LA = BigRowLayout<LOG2K, 0>;
    using LB = BigRowLayout<LOG2K, 1>;
    using LC = BigRowLayout<LOG2K, 2>;
    extern __shared__ __attribute__((aligned(16))) float row_lds[];   // K floats
    __shared__ double red_d[W];
    __shared__ float red_f[W];
    __shared__ int red_i[W];

    const int lane = tid & 63, wave = tid >> 6;
    const int64_t row_off = row * (int64_t)K;

    float v[16][4];
    if constexpr (BF16) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t w[4] = {raw.q[i].x, raw.q[i].y, raw.q[i].z, raw.q[i].w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                v[2 * i + h / 2][2 * (h % 2)] = as_f(w[h] << 16);
                v[2 * i + h / 2][2 * (h % 2) + 1] = as_f(w[h] & 0xFFFF0000u);
            }
        }
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            v[j][0] = as_f(raw.q[j].x); v[j][1] = as_f(raw.q[j].y); v[j][2] = as_f(raw.q[j].z); v[j][3] = as_f(raw.q[j].w);
        }
    }

    if (NORM && rp.ln_gain) {   // uniform: RMS normalisation ahead of the transform (layout A: elements tid*64 + 4j + e)
        __shared__ double red_n[W];
        double ss = 0.0;
#pragma unroll
        for (int j = 0; j < 16; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) ss += (double)v[j][e] * (double)v[j][e];
        const float rn = rms_factor<W>(ss, red_n, lane, wave, K, rp.ln_eps, few_rows);
        const float4* gsrc = reinterpret_cast<const float4*>(rp.ln_gain + bigrow_segment<LOG2K>(tid) * 64);
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float4 gq = gsrc[j];
            v[j][0] = (v[j][0] * rn) * gq.x;
            v[j][1] = (v[j][1] * rn) * gq.y;
            v[j][2] = (v[j][2] * rn) * gq.z;
            v[j][3] = (v[j][3] * rn) * gq.w;
        }
    }

    auto stages_e = [&]() {   // index bits 0, 1: inside a chunk
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float a0 = v[j][0] + v[j][1], a1 = v[j][0] - v[j][1];
            const float a2 = v[j][2] + v[j][3], a3 = v[j][2] - v[j][3];
            v[j][0] = a0 + a2; v[j][2] = a0 - a2;
            v[j][1] = a1 + a3; v[j][3] = a1 - a3;
        }
    };
    auto stages_j = [&](int nstages) {   // the low `nstages` bits of the chunk number, ascending
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            if (b >= nstages) break;
#pragma unroll
            for (int j = 0; j < 16; ++j)
                if (!(j & (1 << b))) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float a = v[j][e], c = v[j | (1 << b)][e];
                        v[j][e] = a + c;
                        v[j | (1 << b)][e] = a - c;
                    }
                }
        }
    };
    // index bits 6-9: between lanes (see above); CTRL = the DPP permutation that reaches the partner, `upper` =
    // this lane's index bit is set
    auto stage_lane = [&](auto ctrl_tag, bool upper) {
        constexpr int CTRL = decltype(ctrl_tag)::value;
        const float c = upper ? -1.0f : 1.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j) lane_butterfly4<CTRL>(v[j], c);
    };
    auto lds_write = [&](auto layout_tag, uint32_t thread) {
        using L = decltype(layout_tag);
        const uint32_t base = swz16(L::qt(thread)) << 4;   // bytes
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            constexpr uint32_t dummy = 0;
            (void)dummy;
            float4* dst = reinterpret_cast<float4*>(reinterpret_cast<char*>(row_lds) + (base ^ (swz16(L::qj(j)) << 4)));
            *dst = make_float4(v[j][0], v[j][1], v[j][2], v[j][3]);
        }
    };
    auto lds_read = [&](auto layout_tag) {
        using L = decltype(layout_tag);
        const uint32_t base = swz16(L::qt(tid)) << 4;
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const float4 t = *reinterpret_cast<const float4*>(reinterpret_cast<const char*>(row_lds) +
                                                              (base ^ (swz16(L::qj(j)) << 4)));
            v[j][0] = t.x; v[j][1] = t.y; v[j][2] = t.z; v[j][3] = t.w;
        }
    };

    stages_e();
    stages_j(4);              // index bits 2-5
    if constexpr (kLaneStages<LOG2K>) {
        const uint32_t seg = bigrow_segment<LOG2K>(tid);
        stage_lane(std::integral_constant<int, 0xB1>{}, seg & 1u);    // index bit 6: lane ^ 1 (quad_perm [1,0,3,2])
        stage_lane(std::integral_constant<int, 0x4E>{}, seg & 2u);    // index bit 7: lane ^ 2 (quad_perm [2,3,0,1])
        stage_lane(std::integral_constant<int, 0x141>{}, seg & 4u);   // index bit 8: lane ^ 7 (row_half_mirror)
        stage_lane(std::integral_constant<int, 0x128>{}, seg & 8u);   // index bit 9: lane ^ 8 (row_ror:8)
        if constexpr (ROWLOOP) __syncthreads();   // after this row's first stages: the wait is mostly over by then
        lds_write(LA{}, seg);
    } else {
        if constexpr (ROWLOOP) __syncthreads();
        lds_write(LA{}, tid);
        __syncthreads();
        lds_read(LB{});
        stages_j(4);              // index bits 6-9
        lds_write(LB{}, tid);     // to the very addresses this thread has just read: no barrier needed before it
    }
    __syncthreads();
    lds_read(LC{});
    before_tail();
    stages_j(LC::stages());   // index bits 10..m-1

    // c_n = (float)(1/sqrt(K)).  For even log2 K it is a power of two: scaling by it commutes exactly
    // with every later rounding (max, fp64 sum, the gain product), so it is applied to the row
    // statistics and folded into the gain instead of costing one multiply per element.
    const float c_n = (float)(1.0 / sqrt((double)K));
    // the sign this thread's values carry out of the lane stages: parity of index bits 6-9, which in layout C
    // are bits 4-7 of q_t(thread); it leaves with the factor below (exactly: a sign flip)
    const float c_s = (kLaneStages<LOG2K> && (__builtin_popcount((LC::qt(tid) >> 4) & 15u) & 1)) ? -c_n : c_n;
    constexpr bool FOLD = (LOG2K % 2) == 0 && BITS != 0;
    if constexpr (!FOLD) {
#pragma unroll
        for (int j = 0; j < 16; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) v[j][e] = v[j][e] * c_s;
    }

    if constexpr (BITS == 0) {
        // transform only: `codes` is the output array and `code_offset` its element type
#pragma unroll
        for (int j = 0; j < 16; ++j)
            store_xr<4>(codes, code_offset, row_off + (int64_t)((LC::qt(tid) ^ LC::qj(j)) << 2), v[j]);
        return;
    }

    float gain, s_d;
    if constexpr (BITS == 8) {
        float m = 0.0f;
#pragma unroll
        for (int j = 0; j < 16; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) m = fmaxf(m, fabsf(v[j][e]));
        m = wave_max(m, few_rows);
        if constexpr (W > 1) {
            if (lane == 0) red_f[wave] = m;
            __syncthreads();
            m = red_f[0];
#pragma unroll
            for (int w = 1; w < W; ++w) m = fmaxf(m, red_f[w]);
        }
        if constexpr (FOLD) m = m * c_n;
        gain = 127.0f / (m + rp.eps);
        s_d = m / 127.0f;
    } else {
        double s = 0.0;
#pragma unroll
        for (int j = 0; j < 16; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) s += (double)fabsf(v[j][e]);
        s = wave_sum(s, few_rows);
        if constexpr (W > 1) {
            if (lane == 0) red_d[wave] = s;
            __syncthreads();
            s = red_d[0];
#pragma unroll
            for (int w = 1; w < W; ++w) s += red_d[w];
        }
        if constexpr (FOLD) s = s * (double)c_n;
        const float beta = (float)(s / (double)K);
        gain = kRoot7 / (beta + rp.eps);
        s_d = beta / kRoot7;
    }

    constexpr float lo = BITS == 8 ? -128.0f : -8.0f;
    constexpr float hi = BITS == 8 ? 127.0f : 7.0f;
    static_assert(!BF6OUT || BITS == 4 || BITS == 0, "bf6 records carry INT4 codes only");
    const float magic = kMagic + (float)code_offset;   // byte forms: the low byte of t + magic is code + offset
    if constexpr (FOLD) gain = gain * c_s;   // (the statistics above took |v| and the positive c_n)
    int isum = 0;
    int8_t* out = codes + row_off + (LC::qt(tid) << 2);
    uint32_t* c24 = reinterpret_cast<uint32_t*>(row_lds);   // BF6OUT: 24 bits of bf6 per chunk, by chunk number
    const uint32_t cbase = LC::qt(tid);
    if constexpr (!BF6OUT) {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            uint32_t packed = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float t = __builtin_amdgcn_fmed3f(v[j][e] * gain, lo, hi);
                const uint32_t bits = as_u(t + magic);
                packed |= (bits & 0xFFu) << (8 * e);
            }
            if (code_sum) isum = __builtin_amdgcn_sdot4((int)packed, 0x01010101, isum, false);   // += the 4 stored bytes
            *reinterpret_cast<uint32_t*>(out + (LC::qj(j) << 2)) = packed;
        }
        isum -= 64 * code_offset;
    } else {
        // The codes as fp32 integers (round to nearest even by adding and removing 1.5 * 2^23, which
        // also turns -0 into +0), then the hardware's 32-value fp32 -> bf6 conversion: exact for
        // integers in [-8, 7].  Its result holds source pair i (one value from each operand) at bits
        // [12i, 12i+12), so with the even elements of 8 chunks in one operand and the odd ones in the
        // other, chunk c of the 8 lands in order at bits [24c, 24c+24) of the six result dwords.
        typedef float v16f __attribute__((ext_vector_type(16)));
        typedef uint32_t v6u __attribute__((ext_vector_type(6)));
        float fsum = 0.0f;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            v16f ev, od;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                float q[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    q[e] = (__builtin_amdgcn_fmed3f(v[8 * half + jj][e] * gain, lo, hi) + kMagic) - kMagic;
                ev[2 * jj] = q[0]; od[2 * jj] = q[1];
                ev[2 * jj + 1] = q[2]; od[2 * jj + 1] = q[3];
            }
            if (code_sum) {   // uniform, and off on the forward path: small integers, exact in any order
#pragma unroll
                for (int i = 0; i < 16; ++i) fsum += ev[i] + od[i];
            }
            const v6u r = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(ev, od, 1.0f);
            // one dword per chunk into LDS by chunk number; bits 24-31 of it are not meaningful
            const uint32_t piece[8] = {r[0], __builtin_amdgcn_alignbit(r[1], r[0], 24),
                                       __builtin_amdgcn_alignbit(r[2], r[1], 16), r[2] >> 8,
                                       r[3], __builtin_amdgcn_alignbit(r[4], r[3], 24),
                                       __builtin_amdgcn_alignbit(r[5], r[4], 16), r[5] >> 8};
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) c24[cbase ^ LC::qj(8 * half + jj)] = piece[jj];
        }
        isum = (int)fsum;
        // Regroup through LDS.  Eight consecutive chunks (32 features, 24 bytes: one record) become six dwords,
        // stored as the record's 16-byte and 8-byte piece by every lane (56 fewer vector instructions per row than
        // the form below, whose even and odd lanes store different pieces: 2-6 % faster at K <= 8192; at K = 16384
        // with fp32 rows 5 % faster, and it needs no spill there).  K = 16384 with bf16 rows keeps four chunks (16
        // features, 12 bytes) per lane and step: there the record form measured 8 % slower (0.125 against 0.116 ms
        // for 8192 rows) although it executes fewer instructions.
        __syncthreads();
        if constexpr (LOG2K < 14 || !BF16) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t rec = tid + NT * i;
                const uint4 c = *reinterpret_cast<const uint4*>(c24 + 8 * rec);
                const uint4 e = *reinterpret_cast<const uint4*>(c24 + 8 * rec + 4);
                store_code_record(codes, row, K, (int)rec,
                                  __builtin_amdgcn_perm(c.y, c.x, 0x04020100u),    // x0 x1 x2 y0
                                  __builtin_amdgcn_perm(c.z, c.y, 0x05040201u),    // y1 y2 z0 z1
                                  __builtin_amdgcn_perm(c.w, c.z, 0x06050402u),    // z2 w0 w1 w2
                                  __builtin_amdgcn_perm(e.y, e.x, 0x04020100u),
                                  __builtin_amdgcn_perm(e.z, e.y, 0x05040201u),
                                  __builtin_amdgcn_perm(e.w, e.z, 0x06050402u));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t quad = tid + NT * i;
                const uint4 c = *reinterpret_cast<const uint4*>(c24 + 4 * quad);
                store_code_quad(codes, row, K, (int)quad,
                                __builtin_amdgcn_perm(c.y, c.x, 0x04020100u),
                                __builtin_amdgcn_perm(c.z, c.y, 0x05040201u),
                                __builtin_amdgcn_perm(c.w, c.z, 0x06050402u));
            }
        }
    }
    if (code_sum) {   // uniform: the fp6 x fp4 GEMM needs no code sum
        isum = wave_sum(isum, few_rows);
        if constexpr (W > 1) {
            if (lane == 0) red_i[wave] = isum;
            __syncthreads();
            isum = 0;
#pragma unroll
            for (int w = 0; w < W; ++w) isum += red_i[w];
        }
        if (tid == 0) code_sum[row] = isum;
    }
    if (tid == 0) s_dequant[row] = s_d;
}

// Each workgroup walks rows blockIdx.x, blockIdx.x + gridDim.x, ...; the grid is sized to what the chip holds
// at once (the LDS row buffer allows only a few workgroups per CU), and the next row's loads are issued
// under the tail of the current row's arithmetic so that their latency is not exposed once per row.  The
// compiler also moves the ~100 per-thread LDS and global address computations out of the row loop and keeps
// them in registers (about 200 VGPRs in all): measured 7-20 % faster than recomputing them per row, and the
// LDS row buffer limits the workgroups per CU before the registers do.
// FEW: at most 64 rows - one row per workgroup and the short-latency reductions.
template <int LOG2K, int BITS, bool BF16, bool BF6OUT, bool NORM, bool FEW>
__global__ __launch_bounds__((1 << LOG2K) / 64, 2) void fwht_quant_bigrow_kernel(
    const void* __restrict__ x, int64_t T, int8_t* __restrict__ codes, float* __restrict__ s_dequant,
    int32_t* __restrict__ code_sum, RowParams rp, int code_offset) {
    int64_t row = blockIdx.x;
    BigRowRaw<BF16> cur;
    bigrow_load<LOG2K, BF16>(x, row, threadIdx.x, cur);
    if constexpr (BITS == 0 || FEW) {   // (transform only: the row loop would cost it registers it lacks)
        fwht_quant_bigrow_body<LOG2K, BITS, BF16, BF6OUT, NORM>(row, threadIdx.x, cur, codes, s_dequant, code_sum, rp,
                                                                code_offset);
        return;
    }
    for (;;) {
        const int64_t next = row + gridDim.x;
        BigRowRaw<BF16> ahead;
        const uint32_t tid = threadIdx.x;
        fwht_quant_bigrow_body<LOG2K, BITS, BF16, BF6OUT, NORM, true>(
            row, tid, cur, codes, s_dequant, code_sum, rp, code_offset,
            [&]() { if (next < T) bigrow_load<LOG2K, BF16>(x, next, tid, ahead); });
        if (next >= T) break;
        cur = ahead;
        row = next;
    }
}

template <int LOG2K, int BITS, bool BF16, bool BF6OUT, bool NORM, bool FEW>
int launch_bigrow_form(const void* x, int64_t T, int8_t* codes, float* s_dequant, int32_t* code_sum, RowParams rp,
                       int code_offset, hipStream_t stream);

template <int LOG2K, int BITS, bool BF16, bool BF6OUT = false>
int launch_bigrow(const void* x, int64_t T, int8_t* codes, float* s_dequant, int32_t* code_sum, RowParams rp,
                  int code_offset, hipStream_t stream) {
    if constexpr (BITS != 0) {
        const bool norm = rp.ln_gain != nullptr;
        if (rp.few_rows)
            return norm ? launch_bigrow_form<LOG2K, BITS, BF16, BF6OUT, true, true>(x, T, codes, s_dequant, code_sum, rp,
                                                                                    code_offset, stream)
                        : launch_bigrow_form<LOG2K, BITS, BF16, BF6OUT, false, true>(x, T, codes, s_dequant, code_sum, rp,
                                                                                     code_offset, stream);
        if (norm)
            return launch_bigrow_form<LOG2K, BITS, BF16, BF6OUT, true, false>(x, T, codes, s_dequant, code_sum, rp,
                                                                              code_offset, stream);
    }
    return launch_bigrow_form<LOG2K, BITS, BF16, BF6OUT, false, false>(x, T, codes, s_dequant, code_sum, rp, code_offset,
                                                                       stream);
}

template <int LOG2K, int BITS, bool BF16, bool BF6OUT, bool NORM, bool FEW>
int launch_bigrow_form(const void* x, int64_t T, int8_t* codes, float* s_dequant, int32_t* code_sum, RowParams rp,
                       int code_offset, hipStream_t stream) {
    constexpr int K = 1 << LOG2K;
    constexpr size_t lds = sizeof(float) * K;
    auto kern = fwht_quant_bigrow_kernel<LOG2K, BITS, BF16, BF6OUT, NORM, FEW>;
    static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
    if (const int rc = allow_dynamic_lds(kern, lds, lds_allowed); rc != HBL_OK) return rc;
    int grid = (int)T;   // one row per workgroup ...
    if constexpr (BITS != 0 && !FEW) {   // ... or as many workgroups as the chip holds at once, walking the rows
        static std::atomic<int> resident[64];
        if (const int rc = resident_workgroups(kern, K / 64, lds, resident, &grid); rc != HBL_OK) return rc;
        if ((int64_t)grid > T) grid = (int)T;
    }
    launch_kernel("fwht_quant_bigrow_kernel", kern, dim3((unsigned)grid), dim3(K / 64), lds, stream, x, T, codes, s_dequant, code_sum, rp,
                       code_offset);
    return after_launch();
}

template <int LOG2K>
int dispatch_bigrow(const void* x, int x_dtype, int64_t T, int bits, RowParams rp, int8_t* codes, float* s_dequant,
                    int32_t* code_sum, int code_offset, hipStream_t stream) {
    const bool bf = x_dtype == HBL_BF16;
    if (code_offset == kCodesBf6)
        return bf ? launch_bigrow<LOG2K, 4, true, true>(x, T, codes, s_dequant, code_sum, rp, 8, stream)
                  : launch_bigrow<LOG2K, 4, false, true>(x, T, codes, s_dequant, code_sum, rp, 8, stream);
    if (bits == 8) return bf ? launch_bigrow<LOG2K, 8, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
                             : launch_bigrow<LOG2K, 8, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
    return bf ? launch_bigrow<LOG2K, 4, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
              : launch_bigrow<LOG2K, 4, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
}

// WITH_H = false: rows of 4096 and more, whose transform belongs to the all-register kernel above - only the
// plain quantiser is compiled from this body for them.
template <int LOG2K, int W, bool WITH_H = true>
int dispatch(const void* x, int x_dtype, int64_t T, int bits, RowParams rp, bool hadamard, int8_t* codes,
             float* s_dequant, int32_t* code_sum, int code_offset, hipStream_t stream) {
    const bool bf = x_dtype == HBL_BF16;
    if constexpr (!WITH_H) {
        if (hadamard) return HBL_E_SHAPE;
    } else if (hadamard) {
        if (bits == 8) return bf ? launch_one<LOG2K, W, 8, true, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
                                 : launch_one<LOG2K, W, 8, false, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
        return bf ? launch_one<LOG2K, W, 4, true, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
                  : launch_one<LOG2K, W, 4, false, true>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
    }
    if (bits == 8) return bf ? launch_one<LOG2K, W, 8, true, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
                             : launch_one<LOG2K, W, 8, false, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
    return bf ? launch_one<LOG2K, W, 4, true, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream)
              : launch_one<LOG2K, W, 4, false, false>(x, T, codes, s_dequant, code_sum, rp, code_offset, stream);
}

// Rows of several projections in one grid (small-batch path): workgroup -> (problem, row), then the
// body the stand-alone launch would run for that problem.  A body that needs fewer than 256 threads
// runs on the first waves only; the other waves end at once, and a workgroup barrier waits only for
// waves that have not ended.
template <int BITS, bool BF16>
__global__ __launch_bounds__(256) void quant_grouped_kernel(const QuantGroupArgs a) {
    const QuantProblem p = a.p[group_index_of(a.row_begin, a.n, (int)blockIdx.x)];
    const int64_t row = (int)blockIdx.x - p.row_begin;
    const int tid = threadIdx.x;
    if (!p.hadamard) {
        quant_generic_body<BITS, BF16>(row, tid, p.x, p.K, p.codes, p.s_dequant, p.code_sum, RowParams{a.eps, p.ln_gain, p.ln_eps, 1}, p.code_offset);
        return;
    }
#define HBL_SMALL_ROW(L2K)                                                                                    \
    case 1 << L2K:                                                                                            \
        if (tid < 64)                                                                                         \
            fwht_quant_body<L2K, 1, BITS, BF16, true>(row, tid, p.x, p.codes, p.s_dequant, p.code_sum, RowParams{a.eps, p.ln_gain, p.ln_eps, 1}, \
                                                      p.code_offset);                                         \
        return;
#define HBL_BIG_ROW(L2K)                                                                                      \
    case 1 << L2K:                                                                                            \
        if (tid < (1 << L2K) / 64) {                                                                          \
            BigRowRaw<BF16> raw;                                                                              \
            bigrow_load<L2K, BF16>(p.x, row, tid, raw);                                                       \
            const RowParams rp{a.eps, p.ln_gain, p.ln_eps, 1};                                                \
            if constexpr (BITS == 4) {                                                                        \
                if (p.code_offset == kCodesBf6) {                                                             \
                    fwht_quant_bigrow_body<L2K, 4, BF16, true, true>(row, tid, raw, p.codes, p.s_dequant, p.code_sum, rp, 8); \
                    return;                                                                                   \
                }                                                                                             \
            }                                                                                                 \
            fwht_quant_bigrow_body<L2K, BITS, BF16, false, true>(row, tid, raw, p.codes, p.s_dequant, p.code_sum, rp, \
                                                                 p.code_offset);                              \
        }                                                                                                     \
        return;
    switch (p.K) {
        HBL_SMALL_ROW(7)
        HBL_SMALL_ROW(8)
        HBL_SMALL_ROW(9)
        HBL_SMALL_ROW(10)
        HBL_SMALL_ROW(11)
        HBL_BIG_ROW(12)
        HBL_BIG_ROW(13)
        HBL_BIG_ROW(14)
        default: return;
    }
#undef HBL_SMALL_ROW
#undef HBL_BIG_ROW
}

}  // namespace

int launch_quant_grouped(const QuantGroupArgs& args, int bits, int x_dtype, hipStream_t stream) {
    int rows = 0;
    size_t lds = 0;
    for (int i = 0; i < args.n; ++i) {
        rows += args.p[i].T;
        if (args.p[i].hadamard && args.p[i].K >= 4096 && sizeof(float) * (size_t)args.p[i].K > lds)
            lds = sizeof(float) * (size_t)args.p[i].K;
    }
    if (rows == 0) return HBL_OK;
    const bool bf = x_dtype == HBL_BF16;
    auto launch = [&](auto kern) -> int {
        static std::atomic<uint64_t> lds_allowed{0};   // per instantiation: devices already set up
        if (const int rc = allow_dynamic_lds(kern, 64 * 1024, lds_allowed); rc != HBL_OK) return rc;
        launch_kernel("quant_grouped_kernel", kern, dim3((unsigned)rows), dim3(256), lds, stream, args);
        return after_launch();
    };
    if (bits == 8) return bf ? launch(quant_grouped_kernel<8, true>) : launch(quant_grouped_kernel<8, false>);
    return bf ? launch(quant_grouped_kernel<4, true>) : launch(quant_grouped_kernel<4, false>);
}

int launch_fwht_only(const void* x, int x_dtype, int64_t T, int64_t K, void* out, int out_dtype, hipStream_t stream) {
    if (T == 0) return HBL_OK;
    const bool bf = x_dtype == HBL_BF16;
    int8_t* o = static_cast<int8_t*>(out);
#define HBL_SMALL(L2K)                                                                                           \
    case 1 << L2K:                                                                                               \
        return bf ? launch_one<L2K, 1, 0, true, true>(x, T, o, nullptr, nullptr, RowParams{0.0f, nullptr, 0.0f, 0}, out_dtype, stream)        \
                  : launch_one<L2K, 1, 0, false, true>(x, T, o, nullptr, nullptr, RowParams{0.0f, nullptr, 0.0f, 0}, out_dtype, stream);
#define HBL_BIG(L2K)                                                                                             \
    case 1 << L2K:                                                                                               \
        return bf ? launch_bigrow<L2K, 0, true, false>(x, T, o, nullptr, nullptr, RowParams{0.0f, nullptr, 0.0f, 0}, out_dtype, stream)       \
                  : launch_bigrow<L2K, 0, false, false>(x, T, o, nullptr, nullptr, RowParams{0.0f, nullptr, 0.0f, 0}, out_dtype, stream);
    switch (K) {
        HBL_SMALL(7)
        HBL_SMALL(8)
        HBL_SMALL(9)
        HBL_SMALL(10)
        HBL_SMALL(11)
        HBL_BIG(12)
        HBL_BIG(13)
        HBL_BIG(14)
        default: return HBL_E_SHAPE;
    }
#undef HBL_SMALL
#undef HBL_BIG
}

int launch_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, int bits, float eps, bool hadamard,
                      int8_t* codes, float* s_dequant, int32_t* code_sum, int code_offset, hipStream_t stream,
                      const float* ln_gain, float ln_eps) {
    if (T == 0) return HBL_OK;
    const RowParams rp = {eps, ln_gain, ln_eps, T <= 64 ? 1 : 0};
    if (code_offset == kCodesBf6 && (bits != 4 || K < 512)) return HBL_E_SHAPE;   // records need 8-element chunks
    if (!hadamard && !is_pow2(K)) return launch_generic(x, x_dtype, T, K, bits, rp, codes, s_dequant, code_sum, code_offset, stream);
    if (hadamard) {
        if (K == 4096) return dispatch_bigrow<12>(x, x_dtype, T, bits, rp, codes, s_dequant, code_sum, code_offset, stream);
        if (K == 8192) return dispatch_bigrow<13>(x, x_dtype, T, bits, rp, codes, s_dequant, code_sum, code_offset, stream);
        if (K == 16384) return dispatch_bigrow<14>(x, x_dtype, T, bits, rp, codes, s_dequant, code_sum, code_offset, stream);
    }
    switch (K) {
        case 128:   return dispatch<7, 1>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 256:   return dispatch<8, 1>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 512:   return dispatch<9, 1>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 1024:  return dispatch<10, 1>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 2048:  return dispatch<11, 1>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 4096:  return dispatch<12, 2, false>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 8192:  return dispatch<13, 4, false>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        case 16384: return dispatch<14, 4, false>(x, x_dtype, T, bits, rp, hadamard, codes, s_dequant, code_sum, code_offset, stream);
        default:    return HBL_E_SHAPE;
    }
}

}  // namespace hbl
