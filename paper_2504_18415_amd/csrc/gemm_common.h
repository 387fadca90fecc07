// Pieces shared by the GEMM translation units (int8 path and fp6 x fp4 path): argument block,
// global->LDS copy, pipeline barrier, dequantising epilogue.
#pragma once

#include "hbl_internal.h"

namespace hbl {
namespace gemm {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int kBK = 128;  // features per pipeline stage = one packed weight tile

__device__ __forceinline__ uint32_t as_u(float f) { return __builtin_bit_cast(uint32_t, f); }

// Wait until at most N of this wave's vector-memory loads are still in flight, then workgroup barrier.
// Written as one asm block: __syncthreads() carries a release fence that the compiler lowers to
// vmcnt(0), which would drain the whole global->LDS pipeline at every stage.  The "memory" clobber
// keeps every load / store on its side of the barrier.
// lgkmcnt(0): this wave's own LDS reads of the buffer about to be recycled have returned.
template <int N>
__device__ __forceinline__ void wait_loads_then_barrier() {
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// One 16-byte-per-lane global -> LDS copy: lane l's 16 bytes at (base + voff) land at LDS byte
// lds_addr + 16*l.  Written in asm so that the address is exactly "SGPR pair + 32-bit VGPR offset"
// (no per-copy vector address arithmetic) and the copy stays where the source puts it.
__device__ __forceinline__ void lds_dma16(uint32_t lds_addr, const void* base, uint32_t voff) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(base)
                 : "memory", "m0");
}

// Output rows leave with the non-temporal hint: y is written once and never read by the kernel, and keeping it
// out of the way of the operand panels in L2 measured 3.5 % faster at N = 32768 (537 MB of output), 3 % at
// N = K = 4096, and no different at N = 12288 and on W_down.
__device__ __forceinline__ void store_y16(uint16_t* dst, uint4 val) {
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store((u32x4){val.x, val.y, val.z, val.w}, reinterpret_cast<u32x4*>(dst));
}

struct GemmArgs {
    const int8_t* codes;      // [T, K]
    const uint32_t* packed;   // tiles [N/32][K/128][64 lanes][4 dwords], sign / magnitude pairs
    const float* s_dequant;   // [T]
    const int32_t* w_row_sum; // [N] sum_k c[o][k]
    int code_offset;          // stored code byte = q + code_offset
    const float* w_scales;    // [groups]
    uint16_t* y;              // [T, N] bf16
    int32_t* acc_out;         // [T, N] (RAW only)
    int T, K, N;
    int rows_per_group;
    int tiles_n, tiles_t;
    // split-K (small T only): workgroup (tile, ks) covers K-blocks [ks*nkb/split_k, (ks+1)*nkb/split_k)
    // and writes its int32 partial tile to partial[ks][T][N]; splitk_reduce_kernel finishes the job
    int split_k;
    int32_t* partial;
};

// Second launch of a split-K GEMM (ternary_gemm.hip): adds the split_k int32 partial tiles and dequantises.
int launch_splitk_reduce(const GemmArgs& a, hipStream_t stream);

// Packed weights (ternary_setup.hip): sign / magnitude bit pairs, 16 weights per dword, placed so that two
// AND and one shift give fp4 operands.  For the int8 matrix cores the same dword is expanded into four
// registers of four signed bytes each, features in natural order:
//   (p >> {0, 1, 4, 5}) & 0x05050505 puts four weights' (magnitude, sign) bits into bits 0 and 2 of four bytes,
//   one byte-permute look-up turns the byte values {0, 1, 5} into {0, +1, -1}, and two more byte permutes per
//   register pair interleave the even- and odd-numbered weights.
__device__ __forceinline__ uint32_t weight_pairs(uint32_t p, int which) {   // which: 0 = b even, 1 = a even, 2 = b odd, 3 = a odd
    const int sh = which == 0 ? 0 : which == 1 ? 1 : which == 2 ? 4 : 5;
    return (p >> sh) & 0x05050505u;
}
__device__ __forceinline__ uint32_t weight_bytes(uint32_t pairs) {          // {0, 1, 5} -> {0x00, 0x01, 0xFF} per byte
    return __builtin_amdgcn_perm(0x0000FF00u, 0x00000100u, pairs);
}
__device__ __forceinline__ uint32_t weight_interleave(uint32_t odd, uint32_t even, int upper) {
    return __builtin_amdgcn_perm(odd, even, upper ? 0x07030602u : 0x05010400u);
}
// The four int8 operand registers of one packed dword (features 16d + 0..15 of the dword's sixteen).
__device__ __forceinline__ v4i expand_weights_i8(uint32_t p) {
    const uint32_t b_even = weight_bytes(weight_pairs(p, 0)), a_even = weight_bytes(weight_pairs(p, 1));
    const uint32_t b_odd = weight_bytes(weight_pairs(p, 2)), a_odd = weight_bytes(weight_pairs(p, 3));
    return v4i{(int)weight_interleave(a_odd, a_even, 0), (int)weight_interleave(a_odd, a_even, 1),
               (int)weight_interleave(b_odd, b_even, 0), (int)weight_interleave(b_odd, b_even, 1)};
}
// 16-byte chunk of a token's 128-byte code row that holds the features packed dword j of a weight tile covers
// for lane half h: features 64 (j >> 1) + 32 h + 16 (j & 1) + 0..15.
__device__ __forceinline__ int code_chunk_of_dword(int j, int h) { return 4 * (j >> 1) + 2 * h + (j & 1); }

// Outer factors of Eq. 1 and Eq. 5/6 on four consecutive output features of one token:
// y = bf16(((float)(acc - corr) * s_d) * alpha), corr = code_offset * sum_k c: the weights are signed, so only
// an offset on the stored codes (INT4 codes travel as q + 8 on this path) leaves a term to remove, exactly,
// in int32.  (ws = the four features' sum_k c, already loaded; ignored when code_offset == 0)
__device__ __forceinline__ uint2 dequant_quad_sums(v4i acc, float sd, float alpha, int code_offset, v4i ws) {
    v4i corr = {0, 0, 0, 0};
    if (code_offset != 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) corr[r] = code_offset * ws[r];
    }
    float v[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) v[r] = ((float)(acc[r] - corr[r]) * sd) * alpha;
    // v_cvt_pk_bf16_f32: round to nearest even, two values per instruction
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const bf16x2 lo = __builtin_convertvector((f32x2){v[0], v[1]}, bf16x2);
    const bf16x2 hi = __builtin_convertvector((f32x2){v[2], v[3]}, bf16x2);
    return make_uint2(__builtin_bit_cast(uint32_t, lo), __builtin_bit_cast(uint32_t, hi));
}
__device__ __forceinline__ uint2 dequant_quad(v4i acc, float sd, float alpha, int code_offset,
                                              const int32_t* w_row_sum) {
    v4i ws = {0, 0, 0, 0};
    if (code_offset != 0) ws = *reinterpret_cast<const v4i*>(w_row_sum);
    return dequant_quad_sums(acc, sd, alpha, code_offset, ws);
}

// WAVES_N x WAVES_T waves; each wave owns TN x TT MFMA tiles (32 features x 32 tokens each).
// LDS stage = [BT tokens x 128 B codes, XOR-swizzled][BN/32 packed weight tiles x 1 KiB].

}  // namespace gemm
}  // namespace hbl
