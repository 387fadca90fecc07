// Transport format of INT4 activation codes between the quantiser launch and the fp6 x fp4 GEMM launch
// (HBL_CODES_BF6): 6 bits per code, no padding - 0.75 byte per feature in HBM.
//
// A code q in [-8, 7] travels as a 6-bit float (e3m2, "bf6"; every such integer is exact).  The 32 codes of
// features [32m, 32m+32) of a token form a 192-bit record, feature i at bits [6i, 6i+6): one lane's B operand
// of v_mfma_f32_32x32x64_f8f6f4.  The buffer is an image of what the GEMM holds in LDS, so that its
// global->LDS copies are plain contiguous 1 KiB pieces:
//   tokens in panels of 128, features in blocks of 128: block (P, kb) at ((P * K/128) + kb) * 12288 bytes holds
//   128 token rows of 96 bytes (4 records);
//   inside a row, the two records of K-step s (64 features; lane half h = 0, 1 reads record 2s + h) occupy the
//   three 16-byte chunks 3s, 3s+1, 3s+2: bits 0..127 of record 2s+h in chunk 3s + 2h, bits 128..191 in half h
//   of chunk 3s + 1 - every operand is one aligned 16-byte and one aligned 8-byte LDS read;
//   row r stores chunk c at slot c ^ ((r >> 3) & 1) and the two halves of chunk 3s+1 swapped when (r >> 4) & 1:
//   with 96-byte rows (24 banks) that makes the 16-byte reads of 16 consecutive rows and the 8-byte reads of 32
//   consecutive rows hit every LDS bank once.
// Rows of the last panel beyond T exist in the buffer and hold whatever was there: every bf6 bit pattern is a
// finite number and the GEMM never stores a row beyond T.
#pragma once

#include <stdint.h>

namespace hbl {

constexpr int kPanelTokens = 128;           // token rows per block
constexpr int kRecordRowBytes = 96;         // one token's 128 features
constexpr int kRecordBlockBytes = kPanelTokens * kRecordRowBytes;   // 12288

// bytes of the record image of [T, K] codes (whole panels)
inline size_t code_record_bytes(int64_t T, int64_t K) {
    return (size_t)((T + kPanelTokens - 1) / kPanelTokens) * (size_t)(K / 128) * kRecordBlockBytes;
}

#if defined(__HIPCC__)
// Byte offsets, inside a token's 96-byte row, of the pieces of the record that holds features 64s + 32h + 0..31
// of the row's 128: its bits 0..127 (16 bytes) and its bits 128..191 (8 bytes).  r = token index mod 128.
__device__ __forceinline__ int record_lo_offset(int r, int s, int h) { return ((3 * s + 2 * h) ^ ((r >> 3) & 1)) << 4; }
__device__ __forceinline__ int record_hi_offset(int r, int s, int h) {
    return (((3 * s + 1) ^ ((r >> 3) & 1)) << 4) + ((h ^ ((r >> 4) & 1)) << 3);
}

// Store the 16 codes of features [16*quad, 16*quad + 16) of token t, given as 96 bits d0 | d1 << 32 | d2 << 64
// (feature 16*quad + i at bits [6i, 6i+6)), into the record image of a [*, K] code buffer.
__device__ __forceinline__ void store_code_quad(int8_t* codes, int64_t t, int K, int quad, uint32_t d0, uint32_t d1,
                                                uint32_t d2) {
    const int r = (int)(t & (kPanelTokens - 1));
    const int kb = quad >> 3, s = (quad >> 2) & 1, h = (quad >> 1) & 1;
    char* row = reinterpret_cast<char*>(codes) +
                ((size_t)(t >> 7) * (size_t)(K >> 7) + (size_t)kb) * kRecordBlockBytes + r * kRecordRowBytes;
    char* lo = row + record_lo_offset(r, s, h);
    if ((quad & 1) == 0) {   // bits 0..95 of the record
        *reinterpret_cast<uint2*>(lo) = make_uint2(d0, d1);
        *reinterpret_cast<uint32_t*>(lo + 8) = d2;
    } else {                 // bits 96..127, then bits 128..191
        *reinterpret_cast<uint32_t*>(lo + 12) = d0;
        *reinterpret_cast<uint2*>(row + record_hi_offset(r, s, h)) = make_uint2(d1, d2);
    }
}

// Store the 32 codes of features [32*rec, 32*rec + 32) of token t - a whole record, given as six dwords (feature
// 32*rec + i at bits [6i, 6i+6)) - as its 16-byte and its 8-byte piece.  The row address is uniform over a
// workgroup that works on one token and the rest is a 32-bit per-lane offset.
__device__ __forceinline__ void store_code_record(int8_t* codes, int64_t t, int K, int rec, uint32_t d0, uint32_t d1,
                                                  uint32_t d2, uint32_t d3, uint32_t d4, uint32_t d5) {
    const int r = (int)(t & (kPanelTokens - 1));
    const int kb = rec >> 2, s = (rec >> 1) & 1, h = rec & 1;
    char* row = reinterpret_cast<char*>(codes) + (size_t)(t >> 7) * (size_t)(K >> 7) * kRecordBlockBytes + r * kRecordRowBytes;
    const uint32_t blk = (uint32_t)kb * kRecordBlockBytes;
    *reinterpret_cast<uint4*>(row + (blk + (uint32_t)record_lo_offset(r, s, h))) = make_uint4(d0, d1, d2, d3);
    *reinterpret_cast<uint2*>(row + (blk + (uint32_t)record_hi_offset(r, s, h))) = make_uint2(d4, d5);
}
#endif

}  // namespace hbl
