// Internal declarations shared by the HIP translation units of libhbitlinear.
// Nothing here is part of the public ABI (see include/hbitlinear.h).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

#include "code_records.h"
#include "hbitlinear.h"

namespace hbl {

// Records a failed HIP call for hbl_last_hip_error() and yields HBL_E_HIP.
int note_hip_error(hipError_t e);

// Per-launch kernel timing (hbl_trace_begin / hbl_trace_end): while a trace is open on the calling thread every
// kernel launch of the library goes out with a start / stop event pair of its own, which the runtime fills with
// the dispatch's own device timestamps (no marker packets between the kernels, so the launches overlap their
// dispatch with the previous kernel exactly as untraced launches do).
struct LaunchTrace {
    hipEvent_t* start;
    hipEvent_t* stop;
    const char** names;
    int capacity;
    int count;      // launches seen since hbl_trace_begin (may exceed capacity: the excess is not timed)
};
LaunchTrace* current_trace();   // the calling thread's open trace, or nullptr

template <typename... KArgs, typename... Args>
inline void launch_kernel(const char* name, void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds,
                          hipStream_t stream, Args&&... args) {
    LaunchTrace* tr = current_trace();
    if (tr != nullptr) {
        const int i = tr->count++;
        if (i < tr->capacity) {
            tr->names[i] = name;
            hipExtLaunchKernelGGL(kern, grid, block, (uint32_t)lds, stream, tr->start[i], tr->stop[i], 0,
                                  static_cast<KArgs>(args)...);
            return;
        }
    }
    hipLaunchKernelGGL(kern, grid, block, lds, stream, static_cast<KArgs>(args)...);
}

inline int after_launch() {
    hipError_t e = hipGetLastError();
    return e == hipSuccess ? HBL_OK : note_hip_error(e);
}

// Allow `kern` more than 48 KiB of dynamic LDS.  The attribute belongs to the (function, device) pair: set
// once per device this process launches on (`done` is the caller's per-instantiation mask of devices, bit =
// device ordinal mod 64).
template <typename Kernel>
inline int allow_dynamic_lds(Kernel kern, size_t bytes, std::atomic<uint64_t>& done) {
    if (bytes <= 48 * 1024) return HBL_OK;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error(e);
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return HBL_OK;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) return note_hip_error(e);
    done.fetch_or(bit, std::memory_order_release);
    return HBL_OK;
}

// Number of workgroups of `kern` (threads per workgroup, dynamic LDS bytes) that the current device holds at
// once: occupancy per CU times the CU count, asked once per (kernel, device).  `cache` is the caller's
// per-instantiation table of 64 zero-initialised slots (device ordinal mod 64).
template <typename Kernel>
inline int resident_workgroups(Kernel kern, int threads, size_t lds_bytes, std::atomic<int>* cache, int* out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error(e);
    std::atomic<int>& slot = cache[dev & 63];
    int n = slot.load(std::memory_order_acquire);
    if (n == 0) {
        int per_cu = 0, cus = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), threads, lds_bytes);
        if (e != hipSuccess) return note_hip_error(e);
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return note_hip_error(e);
        n = (per_cu < 1 ? 1 : per_cu) * (cus < 1 ? 1 : cus);
        slot.store(n, std::memory_order_release);
    }
    *out = n;
    return HBL_OK;
}

inline bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Split-K factor of the small-T (decode) GEMM: split K only until there are enough workgroups (128
// output rows each) to occupy the chip, and never below 4 K-blocks of 128 per workgroup.  Every
// split costs a second launch (the reduction) and T*N*4 bytes of partials per slice.
constexpr int kDecodeWgTarget = 192;
inline int decode_split_k(int64_t T, int64_t K, int64_t N) {
    if (T > 64 || T <= 0) return 1;
    const int64_t nkb = K / 128, groups = (N + 127) / 128;
    int sk = 1;
    while ((int64_t)sk * groups < kDecodeWgTarget && nkb % (sk * 2) == 0 && nkb / (sk * 2) >= 4) sk *= 2;
    return sk;
}

// Layout of the forward workspace: codes (one byte per code [T,K], or the record image) | float s_dequant [T],
// and | int32 partial [split_k][T][N] for T <= 64 or a split K range.
// K split of the fp6 x fp4 prefill GEMM at mid-size batches: between 65 tokens and about a thousand a long-K
// projection has too few output tiles (128 x 128) to give most CUs a workgroup, so the K range is cut until about
// 256 workgroups exist, each keeping at least 8 K-blocks of 128; the int32 partial tiles then take one more launch.
// Only for K >= 8192: at K = 4096 the unsplit call is short already and the extra launch costs more than it saves
// (measured: W_down at 96-512 tokens 48-52 us -> 26-45 us; K = 4096 projections 18-20 us -> 21-29 us).
inline int prefill_split_k(int64_t T, int64_t K, int64_t N) {
    if (T <= 64 || K < 8192) return 1;
    const int64_t tiles = ((N + 127) / 128) * ((T + 127) / 128), nkb = K / 128;
    int sk = 1;
    while (sk < 8 && tiles * sk * 2 <= 256 && nkb % (sk * 2) == 0 && nkb / (sk * 2) >= 8) sk *= 2;
    return sk;
}

// Largest K split the small-batch streaming GEMM may choose (sizes the partial buffers).
constexpr int kMaxDecodeSplit = 4;

struct Workspace {
    int8_t* codes;
    float* s_dequant;
    int32_t* partial;
    size_t bytes;
};
// with_partial = false: no room for partial tiles (the kernels then keep every K range in one workgroup).
// tile_rows: 32 or 64 when the projection runs in a group whose largest member has 17-32 / 33-64 tokens (the
// small-batch kernel's form, and with it the shape of its slices, follows the largest member), else 0.
inline Workspace carve_workspace(void* base, int64_t T, int64_t K, int64_t N, bool with_partial = true, int tile_rows = 0) {
    Workspace w;
    size_t off = 0;
    w.codes = reinterpret_cast<int8_t*>(static_cast<char*>(base) + off);
    {   // one byte per code, or the record image (0.75 byte per code, whole panels of 128 tokens)
        const size_t bytes = static_cast<size_t>(T) * static_cast<size_t>(K), rec = code_record_bytes(T, K);
        off += round_up(bytes > rec ? bytes : rec, 256);
    }
    w.s_dequant = reinterpret_cast<float*>(static_cast<char*>(base) + off);
    off += round_up(static_cast<size_t>(T) * sizeof(float), 256);
    w.partial = nullptr;
    // small batches: room for the K split of either small-batch kernel pair (the streaming kernel's plan cuts a
    // K range into at most kMaxDecodeSplit slices)
    int split = T <= 64 ? decode_split_k(T, K, N) : prefill_split_k(T, K, N);
    if (T <= 64 && split < kMaxDecodeSplit) split = kMaxDecodeSplit;
    if (with_partial && (T <= 64 || split > 1)) {
        w.partial = reinterpret_cast<int32_t*>(static_cast<char*>(base) + off);
        // (17 to 64 tokens: the small-batch kernel keeps its slices as whole tiles of 32 tokens x 128 features)
        size_t rows = static_cast<size_t>(T);
        if (T <= 64) {
            int tr = T > 16 ? (T <= 32 ? 32 : 64) : 0;
            if (tile_rows > tr) tr = tile_rows;
            if (tr != 0) rows = static_cast<size_t>(tr);
        }
        const size_t cols = T <= 64 ? round_up(static_cast<size_t>(N), 128) : static_cast<size_t>(N);
        off += round_up(static_cast<size_t>(split) * rows * cols * sizeof(int32_t), 256);
    }
    w.bytes = off;
    return w;
}

// Launchers (defined in the .hip files). All validate nothing: callers in api.hip do.
// Codes are stored as code + code_offset (0, or 8 for INT4 so that the stored bytes are 0..15), or -
// code_offset == kCodesBf6 - as bf6 records (see fwht_quant.hip; INT4 with K >= 512).
constexpr int kCodesBf6 = 6;
// INT4 activations on rows of 512 features and more travel as bf6 records and meet the weights on the fp6 x fp4
// matrix cores, at every batch size; INT8 activations and shorter rows travel as bytes to the int8 matrix cores.
inline bool bf6_path_supported(int64_t K, int bits) { return bits == 4 && K >= 512; }
// ln_gain != nullptr: RMS-normalise each row with that gain vector [K] and ln_eps first (LN of Eq. 7).
int launch_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, int bits, float eps, bool hadamard,
                      int8_t* codes, float* s_dequant, int32_t* code_sum, int code_offset, hipStream_t stream,
                      const float* ln_gain = nullptr, float ln_eps = 0.0f);

// Transform only: out[t] = Hadamard(x[t]) as fp32 or bf16 (K a power of two, 128..16384).
// Low-bit head states (kv_quant.hip)
bool kv_shape_ok(int64_t rows, int64_t d, int bits);
int launch_kv_quant(const void* x, int x_dtype, int64_t rows, int64_t d, int bits, float eps, void* packed,
                    float* scales, hipStream_t stream);
int launch_kv_dequant(const void* packed, const float* scales, int64_t rows, int64_t d, int bits, void* out,
                      int out_dtype, hipStream_t stream);
int launch_fwht_only(const void* x, int x_dtype, int64_t T, int64_t K, void* out, int out_dtype, hipStream_t stream);

// Workgroup tiles of the two prefill GEMM kernels.  kTileAuto is the choice every forward call makes from the
// shape; the others let the parity tests run a given tile on a shape of their own.
constexpr int kTileAuto = -1, kTileSquare = 0 /*256 x 256*/, kTileSmall = 1 /*128 x 128*/,
              kTileWide = 2 /*512 features x 128 tokens*/, kTileSplitK = 3 /*128 x 128, K cut over workgroups*/;

// GEMM + epilogue. If acc_out != nullptr the raw int32 accumulators are written
// (no scales, no code_sum needed); otherwise y (bf16) is written.
int launch_ternary_gemm(const int8_t* codes, int code_offset, int64_t T, int64_t K, const void* packed, int64_t N,
                        const float* s_dequant, const float* w_scales,
                        int64_t n_scale_groups, void* y_bf16, int32_t* acc_out, int32_t* splitk_partial,
                        hipStream_t stream, int tile = kTileAuto);

// GEMM + epilogue on the fp6 x fp4 matrix-core path: codes as bf6 records; exact, INT4 activations only.
// acc_out != nullptr: the raw accumulators as int32 [T, N] instead of y.
int launch_ternary_gemm_f6f4(const int8_t* code_records, int64_t T, int64_t K, const void* packed, int64_t N,
                             const float* s_dequant, const float* w_scales, int64_t n_scale_groups, void* y_bf16,
                             hipStream_t stream, int32_t* splitk_partial = nullptr, int32_t* acc_out = nullptr,
                             int tile = kTileAuto);

// ---------------------------------------------------------------------------------------------
// Grouped small-batch path: up to kMaxGroup independent projections (T <= 64 each) served by one
// quantiser launch and one GEMM launch (a K range split over workgroups is reduced by the last of them to
// finish).  The argument blocks travel by value as kernel arguments: no table in device memory.
constexpr int kMaxGroup = 8;

struct QuantProblem {
    const void* x;        // [T, K] bf16 / fp32
    int8_t* codes;        // [T, K] out
    float* s_dequant;     // [T] out
    int32_t* code_sum;    // [T] out
    int T, K;
    int hadamard;
    int code_offset;
    int row_begin;        // first workgroup (= row) of this problem in the grouped grid
    const float* ln_gain; // [K] RMS-norm gain ahead of the transform, or nullptr
    float ln_eps;
};
// (n and the begin arrays come first: a workgroup finds its problem from one cache line of the argument
// block and then loads that problem only - reading all kMaxGroup problems cost ~0.7 us at kernel start)
struct QuantGroupArgs {
    int n;
    float eps;
    int row_begin[kMaxGroup];   // = p[i].row_begin
    QuantProblem p[kMaxGroup];
};
int launch_quant_grouped(const QuantGroupArgs& args, int bits, int x_dtype, hipStream_t stream);

struct DecodeProblem {
    const int8_t* codes;       // [T, K] stored as code + code_offset
    const uint32_t* packed;    // weight tiles
    const float* s_dequant;    // [T]
    const int32_t* w_row_sum;  // [N]
    const float* w_scales;     // [groups]
    uint16_t* y;               // [T, N] bf16
    int32_t* partial;          // [ksplit][T][N] when the K range is split over workgroups, else unused
    int T, K, N;
    int rows_per_group;
    int code_offset;           // int8 path: stored code byte = q + code_offset
    int f6;                    // codes are bf6 records (record image): the fp6 x fp4 matrix cores do the work
    int ksplit;                // K slices per row tile
    int wg_begin;              // first workgroup of this problem in the GEMM grid
    int arrive_begin;          // first arrival counter of this problem (K split over workgroups, reduced in the kernel)
};
struct DecodeArgs {
    int n;
    int wg_begin[kMaxGroup];    // = p[i].wg_begin (filled with it by the launch plan)
    unsigned int* arrive;       // arrival counters of this launch (set by the launch when some K range is split over workgroups)
    DecodeProblem p[kMaxGroup];
};
// Index of the problem workgroup `wg` belongs to: the last one whose first workgroup is not beyond it.
__host__ __device__ inline int group_index_of(const int* begin, int n, int wg) {
    int idx = 0;
#pragma unroll
    for (int i = 1; i < kMaxGroup; ++i)
        if (i < n && wg >= begin[i]) idx = i;
    return idx;
}
// Fills ksplit / wg_begin / arrive_begin and launches.  Every problem needs T <= 64.
int launch_decode_gemm(DecodeArgs& args, hipStream_t stream);
// The launch plan launch_decode_gemm would use (K splits, grid sizes), without launching: host logic only.
int decode_plan_for_tests(DecodeArgs& args, int* wgs, int* arrival_counters);
// Whether a single projection with T <= 16 is better served by the streaming form of that launch than
// by the split-K pair of launch_ternary_gemm.
bool decode_stream_preferred(int64_t T, int64_t K, int64_t N);

// Packed weight buffer: N*K/4 bytes of 2-bit tiles (one form, read by every GEMM kernel), then N int32 row sums
// of the ternary codes.
inline size_t packed_tile_bytes(int64_t N, int64_t K) { return (size_t)N * (size_t)K / 4; }
inline size_t packed_total_bytes(int64_t N, int64_t K) { return packed_tile_bytes(N, K) + (size_t)N * sizeof(int32_t); }

int launch_ternarize(const float* W, int64_t count, float eps, int8_t* codes, float* alpha, void* workspace,
                     hipStream_t stream);
size_t ternarize_workspace_bytes(int64_t count);
int launch_pack(const int8_t* codes, int64_t N, int64_t K, void* packed, hipStream_t stream);
int launch_unpack(const void* packed, int64_t N, int64_t K, int8_t* codes, hipStream_t stream);

}  // namespace hbl
