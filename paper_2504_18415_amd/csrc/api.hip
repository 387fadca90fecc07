// C-ABI entry points of libhbitlinear: argument validation and kernel sequencing only.
#include <vector>

#include "hbl_internal.h"
#include "hbl_test_exports.h"

namespace hbl {

static thread_local int g_last_hip_error = 0;

namespace {
// The calling thread's kernel-timing trace (hbl_trace_begin / hbl_trace_end).
struct TraceState {
    LaunchTrace view{};
    std::vector<hipEvent_t> start, stop;
    std::vector<const char*> names;
    bool open = false;
};
thread_local TraceState g_trace;
}  // namespace

LaunchTrace* current_trace() { return g_trace.open ? &g_trace.view : nullptr; }

// Scratch of hbl_bitlinear_forward_small, the entry point that allocates nothing: it plays the part the
// caller's workspace plays in the other forward calls (activation codes and per-token scales; no room for partial
// tiles, so the kernels keep every K range inside one workgroup).  One copy per GPU, held until the process ends.
// In host code the array's name is only a handle for hipGetSymbolAddress: the device address, asked once per
// device, is what is passed on.
constexpr size_t kSmallScratchBytes = (size_t)2 << 20;   // codes of 64 tokens x 16384 features: 1.5 MiB as records
static __device__ __align__(256) unsigned char scratch[kSmallScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

int scratch_of_current_device(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return note_hip_error(e);
    if (dev < 0 || dev >= kMaxDevices) return HBL_E_SHAPE;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p == nullptr) {   // first call on this device (it is current): every GPU holds its own copy of the array
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return note_hip_error(e);
        if (p == nullptr) return note_hip_error(hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return HBL_OK;
}
}  // namespace

int note_hip_error(hipError_t e) {
    g_last_hip_error = (int)e;
    return HBL_E_HIP;
}

namespace {

// INT4 codes on the int8 path travel as code + 8 (bytes 0..15): same results, fewer toggling multiplier inputs.
int small_code_offset(int bits) { return bits == 4 ? 8 : 0; }

int check_gemm_shape(int64_t T, int64_t K, int64_t N, bool hadamard) {
    if (T < 0 || T > (1 << 24)) return HBL_E_SHAPE;
    if (K < 128 || K > 16384 || (K % 128) != 0) return HBL_E_SHAPE;
    if (hadamard && !is_pow2(K)) return HBL_E_SHAPE;
    if (N < 32 || (N % 32) != 0 || N > (1 << 24)) return HBL_E_SHAPE;
    if (T * N >= ((int64_t)1 << 40)) return HBL_E_SHAPE;
    return HBL_OK;
}

// Argument checks of one forward problem (everything but the workspace size).
int check_forward_args(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                       const float* w_scales, int64_t groups, int bits, const void* y, const void* workspace,
                       bool hadamard) {
    if (bits != 4 && bits != 8) return HBL_E_BITS;
    if (x_dtype != HBL_F32 && x_dtype != HBL_BF16) return HBL_E_DTYPE;
    int rc = check_gemm_shape(T, K, N, hadamard);
    if (rc != HBL_OK) return rc;
    if (groups < 1 || (N % groups) != 0 || ((N / groups) % 32) != 0) return HBL_E_SHAPE;
    if (T == 0) return HBL_OK;
    if (!x || !Wq_packed || !w_scales || !y || !workspace) return HBL_E_NULL;
    if (!aligned16(x) || !aligned16(Wq_packed) || !aligned16(y) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return HBL_E_ALIGN;
    return HBL_OK;
}

void fill_decode_problem(DecodeProblem& dp, const Workspace& ws, int64_t T, int64_t K, const void* Wq_packed,
                         int64_t N, const float* w_scales, int64_t groups, int bits, void* y) {
    dp.codes = ws.codes;
    dp.packed = static_cast<const uint32_t*>(Wq_packed);
    dp.s_dequant = ws.s_dequant;
    dp.w_row_sum = reinterpret_cast<const int32_t*>(static_cast<const char*>(Wq_packed) + packed_tile_bytes(N, K));
    dp.w_scales = w_scales;
    dp.y = static_cast<uint16_t*>(y);
    dp.partial = ws.partial;
    dp.T = (int)T;
    dp.K = (int)K;
    dp.N = (int)N;
    dp.rows_per_group = (int)(N / groups);
    dp.f6 = bf6_path_supported(K, bits) ? 1 : 0;
    dp.code_offset = dp.f6 ? 0 : small_code_offset(bits);
}

// Form of the codes between the two launches of a forward call.
int code_form_for(int64_t K, int bits) { return bf6_path_supported(K, bits) ? kCodesBf6 : small_code_offset(bits); }

int forward(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
            const float* w_scales, int64_t groups, int bits, float eps, void* y, void* workspace,
            size_t workspace_bytes, void* stream, bool hadamard, const float* ln_gain = nullptr,
            float ln_eps = 0.0f, bool with_partial = true) {
    int rc = check_forward_args(x, x_dtype, T, K, Wq_packed, N, w_scales, groups, bits, y, workspace, hadamard);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (workspace_bytes < carve_workspace(nullptr, T, K, N, with_partial).bytes) return HBL_E_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Workspace ws = carve_workspace(workspace, T, K, N, with_partial);
    const int code_form = code_form_for(K, bits);
    rc = launch_fwht_quant(x, x_dtype, T, K, bits, eps, hadamard, ws.codes, ws.s_dequant, nullptr, code_form, s, ln_gain,
                           ln_eps);
    if (rc != HBL_OK) return rc;
    // a small batch: the weight-streaming kernel (always on the record path; on the byte path unless the plain
    // split-K pair suits the shape better)
    if (T <= 64 && (code_form == kCodesBf6 || decode_stream_preferred(T, K, N))) {
        DecodeArgs da = {};
        da.n = 1;
        fill_decode_problem(da.p[0], ws, T, K, Wq_packed, N, w_scales, groups, bits, y);
        if (code_form != kCodesBf6) da.p[0].partial = nullptr;   // byte path: the streaming form only
        return launch_decode_gemm(da, s);
    }
    // INT4 at prefill sizes: bf6 code records and the fp6 x fp4 matrix cores (exact, twice the int8 MFMA rate)
    if (code_form == kCodesBf6)
        return launch_ternary_gemm_f6f4(ws.codes, T, K, Wq_packed, N, ws.s_dequant, w_scales, groups, y, s, ws.partial);
    return launch_ternary_gemm(ws.codes, code_form, T, K, Wq_packed, N, ws.s_dequant, w_scales, groups, y, nullptr,
                               ws.partial, s);
}

// Workspace region of one problem of a grouped call: large enough for the grouped launches (partials
// for the largest K split they may choose) and for the stand-alone forward call.
size_t group_region_bytes(const hbl_problem& q, int tile_rows) {
    if (q.T <= 0 || q.K <= 0 || q.N <= 0) return 256;
    return carve_workspace(nullptr, q.T, q.K, q.N, true, tile_rows).bytes;
}
// Token rows of the slices the small-batch kernel keeps for a group: set by the largest member that takes that
// kernel (0: at most 16 tokens everywhere, no slices).
int group_tile_rows(const hbl_problem* problems, int n) {
    int64_t max_t = 0;
    for (int i = 0; i < n; ++i)
        if (problems[i].T <= 64 && problems[i].T > max_t) max_t = problems[i].T;
    return max_t <= 16 ? 0 : (max_t <= 32 ? 32 : 64);
}

}  // namespace
}  // namespace hbl

using namespace hbl;

extern "C" {

const char* hbl_strerror(int status) {
    switch (status) {
        case HBL_OK: return "ok";
        case HBL_E_NULL: return "a required pointer is NULL";
        case HBL_E_SHAPE: return "unsupported shape (K: multiple of 128 in [128,16384], power of two with Hadamard; N: multiple of 32; T >= 0)";
        case HBL_E_BITS: return "bits must be 4 or 8";
        case HBL_E_DTYPE: return "x_dtype must be HBL_F32 or HBL_BF16";
        case HBL_E_WORKSPACE: return "workspace too small";
        case HBL_E_HIP: return "a HIP call failed (see hbl_last_hip_error)";
        case HBL_E_ALIGN: return "pointer not sufficiently aligned";
        case HBL_E_SCRATCH: return "problem too large for the static scratch of the allocation-free entry point (T <= 64)";
        default: return "unknown status";
    }
}

int hbl_last_hip_error(void) { return g_last_hip_error; }

size_t hbl_ternarize_workspace_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0) return 0;
    return ternarize_workspace_bytes(N * K);
}

int hbl_ternarize_weights_absmean(const float* W, int64_t N, int64_t K, float eps, int8_t* codes, float* alpha,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    if (!W || !codes || !alpha || !workspace) return HBL_E_NULL;
    if (N <= 0 || K <= 0 || N > ((int64_t)1 << 40) / K) return HBL_E_SHAPE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 7u) != 0) return HBL_E_ALIGN;
    if (workspace_bytes < hbl_ternarize_workspace_bytes(N, K)) return HBL_E_WORKSPACE;
    return launch_ternarize(W, N * K, eps, codes, alpha, workspace, static_cast<hipStream_t>(stream));
}

size_t hbl_packed_bytes(int64_t N, int64_t K) {
    if (N <= 0 || K <= 0) return 0;
    return packed_total_bytes(N, K);
}

int hbl_pack_ternary_2bit(const int8_t* codes, int64_t N, int64_t K, void* packed, void* stream) {
    if (!codes || !packed) return HBL_E_NULL;
    int rc = check_gemm_shape(0, K, N, false);
    if (rc != HBL_OK) return rc;
    if (!aligned16(codes) || !aligned16(packed)) return HBL_E_ALIGN;
    return launch_pack(codes, N, K, packed, static_cast<hipStream_t>(stream));
}

int hbl_unpack_ternary_2bit(const void* packed, int64_t N, int64_t K, int8_t* codes, void* stream) {
    if (!codes || !packed) return HBL_E_NULL;
    int rc = check_gemm_shape(0, K, N, false);
    if (rc != HBL_OK) return rc;
    if (!aligned16(codes) || !aligned16(packed)) return HBL_E_ALIGN;
    return launch_unpack(packed, N, K, codes, static_cast<hipStream_t>(stream));
}

size_t hbl_workspace_bytes(int64_t T, int64_t K, int64_t N, int bits) {
    (void)bits;
    if (T <= 0 || K <= 0 || N <= 0) return 256;
    return carve_workspace(nullptr, T, K, N).bytes;
}

int hbl_hbitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                           const float* w_scales, int64_t n_scale_groups, int bits, float eps, void* y,
                           void* workspace, size_t workspace_bytes, void* stream) {
    return forward(x, x_dtype, T, K, Wq_packed, N, w_scales, n_scale_groups, bits, eps, y, workspace,
                   workspace_bytes, stream, true);
}

int hbl_plain_bitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                                const float* w_scales, int64_t n_scale_groups, int bits, float eps, void* y,
                                void* workspace, size_t workspace_bytes, void* stream) {
    return forward(x, x_dtype, T, K, Wq_packed, N, w_scales, n_scale_groups, bits, eps, y, workspace,
                   workspace_bytes, stream, false);
}

int hbl_bitlinear_forward_small(const void* x, int x_dtype, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                                const float* w_scales, int64_t n_scale_groups, int bits, float eps, int hadamard,
                                void* y, void* stream) {
    // argument errors first (same order as the other forward calls), with a stand-in workspace pointer
    int rc = check_forward_args(x, x_dtype, T, K, Wq_packed, N, w_scales, n_scale_groups, bits, y,
                                reinterpret_cast<const void*>(uintptr_t{256}), hadamard != 0);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (T > 64 || carve_workspace(nullptr, T, K, N, false).bytes > kSmallScratchBytes) return HBL_E_SCRATCH;
    void* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != HBL_OK) return rc;
    return forward(x, x_dtype, T, K, Wq_packed, N, w_scales, n_scale_groups, bits, eps, y, ws, kSmallScratchBytes,
                   stream, hadamard != 0, nullptr, 0.0f, false);
}

size_t hbl_grouped_workspace_bytes(const hbl_problem* problems, int n_problems) {
    size_t total = 256;
    if (!problems) return total;
    const int tile_rows = group_tile_rows(problems, n_problems);
    for (int i = 0; i < n_problems; ++i) total += group_region_bytes(problems[i], tile_rows);
    return total;
}

int hbl_bitlinear_forward_grouped(const hbl_problem* problems, int n_problems, float eps, void* workspace,
                                  size_t workspace_bytes, void* stream) {
    if (n_problems < 0) return HBL_E_SHAPE;
    if (n_problems == 0) return HBL_OK;
    if (!problems) return HBL_E_NULL;
    bool grouped = n_problems <= kMaxGroup;
    bool any_rows = false;
    for (int i = 0; i < n_problems; ++i) {
        const hbl_problem& q = problems[i];
        const int rc = check_forward_args(q.x, q.x_dtype, q.T, q.K, q.Wq_packed, q.N, q.w_scales, q.n_scale_groups,
                                          q.bits, q.y, workspace, q.hadamard != 0);
        if (rc != HBL_OK) return rc;
        if (q.ln_gain && (reinterpret_cast<uintptr_t>(q.ln_gain) & 15u) != 0) return HBL_E_ALIGN;
        if (q.T > 64 || q.bits != problems[0].bits || q.x_dtype != problems[0].x_dtype) grouped = false;
        any_rows = any_rows || q.T > 0;
    }
    if (!any_rows) return HBL_OK;
    if (!workspace) return HBL_E_NULL;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return HBL_E_ALIGN;
    if (workspace_bytes < hbl_grouped_workspace_bytes(problems, n_problems)) return HBL_E_WORKSPACE;
    char* base = static_cast<char*>(workspace);
    const int tile_rows = group_tile_rows(problems, n_problems);
    if (!grouped) {
        for (int i = 0; i < n_problems; ++i) {
            const hbl_problem& q = problems[i];
            const size_t region = group_region_bytes(q, tile_rows);
            const int rc = forward(q.x, q.x_dtype, q.T, q.K, q.Wq_packed, q.N, q.w_scales, q.n_scale_groups, q.bits, eps,
                                   q.y, base, region, stream, q.hadamard != 0, q.ln_gain, q.ln_eps);
            if (rc != HBL_OK) return rc;
            base += region;
        }
        return HBL_OK;
    }
    QuantGroupArgs qa = {};
    DecodeArgs da = {};
    qa.eps = eps;
    int rows = 0;
    for (int i = 0; i < n_problems; ++i) {
        const hbl_problem& q = problems[i];
        const size_t region = group_region_bytes(q, tile_rows);
        if (q.T > 0) {
            const Workspace ws = carve_workspace(base, q.T, q.K, q.N, true, tile_rows);
            QuantProblem& qp = qa.p[qa.n++];
            qp.x = q.x;
            qp.codes = ws.codes;
            qp.s_dequant = ws.s_dequant;
            qp.code_sum = nullptr;
            qp.T = (int)q.T;
            qp.K = (int)q.K;
            qp.hadamard = q.hadamard != 0;
            qp.code_offset = code_form_for(q.K, q.bits);
            qp.row_begin = qa.row_begin[qa.n - 1] = rows;
            qp.ln_gain = q.ln_gain;
            qp.ln_eps = q.ln_eps;
            rows += (int)q.T;
            fill_decode_problem(da.p[da.n++], ws, q.T, q.K, q.Wq_packed, q.N, q.w_scales, q.n_scale_groups, q.bits, q.y);
        }
        base += region;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int rc = launch_quant_grouped(qa, problems[0].bits, problems[0].x_dtype, s);
    if (rc != HBL_OK) return rc;
    return launch_decode_gemm(da, s);
}

int hbl_ln_bitlinear_forward(const void* x, int x_dtype, int64_t T, int64_t K, const float* ln_gain, float ln_eps,
                             int hadamard, const void* Wq_packed, int64_t N, const float* w_scales,
                             int64_t n_scale_groups, int bits, float eps, void* y, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (T > 0 && !ln_gain) return HBL_E_NULL;
    if (!aligned16(ln_gain)) return HBL_E_ALIGN;
    return forward(x, x_dtype, T, K, Wq_packed, N, w_scales, n_scale_groups, bits, eps, y, workspace,
                   workspace_bytes, stream, hadamard != 0, ln_gain, ln_eps);
}

int hbl_ln_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, const float* ln_gain, float ln_eps, int bits,
                      float eps, int hadamard, int code_offset, int8_t* codes, float* s_dequant, int32_t* code_sum,
                      void* stream) {
    if (code_offset != HBL_CODES_INT8 && !((code_offset == HBL_CODES_UINT4_PLUS8 || code_offset == HBL_CODES_BF6) && bits == 4))
        return HBL_E_BITS;
    if (code_offset == HBL_CODES_BF6 && K < 512) return HBL_E_SHAPE;
    if (bits != 4 && bits != 8) return HBL_E_BITS;
    if (x_dtype != HBL_F32 && x_dtype != HBL_BF16) return HBL_E_DTYPE;
    int rc = check_gemm_shape(T, K, 32, hadamard != 0);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (!x || !codes || !s_dequant || !ln_gain) return HBL_E_NULL;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(ln_gain)) return HBL_E_ALIGN;
    return launch_fwht_quant(x, x_dtype, T, K, bits, eps, hadamard != 0, codes, s_dequant, code_sum, code_offset,
                             static_cast<hipStream_t>(stream), ln_gain, ln_eps);
}

int hbl_test_grouped_plan(const hbl_problem* problems, int n_problems, int* ksplit, int* gemm_workgroups,
                           int* arrival_counters, int* single_call_streams) {
    if (!problems || !ksplit || !gemm_workgroups || !arrival_counters || !single_call_streams) return HBL_E_NULL;
    if (n_problems < 1 || n_problems > kMaxGroup) return HBL_E_SHAPE;
    DecodeArgs da = {};
    static int32_t dummy_partial;
    for (int i = 0; i < n_problems; ++i) {
        const hbl_problem& q = problems[i];
        if (q.T < 1 || q.T > 64) return HBL_E_SHAPE;
        const int rc = check_gemm_shape(q.T, q.K, q.N, q.hadamard != 0);
        if (rc != HBL_OK) return rc;
        DecodeProblem& dp = da.p[da.n++];
        dp.T = (int)q.T;
        dp.K = (int)q.K;
        dp.N = (int)q.N;
        dp.partial = &dummy_partial;   // the grouped call always brings a partial buffer
        single_call_streams[i] = decode_stream_preferred(q.T, q.K, q.N) ? 1 : 0;
    }
    const int rc = decode_plan_for_tests(da, gemm_workgroups, arrival_counters);
    if (rc != HBL_OK) return rc;
    for (int i = 0; i < n_problems; ++i) ksplit[i] = da.p[i].ksplit;
    return HBL_OK;
}

size_t hbl_code_bytes(int64_t T, int64_t K, int code_form) {
    if (T < 0 || K < 128 || K > 16384 || (K % 128) != 0) return 0;
    if (code_form == HBL_CODES_INT8 || code_form == HBL_CODES_UINT4_PLUS8) return (size_t)T * (size_t)K;
    if (code_form == HBL_CODES_BF6) return K >= 512 ? code_record_bytes(T, K) : 0;
    return 0;
}

int hbl_fwht_quant(const void* x, int x_dtype, int64_t T, int64_t K, int bits, float eps, int hadamard,
                   int code_offset, int8_t* codes, float* s_dequant, int32_t* code_sum, void* stream) {
    if (code_offset != HBL_CODES_INT8 && !((code_offset == HBL_CODES_UINT4_PLUS8 || code_offset == HBL_CODES_BF6) && bits == 4))
        return HBL_E_BITS;
    if (code_offset == HBL_CODES_BF6 && K < 512) return HBL_E_SHAPE;
    if (bits != 4 && bits != 8) return HBL_E_BITS;
    if (x_dtype != HBL_F32 && x_dtype != HBL_BF16) return HBL_E_DTYPE;
    int rc = check_gemm_shape(T, K, 32, hadamard != 0);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (!x || !codes || !s_dequant) return HBL_E_NULL;
    if (!aligned16(x) || !aligned16(codes)) return HBL_E_ALIGN;
    return launch_fwht_quant(x, x_dtype, T, K, bits, eps, hadamard != 0, codes, s_dequant, code_sum, code_offset,
                             static_cast<hipStream_t>(stream));
}

int hbl_fwht(const void* x, int x_dtype, int64_t T, int64_t K, void* out, int out_dtype, void* stream) {
    if ((x_dtype != HBL_F32 && x_dtype != HBL_BF16) || (out_dtype != HBL_F32 && out_dtype != HBL_BF16))
        return HBL_E_DTYPE;
    int rc = check_gemm_shape(T, K, 32, true);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (!x || !out) return HBL_E_NULL;
    if (!aligned16(x) || !aligned16(out)) return HBL_E_ALIGN;
    return launch_fwht_only(x, x_dtype, T, K, out, out_dtype, static_cast<hipStream_t>(stream));
}

size_t hbl_kv_packed_bytes(int64_t rows, int64_t d, int bits) {
    if (!kv_shape_ok(rows, d, bits)) return 0;
    return (size_t)rows * (size_t)d * (size_t)bits / 8;
}

int hbl_kv_quant_absmax(const void* x, int x_dtype, int64_t rows, int64_t d, int bits, float eps, void* packed,
                        float* scales, void* stream) {
    if (bits != 8 && bits != 4 && bits != 3) return HBL_E_BITS;
    if (x_dtype != HBL_F32 && x_dtype != HBL_BF16) return HBL_E_DTYPE;
    if (!kv_shape_ok(rows, d, bits)) return HBL_E_SHAPE;
    if (rows == 0) return HBL_OK;
    if (!x || !packed || !scales) return HBL_E_NULL;
    if (!aligned16(x) || !aligned16(packed)) return HBL_E_ALIGN;
    return launch_kv_quant(x, x_dtype, rows, d, bits, eps, packed, scales, static_cast<hipStream_t>(stream));
}

int hbl_kv_dequant(const void* packed, const float* scales, int64_t rows, int64_t d, int bits, void* out,
                   int out_dtype, void* stream) {
    if (bits != 8 && bits != 4 && bits != 3) return HBL_E_BITS;
    if (out_dtype != HBL_F32 && out_dtype != HBL_BF16) return HBL_E_DTYPE;
    if (!kv_shape_ok(rows, d, bits)) return HBL_E_SHAPE;
    if (rows == 0) return HBL_OK;
    if (!packed || !scales || !out) return HBL_E_NULL;
    if (!aligned16(packed) || !aligned16(out)) return HBL_E_ALIGN;
    return launch_kv_dequant(packed, scales, rows, d, bits, out, out_dtype, static_cast<hipStream_t>(stream));
}

int hbl_gemm_i32(const int8_t* codes, int64_t T, int64_t K, const void* Wq_packed, int64_t N, int32_t* acc,
                 void* stream) {
    int rc = check_gemm_shape(T, K, N, false);
    if (rc != HBL_OK) return rc;
    if (T == 0) return HBL_OK;
    if (!codes || !Wq_packed || !acc) return HBL_E_NULL;
    if (!aligned16(codes) || !aligned16(Wq_packed) || !aligned16(acc)) return HBL_E_ALIGN;
    return launch_ternary_gemm(codes, 0, T, K, Wq_packed, N, nullptr, nullptr, 1, nullptr, acc, nullptr,
                               static_cast<hipStream_t>(stream));
}

int hbl_gemm_i32_bf6(const void* code_records, int64_t T, int64_t K, const void* Wq_packed, int64_t N, int32_t* acc,
                     void* workspace, size_t workspace_bytes, void* stream) {
    int rc = check_gemm_shape(T, K, N, false);
    if (rc != HBL_OK) return rc;
    if (K < 512) return HBL_E_SHAPE;
    if (T == 0) return HBL_OK;
    if (!code_records || !Wq_packed || !acc || !workspace) return HBL_E_NULL;
    if (!aligned16(code_records) || !aligned16(Wq_packed) || !aligned16(acc) ||
        (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0)
        return HBL_E_ALIGN;
    if (workspace_bytes < hbl_workspace_bytes(T, K, N, 4)) return HBL_E_WORKSPACE;
    const Workspace ws = carve_workspace(workspace, T, K, N);
    return launch_ternary_gemm_f6f4(static_cast<const int8_t*>(code_records), T, K, Wq_packed, N, nullptr, nullptr, 1,
                                    nullptr, static_cast<hipStream_t>(stream), T > 64 ? ws.partial : nullptr, acc);
}

int hbl_test_gemm_i32_tile(const void* codes, int code_form, int64_t T, int64_t K, const void* Wq_packed, int64_t N,
                           int32_t* acc, int tile, void* partial, size_t partial_bytes, void* stream) {
    if (code_form != HBL_CODES_INT8 && code_form != HBL_CODES_BF6) return HBL_E_BITS;
    if (tile < kTileSquare || tile > kTileSplitK) return HBL_E_SHAPE;
    int rc = check_gemm_shape(T, K, N, false);
    if (rc != HBL_OK) return rc;
    if (T <= 64 || (code_form == HBL_CODES_BF6 && K < 512)) return HBL_E_SHAPE;
    if (!codes || !Wq_packed || !acc) return HBL_E_NULL;
    if (!aligned16(codes) || !aligned16(Wq_packed) || !aligned16(acc) || !aligned16(partial)) return HBL_E_ALIGN;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (tile == kTileSplitK) {
        // the K cut the launcher will take: the forward's own for this shape, else 4 (or 2) slices
        if (code_form != HBL_CODES_BF6) return HBL_E_SHAPE;
        int split = prefill_split_k(T, K, N);
        if (split == 1) split = (K / 128) % 4 == 0 ? 4 : ((K / 128) % 2 == 0 ? 2 : 1);
        if (!partial || partial_bytes < (size_t)split * T * N * sizeof(int32_t)) return HBL_E_WORKSPACE;
    }
    if (code_form == HBL_CODES_BF6)
        return launch_ternary_gemm_f6f4(static_cast<const int8_t*>(codes), T, K, Wq_packed, N, nullptr, nullptr, 1,
                                        nullptr, s, tile == kTileSplitK ? static_cast<int32_t*>(partial) : nullptr, acc,
                                        tile);
    return launch_ternary_gemm(static_cast<const int8_t*>(codes), 0, T, K, Wq_packed, N, nullptr, nullptr, 1, nullptr,
                               acc, nullptr, s, tile);
}

int hbl_trace_begin(int max_launches) {
    if (max_launches < 1 || max_launches > (1 << 20)) return HBL_E_SHAPE;
    TraceState& t = g_trace;
    if (t.open) return HBL_E_SHAPE;
    while ((int)t.start.size() < max_launches) {
        hipEvent_t a = nullptr, b = nullptr;
        hipError_t e = hipEventCreate(&a);
        if (e == hipSuccess) e = hipEventCreate(&b);
        if (e != hipSuccess) {
            if (a) (void)hipEventDestroy(a);
            return note_hip_error(e);
        }
        t.start.push_back(a);
        t.stop.push_back(b);
    }
    t.names.assign(t.start.size(), nullptr);
    t.view = LaunchTrace{t.start.data(), t.stop.data(), t.names.data(), max_launches, 0};
    t.open = true;
    return HBL_OK;
}

int hbl_trace_end(float* ms, const char** kernel_names, int capacity, int* n_launches) {
    TraceState& t = g_trace;
    if (!t.open) return HBL_E_SHAPE;
    t.open = false;
    const int seen = t.view.count;
    const int timed = seen < t.view.capacity ? seen : t.view.capacity;
    if (n_launches) *n_launches = seen;
    for (int i = 0; i < timed && i < capacity; ++i) {
        hipError_t e = hipEventSynchronize(t.stop[i]);
        float v = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&v, t.start[i], t.stop[i]);
        if (e != hipSuccess) return note_hip_error(e);
        if (ms) ms[i] = v;
        if (kernel_names) kernel_names[i] = t.names[i];
    }
    return HBL_OK;
}

int hbl_gemm_dequant_bf16(const int8_t* codes, int code_offset, const float* s_dequant, const int32_t* code_sum,
                          int64_t T, int64_t K, const void* Wq_packed, int64_t N, const float* w_scales,
                          int64_t n_scale_groups, void* y, void* stream) {
    if (code_offset != HBL_CODES_INT8 && code_offset != HBL_CODES_UINT4_PLUS8 && code_offset != HBL_CODES_BF6)
        return HBL_E_BITS;
    int rc = check_gemm_shape(T, K, N, false);
    if (rc != HBL_OK) return rc;
    if (n_scale_groups < 1 || (N % n_scale_groups) != 0 || ((N / n_scale_groups) % 32) != 0) return HBL_E_SHAPE;
    if (T == 0) return HBL_OK;
    (void)code_sum;   // no kernel needs it: the packed weights are signed
    if (!codes || !s_dequant || !Wq_packed || !w_scales || !y) return HBL_E_NULL;
    if (!aligned16(codes) || !aligned16(Wq_packed) || !aligned16(y)) return HBL_E_ALIGN;
    if (code_offset == HBL_CODES_BF6)
        return launch_ternary_gemm_f6f4(codes, T, K, Wq_packed, N, s_dequant, w_scales, n_scale_groups, y,
                                        static_cast<hipStream_t>(stream));
    return launch_ternary_gemm(codes, code_offset, T, K, Wq_packed, N, s_dequant, w_scales, n_scale_groups, y, nullptr,
                               nullptr, static_cast<hipStream_t>(stream));
}

}  // extern "C"
