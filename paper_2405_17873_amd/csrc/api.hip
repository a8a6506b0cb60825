// C ABI of the library: argument validation on the host, workspace carving, launch sequencing.
// No entry point allocates device memory or synchronises.
#include <atomic>
#include <mutex>

#include "mq_common.h"

namespace mq {
static std::atomic<int> g_last_hip_error{0};
void set_hip_error(int e) { g_last_hip_error.store(e); }

static inline bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }
static inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }
static inline bool bits_ok(int b) { return b == 2 || b == 3 || b == 4 || b == 8; }
// 16: unquantised 16-bit weights, accepted by the packers and by the weight-only linear
static inline bool bits_ok16(int b) { return bits_ok(b) || b == 16; }

// Workspace of the 8-bit-activation path.
struct A8Workspace {
    ActParams* params;
    float* partials;
    int32_t* rowsum;
    int8_t* a8;
    static size_t bytes(long M, long K) {
        const size_t Kp = ((size_t)K + 127) / 128 * 128;  // int8 rows are padded to whole 128-k stages
        return 256 + up256(sizeof(float) * 2 * (size_t)act_quant_partial_slots()) + up256(4 * (size_t)M) +
               up256((size_t)M * Kp) + 256;
    }
    A8Workspace(void* ws, long M, long K) {
        uint8_t* p = (uint8_t*)ws;
        params = (ActParams*)p;
        p += 256;
        partials = (float*)p;
        p += up256(sizeof(float) * 2 * (size_t)act_quant_partial_slots());
        rowsum = (int32_t*)p;
        p += up256(4 * (size_t)M);
        a8 = (int8_t*)p;
        (void)K;
    }
};

// Upper bound of what the split of an [M,K] x [N,K] GEMM's reduction over workgroups can use: arrival counters of the
// smallest tile (64 x 64) plus `parts` partial accumulator sets over the output padded to the largest splitting tile
// (128 x 128).  The automatic choice splits only where there are at most 64 tiles and at least 16 pipeline stages, into
// at most min(16, stages / 4) parts; a forced part count (test hook) is taken as it is.
size_t split_workspace_bytes(long M, long N, long K) {
    if (M <= 0 || N <= 0 || K <= 0) return 0;
    const long Mp = (M + 127) / 128 * 128, Np = (N + 127) / 128 * 128;
    long parts = 0;
    if (forced_splits() > 1) {
        parts = forced_splits();
    } else if (forced_splits() == 0 && (Mp / 128) * (Np / 128) <= 64 && K / 64 >= 16) {
        parts = K / 64 / 4;
        parts = parts > 16 ? 16 : parts;
    }
    if (parts <= 1) return 0;
    return up256((size_t)(Mp / 64) * (Np / 64) * 4) + (size_t)parts * Mp * Np * 4 + 256;
}

static int check_linear_common(const void* x, int M, int K, int ldx, const void* packed, int N, int layout,
                               const float* w_scale, const int32_t* w_zp, const void* bias, const void* y, int ldy,
                               bool need_params = true) {
    if (!x || !packed || !y) return MQ_ERR_BAD_ARG;
    if (need_params && (!w_scale || !w_zp)) return MQ_ERR_BAD_ARG;
    if (M <= 0 || K <= 0 || N <= 0 || ldx < K || ldy < N) return MQ_ERR_BAD_SHAPE;
    if (layout != MQ_LAYOUT_KERNEL) return MQ_ERR_UNSUPPORTED_LAYOUT;
    if (K % 64 != 0 || N % 8 != 0 || ldx % 8 != 0 || ldy % 8 != 0) return MQ_ERR_BAD_SHAPE;
    // lane offsets into X and into the packed weights are 32-bit
    if ((long)M * ldx * 2 >= (1L << 31) || (long)(N + 31) * K >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if (!aligned(x, 16) || !aligned(packed, 16) || (w_scale && !aligned(w_scale, 16)) ||
        (w_zp && !aligned(w_zp, 16)) || !aligned(y, 16) || (bias && !aligned(bias, 8)))
        return MQ_ERR_BAD_ARG;
    return MQ_OK;
}

// Optional residual operand: [M, ldr] 16-bit values, may be the output tensor itself.
static int check_residual(const void* residual, long ldr, int N) {
    if (!residual) return MQ_OK;
    if (ldr < N || ldr % 4 != 0) return MQ_ERR_BAD_SHAPE;
    if (!aligned(residual, 8)) return MQ_ERR_BAD_ARG;
    return MQ_OK;
}

static int qlinear_a8(const void* x, int M, int K, int ldx, RowMap in_map, const void* packed, int N, int layout,
                      int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                      const float* act_scale, const int32_t* act_zp, const void* bias, void* y, int ldy, RowMap out_map,
                      int32_t* acc_debug, float* act_scale_out, int32_t* act_zp_out, void* ws, size_t ws_bytes,
                      const void* residual, int ldr, hipStream_t st, const BosWork* bos = nullptr) {
    int rc = check_linear_common(x, M, K, ldx, packed, N, layout, w_scale, w_zp, bias, y, ldy);
    if (rc) return rc;
    if ((rc = check_residual(residual, ldr, N))) return rc;
    if (!w_colsum || !ws) return MQ_ERR_BAD_ARG;
    if ((act_scale == nullptr) != (act_zp == nullptr)) return MQ_ERR_BAD_ARG;
    if (!aligned(w_colsum, 16) || !aligned(ws, 256) || (acc_debug && !aligned(acc_debug, 16))) return MQ_ERR_BAD_ARG;
    if ((long)255 * 255 * K >= (1L << 31)) return MQ_ERR_OVERFLOW_RISK;
    const size_t base = A8Workspace::bytes(M, K);
    if (ws_bytes < base) return MQ_ERR_WORKSPACE_TOO_SMALL;
    // (a forced split that the rest of the workspace cannot hold must fail before anything is launched)
    if (forced_splits() > 1 && ws_bytes - base < split_workspace_bytes(M, N, K)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    A8Workspace w(ws, M, K);
    rc = launch_act_quant(x, M, K, ldx, in_map, act_scale, act_zp, w.a8, w.rowsum, w.params, w.partials,
                          act_scale_out, act_zp_out, bos, st);
    if (rc) return rc;
    // what lies beyond the activation workspace serves the split of the reduction over workgroups
    return launch_gemm_a8(w.a8, w.rowsum, w.params, M, K, packed, N, w_bits, w_signed, w_scale, w_zp, w_colsum, bias,
                          y, ldy, out_map, acc_debug, residual, ldr, (uint8_t*)ws + base, ws_bytes - base, st);
}

// ---- built-in workspace ---------------------------------------------------------------------------------------
// For callers that cannot allocate (code under graph capture, serving loops, harnesses that forbid it):
// mq_qlinear_a8_builtin_ws runs the 8-bit-activation linear with its workspace in this file-scope device array.  In
// host code the array's name is only a stand-in, not a device address: its address on the current device is looked
// up once per device and kept, and host code uses that pointer everywhere.  Every GPU the library runs on holds its
// own copy of the array until the process ends.
static constexpr size_t kBuiltinWsBytes = 48u << 20;
static __device__ __align__(256) uint8_t scratch[kBuiltinWsBytes];

static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[64] = {};  // per device

static int builtin_workspace(void** out) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= 64) {
        set_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidDevice));
        return MQ_ERR_HIP;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            set_hip_error((int)(e != hipSuccess ? e : hipErrorInvalidSymbol));
            return MQ_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MQ_OK;
}
}  // namespace mq

using namespace mq;

extern "C" {

int mq_version(void) { return 1; }
int mq_last_hip_error(void) { return g_last_hip_error.load(); }
void mq_tune_force_tile(int tile) { set_force_tile(tile); }
void mq_tune_force_splits(int parts) { set_force_splits(parts); }
void mq_tune_force_band(int rows) { set_force_band(rows); }
void mq_prof_phase_buffer(long long* clk, long workgroups) { set_phase_buffer(clk, workgroups); }
int mq_prof_enable(int on) { return prof_enable(on); }
int mq_prof_num_slots(void) { return prof_num_slots(); }
int mq_prof_read(int slot, char* name_host, int name_cap, long long* launches_host, double* ms_host,
                 double* ops_host, double* bytes_host) {
    return prof_read(slot, name_host, name_cap, launches_host, ms_host, ops_host, bytes_host);
}
int mq_prof_reset(void) { return prof_reset(); }
int mq_prof_filter(int slot, int stride) { return prof_filter(slot, stride); }
int mq_prof_copy(void* dst, const void* src, size_t bytes, void* stream) {
    return prof_copy(dst, src, bytes, (hipStream_t)stream);
}
int mq_prof_microbench(int kind, void* buf, size_t buf_bytes, double* ms_host, void* stream) {
    return prof_microbench(kind, buf, buf_bytes, ms_host, (hipStream_t)stream);
}
double mq_prof_bracket_overhead_us(void* stream) { return prof_bracket_overhead_us((hipStream_t)stream); }

int mq_quantize_weights(const void* w, int N, int K, int bits, int symmetric, int dtype, uint8_t* codes, float* scale,
                        int32_t* zp, void* stream) {
    if (!w || !codes || !scale || !zp) return MQ_ERR_BAD_ARG;
    if (dtype != MQ_F16 && dtype != MQ_BF16) return MQ_ERR_BAD_ARG;
    if (N <= 0 || K <= 0) return MQ_ERR_BAD_SHAPE;
    if (!bits_ok(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    return launch_quantize_weights(w, N, K, bits, symmetric ? 1 : 0, dtype, codes, scale, zp, (hipStream_t)stream);
}

size_t mq_packed_bytes(int N, int K, int bits, int layout) {
    if (N <= 0 || K <= 0 || !bits_ok16(bits)) return 0;
    if (layout == MQ_LAYOUT_CANONICAL) {
        if (((long)K * bits) % 8 != 0) return 0;
        return (size_t)N * ((size_t)K * bits / 8);
    }
    if (layout == MQ_LAYOUT_KERNEL) {
        if (K % 64 != 0) return 0;
        return (size_t)((N + 31) / 32) * (K / 64) * kl_tile_bytes(bits);
    }
    return 0;
}

int mq_pack_weights(const uint8_t* codes, int N, int K, int bits, int layout, int codes_signed, void* packed,
                    int32_t* colsum, void* stream) {
    if (!codes || !packed) return MQ_ERR_BAD_ARG;
    if (N <= 0 || K <= 0) return MQ_ERR_BAD_SHAPE;
    if (!bits_ok16(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    if (layout != MQ_LAYOUT_CANONICAL && layout != MQ_LAYOUT_KERNEL) return MQ_ERR_UNSUPPORTED_LAYOUT;
    if (codes_signed && bits != 8) return MQ_ERR_BAD_ARG;
    if (bits == 16 && colsum) return MQ_ERR_BAD_ARG;  // no code sums of unquantised weights
    if (mq_packed_bytes(N, K, bits, layout) == 0) return MQ_ERR_BAD_SHAPE;
    if (layout == MQ_LAYOUT_KERNEL && !aligned(packed, 16)) return MQ_ERR_BAD_ARG;
    return launch_pack(codes, N, K, bits, layout, codes_signed ? 1 : 0, packed, colsum, (hipStream_t)stream);
}

int mq_unpack_weights(const void* packed, int N, int K, int bits, int layout, uint8_t* codes, void* stream) {
    if (!codes || !packed) return MQ_ERR_BAD_ARG;
    if (N <= 0 || K <= 0) return MQ_ERR_BAD_SHAPE;
    if (!bits_ok16(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    if (layout != MQ_LAYOUT_CANONICAL && layout != MQ_LAYOUT_KERNEL) return MQ_ERR_UNSUPPORTED_LAYOUT;
    if (mq_packed_bytes(N, K, bits, layout) == 0) return MQ_ERR_BAD_SHAPE;
    if (layout == MQ_LAYOUT_KERNEL && !aligned(packed, 16)) return MQ_ERR_BAD_ARG;
    return launch_unpack(packed, N, K, bits, layout, codes, (hipStream_t)stream);
}

size_t mq_split_workspace_bytes(int M, int N, int K) { return split_workspace_bytes(M, N, K); }

int mq_qlinear_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, int bits, int layout,
                      const float* w_scale, const int32_t* w_zp, const void* bias, void* y, int ldy, int dtype,
                      const void* residual, int ldr, void* ws, size_t ws_bytes, void* stream) {
    if (!bits_ok16(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    if (dtype != MQ_F16 && dtype != MQ_BF16) return MQ_ERR_BAD_ARG;
    int rc = check_linear_common(x, M, K, ldx, packed, N, layout, w_scale, w_zp, bias, y, ldy, bits != 16);
    if (rc) return rc;
    if ((rc = check_residual(residual, ldr, N))) return rc;
    // (lane offsets into the weights are 32-bit byte offsets: unquantised weights take two bytes per element)
    if (bits == 16 && (long)(N + 31) * K * 2 >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if (bits == 16) w_scale = nullptr, w_zp = nullptr;  // 16-bit weights are used as they are
    if (ws && !aligned(ws, 256)) return MQ_ERR_BAD_ARG;
    if (!ws) ws_bytes = 0;
    if (forced_splits() > 1 && ws_bytes < split_workspace_bytes(M, N, K)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    return launch_gemm_w_only(x, M, K, ldx, packed, N, bits, w_scale, w_zp, bias, y, ldy, dtype, residual, ldr, ws,
                              ws_bytes, (hipStream_t)stream);
}

size_t mq_a8_row_bytes(int K) { return K > 0 ? ((size_t)K + 127) / 128 * 128 : 0; }

int mq_qlinear_a8_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int w_bits, int layout,
                        int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                        const float* act_scale, const int32_t* act_zp, const void* bias, const float* out_scale,
                        const int32_t* out_zp, int8_t* a8_out, void* h16_out, int ldh, float* act_scale_out,
                        int32_t* act_zp_out, void* ws, size_t ws_bytes, void* stream) {
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    if (H <= 0 || H % 32 != 0 || H > (1 << 29)) return MQ_ERR_BAD_SHAPE;
    // x, weights of 2H rows; the fp16 product (if asked for) stands in for y in the common checks
    int rc = check_linear_common(x, M, K, ldx, packed, 2 * H, layout, w_scale, w_zp, bias, a8_out, 2 * H);
    if (rc) return rc;
    if (!w_colsum || !ws || !out_scale || !out_zp) return MQ_ERR_BAD_ARG;
    if ((act_scale == nullptr) != (act_zp == nullptr)) return MQ_ERR_BAD_ARG;
    if (!aligned(w_colsum, 16) || !aligned(ws, 256)) return MQ_ERR_BAD_ARG;
    if (h16_out && (!aligned(h16_out, 16) || ldh < H || ldh % 8 != 0)) return MQ_ERR_BAD_ARG;
    if ((long)M * (long)mq_a8_row_bytes(H) >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if ((long)255 * 255 * K >= (1L << 31)) return MQ_ERR_OVERFLOW_RISK;
    if (ws_bytes < A8Workspace::bytes(M, K)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    A8Workspace w(ws, M, K);
    rc = launch_act_quant(x, M, K, ldx, RowMap{0, 0, 0}, act_scale, act_zp, w.a8, w.rowsum, w.params, w.partials,
                          act_scale_out, act_zp_out, nullptr, st);
    if (rc) return rc;
    return launch_gemm_a8_geglu(w.a8, w.rowsum, w.params, M, K, packed, H, w_bits, w_signed ? 1 : 0, w_scale, w_zp,
                                w_colsum, bias, out_scale, out_zp, a8_out, h16_out, ldh, nullptr, nullptr, st);
}

// Dynamic output parameters: behind the input's workspace lie the parameters of the output pass, one (min, max)
// pair per workgroup of the gated projection (at most one per 128 rows x 64 gated columns) and the row sums that
// the quantise kernel writes beside its codes (the consumer takes its own inside its main loop).
static size_t geglu_dynamic_pairs(long M, long H) { return (size_t)((M + 127) / 128) * (size_t)((H + 127) / 128 * 2); }

size_t mq_qlinear_a8_geglu_dynamic_workspace_bytes(int M, int K, int H) {
    if (M <= 0 || K <= 0 || H <= 0) return 0;
    return A8Workspace::bytes(M, K) + 256 + up256(8 * geglu_dynamic_pairs(M, H)) + up256(4 * (size_t)M);
}

int mq_qlinear_a8_geglu_dynamic(const void* x, int M, int K, int ldx, const void* packed, int H, int w_bits,
                                int layout, int w_signed, const float* w_scale, const int32_t* w_zp,
                                const int32_t* w_colsum, const float* act_scale, const int32_t* act_zp,
                                const void* bias, void* h16, int ldh, int8_t* a8_out, float* out_scale_out,
                                int32_t* out_zp_out, float* act_scale_out, int32_t* act_zp_out, void* ws,
                                size_t ws_bytes, void* stream) {
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    if (H <= 0 || H % 32 != 0 || H > (1 << 29)) return MQ_ERR_BAD_SHAPE;
    int rc = check_linear_common(x, M, K, ldx, packed, 2 * H, layout, w_scale, w_zp, bias, a8_out, 2 * H);
    if (rc) return rc;
    if (!w_colsum || !ws || !h16 || !out_scale_out || !out_zp_out) return MQ_ERR_BAD_ARG;
    if ((act_scale == nullptr) != (act_zp == nullptr)) return MQ_ERR_BAD_ARG;
    if (!aligned(w_colsum, 16) || !aligned(ws, 256) || !aligned(h16, 16)) return MQ_ERR_BAD_ARG;
    if (ldh < H || ldh % 8 != 0) return MQ_ERR_BAD_SHAPE;
    if ((long)M * (long)mq_a8_row_bytes(H) >= (1L << 31) || (long)M * ldh * 2 >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if ((long)255 * 255 * K >= (1L << 31)) return MQ_ERR_OVERFLOW_RISK;
    if (ws_bytes < mq_qlinear_a8_geglu_dynamic_workspace_bytes(M, K, H)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    A8Workspace w(ws, M, K);
    uint8_t* q = (uint8_t*)ws + A8Workspace::bytes(M, K);
    ActParams* out_params = (ActParams*)q;
    float* pairs = (float*)(q + 256);
    int32_t* out_rowsum = (int32_t*)(q + 256 + up256(8 * geglu_dynamic_pairs(M, H)));
    rc = launch_act_quant(x, M, K, ldx, RowMap{0, 0, 0}, act_scale, act_zp, w.a8, w.rowsum, w.params, w.partials,
                          act_scale_out, act_zp_out, nullptr, st);
    if (rc) return rc;
    int n_pairs = 0;
    rc = launch_gemm_a8_geglu(w.a8, w.rowsum, w.params, M, K, packed, H, w_bits, w_signed ? 1 : 0, w_scale, w_zp,
                              w_colsum, bias, nullptr, nullptr, nullptr, h16, ldh, pairs, &n_pairs, st);
    if (rc) return rc;
    if (n_pairs <= 0 || (size_t)n_pairs > geglu_dynamic_pairs(M, H)) return MQ_ERR_BAD_SHAPE;  // (cannot happen)
    // the ordinary dynamic quantisation of the fp16 product, minus its pass for the range
    return launch_act_quant(h16, M, H, ldh, RowMap{0, 0, 0}, nullptr, nullptr, a8_out, out_rowsum, out_params, pairs,
                            out_scale_out, out_zp_out, nullptr, st, n_pairs);
}

int mq_qlinear_w_only_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int bits, int layout,
                            const float* w_scale, const int32_t* w_zp, const void* bias, void* h, int ldh,
                            void* stream) {
    if (!bits_ok(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    if (H <= 0 || H % 32 != 0 || H > (1 << 29)) return MQ_ERR_BAD_SHAPE;
    int rc = check_linear_common(x, M, K, ldx, packed, 2 * H, layout, w_scale, w_zp, bias, h, 2 * H);
    if (rc) return rc;
    if (ldh < H || ldh % 8 != 0) return MQ_ERR_BAD_SHAPE;
    return launch_gemm_w_only_geglu(x, M, K, ldx, packed, H, bits, w_scale, w_zp, bias, h, ldh, nullptr, nullptr,
                                    nullptr, (hipStream_t)stream);
}

int mq_qlinear_w_only_geglu_a8(const void* x, int M, int K, int ldx, const void* packed, int H, int bits, int layout,
                               const float* w_scale, const int32_t* w_zp, const void* bias, const float* out_scale,
                               const int32_t* out_zp, int8_t* a8_out, void* h16_out, int ldh, void* stream) {
    if (!bits_ok(bits) || bits == 16) return MQ_ERR_UNSUPPORTED_BITS;
    if (H <= 0 || H % 32 != 0 || H > (1 << 29)) return MQ_ERR_BAD_SHAPE;
    int rc = check_linear_common(x, M, K, ldx, packed, 2 * H, layout, w_scale, w_zp, bias, a8_out, 2 * H);
    if (rc) return rc;
    if (!out_scale || !out_zp) return MQ_ERR_BAD_ARG;
    if (h16_out && (!aligned(h16_out, 16) || ldh < H || ldh % 8 != 0)) return MQ_ERR_BAD_ARG;
    if ((long)M * (long)mq_a8_row_bytes(H) >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    return launch_gemm_w_only_geglu(x, M, K, ldx, packed, H, bits, w_scale, w_zp, bias, h16_out, ldh, out_scale, out_zp,
                                    a8_out, (hipStream_t)stream);
}

int mq_qlinear_a8_codes(const int8_t* a8, int M, int K, int lda, const float* act_scale, const int32_t* act_zp,
                        const void* packed, int N, int w_bits, int layout, int w_signed, const float* w_scale,
                        const int32_t* w_zp, const int32_t* w_colsum, const void* bias, void* y, int ldy,
                        int32_t* acc_debug, const void* residual, int ldr, void* stream) {
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    if (!a8 || !act_scale || !act_zp || !packed || !w_scale || !w_zp || !w_colsum || !y) return MQ_ERR_BAD_ARG;
    if (M <= 0 || K <= 0 || N <= 0 || ldy < N) return MQ_ERR_BAD_SHAPE;
    if (layout != MQ_LAYOUT_KERNEL) return MQ_ERR_UNSUPPORTED_LAYOUT;
    if (K % 64 != 0 || N % 8 != 0 || ldy % 8 != 0) return MQ_ERR_BAD_SHAPE;
    if (lda % 128 != 0 || (size_t)lda < mq_a8_row_bytes(K)) return MQ_ERR_BAD_SHAPE;
    if ((long)M * lda >= (1L << 31) || (long)(N + 31) * K >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if (!aligned(a8, 16) || !aligned(packed, 16) || !aligned(w_scale, 16) || !aligned(w_zp, 16) ||
        !aligned(w_colsum, 16) || !aligned(y, 16) || (bias && !aligned(bias, 8)) ||
        (acc_debug && !aligned(acc_debug, 16)))
        return MQ_ERR_BAD_ARG;
    if ((long)255 * 255 * K >= (1L << 31)) return MQ_ERR_OVERFLOW_RISK;
    if (int rc = check_residual(residual, ldr, N)) return rc;
    return launch_gemm_a8_codes(a8, lda, act_scale, act_zp, M, K, packed, N, w_bits, w_signed ? 1 : 0, w_scale, w_zp,
                                w_colsum, bias, y, ldy, acc_debug, residual, ldr, (hipStream_t)stream);
}

static int check_conv_common(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N,
                             int layout, const float* w_scale, const int32_t* w_zp, const void* bias, const void* y) {
    if (!x || !packed || !w_scale || !w_zp || !y) return MQ_ERR_BAD_ARG;
    if (B <= 0 || H <= 0 || W <= 0 || Cin <= 0 || N <= 0 || (stride != 1 && stride != 2)) return MQ_ERR_BAD_SHAPE;
    if (layout != MQ_LAYOUT_KERNEL) return MQ_ERR_UNSUPPORTED_LAYOUT;
    if (Cin % 64 != 0 || N % 8 != 0) return MQ_ERR_BAD_SHAPE;
    const long M = (long)B * H * W;
    // lane offsets into X, Y rows and the packed weights are 32-bit
    if (M * Cin * 2 >= (1L << 31) || M >= (1L << 31) / 4 || (long)(N + 31) * 9 * Cin >= (1L << 31)) return MQ_ERR_BAD_SHAPE;
    if (!aligned(x, 16) || !aligned(packed, 16) || !aligned(w_scale, 16) || !aligned(w_zp, 16) || !aligned(y, 16) ||
        (bias && !aligned(bias, 8)))
        return MQ_ERR_BAD_ARG;
    return MQ_OK;
}

int mq_conv3x3_w_only(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int bits,
                      int layout, const float* w_scale, const int32_t* w_zp, const void* bias, void* y,
                      const void* residual, void* stream) {
    if (!bits_ok(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    int rc = check_conv_common(x, B, H, W, Cin, stride, packed, N, layout, w_scale, w_zp, bias, y);
    if (rc) return rc;
    if ((rc = check_residual(residual, N, N))) return rc;
    return launch_conv3x3_w_only(x, B, H, W, Cin, stride, packed, N, bits, w_scale, w_zp, bias, y, residual,
                                 (hipStream_t)stream);
}

int mq_conv_tap_sums(const uint8_t* codes, int N, int Cin, int bits, int codes_signed, int32_t* tapsum, void* stream) {
    if (!codes || !tapsum) return MQ_ERR_BAD_ARG;
    if (N <= 0 || Cin <= 0) return MQ_ERR_BAD_SHAPE;
    if (!bits_ok(bits)) return MQ_ERR_UNSUPPORTED_BITS;
    if (codes_signed && bits != 8) return MQ_ERR_BAD_ARG;
    return launch_tap_sums(codes, N, Cin, bits, codes_signed ? 1 : 0, tapsum, (hipStream_t)stream);
}

size_t mq_conv3x3_a8_workspace_bytes(int B, int H, int W, int Cin) {
    if (B <= 0 || H <= 0 || W <= 0 || Cin <= 0) return 0;
    return A8Workspace::bytes((long)B * H * W, Cin);
}

int mq_conv3x3_a8(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int w_bits,
                  int layout, int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                  const int32_t* w_tapsum, const float* act_scale, const int32_t* act_zp, const void* bias, void* y,
                  int32_t* acc_debug, const void* residual, float* act_scale_out, int32_t* act_zp_out, void* ws,
                  size_t ws_bytes, void* stream) {
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    int rc = check_conv_common(x, B, H, W, Cin, stride, packed, N, layout, w_scale, w_zp, bias, y);
    if (rc) return rc;
    if ((rc = check_residual(residual, N, N))) return rc;
    if (!w_colsum || !w_tapsum || !ws) return MQ_ERR_BAD_ARG;
    if ((act_scale == nullptr) != (act_zp == nullptr)) return MQ_ERR_BAD_ARG;
    if (!aligned(w_colsum, 16) || !aligned(w_tapsum, 4) || !aligned(ws, 256) || (acc_debug && !aligned(acc_debug, 16)))
        return MQ_ERR_BAD_ARG;
    if ((long)255 * 255 * 9 * Cin >= (1L << 31)) return MQ_ERR_OVERFLOW_RISK;
    const long M = (long)B * H * W;
    if (M >= (1L << 31) / 8) return MQ_ERR_BAD_SHAPE;
    if (ws_bytes < A8Workspace::bytes(M, Cin)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    hipStream_t st = (hipStream_t)stream;
    A8Workspace w(ws, M, Cin);
    rc = launch_act_quant(x, (int)M, Cin, Cin, RowMap{0, 0, 0}, act_scale, act_zp, w.a8, w.rowsum, w.params, w.partials,
                          act_scale_out, act_zp_out, nullptr, st);
    if (rc) return rc;
    return launch_conv3x3_a8(w.a8, w.params, B, H, W, Cin, stride, packed, N, w_bits, w_signed ? 1 : 0, w_scale, w_zp, w_colsum,
                             w_tapsum, bias, y, acc_debug, residual, st);
}

size_t mq_qlinear_a8_workspace_bytes(int M, int K) {
    if (M <= 0 || K <= 0) return 0;
    return A8Workspace::bytes(M, K);
}

int mq_qlinear_w8a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout, int w_signed,
                    const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale,
                    const int32_t* act_zp, const void* bias, void* y, int ldy, int32_t* acc_debug,
                    const void* residual, int ldr, float* act_scale_out, int32_t* act_zp_out, void* ws, size_t ws_bytes,
                    void* stream) {
    return qlinear_a8(x, M, K, ldx, RowMap{0, 0, 0}, packed, N, layout, 8, w_signed ? 1 : 0, w_scale, w_zp, w_colsum,
                      act_scale, act_zp, bias, y, ldy, RowMap{0, 0, 0}, acc_debug, act_scale_out, act_zp_out, ws,
                      ws_bytes, residual, ldr, (hipStream_t)stream);
}

int mq_qlinear_w4a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout, const float* w_scale,
                    const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale, const int32_t* act_zp,
                    const void* bias, void* y, int ldy, int32_t* acc_debug, const void* residual, int ldr,
                    float* act_scale_out, int32_t* act_zp_out, void* ws, size_t ws_bytes, void* stream) {
    return qlinear_a8(x, M, K, ldx, RowMap{0, 0, 0}, packed, N, layout, 4, 0, w_scale, w_zp, w_colsum, act_scale,
                      act_zp, bias, y, ldy, RowMap{0, 0, 0}, acc_debug, act_scale_out, act_zp_out, ws, ws_bytes,
                      residual, ldr, (hipStream_t)stream);
}

int mq_qlinear_w2a8(const void* x, int M, int K, int ldx, const void* packed, int N, int layout, const float* w_scale,
                    const int32_t* w_zp, const int32_t* w_colsum, const float* act_scale, const int32_t* act_zp,
                    const void* bias, void* y, int ldy, int32_t* acc_debug, const void* residual, int ldr,
                    float* act_scale_out, int32_t* act_zp_out, void* ws, size_t ws_bytes, void* stream) {
    return qlinear_a8(x, M, K, ldx, RowMap{0, 0, 0}, packed, N, layout, 2, 0, w_scale, w_zp, w_colsum, act_scale,
                      act_zp, bias, y, ldy, RowMap{0, 0, 0}, acc_debug, act_scale_out, act_zp_out, ws, ws_bytes,
                      residual, ldr, (hipStream_t)stream);
}

size_t mq_builtin_workspace_bytes(void) { return kBuiltinWsBytes; }

int mq_qlinear_a8_builtin_ws(const void* x, int M, int K, int ldx, const void* packed, int N, int w_bits, int layout,
                             int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                             const float* act_scale, const int32_t* act_zp, const void* bias, void* y, int ldy,
                             int32_t* acc_debug, const void* residual, int ldr, float* act_scale_out,
                             int32_t* act_zp_out, void* stream) {
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    if (M <= 0 || K <= 0) return MQ_ERR_BAD_SHAPE;
    // the size limit is checked before the device is touched
    if (A8Workspace::bytes(M, K) > kBuiltinWsBytes) return MQ_ERR_WORKSPACE_TOO_SMALL;
    void* ws = nullptr;
    if (int rc = builtin_workspace(&ws)) return rc;
    return qlinear_a8(x, M, K, ldx, RowMap{0, 0, 0}, packed, N, layout, w_bits, w_signed ? 1 : 0, w_scale, w_zp, w_colsum,
                      act_scale, act_zp, bias, y, ldy, RowMap{0, 0, 0}, acc_debug, act_scale_out, act_zp_out, ws,
                      kBuiltinWsBytes, residual, ldr, (hipStream_t)stream);
}

size_t mq_bos_aware_kv_proj_workspace_bytes(int B, int T, int K) {
    if (B <= 0 || T <= 0 || K <= 0) return 0;
    return A8Workspace::bytes((long)B * T, K);
}

int mq_bos_aware_kv_proj(const void* ctx, int B, int T, int K, const void* packed, int N, int w_bits, int layout,
                         int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                         const void* w_f16, const void* bos_out, const float* act_scale, const int32_t* act_zp,
                         const void* bias, void* y, int naive_all_rows, float* act_scale_out, int32_t* act_zp_out,
                         void* ws, size_t ws_bytes, void* stream) {
    if (B <= 0 || T <= 0) return MQ_ERR_BAD_SHAPE;
    if (w_bits != 2 && w_bits != 4 && w_bits != 8) return MQ_ERR_UNSUPPORTED_BITS;
    if (w_bits != 8 && w_signed) return MQ_ERR_BAD_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (naive_all_rows)
        return qlinear_a8(ctx, B * T, K, K, RowMap{0, 0, 0}, packed, N, layout, w_bits, w_signed ? 1 : 0, w_scale, w_zp,
                          w_colsum, act_scale, act_zp, bias, y, N, RowMap{0, 0, 0}, nullptr, act_scale_out, act_zp_out,
                          ws, ws_bytes, nullptr, 0, st);
    if ((w_f16 == nullptr) == (bos_out == nullptr)) return MQ_ERR_BAD_ARG;
    if (w_f16 && !aligned(w_f16, 16)) return MQ_ERR_BAD_ARG;
    if (ws_bytes < mq_bos_aware_kv_proj_workspace_bytes(B, T, K)) return MQ_ERR_WORKSPACE_TOO_SMALL;
    const BosWork bw{(const _Float16*)ctx, B, T, K, N, (const _Float16*)w_f16, (const _Float16*)bos_out,
                     (const _Float16*)bias, (_Float16*)y};
    if (T > 1) {
        // (the BOS rows ride along as extra workgroups of the activation-quantise launch)
        const RowMap body{T - 1, T, 1};  // logical row r -> token 1 + r % (T-1) of prompt r / (T-1)
        return qlinear_a8(ctx, B * (T - 1), K, K, body, packed, N, layout, w_bits, w_signed ? 1 : 0, w_scale, w_zp,
                          w_colsum, act_scale, act_zp, bias, y, N, body, nullptr, act_scale_out, act_zp_out, ws,
                          ws_bytes, nullptr, 0, st, &bw);
    }
    int rc = check_linear_common(ctx, B, K, K, packed, N, layout, w_scale, w_zp, bias, y, N);
    if (rc) return rc;
    return launch_bos_rows(bw, st);
}

}  // extern "C"
