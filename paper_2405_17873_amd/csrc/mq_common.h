// Shared declarations of the gfx950 quantized-linear library: status codes, the tile-major
// "kernel layout" of packed weights, small device helpers and the internal launcher prototypes.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/mixdq.h"

namespace mq {

// ---------------------------------------------------------------------------------------------
// Kernel layout of packed weights
//
// The N x K code matrix is cut into tiles of 32 output channels x 64 input channels.  Tile (g, c)
// (g = n / 32, c = k / 64) starts at byte ((g * (K/64) + c) * 256 * bits).  Inside a tile the unit is
// the "lane chunk": the 32 codes k' = 0..31 of channel j = n % 32 in k-half kb = (k % 64) / 32, owned
// by lane L = kb * 32 + j of the wave that will feed them to a 32x32 MFMA (operand row j, k-slice kb).
// A wave therefore fetches a whole tile with one fully contiguous load per 16 bytes of lane chunk.
//
//   4 bit: chunk = 16 B at L*16; word wd holds codes 8wd..8wd+7, pair p=(c[2p],c[2p+1]) of that group in
//          bits [4p,4p+4) and [16+4p,16+4p+4)  -> (w >> 4p) & 0x000F000F is a ready half2 mantissa pair.
//   2 bit: chunk = 8 B at L*8; word wd holds codes 16wd..16wd+15, pair p in bits [2p,2p+2) and [16+2p,..).
//   3 bit: chunk = 12 B at L*12; pairs 0..14: word t=p/5, field f=p%5 in bits [3f,3f+3) and [16+3f,..);
//          pair 15 is scattered: bit i of c[30] in bit 15 of word i, bit i of c[31] in bit 31 of word i.
//   8 bit: two 16-byte pieces per lane: piece h (codes 16h..16h+15) at h*1024 + L*16; inside every group of
//          8 codes the byte order is c0,c4,c1,c5,c2,c6,c3,c7 (the order in which a 4-bit word widens to
//          bytes, so that int8 activations are stored once in an order that suits both widths).
// ---------------------------------------------------------------------------------------------

__host__ __device__ inline int kl_tile_bytes(int bits) { return 256 * bits; }
__host__ __device__ inline int kl_chunk_bytes(int bits) { return bits == 8 ? 16 : 4 * bits; }  // per piece

// Order in which the 8 activations of a group are stored for the int8 GEMM (see the 8-bit note above).
__host__ __device__ inline int k8_perm(int p) { return ((p & 1) << 2) | (p >> 1); }  // 0,4,1,5,2,6,3,7

void set_hip_error(int e);

#define MQ_HIP_CHECK_LAUNCH()                       \
    do {                                            \
        hipError_t e__ = hipGetLastError();         \
        if (e__ != hipSuccess) {                    \
            mq::set_hip_error((int)e__);            \
            return MQ_ERR_HIP;                      \
        }                                           \
    } while (0)

// Activation parameters as the integer GEMM reads them (device memory, written by the quantise kernel).
struct ActParams {
    float scale;
    int32_t zp;
};

// Row view: logical row r of the activation matrix lives at physical row
//   (r / rows_per_group) * group_stride + r % rows_per_group + row_offset      (rows_per_group > 0)
// which expresses "tokens 1..T-1 of every prompt" without a gather; rows_per_group == 0 means identity.
struct RowMap {
    int rows_per_group;
    int group_stride;
    int row_offset;
    __host__ __device__ inline long phys(long r) const {
        if (rows_per_group <= 0) return r;
        return (r / rows_per_group) * (long)group_stride + (r % rows_per_group) + row_offset;
    }
};

// Division of a 32-bit unsigned number by a divisor that the host knows: the quotient estimate from the high half
// of t * floor(2^32 / d) is at most one too small (for any t < 2^32, d >= 1), which one comparison corrects.  An
// integer division in device code costs about forty instructions, and a kernel's prologue has several of them on its
// critical path.
struct FastDiv {
    uint32_t d, inv;
    static FastDiv make(uint32_t d_) {
        FastDiv f;
        f.d = d_ ? d_ : 1;
        f.inv = f.d == 1 ? 0xFFFFFFFFu : (uint32_t)((1ULL << 32) / f.d);
        return f;
    }
    __device__ inline void divmod(uint32_t t, uint32_t& q, uint32_t& r) const {
        q = __umulhi(t, inv);
        r = t - q * d;
        if (r >= d) {
            q += 1;
            r -= d;
        }
    }
};

// ---- launchers implemented in the .hip files (all validate nothing: api.cpp has done it) ----
int launch_quantize_weights(const void* w, int N, int K, int bits, int symmetric, int dtype, uint8_t* codes,
                            float* scale, int32_t* zp, hipStream_t st);
int launch_pack(const uint8_t* codes, int N, int K, int bits, int layout, int codes_signed, void* packed,
                int32_t* colsum, hipStream_t st);
int launch_unpack(const void* packed, int N, int K, int bits, int layout, uint8_t* codes, hipStream_t st);

// BOS rows of one BOS-aware K/V projection: ctx [B,T,K] fp16, unquantised weights [N,K] fp16 or the pre-computed
// vector [N] (exactly one of the two), optional bias, output [B,T,N] (only token 0 of each prompt is written).
struct BosWork {
    const _Float16* ctx;
    int B, T, K, N;
    const _Float16* w_f16;
    const _Float16* bos_out;
    const _Float16* bias;
    _Float16* y;
};

// Activation min/max partials -> parameters -> int8 copy (a' = code - 128, groups of 8 in k8_perm order)
// and per-row sums of a'.  bos (optional): BOS rows computed by extra workgroups of the quantise launch.
int launch_act_quant(const void* x, int M, int K, int ldx, RowMap in_map, const float* act_scale,
                     const int32_t* act_zp, int8_t* a8, int32_t* rowsum, ActParams* params, float* partials,
                     float* act_scale_out, int32_t* act_zp_out, const BosWork* bos, hipStream_t st,
                     int given_partials = 0);
int act_quant_partial_slots();

int launch_gemm_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, int bits,
                       const float* w_scale, const int32_t* w_zp, const void* bias, void* y, int ldy, int dtype,
                       const void* res, int ldr, void* split_ws, size_t split_ws_bytes, hipStream_t st);

int launch_gemm_a8(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                   const void* packed, int N, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                   const int32_t* w_colsum, const void* bias, void* y, int ldy, RowMap out_map, int32_t* acc_debug,
                   const void* res, int ldr, void* split_ws, size_t split_ws_bytes, hipStream_t st);

int launch_gemm_a8_geglu(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                         const void* packed, int H, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                         const int32_t* w_colsum, const void* bias, const float* out_scale, const int32_t* out_zp,
                         int8_t* a8_out, void* h16, int ldh, float* mm_out, int* mm_pairs, hipStream_t st);
int launch_gemm_w_only_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int bits,
                             const float* w_scale, const int32_t* w_zp, const void* bias, void* h16, int ldh,
                             const float* out_scale, const int32_t* out_zp, int8_t* a8_out, hipStream_t st);
int launch_gemm_a8_codes(const int8_t* a8, long lda, const float* act_scale, const int32_t* act_zp, int M, int K,
                         const void* packed, int N, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                         const int32_t* w_colsum, const void* bias, void* y, int ldy, int32_t* acc_debug,
                         const void* res, int ldr, hipStream_t st);

int launch_conv3x3_w_only(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int bits,
                          const float* w_scale, const int32_t* w_zp, const void* bias, void* y, const void* res,
                          hipStream_t st);
int launch_conv3x3_a8(const int8_t* a8, const ActParams* params, int B, int H, int W, int Cin, int stride, const void* packed, int N,
                      int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                      const int32_t* w_tapsum, const void* bias, void* y, int32_t* acc_debug, const void* res,
                      hipStream_t st);
int launch_tap_sums(const uint8_t* codes, int N, int Cin, int bits, int codes_signed, int32_t* tapsum, hipStream_t st);

void set_force_tile(int t);
void set_force_splits(int n);
int forced_splits();
void set_force_band(int n);
void set_phase_buffer(long long* p, long workgroups);

// ---- optional per-kernel event timing (prof.hip) ----
enum { PROF_GEMM_TILES = 7, PROF_GEMM_BITS = 5, PROF_GEMM_FAMILIES = 7, PROF_ACT_MINMAX = PROF_GEMM_FAMILIES * PROF_GEMM_BITS * PROF_GEMM_TILES, PROF_ACT_QUANTIZE, PROF_BOS_ROWS };
int prof_num_slots();
int prof_gemm_slot(int family /*0 weight-only fp16, 1 int8, 2 weight-only bf16, 3 int8 gated projection, 4 int8 on codes, 5 weight-only convolution, 6 int8 convolution*/,
                   int bits, int tile);
bool prof_enabled();
bool prof_wants(int slot);
int prof_filter(int slot, int stride);
void prof_name_slot(int slot, const char* name);
int prof_enable(int on);
bool prof_begin(hipStream_t st, hipEvent_t* a, hipEvent_t* b);
void prof_end(hipEvent_t a, hipEvent_t b, hipStream_t st, int slot, double ops, double bytes);
int prof_read(int slot, char* name, int name_cap, long long* launches, double* ms, double* ops, double* bytes);
int prof_reset();
double prof_bracket_overhead_us(hipStream_t st);
int prof_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
int prof_microbench(int kind, void* buf, size_t buf_bytes, double* ms_host, hipStream_t st);

struct ProfScope {
    bool open = false;
    hipEvent_t a, b;
    int slot;
    hipStream_t st;
    double ops, bytes;
    ProfScope(hipStream_t s, int slot_, double ops_, double bytes_) : slot(slot_), st(s), ops(ops_), bytes(bytes_) {
        if (prof_enabled() && prof_wants(slot)) open = prof_begin(st, &a, &b);
    }
    ~ProfScope() {
        if (open) prof_end(a, b, st, slot, ops, bytes);
    }
};

int launch_bos_rows(const BosWork& bw, hipStream_t st);

}  // namespace mq
