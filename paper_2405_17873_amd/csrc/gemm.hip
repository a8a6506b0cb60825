// MFMA GEMMs of the quantized-linear hot path for gfx950 (64-wide wavefronts, 32x32 MFMA tiles).
//
//   weight-only : Y = X . dequant(Wq)^T      fp16 / bf16 MFMA (v_mfma_f32_32x32x16_f16 / _bf16), fp32 accumulate
//                 (paper App. C item 2: weight-only layers keep 16-bit floating-point compute; also the layers kept
//                 at 16 bits, Sec. 4.2, whose weights pass unquantised)
//   int8        : ACC = A8 . W8^T            int8 MFMA (v_mfma_i32_32x32x32_i8), int32 accumulate
//                 (paper Sec. 4.3 / App. C item 4: integer GEMM for W8A8; 4-bit codes widened for W4A8)
// and, on the same skeleton, selected by the kernel's MODE: the gated feed-forward projection whose epilogue emits
// value * gelu(gate) as 8-bit codes or fp16, the int8 GEMM on activations that arrive as codes, and the 3x3
// convolution (Sec. 4.1: convolutions are quantised like linears) by addressing the filter taps in the activation loads.
//
// Shared structure
//   * One workgroup = WGM x WGN waves (x KS groups that split k); each wave owns TM x TN MFMA tiles of 32x32.
//   * Both operands go HBM -> LDS directly (buffer loads with the LDS bit: no staging registers) through a
//     pipeline of 2..8 LDS stages with hand-placed vmcnt waits and one barrier per stage; the hand-over to the
//     next stage sits in the middle of a stage, behind the MFMAs of its last two k-steps.
//   * Activations: 128 bytes of K per row per stage, 16-byte pieces XOR-swizzled (on the global side of the
//     copy) so that ds_read_b128 of 32 consecutive rows is conflict free.
//   * Weights stay PACKED in LDS: the kernel layout stores, for every 32-channel x 64-k tile, the 64 lane
//     chunks in lane order, so a tile is copied with one contiguous wave access and a lane later reads its own
//     chunk with one conflict-free ds_read; codes are widened in registers, right before the MFMA.
//   * The MFMA is issued with the weight fragment as the first operand: the 32x32 result then holds, per
//     lane, 4 consecutive output channels of one activation row; the epilogue transposes through LDS and stores
//     16-byte row segments.
//   * k-order inside a stage is permuted identically for both operands (a sum does not care), chosen so
//     that every lane's global and LDS accesses are 16 bytes wide.
//   * Few tiles and a long reduction: several workgroups per tile, partial sums through the caller's workspace,
//     the last-arriving workgroup adds them in a fixed order (no waiting).
//   * Optional residual operand (a skip connection, or the output of the other half of a split concatenated
//     input, Sec. 4.1): a kernel variant (RES) loads it in the accumulator layout and adds it in fp32 before the
//     one rounding; kernels without it contain none of this.
#include <stdio.h>

#include <mutex>
#include <type_traits>

#include "mq_common.h"

namespace mq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef int int16v __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));
typedef uint32_t uint3v __attribute__((ext_vector_type(3)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Swizzle of the 16-byte piece index inside a 128-byte LDS row.  Distinct over any 8 consecutive rows and,
// together with the row parity, over any 16 consecutive rows.
__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ half2v as_h2(uint32_t u) { return __builtin_bit_cast(half2v, u); }
__device__ __forceinline__ uint32_t h2_bits(half2v h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half2v splat(float v) {
    half2v r;
    r[0] = (_Float16)v;
    r[1] = (_Float16)v;
    return r;
}

// ---------------------------------------------------------------------------------------------
// Code -> fp16 widening.  0x6400 is 1024.0 in fp16; OR-ing a small integer into its mantissa gives
// 1024 + q (or 1024 + 2^s q for a field that sits s bits up), and one packed add or fma brings it to
// the exact integer q - z.  All intermediate values are integers below 2048, so nothing rounds.
// ---------------------------------------------------------------------------------------------
template <int BITS>
struct WChunk {
    static constexpr int WORDS = BITS == 8 ? 8 : BITS;  // 32-bit words per lane per 64-k tile (16: unquantised)
    uint32_t w[WORDS];
};

// (w & mask) | magic in one instruction.  The compiler emits v_and + v_or here, each with its own 32-bit literal: the
// three-operand form takes no literals on this target, so the mask is handed over in a scalar register and the magic
// number in a vector register (both loop invariant).  It is a third of the widening work of the 2/3/4-bit codes.
__device__ __forceinline__ uint32_t and_or(uint32_t w, uint32_t mask, uint32_t magic) {
    uint32_t r;
    asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(r) : "v"(w), "s"(mask), "v"(magic));
    return r;
}

template <int SHIFT>
__device__ __forceinline__ half2v field_to_h2(uint32_t w, uint32_t mask, int z) {
    // field value sits at bit SHIFT of each half: magic|field = 1024 + 2^SHIFT q
    const half2v v = as_h2(and_or(w, mask, 0x64006400u));
    if constexpr (SHIFT == 0) {
        return v - splat((float)(1024 + z));
    } else {
        constexpr float inv = 1.0f / (float)(1 << SHIFT);
        return v * splat(inv) - splat((float)((1024 >> SHIFT) + z));
    }
}

// Fragment for MFMA step s (8 consecutive k of this lane's 32): four half2 pairs.
template <int BITS>
__device__ __forceinline__ half8 dequant_step(const WChunk<BITS>& c, int s, int z);

template <>
__device__ __forceinline__ half8 dequant_step<4>(const WChunk<4>& c, int s, int z) {
    uint32_t w = c.w[s];
    half2v p0 = field_to_h2<0>(w, 0x000F000Fu, z);
    half2v p1 = field_to_h2<4>(w, 0x00F000F0u, z);
    w >>= 8;
    half2v p2 = field_to_h2<0>(w, 0x000F000Fu, z);
    half2v p3 = field_to_h2<4>(w, 0x00F000F0u, z);
    return half8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

template <>
__device__ __forceinline__ half8 dequant_step<2>(const WChunk<2>& c, int s, int z) {
    uint32_t w = c.w[s >> 1];
    if (s & 1) w >>= 8;
    half2v p0 = field_to_h2<0>(w, 0x00030003u, z);
    half2v p1 = field_to_h2<2>(w, 0x000C000Cu, z);
    half2v p2 = field_to_h2<4>(w, 0x00300030u, z);
    half2v p3 = field_to_h2<6>(w, 0x00C000C0u, z);
    return half8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// 3 bit: pair p (0..14) is field p%5 of word p/5; fields 0..2 are read in place, fields 3,4 after >> 9.
template <int F>
__device__ __forceinline__ half2v field3(uint32_t w, int z) {
    if constexpr (F == 0) return field_to_h2<0>(w, 0x00070007u, z);
    if constexpr (F == 1) return field_to_h2<3>(w, 0x00380038u, z);
    if constexpr (F == 2) return field_to_h2<6>(w, 0x01C001C0u, z);
    if constexpr (F == 3) return field_to_h2<0>(w >> 9, 0x00070007u, z);
    return field_to_h2<3>(w >> 9, 0x00380038u, z);
}

template <>
__device__ __forceinline__ half8 dequant_step<3>(const WChunk<3>& c, int s, int z) {
    half2v p0, p1, p2, p3;
    if (s == 0) {
        p0 = field3<0>(c.w[0], z);
        p1 = field3<1>(c.w[0], z);
        p2 = field3<2>(c.w[0], z);
        p3 = field3<3>(c.w[0], z);
    } else if (s == 1) {
        p0 = field3<4>(c.w[0], z);
        p1 = field3<0>(c.w[1], z);
        p2 = field3<1>(c.w[1], z);
        p3 = field3<2>(c.w[1], z);
    } else if (s == 2) {
        p0 = field3<3>(c.w[1], z);
        p1 = field3<4>(c.w[1], z);
        p2 = field3<0>(c.w[2], z);
        p3 = field3<1>(c.w[2], z);
    } else {
        p0 = field3<2>(c.w[2], z);
        p1 = field3<3>(c.w[2], z);
        p2 = field3<4>(c.w[2], z);
        const uint32_t t = ((c.w[0] >> 15) & 0x00010001u) | ((c.w[1] >> 14) & 0x00020002u) |
                           ((c.w[2] >> 13) & 0x00040004u);
        p3 = field_to_h2<0>(t, 0x00070007u, z);
    }
    return half8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// 8 bit: step s uses the two words of group (s & 1) in piece (s >> 1): bytes c0,c4,c1,c5 | c2,c6,c3,c7.
template <>
__device__ __forceinline__ half8 dequant_step<8>(const WChunk<8>& c, int s, int z) {
    const uint32_t wa = c.w[(s >> 1) * 4 + (s & 1) * 2], wb = c.w[(s >> 1) * 4 + (s & 1) * 2 + 1];
    const half2v zz = splat((float)(1024 + z));
    // v_perm_b32: selector bytes 0..3 pick bytes of the second source, 4..7 of the first
    half2v p0 = as_h2(__builtin_amdgcn_perm(0x64646464u, wa, 0x04020400u)) - zz;  // c0,c1
    half2v p1 = as_h2(__builtin_amdgcn_perm(0x64646464u, wb, 0x04020400u)) - zz;  // c2,c3
    half2v p2 = as_h2(__builtin_amdgcn_perm(0x64646464u, wa, 0x04030401u)) - zz;  // c4,c5
    half2v p3 = as_h2(__builtin_amdgcn_perm(0x64646464u, wb, 0x04030401u)) - zz;  // c6,c7
    return half8{p0[0], p0[1], p1[0], p1[1], p2[0], p2[1], p3[0], p3[1]};
}

// 16 bit: the weights are unquantised fp16 (or bf16) values, piece s is the operand of step s as it stands.
template <>
__device__ __forceinline__ half8 dequant_step<16>(const WChunk<16>& c, int s, int) {
    const uint4v v = {c.w[4 * s], c.w[4 * s + 1], c.w[4 * s + 2], c.w[4 * s + 3]};
    return __builtin_bit_cast(half8, v);
}

// bfloat16 variant: the widened weights are small integers (|q - z| <= 255), exact in fp16 and in bf16 alike, so
// the fp16 fragment is converted pair by pair: two fp16 -> fp32 conversions and one byte permute that keeps the
// upper halves (which for these values is the exact bf16).
__device__ __forceinline__ bf16x8 half8_to_bf16x8(half8 h) {
    uint4v o;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const uint32_t f0 = __float_as_uint((float)h[2 * p]), f1 = __float_as_uint((float)h[2 * p + 1]);
        o[p] = __builtin_amdgcn_perm(f1, f0, 0x07060302u);
    }
    return __builtin_bit_cast(bf16x8, o);
}

__device__ __forceinline__ float bf16_bits_to_float(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

// ---------------------------------------------------------------------------------------------
// Buffer addressing.  Both operands are read through buffer resources: a lane's offset is a 32-bit
// register computed once, the k advance is a scalar offset, and anything past the end of the buffer reads
// as zero instead of faulting (rows beyond M, the k padding of the int8 activation copy).
// ---------------------------------------------------------------------------------------------
typedef __attribute__((address_space(3))) void* lds_ptr_t;

// Raw buffer resource (stride 0): base address, byte extent, gfx9-family format word.
typedef int int4s __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4s make_rsrc(const void* p, uint32_t bytes) {
    const uint64_t a = (uint64_t)(uintptr_t)p;
    int4s r;
    r[0] = (int)(uint32_t)a;
    r[1] = (int)(uint32_t)((a >> 32) & 0xFFFFu);
    r[2] = (int)bytes;
    r[3] = 0x00020000;
    // the descriptor is wave-uniform: keep it in scalar registers
    r[0] = __builtin_amdgcn_readfirstlane(r[0]);
    r[1] = __builtin_amdgcn_readfirstlane(r[1]);
    r[2] = __builtin_amdgcn_readfirstlane(r[2]);
    return r;
}

// 16 bytes per lane from the buffer straight into LDS: lane L of the wave writes lds_wave_base + 16 * L; a lane
// whose offset lies past the end of the buffer writes zeros.  Issued as inline assembly on purpose: the compiler
// would otherwise order every later LDS read behind ALL pending loads of this kind (it cannot tell the stage being
// filled from the stage being read), which serialises the pipeline.  The waits are placed by hand (vmcnt below).
__device__ __forceinline__ void dma_to_lds_b128(int4s rsrc, uint32_t lds_wave_base, int voff, int soff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dwordx4 %1, %2, %3 offen lds"
        :
        : "s"(lds_wave_base), "v"(voff), "s"(rsrc), "s"(soff)
        : "memory");  // m0 is a reserved register: the compiler rewrites it before each of its own uses
}

// The same for 4 bytes per lane (256 contiguous bytes per wave).
__device__ __forceinline__ void dma_to_lds_b32(int4s rsrc, uint32_t lds_wave_base, int voff, int soff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "buffer_load_dword %1, %2, %3 offen lds"
        :
        : "s"(lds_wave_base), "v"(voff), "s"(rsrc), "s"(soff)
        : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// A lane's chunk of one 64-k weight tile, read from the tile's LDS copy (lane order, so consecutive lanes read
// consecutive addresses).
template <int BITS>
__device__ __forceinline__ void read_chunk(WChunk<BITS>& c, const uint8_t* tile, int lane) {
    if constexpr (BITS == 4) {
        const uint4v v = *(const uint4v*)(tile + lane * 16);
        c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3];
    } else if constexpr (BITS == 2) {
        const uint2v v = *(const uint2v*)(tile + lane * 8);
        c.w[0] = v[0]; c.w[1] = v[1];
    } else if constexpr (BITS == 3) {
        const uint32_t* p = (const uint32_t*)(tile + lane * 12);
        c.w[0] = p[0]; c.w[1] = p[1]; c.w[2] = p[2];
    } else if constexpr (BITS == 16) {
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4v v = *(const uint4v*)(tile + s * 1024 + lane * 16);
            c.w[4 * s] = v[0]; c.w[4 * s + 1] = v[1]; c.w[4 * s + 2] = v[2]; c.w[4 * s + 3] = v[3];
        }
    } else {
        const uint4v v0 = *(const uint4v*)(tile + lane * 16);
        const uint4v v1 = *(const uint4v*)(tile + 1024 + lane * 16);
        c.w[0] = v0[0]; c.w[1] = v0[1]; c.w[2] = v0[2]; c.w[3] = v0[3];
        c.w[4] = v1[0]; c.w[5] = v1[1]; c.w[6] = v1[2]; c.w[7] = v1[3];
    }
}

// xflip = 0x80808080 turns unsigned 8-bit codes q into the signed bytes q - 128 (0 for signed codes).
template <int WBITS>
__device__ __forceinline__ int4v widen_step(const WChunk<WBITS>& c, int s /*0..1 inside the 64-k tile*/,
                                            uint32_t xflip) {
    if constexpr (WBITS == 8) {
        return int4v{(int)(c.w[4 * s] ^ xflip), (int)(c.w[4 * s + 1] ^ xflip), (int)(c.w[4 * s + 2] ^ xflip),
                     (int)(c.w[4 * s + 3] ^ xflip)};
    } else if constexpr (WBITS == 2) {
        // Word s holds codes 16s..16s+15, pair (c[2p], c[2p+1]) in bits [2p, 2p+2) and [16+2p, 16+2p+2):
        // (w >> 2t) & 0x03030303 = bytes c[2t], c[2t+8], c[2t+1], c[2t+9].  The activations of a group of 8 sit in
        // the order 0,4,1,5,2,6,3,7: two byte permutes per pair of extracts put the codes in that order.
        const uint32_t w = c.w[s];
        const uint32_t e0 = w & 0x03030303u, e1 = (w >> 2) & 0x03030303u, e2 = (w >> 4) & 0x03030303u,
                       e3 = (w >> 6) & 0x03030303u;
        // v_perm_b32: selector bytes 0..3 pick bytes of the second source, 4..7 of the first
        return int4v{(int)__builtin_amdgcn_perm(e2, e0, 0x06020400u),   // c0,c4,c1,c5
                     (int)__builtin_amdgcn_perm(e3, e1, 0x06020400u),   // c2,c6,c3,c7
                     (int)__builtin_amdgcn_perm(e2, e0, 0x07030501u),   // c8,c12,c9,c13
                     (int)__builtin_amdgcn_perm(e3, e1, 0x07030501u)};  // c10,c14,c11,c15
    } else {
        const uint32_t w0 = c.w[2 * s], w1 = c.w[2 * s + 1];
        return int4v{(int)(w0 & 0x0F0F0F0Fu), (int)((w0 >> 4) & 0x0F0F0F0Fu), (int)(w1 & 0x0F0F0F0Fu),
                     (int)((w1 >> 4) & 0x0F0F0F0Fu)};
    }
}

// ---------------------------------------------------------------------------------------------
// GELU of the gated feed-forward epilogue: gelu(g) = 0.5 g (1 + erf(g / sqrt 2)), single fp32 operations without
// contraction, library call or division, with erf(x) = 1 - exp(-x P(x)) on [0, 4.3] (x is held at 4.3 beyond), P a
// degree-6 polynomial fitted to -ln(erfc(x)) / x (error of the fit below 2e-7), and the exponential by the hardware's
// 2^t instruction (1 ulp, i.e. 1.2e-7 of a value that is at most 1; the rounding of its argument, at most 30 in
// magnitude, matters only where exp(-t) is below 1e-8): |error of erf| < 3e-7.  A range reduction with a degree-6
// polynomial in its place costs twelve more instructions per element: the gated feed-forward pair runs 2 to 3 %
// slower with it.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float gelu32(float g) {
    const float x = fminf(__fmul_rn(fabsf(g), 0.70710678f), 4.3f);
    float p = -5.95750535e-05f;
    p = __fmaf_rn(p, x, 0.000253331062f);
    p = __fmaf_rn(p, x, 0.00176583871f);
    p = __fmaf_rn(p, x, -0.0206223261f);
    p = __fmaf_rn(p, x, 0.103378408f);
    p = __fmaf_rn(p, x, 0.636503041f);
    p = __fmaf_rn(p, x, 1.12838686f);
    const float e = __builtin_amdgcn_exp2f(__fmul_rn(__fmul_rn(p, x), -1.44269504f));  // v_exp_f32: 2^t, 1 ulp
    const float erf_g = copysignf(__fsub_rn(1.0f, e), g);
    return __fmul_rn(__fmul_rn(0.5f, g), __fadd_rn(1.0f, erf_g));
}

// ---------------------------------------------------------------------------------------------
// The GEMM kernel.  I8 == false: weight-only, fp16 activations straight from X, 64 k per stage.
//                   I8 == true : int8 activation copy (row stride Kp = K rounded up to 128, padding zero),
//                                128 k per stage = two 64-k weight tiles.
// A stage of the activation operand is BM rows x 128 bytes.  It is brought in by buffer loads that write LDS
// directly (each lane 16 bytes, a wave instruction fills 8 rows), XOR-swizzled on the global side so that the
// later ds_read_b128 of 32 consecutive rows is conflict free.  S LDS stages rotate; the loads of the next S-1 stages
// are in flight while a stage is multiplied.
// ---------------------------------------------------------------------------------------------
struct GemmArgs {
    const void* a;        // X fp16 [M, lda] or int8 copy [M, Kp]
    long a_row_bytes;     // byte stride between rows of a
    uint32_t a_bytes;     // valid extent of a in bytes
    const uint8_t* packed;
    uint32_t packed_bytes;
    int M, N, K;          // K: true reduction length
    int k_stages;         // number of 128-byte stages
    const float* w_scale;
    const int32_t* w_zp;
    const uint16_t* bias;  // fp16 or bf16 bits
    uint16_t* y;
    long ldy;
    int tiles_m, tiles_n;
    int band_rows;        // row blocks per band of the workgroup -> tile map (>= 1)
    FastDiv fd_band_tiles, fd_band_rows, fd_last_rows;  // divisors of that map: tiles per band, rows of a band, of the last
    FastDiv fd_splits;
    int kt_q, kt_r;       // pipeline stages per part of a split reduction: kt_q, and one more for the first kt_r parts
    // int8 only
    const int32_t* rowsum;
    const ActParams* params;
    const int32_t* w_colsum;
    int w_off;
    long long* phase_clk;  // optional: 4 shader-clock samples per workgroup (start, loop, epilogue, end)
    RowMap out_map;
    int32_t* acc_debug;
    // split of the reduction over `splits` workgroups per tile (1 = none): partial accumulators in `partial`
    // ([tile][split][BM * BN] 4-byte values, register order), one arrival counter per tile (cleared before the launch)
    int splits;
    uint32_t* partial;
    uint32_t* counters;
    // (host side only) the caller's workspace that partial sums and counters are carved from; may be null
    void* split_ws;
    size_t split_ws_bytes;
    // MODE 1 (gated feed-forward projection, 8-bit output): N = 2H weight rows; codes of the gated product go to
    // a8_out (row stride ld8 bytes, the int8 activation layout), optionally the product itself as fp16 to y
    const float* out_scale_p;
    const int32_t* out_zp_p;
    int8_t* a8_out;
    // optional (int8 gated projection): one (min, max) pair per workgroup over the fp16 gated products it wrote
    float* mm_out;
    long ld8;
    // MODE 2 (activations arrive as int8 codes): their parameters; row sums are taken inside the main loop
    const float* act_scale_p;
    const int32_t* act_zp_p;
    // MODE 3 / 4 (3x3 convolution, stride 1, zero padding 1, channels-last): a is the [B*H*W, Cin] activation tensor
    // (a_row_bytes per pixel), K = 9 * Cin, row m is output pixel m; the k order is (filter row, filter column, c)
    int conv_h, conv_w;      // input image
    int conv_ho, conv_wo;    // output image: (H - 1) / stride + 1, likewise W; M = B * conv_ho * conv_wo
    int conv_stride;         // 1 or 2: output pixel (i, j) is centred on input pixel (stride * i, stride * j)
    int conv_cpt;            // 64-channel chunks per filter tap (Cin / 64)
    uint32_t conv_cpt_inv;   // ceil(2^32 / conv_cpt) for conv_cpt > 1
    const int32_t* w_tapsum; // MODE 4: [9][N] sums of the weight codes per filter tap
    // optional residual [M, ldr] (16-bit, the dtype of y; rows as the rows of y): added in fp32 before the rounding
    const uint16_t* res;
    long ldr;
};

// Workgroup id -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each with its own L2),
// so the ids an XCD receives are mapped onto a contiguous run of tiles.  The run walks the tile grid in bands of
// `band_rows` row blocks, inside a band column by column: the workgroups an XCD runs at the same time then cover
// band_rows row blocks times a few column blocks, the band's activation rows stay in that L2 while the band walks
// along N, and every weight tile is fetched once per band instead of once per row block.
__device__ __forceinline__ void tile_of_block(int bid, const GemmArgs& g, int& bm, int& bn) {
    const int total = g.tiles_m * g.tiles_n;
    const int per = total >> 3;  // tiles of the leftover (total % 8) keep their own index
    const uint32_t t = (uint32_t)(bid < (per << 3) ? (bid & 7) * per + (bid >> 3) : bid);
    uint32_t band, r, col, row;
    g.fd_band_tiles.divmod(t, band, r);
    const int first = (int)band * g.band_rows;
    if (g.tiles_m - first < g.band_rows)  // (the last band may be lower)
        g.fd_last_rows.divmod(r, col, row);
    else
        g.fd_band_rows.divmod(r, col, row);
    bn = (int)col;
    bm = first + (int)row;
}

// LDS plan of one workgroup: S stages, each KS sub-stages of [activation tile BM x 128 B][weight tiles]; a 1 KB sink
// for padding loads; the per-channel epilogue constants.  The accumulator exchange (KS == 2) and the epilogue staging
// reuse the stages.
//
// KS == 2 splits the reduction inside the workgroup: a second group of WGM x WGN waves works on the same output
// tile and takes every other 128-byte k step.  It is for problems with few tiles: a compute unit then still has two
// waves per SIMD to alternate between while fragments travel from LDS, without any extra global traffic; the two
// accumulator sets meet once, through LDS, before the epilogue.
template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int S, int KS>
struct GemmPlan {
    static constexpr int NWG = WGM * WGN;                     // waves of one group
    static constexpr int NW = NWG * KS, NT = NW * 64;
    static constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    static constexpr int CH = I8 ? 2 : 1;                     // 64-k weight tiles per 128-byte k step
    static constexpr int A_BYTES = BM * 128;
    static constexpr int BSLOT = BITS == 16 ? 4096 : BITS == 8 ? 2048 : 1024;  // LDS slot of one weight tile
    static constexpr int PIECES = BITS == 16 ? 4 : BITS == 8 ? 2 : 1;           // 1 KB wave loads per weight tile
    static constexpr int NBT = (BN / 32) * CH;                // weight tiles per sub-stage
    static constexpr int B_BYTES = NBT * BSLOT;
    static constexpr int SUB_BYTES = A_BYTES + B_BYTES;
    static constexpr int STAGE_BYTES = KS * SUB_BYTES;
    static constexpr int NAI = KS * (BM / 8);                 // LDS-writing loads per stage, activations
    static constexpr int DMA_A = NAI / NW;                    // ... per wave
    static constexpr int NBI1 = NBT * PIECES;                 // LDS-writing loads per sub-stage, weights
    static constexpr int NBI = KS * NBI1;
    static constexpr int DMA_B = (NBI + NW - 1) / NW;         // per wave (padded with loads into the sink)
    static constexpr int OPS = DMA_A + DMA_B;                 // vector-memory operations per wave per stage
    static constexpr int SINK = S * STAGE_BYTES;
    static constexpr int CONSTS = SINK + 1024;
    static constexpr int LDS_BYTES = CONSTS + BN * 16;
    static_assert(NAI % NW == 0, "tile rows must split over the waves");
};

// MODE 0: Y = linear(X).  MODE 1 (int8, two channel tiles per wave): gated feed-forward projection; the wave's first
// channel tile is a value tile, its second the gate tile of the same 32 columns, and the epilogue emits
// value * gelu(gate) as 8-bit codes for the next integer GEMM.  MODE 2 (int8): the activations arrive as codes with
// their parameters; the row sums the epilogue needs are accumulated in the main loop.  MODE 3 / 4: 3x3 convolution
// (16-bit / 8-bit activations).  MODE 5 (int8): the gated projection of MODE 1 without output parameters: it writes
// the fp16 product and one (min, max) pair per workgroup, from which the codes follow in a pass of their own.
// MODE 6 (16-bit activations): the gated projection of the weight-only path with MODE 1's 8-bit output.
template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int S, int KS, bool BF = false, int MODE = 0,
          bool RES = false>
__global__ __launch_bounds__(WGM* WGN* KS * 64,
                             (TM * TN <= 8 && GemmPlan<I8, BITS, WGM, WGN, TM, TN, S, KS>::LDS_BYTES <= 80 * 1024) ? 2 : 1)
void gemm_kernel(const GemmArgs g) {
    static_assert(!(I8 && BF), "the int8 path writes fp16");
    constexpr bool GEGLU = MODE == 1 || MODE == 5 || MODE == 6, RS_INLINE = MODE == 2 || MODE == 4, CONV = MODE == 3 || MODE == 4;
    constexpr bool RANGE = MODE == 5;    // gated projection that leaves the fp16 product and its range, no codes
    constexpr bool CODES16 = MODE == 6;  // gated projection of the 16-bit-activation path that emits 8-bit codes
    static_assert(MODE == 0 || KS == 1, "the special modes have no in-workgroup k split");
    static_assert(!(RES && GEGLU), "the gated projection takes no residual");
    static_assert(!RANGE || (I8 && !BF), "the range output belongs to the int8 gated projection");
    static_assert(!CODES16 || (!I8 && !BF), "MODE 6 is the fp16 weight-only gated projection with 8-bit output");
    static_assert((MODE != 2 && MODE != 4) || I8, "int8 modes");
    static_assert(MODE != 3 || !I8, "MODE 3 is the weight-only convolution");
    static_assert(!GEGLU || TN == 2, "value tile and gate tile per wave");
    using P = GemmPlan<I8, BITS, WGM, WGN, TM, TN, S, KS>;
    constexpr int NW = P::NW, NT = P::NT, BM = P::BM, BN = P::BN, CH = P::CH;
    constexpr int STAGE_BYTES = P::STAGE_BYTES;
    using acc_t = typename std::conditional<I8, int16v, float16v>::type;
    using frag_t = typename std::conditional<I8, int4v, half8>::type;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int grp = wv / P::NWG, wvg = wv % P::NWG;  // k-split group, wave inside the group
    const int wm = wvg / WGN, wn = wvg % WGN;
    int bm, bn;
    // (the large wave tile has no registers to spare for the split of the reduction over workgroups, and no use
    // for it: its problems have hundreds of tiles)
    constexpr bool CAN_SPLIT = TM * TN <= 4 && MODE == 0;
    const int splits = CAN_SPLIT ? g.splits : 1;
    uint32_t tile_u = blockIdx.x, sp_u = 0;  // sp: which part of the reduction this workgroup takes
    if (splits > 1) g.fd_splits.divmod(blockIdx.x, tile_u, sp_u);
    const int tile_id = (int)tile_u, sp = (int)sp_u;
    tile_of_block(tile_id, g, bm, bn);
    // n0: first output column of the workgroup (MODE 1: first gated column; it covers BN / 2 of them)
    const int m0 = bm * BM, n0 = GEGLU ? bn * (BN / 2) : bn * BN;
    const int KC = g.K >> 6;
    const int G = (g.N + 31) >> 5;
    const int H = g.N >> 1;  // MODE 1: gated columns
    // local 32-channel group (wave column * TN + channel tile) -> group of weight rows, clamped to an existing one
    auto group_of = [&](int gt) {
        int gi = GEGLU ? ((gt % TN) ? (H >> 5) : 0) + (n0 >> 5) + gt / TN : (n0 >> 5) + gt;
        return gi < G ? gi : G - 1;
    };
    const int l31 = lane & 31, kb = lane >> 5;
    const uint32_t xflip = (I8 && g.w_off) ? 0x80808080u : 0u;
    constexpr int TILE_B = 256 * BITS;
    constexpr int OOB = 0x7FFFF000;  // an offset past the end of any buffer this library accepts

    const int4s ra = make_rsrc(g.a, g.a_bytes);
    const int4s rb = make_rsrc(g.packed, g.packed_bytes);
    const uint32_t lds_base = (uint32_t)(uintptr_t)lds;

    // activation loads: lane -> (row, physical slot) of an 8-row group; it fetches the logical piece slot ^ swz(row).
    // Rows past M get an offset past the end of the buffer and therefore read as zero.
    int a_voff[P::DMA_A];
    uint32_t a_lds[P::DMA_A];
    int a_sub[KS == 2 ? P::DMA_A : 1];  // k-split tiles: which of the stage's two k steps the load belongs to
    int a_half[CONV ? P::DMA_A : 1];
    uint32_t a_taps[CONV ? P::DMA_A : 1];
    // convolution: which of the 9 filter taps (bit r * 3 + s) of output pixel m read inside the image
    auto tap_mask = [&](int m) -> uint32_t {
        if (m >= g.M) return 0u;
        const int j = (m % g.conv_wo) * g.conv_stride, i = ((m / g.conv_wo) % g.conv_ho) * g.conv_stride;
        const uint32_t rows = (i > 0 ? 1u : 0u) | 2u | (i + 1 < g.conv_h ? 4u : 0u);
        const uint32_t cols = (j > 0 ? 1u : 0u) | 2u | (j + 1 < g.conv_w ? 4u : 0u);
        uint32_t mk = 0;
#pragma unroll
        for (int r = 0; r < 3; ++r)
            if (rows >> r & 1u) mk |= cols << (3 * r);
        return mk;
    };
#pragma unroll
    for (int i = 0; i < P::DMA_A; ++i) {
        const int j = i * NW + wv;
        const int sub = j / (BM / 8), row0 = (j % (BM / 8)) * 8;
        const int row = row0 + (lane >> 3);
        const int piece = (lane & 7) ^ swz(row);
        a_voff[i] = m0 + row < g.M ? (int)((long)(m0 + row) * g.a_row_bytes + sub * 128 + piece * 16) : OOB;
        if constexpr (KS == 2) a_sub[i] = sub;
        a_lds[i] = __builtin_amdgcn_readfirstlane((uint32_t)(sub * P::SUB_BYTES + row0 * 128));
        if constexpr (CONV) {
            // row = output pixel; the lane's 16 bytes of a stage lie in one 64-channel chunk (int8: piece / 4 says
            // which of the stage's two), i.e. in one filter tap: per stage it adds that tap's pixel offset, or
            // reads nothing (zero) where the tap falls outside the image
            const int mo = m0 + row < g.M ? m0 + row : g.M - 1;  // (rows past M read nothing: their tap mask is empty)
            const int per_image = g.conv_ho * g.conv_wo;
            const int bi = mo / per_image, rem = mo - bi * per_image;
            const int io = rem / g.conv_wo, jo = rem - io * g.conv_wo;
            const long centre = ((long)bi * g.conv_h + io * g.conv_stride) * g.conv_w + jo * g.conv_stride;
            a_voff[i] = (int)(centre * g.a_row_bytes) + (I8 ? (piece & 3) : piece) * 16;
            a_half[i] = I8 ? piece >> 2 : 0;
            a_taps[i] = tap_mask(m0 + row);
        }
    }
    // weight loads: instruction jj of a sub-stage copies piece jj % PCS of weight tile jj / PCS (tile = channel group,
    // chunk)
    constexpr int PCS = P::PIECES;
    constexpr int VALID_LANES = BITS >= 8 ? 64 : 16 * BITS;  // lanes of a 16-byte-per-lane copy that hold tile data
    int b_voff[P::DMA_B];
    uint32_t b_lds[P::DMA_B];
    constexpr bool B_TAIL = I8 || KS == 2;  // a stage may reach past the last 64-k weight tile of the reduction
    int b_chunk[B_TAIL ? P::DMA_B : 1];     // the load's 64-k tile inside its stage
#pragma unroll
    for (int i = 0; i < P::DMA_B; ++i) {
        const int j = i * NW + wv;
        const int sub = j / P::NBI1, jj = j % P::NBI1;
        const int t = jj / PCS, piece = jj % PCS;
        const int gt = t / CH, cc = t % CH;
        const int gi = group_of(gt);
        const bool on = j < P::NBI && lane < VALID_LANES;
        b_voff[i] = on ? (gi * KC + sub * CH + cc) * TILE_B + piece * 1024 + lane * 16 : OOB;
        if constexpr (B_TAIL) b_chunk[i] = sub * CH + cc;
        b_lds[i] = __builtin_amdgcn_readfirstlane(
            j < P::NBI ? (uint32_t)(sub * P::SUB_BYTES + P::A_BYTES + t * P::BSLOT + piece * 1024) : (uint32_t)0xFFFFFFFFu);
    }

    // Weight zero points of the 16-bit-activation path (the int8 path corrects for them in the epilogue): an ordinary
    // load here would be waited for by the compiler with a count that ignores the LDS-writing loads, i.e. until all
    // prologue stages have landed.  So the zero points of the workgroup's channels travel like a stage: one
    // LDS-writing load per 64 channels, issued first (the oldest entry of the counter), into the slot that the int8
    // epilogue uses for its own constants; every lane picks its channel's value up after the first barrier.
    constexpr bool ZP_LDS = !I8 && BITS != 16;
    constexpr int ZP_SLOT = P::CONSTS + 2 * BN * 4;
    if constexpr (ZP_LDS) {
        if (wv < BN / 64) {
            const int ch = wv * 64 + lane;
            int n = group_of(ch >> 5) * 32 + (ch & 31);
            n = n < g.N ? n : g.N - 1;
            const int4s rz = make_rsrc(g.w_zp, (uint32_t)g.N * 4u);
            dma_to_lds_b32(rz, __builtin_amdgcn_readfirstlane(lds_base + ZP_SLOT + wv * 256), n * 4, 0);
        }
    }
    int zc[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) zc[tn] = 0;

    // Without an in-workgroup k split every wave's first k step exists, so its MFMAs take the constant zero as their
    // third operand and the accumulators need no clearing (16 vector instructions per MFMA tile otherwise).
    constexpr bool ZERO_C = KS == 1 && !CONV;  // (the convolution kernels have no registers to spare for the second copy of step 0)
    acc_t acc[TM][TN];
    if constexpr (!ZERO_C) {
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;
    }

    // Per-channel epilogue inputs of the workgroup's BN channels: thread t fetches those of channel n0 + t now and
    // keeps them in registers; they are combined and parked in LDS after the loop.  These ordinary loads are issued
    // BEFORE the first LDS-writing load, so that they are the oldest entries of the vector-memory counter and the
    // hand-counted waits below see only the stage loads behind them.
    static_assert(BN <= NT, "one thread per channel");
    float c_scale = 0.0f;
    uint32_t c_bias_bits = 0;  // converted where it is used, after the loop: a conversion here would wait for the load
    int c_zp = 0, c_colsum = 0;
    // (the activation parameters are the same for every thread: loaded outside the divergent branch they stay in
    // scalar registers, and nothing waits for them before the epilogue)
    float c_sx = 1.0f;
    int c_zx = 0;
    if constexpr (I8) {
        c_sx = RS_INLINE ? *g.act_scale_p : g.params->scale;
        c_zx = RS_INLINE ? *g.act_zp_p : g.params->zp;
    }
    if (threadIdx.x < BN) {
        int n = group_of((int)threadIdx.x >> 5) * 32 + ((int)threadIdx.x & 31);
        n = n < g.N ? n : g.N - 1;
        c_scale = BITS == 16 ? 1.0f : g.w_scale[n];
        if (g.bias) c_bias_bits = g.bias[n];
        if constexpr (I8) {
            c_zp = g.w_zp[n];
            c_colsum = g.w_colsum[n];
        }
    }
    int rsum[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = m0 + (wm * TM + tm) * 32 + l31;
        rsum[tm] = (I8 && !RS_INLINE) ? g.rowsum[m < g.M ? m : g.M - 1] : 0;
    }

    // Every wave issues exactly OPS loads per stage (padding loads go to the sink), so that "at most n * OPS loads
    // outstanding" means "all but the n youngest stages have landed" for every wave alike.
    const int KSTEPS = g.k_stages;                // 128-byte k steps
    const int KT_ALL = (KSTEPS + KS - 1) / KS;    // pipeline stages of the whole reduction
    const int kt0 = splits > 1 ? sp * g.kt_q + (sp < g.kt_r ? sp : g.kt_r) : 0;
    const int KT = splits > 1 ? g.kt_q + (sp < g.kt_r ? 1 : 0) : KT_ALL;  // ... of this workgroup
    // The k advance of a stage travels in the load's scalar offset, which the hardware leaves out of its range check
    // (only the lane's own offset is compared with the extent of the buffer).  The last stage may hold a 64-k weight
    // tile or (k-split tiles) a whole k step that does not exist: int8 stages are two weight tiles long and K / 64 may
    // be odd, a k-split stage is two k steps long and their number may be odd.  Loads of such phantom pieces get the
    // out-of-range lane offset, so nothing outside the operands is ever addressed.
    auto issue = [&](int stage, int buf) {
        const int step0 = (kt0 + stage) * KS;  // first k step of the stage
        const int soff_a = __builtin_amdgcn_readfirstlane(step0 * 128);
        const int soff_b = __builtin_amdgcn_readfirstlane(step0 * CH * TILE_B);
        const uint32_t sb = lds_base + buf * STAGE_BYTES;
        const bool tail_a = KS == 2 && step0 + 1 >= KSTEPS;
        const bool tail_b = B_TAIL && (step0 + KS) * CH > KC;
        if constexpr (CONV) {
            // the stage's 64-channel chunks -> (filter tap, chunk inside the tap) -> byte offset from the output pixel
            int tap[CH], delta[CH];
#pragma unroll
            for (int h = 0; h < CH; ++h) {
                const uint32_t ci = (uint32_t)(kt0 + stage) * CH + h;
                const uint32_t t = g.conv_cpt > 1 ? __umulhi(ci, g.conv_cpt_inv) : ci;
                const int cc = (int)(ci - t * g.conv_cpt);
                tap[h] = ci < (uint32_t)KC ? (int)t : 31;  // past the end of K (int8 padding of the last stage): no tap
                delta[h] = (((int)t / 3 - 1) * g.conv_w + ((int)t % 3 - 1)) * (int)g.a_row_bytes + cc * (I8 ? 64 : 128);
            }
#pragma unroll
            for (int i = 0; i < P::DMA_A; ++i) {
                const int t = CH == 2 && a_half[i] ? tap[CH - 1] : tap[0];
                const int d = CH == 2 && a_half[i] ? delta[CH - 1] : delta[0];
                const int voff = (a_taps[i] >> t) & 1u ? a_voff[i] + d : OOB;
                dma_to_lds_b128(ra, __builtin_amdgcn_readfirstlane(sb + a_lds[i]), voff, 0);
            }
        } else if (tail_a) {
            if constexpr (KS == 2) {
#pragma unroll
                for (int i = 0; i < P::DMA_A; ++i)
                    dma_to_lds_b128(ra, __builtin_amdgcn_readfirstlane(sb + a_lds[i]),
                                    step0 + a_sub[i] < KSTEPS ? a_voff[i] : OOB, soff_a);
            }
        } else {
#pragma unroll
            for (int i = 0; i < P::DMA_A; ++i)
                dma_to_lds_b128(ra, __builtin_amdgcn_readfirstlane(sb + a_lds[i]), a_voff[i], soff_a);
        }
        if (tail_b) {
            if constexpr (B_TAIL) {
#pragma unroll
                for (int i = 0; i < P::DMA_B; ++i)
                    dma_to_lds_b128(rb, __builtin_amdgcn_readfirstlane(b_lds[i] == 0xFFFFFFFFu ? lds_base + P::SINK : sb + b_lds[i]),
                                    step0 * CH + b_chunk[i] < KC ? b_voff[i] : OOB, soff_b);
            }
        } else {
#pragma unroll
            for (int i = 0; i < P::DMA_B; ++i)
                dma_to_lds_b128(rb, __builtin_amdgcn_readfirstlane(b_lds[i] == 0xFFFFFFFFu ? lds_base + P::SINK : sb + b_lds[i]),
                                b_voff[i], soff_b);
        }
    };

    // LDS read offsets of this lane: row l31 of the wave's first tile, one register per MFMA step
    const int sw = swz(l31);
    uint32_t rd[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int piece = I8 ? ((s >> 1) * 4 + kb * 2 + (s & 1)) : (kb * 4 + s);
        rd[s] = (uint32_t)(wm * TM * 32 * 128 + l31 * 128 + ((piece ^ sw) << 4));
    }

    long long t0 = 0, t1 = 0, t2 = 0;
    if (g.phase_clk) t0 = clock64();
#pragma unroll
    for (int s = 0; s < S; ++s)
        if (s < KT) issue(s, s);
    if (g.phase_clk) t1 = clock64();

    // Main loop.  A 32-cycle MFMA leaves room for about five vector ALU instructions on its SIMD (measured: four
    // behind every MFMA cost nothing, eight cost 37 % more time than the MFMAs alone), and a workgroup has one wave
    // per SIMD, so the widening work is spread between the MFMAs and every latency is covered by the wave's own MFMAs:
    //   * the activation fragments of steps 1..3 are requested one or two steps ahead (four register sets);
    //   * the hand-over to the next stage (wait for its loads, barrier, refill of the buffer just read, request of
    //     its first fragments) sits in the MIDDLE of a stage, after the last LDS read of the current stage has
    //     returned and before the MFMAs of steps 2 and 3, which then run while the barrier settles and the first
    //     fragments of the next stage travel.
    WChunk<BITS> wq[TN][CH];
    frag_t xf[4][TM];
    auto request_first = [&](const uint8_t* abuf) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int c = 0; c < CH; ++c)
                read_chunk<BITS>(wq[tn][c], abuf + P::A_BYTES + ((wn * TN + tn) * CH + c) * P::BSLOT, lane);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[0][tm] = *(const frag_t*)(abuf + rd[0] + tm * 32 * 128);
    };
    auto widen = [&](frag_t (&wf)[TN], int s) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            if constexpr (I8)
                wf[tn] = widen_step<BITS>(wq[tn][s >> 1], s & 1, xflip);
            else
                wf[tn] = dequant_step<BITS>(wq[tn][0], s, zc[tn]);
            if constexpr (BF && BITS != 16) wf[tn] = __builtin_bit_cast(half8, half8_to_bf16x8(wf[tn]));  // bf16 bits now
        }
    };
    auto multiply = [&](const frag_t (&wf)[TN], int s, auto fresh_c) {
        constexpr bool FRESH = decltype(fresh_c)::value;  // the accumulators start here: C = 0
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                acc_t c;
                if constexpr (FRESH) {
#pragma unroll
                    for (int i = 0; i < 16; ++i) c[i] = 0;
                } else {
                    c = acc[tm][tn];
                }
                if constexpr (I8)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[tn], xf[s][tm], c, 0, 0, 0);
                else if constexpr (BF)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, wf[tn]), __builtin_bit_cast(bf16x8, xf[s][tm]), c, 0, 0, 0);
                else
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[tn], xf[s][tm], c, 0, 0, 0);
            }
        if constexpr (RS_INLINE) {  // this lane's share of the row sums of the stored activations (bytes a' = code - 128)
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int4v a = __builtin_bit_cast(int4v, xf[s][tm]);
#pragma unroll
                for (int i = 0; i < 4; ++i) rsum[tm] = __builtin_amdgcn_sdot4(a[i], 0x01010101, rsum[tm], false);
            }
        }
    };

    // stage 0 must have landed; the younger stages stay in flight
    constexpr int W_FIRST = (S - 1) * P::OPS <= 63 ? (S - 1) * P::OPS : (S > 2 ? (S - 2) * P::OPS : 0);
    if (KT >= S)
        wait_vmcnt<W_FIRST>();
    else
        wait_vmcnt<0>();
    __syncthreads();
    if constexpr (ZP_LDS) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) zc[tn] = *(const int*)(lds + ZP_SLOT + ((wn * TN + tn) * 32 + l31) * 4);
    }
    request_first(lds + grp * P::SUB_BYTES);

    int buf = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const uint8_t* abuf = lds + buf * STAGE_BYTES + grp * P::SUB_BYTES;
        // odd tail of a k-split: the last k step of group 1 does not exist (it still takes part in the barriers)
        const bool live = KS == 1 || (kt0 + kt) * KS + grp < KSTEPS;
        frag_t wf[2][TN];
        // step 0
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[1][tm] = *(const frag_t*)(abuf + rd[1] + tm * 32 * 128);
        __builtin_amdgcn_sched_barrier(0);
        widen(wf[0], 0);
        if (ZERO_C && kt == 0)
            multiply(wf[0], 0, std::true_type{});
        else if (live)
            multiply(wf[0], 0, std::false_type{});
        __builtin_amdgcn_sched_barrier(0);
        // step 1: the last LDS reads of this stage
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[2][tm] = *(const frag_t*)(abuf + rd[2] + tm * 32 * 128);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) xf[3][tm] = *(const frag_t*)(abuf + rd[3] + tm * 32 * 128);
        __builtin_amdgcn_sched_barrier(0);
        widen(wf[1], 1);
        if (live) multiply(wf[1], 1, std::false_type{});
        __builtin_amdgcn_sched_barrier(0);
        // the packed weights of this stage are widened completely before their registers are reused
        widen(wf[0], 2);
        widen(wf[1], 3);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)  // materialise them here (the compiler would otherwise sink them past the branch)
            asm volatile("" : "+v"(wf[0][tn]), "+v"(wf[1][tn]));
        __builtin_amdgcn_sched_barrier(0);
        int nb = buf + 1 == S ? 0 : buf + 1;
        if (kt + 1 < KT) {
            // hand-over: stage kt+1 must have landed (the S-2 stages behind it may stay in flight while they exist);
            // the barrier also says that every wave holds its last fragments of stage kt, so its buffer is refilled
            if (S > 2 && kt + S - 1 < KT)
                wait_vmcnt<(S > 2 ? (S - 2) * P::OPS : 0)>();
            else
                wait_vmcnt<0>();
            __syncthreads();
            if (kt + S < KT) issue(kt + S, buf);
            request_first(lds + nb * STAGE_BYTES + grp * P::SUB_BYTES);
        }
        __builtin_amdgcn_sched_barrier(0);
        if (live) {
            multiply(wf[0], 2, std::false_type{});
            multiply(wf[1], 3, std::false_type{});
        }
        __builtin_amdgcn_sched_barrier(0);
        buf = nb;
    }
    __syncthreads();  // every wave is done reading the stages: what follows may overwrite them

    if constexpr (RS_INLINE) {  // lanes l and l + 32 hold the two k-halves of row l's sum
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) rsum[tm] += __shfl_xor(rsum[tm], 32, 64);
    }

    // Park the per-channel constants in LDS behind the stages: multiplier, additive term and (int8) the two
    // zero-point corrections.
    //   weight-only: y = acc * s_w[n] + bias[n]
    //   int8: stored operands are a' = qx - 128 and b' = qw - w_off; with dx = 128 - z_x, dw = w_off - z_w[n]:
    //         ACC = raw + dw * rowsum_a'[m] + dx * (colsum_b'[n] + K * dw),  colsum_b' = colsum - K * w_off,
    //         y = ACC * (s_x * s_w[n]) + bias[n].  Wrap-around int32 arithmetic is exact because ACC itself fits.
    float* ch_mul = (float*)(lds + P::CONSTS);
    float* ch_add = ch_mul + BN;
    int* ch_dw = (int*)(ch_add + BN);
    int* ch_cn = ch_dw + BN;
    if (threadIdx.x < BN) {
        const int t = threadIdx.x;
        if constexpr (I8) {
            // (nothing derived from the activation parameters is computed before this point: the arithmetic would
            // wait for their load at the top of the kernel, ahead of the first stage's requests)
            asm volatile("" : "+s"(c_zx), "+s"(c_sx));
            const int dx = 128 - c_zx;
            const int dw = g.w_off - c_zp;
            ch_dw[t] = dw;
            ch_cn[t] = dx * (c_colsum - g.K * g.w_off + g.K * dw);
        }
        ch_mul[t] = c_scale * c_sx;
        asm volatile("" : "+v"(c_bias_bits));  // (keeps the compiler from moving the conversion up to the load)
        ch_add[t] = BF ? bf16_bits_to_float((uint16_t)c_bias_bits)
                       : (float)__builtin_bit_cast(_Float16, (uint16_t)c_bias_bits);
    }

    // k-split: the two groups' partial sums meet through LDS ([register quad][lane], 16 bytes per lane).  With an
    // even number of row slabs per wave each group finishes half of them (it sends the other half across and adds
    // what it receives), so both groups take part in the epilogue; otherwise group 1 sends everything to group 0.
    constexpr bool SPLIT_EPI = KS == 2 && TM % 2 == 0;
    constexpr int TMX = SPLIT_EPI ? TM / 2 : TM;  // slabs one wave sends
    auto owner = [](int tm) { return SPLIT_EPI ? (tm & 1) : 0; };
    if constexpr (KS == 2) {
        using quad_t = typename std::conditional<I8, int4v, float4v>::type;
        constexpr int XW = TMX * TN * 4 * 1024;  // bytes one wave sends
        static_assert(P::NWG * (SPLIT_EPI ? 2 : 1) * XW <= S * STAGE_BYTES, "accumulator exchange must fit the stages");
        auto area = [&](int writer) { return lds + (SPLIT_EPI ? wvg * 2 + writer : wvg) * XW + lane * 16; };
        uint8_t* out = area(grp);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (owner(tm) == grp) continue;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    quad_t v;
#pragma unroll
                    for (int r = 0; r < 4; ++r) v[r] = acc[tm][tn][4 * q + r];
                    *(quad_t*)(out + (((SPLIT_EPI ? tm >> 1 : tm) * TN + tn) * 4 + q) * 1024) = v;
                }
        }
        __syncthreads();
        const uint8_t* in = area(1 - grp);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (owner(tm) != grp) continue;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const quad_t v = *(const quad_t*)(in + (((SPLIT_EPI ? tm >> 1 : tm) * TN + tn) * 4 + q) * 1024);
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[tm][tn][4 * q + r] += v[r];
                }
        }
        __syncthreads();
    }

    if constexpr (KS == 1) __syncthreads();  // constants visible (the k-split exchange above has its own barriers)

    // Reduction split over workgroups: every workgroup stores its partial sums (register order, one 4-byte value per
    // lane per store: fully coalesced; rows past M skipped), then takes a ticket; the one that draws the last ticket
    // adds the partial sums of all parts, its own included, in part order (so the result does not depend on which
    // workgroup came last) and goes on to the epilogue; the others are done.  Nobody waits for anybody.
    // The partial sums are written and read with device-scope atomic accesses (write-through stores, loads that
    // bypass the L2 of the reader's XCD); every wave waits for its stores to complete, the workgroup meets at a
    // barrier, and one thread draws the ticket with a device-scope acquire-release read-modify-write, which orders
    // the stores of this workgroup before the ticket and the loads of the last workgroup after it.
    if (CAN_SPLIT && splits > 1) {
        using elem_t = typename std::conditional<I8, int, float>::type;
        const size_t tile_elems = (size_t)BM * BN;
        elem_t* mine = (elem_t*)(g.partial + ((size_t)tile_id * splits + sp) * tile_elems);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (KS > 1 && owner(tm) != grp) continue;
            if (m0 + (wm * TM + tm) * 32 + l31 >= g.M) continue;
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    __hip_atomic_store(mine + (((wvg * TM + tm) * TN + tn) * 16 + i) * 64 + lane, (elem_t)acc[tm][tn][i],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        wait_vmcnt<0>();  // this wave's stores have completed (reached the level all compute units see)
        __syncthreads();
        uint32_t* ticket = (uint32_t*)(lds + P::SINK);  // the sink of padding loads is idle by now
        if (threadIdx.x == 0)
            *ticket = __hip_atomic_fetch_add(g.counters + tile_id, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (*ticket != (uint32_t)(splits - 1)) return;  // (the counters are cleared on the stream before every launch)
#pragma unroll
        for (int tm = 0; tm < TM; ++tm)
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;
        // (the loads of PU parts are requested together where the registers allow; the additions keep part order)
        constexpr int PU = TM * TN == 1 ? 4 : 1;
        for (int part0 = 0; part0 < splits; part0 += PU) {
            elem_t v[PU][TM][TN][16];
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int part = part0 + u < splits ? part0 + u : splits - 1;
                const elem_t* theirs = (const elem_t*)(g.partial + ((size_t)tile_id * splits + part) * tile_elems);
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    if (KS > 1 && owner(tm) != grp) continue;
                    if (m0 + (wm * TM + tm) * 32 + l31 >= g.M) continue;
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int i = 0; i < 16; ++i)
                            v[u][tm][tn][i] =
                                __hip_atomic_load(theirs + (((wvg * TM + tm) * TN + tn) * 16 + i) * 64 + lane,
                                                  __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                if (part0 + u >= splits) break;
#pragma unroll
                for (int tm = 0; tm < TM; ++tm) {
                    if (KS > 1 && owner(tm) != grp) continue;
                    if (m0 + (wm * TM + tm) * 32 + l31 >= g.M) continue;
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[tm][tn][i] += v[u][tm][tn][i];
                }
            }
        }
    }
    if (g.phase_clk) t2 = clock64();
    // ---------------------------------------------------------------- epilogue
    // Result element v of a lane is channel 8*(v/4) + 4*kb + v%4 of its 32-channel tile, activation row l31:
    // four consecutive channels of ONE row per lane, so a direct store would scatter 8-byte pieces over 32 rows.
    // Instead every wave transposes through its own slice of the (now idle) LDS stages, in slabs of 32 rows by the
    // wave's TN channel tiles: finished fp16 values are written as 8-byte pieces into a [32 rows][TN*32 channels]
    // image (16-byte chunks XOR-swizzled by row), read back as 16 bytes per lane along rows, and stored with 4*TN
    // lanes covering one contiguous row segment of TN*64 bytes.
    if constexpr (GEGLU) {
        // value * gelu(gate) -> 8-bit codes in the int8 activation layout (a' = code - 128, groups of 8 columns in
        // the order 0,4,1,5,2,6,3,7, columns from H to the row stride zero), optionally the product itself as fp16.
        // A lane holds four consecutive columns of one row; the lane 32 further on holds the other four of the same
        // group of 8, so the two swap their packed words and each keeps one of the group's two output words.
        // Rows are staged through LDS (32 rows x 32 bytes per wave) and leave as 16-byte pieces.
        // (without output parameters the kernel only writes the product and its range: the codes follow in a pass of
        // their own once the range of the whole tensor is known)
        constexpr bool want_codes = (I8 && !RANGE) || CODES16;
        float inv_o = 0.0f, zf_o = 0.0f;
        if constexpr (want_codes) {
            inv_o = __fdiv_rn(1.0f, *g.out_scale_p);
            zf_o = (float)*g.out_zp_p;
        }
        float hmn = INFINITY, hmx = -INFINITY;
        static_assert(P::NWG * 3072 <= S * STAGE_BYTES, "epilogue staging must fit the LDS stages");
        uint8_t* ep8 = lds + wvg * 3072;
        uint8_t* ep16 = ep8 + 1024;
        const int col0 = n0 + wn * 32;  // first gated column of this wave
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            const int mt0 = m0 + (wm * TM + tm) * 32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cl_v = (wn * TN) * 32 + 8 * q + 4 * kb, cl_g = cl_v + 32;
                const float4v mul_v = *(const float4v*)(ch_mul + cl_v), add_v = *(const float4v*)(ch_add + cl_v);
                const float4v mul_g = *(const float4v*)(ch_mul + cl_g), add_g = *(const float4v*)(ch_add + cl_g);
                int4v dw_v = {0, 0, 0, 0}, cn_v = dw_v, dw_g = dw_v, cn_g = dw_v;
                if constexpr (I8) {
                    dw_v = *(const int4v*)(ch_dw + cl_v), cn_v = *(const int4v*)(ch_cn + cl_v);
                    dw_g = *(const int4v*)(ch_dw + cl_g), cn_g = *(const int4v*)(ch_cn + cl_g);
                }
                uint32_t word = 0;
                half4 hh;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float lv, lg;
                    if constexpr (I8) {
                        const int av = acc[tm][0][4 * q + r] + __mul24(dw_v[r], rsum[tm]) + cn_v[r];
                        const int ag = acc[tm][1][4 * q + r] + __mul24(dw_g[r], rsum[tm]) + cn_g[r];
                        lv = __fmaf_rn((float)av, mul_v[r], add_v[r]);
                        lg = __fmaf_rn((float)ag, mul_g[r], add_g[r]);
                    } else {
                        lv = __fmaf_rn(acc[tm][0][4 * q + r], mul_v[r], add_v[r]);
                        lg = __fmaf_rn(acc[tm][1][4 * q + r], mul_g[r], add_g[r]);
                    }
                    const float h = __fmul_rn(lv, gelu32(lg));
                    if constexpr (want_codes) {
                        float t = __fadd_rn(rintf(__fmul_rn(h, inv_o)), zf_o);
                        t = fminf(fmaxf(t, 0.0f), 255.0f);
                        const int code = col0 + 8 * q + 4 * kb + r < H ? (int)t - 128 : 0;
                        word |= ((uint32_t)code & 255u) << (8 * r);
                    }
                    if constexpr (BF)
                        hh[r] = __builtin_bit_cast(_Float16, float_to_bf16_bits(h));
                    else
                        hh[r] = (_Float16)h;
                }
                if constexpr (RANGE) {  // range of the values as they are stored (fp16), real rows and columns only
                    const bool row_ok = mt0 + l31 < g.M;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const bool ok = row_ok && col0 + 8 * q + 4 * kb + r < H;
                        const float hv = (float)hh[r];
                        hmn = fminf(hmn, ok ? hv : INFINITY);
                        hmx = fmaxf(hmx, ok ? hv : -INFINITY);
                    }
                }
                if constexpr (want_codes) {
                    const uint32_t other = (uint32_t)__shfl_xor((int)word, 32, 64);
                    const uint32_t lo = kb ? other : word, hi = kb ? word : other;  // columns 0..3 and 4..7 of the group
                    // v_perm_b32: selector bytes 0..3 pick bytes of the second source, 4..7 of the first
                    const uint32_t out = kb ? __builtin_amdgcn_perm(hi, lo, 0x07030602u) : __builtin_amdgcn_perm(hi, lo, 0x05010400u);
                    *(uint32_t*)(ep8 + l31 * 32 + q * 8 + kb * 4) = out;
                }
                if (g.y) *(half4*)(ep16 + l31 * 64 + q * 16 + kb * 8) = hh;
            }
            __builtin_amdgcn_wave_barrier();
            if constexpr (want_codes) {
                const int row = lane >> 1, half = lane & 1;
                const uint4v v = *(const uint4v*)(ep8 + row * 32 + half * 16);
                const int m = mt0 + row, col = col0 + half * 16;
                if (m < g.M && col < g.ld8) __builtin_nontemporal_store(v, (uint4v*)(g.a8_out + (long)m * g.ld8 + col));
            }
            if (g.y) {
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int idx = i * 64 + lane, row = idx >> 2, c = idx & 3;
                    const uint4v v = *(const uint4v*)(ep16 + row * 64 + c * 16);
                    const int m = mt0 + row, col = col0 + c * 8;
                    if (m < g.M && col < H) __builtin_nontemporal_store(v, (uint4v*)(g.y + (long)m * g.ldy + col));
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
        if constexpr (RANGE) {  // one pair per workgroup: waves meet through the (idle) sink of the padding loads
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) {
                hmn = fminf(hmn, __shfl_xor(hmn, off, 64));
                hmx = fmaxf(hmx, __shfl_xor(hmx, off, 64));
            }
            float* mm = (float*)(lds + P::SINK);
            if (lane == 0) {
                mm[2 * wv] = hmn;
                mm[2 * wv + 1] = hmx;
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                float a = mm[0], b = mm[1];
#pragma unroll
                for (int i = 1; i < NW; ++i) {
                    a = fminf(a, mm[2 * i]);
                    b = fmaxf(b, mm[2 * i + 1]);
                }
                g.mm_out[2 * blockIdx.x] = a;
                g.mm_out[2 * blockIdx.x + 1] = b;
            }
        }
    } else {
    static_assert(TN == 1 || TN == 2 || TN == 4, "channel tiles per wave: 1, 2 or 4");
    constexpr int EP_BYTES = 32 * TN * 64;          // staging bytes of one 32-row slab of a wave
    constexpr int EW = SPLIT_EPI ? NW : P::NWG;     // storing waves
    // Where the idle stages have the room, a wave stages all its slabs at once: the per-channel constants of a
    // register quad are then read from LDS once and serve every slab (a wave that reads them again for each slab
    // spends most of its epilogue waiting for LDS), and one pass of stores follows one pass of conversions.
    constexpr bool ALL_SLABS = KS == 1 && !RES && EW * TM * EP_BYTES <= S * STAGE_BYTES;
    constexpr int WAVE_EP = ALL_SLABS ? TM * EP_BYTES : EP_BYTES;
    static_assert(EW * WAVE_EP <= S * STAGE_BYTES, "epilogue staging must fit the LDS stages");
    uint8_t* ep = lds + (SPLIT_EPI ? wv : wvg) * WAVE_EP;
    const int nw0 = n0 + wn * TN * 32;  // first channel of this wave
    constexpr int CPR = TN * 4;              // 16-byte chunks per staged row
    constexpr int ROWS_PER_PASS = 64 / CPR;  // rows one store instruction covers
    // The chunk index is XOR-ed with the row bits ABOVE those that already separate rows inside one 256-byte
    // turn of the banks (16 / CPR rows): the 8-byte writes of 32 rows then fall on 16 different bank pairs instead
    // of 4 (64-byte rows) or 8 (128-byte rows), and the 16-byte reads of whole rows stay conflict free.
    constexpr int RSH = CPR == 4 ? 2 : (CPR == 8 ? 1 : 0);

    // Residual pieces arrive in the accumulator layout (8 bytes per lane: four channels of the lane's row), all of a
    // 32-row slab at once and, where a wave stores several slabs, one slab ahead of the stores.
    auto load_res = [&](int tm, half4 (&dst)[TN][4]) {
        const int m = m0 + (wm * TM + tm) * 32 + l31;
        long rr = m;
        if constexpr (I8) rr = g.out_map.phys(m);
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = nw0 + tn * 32 + 8 * q + 4 * kb;
                half4 z = {0, 0, 0, 0};
                dst[tn][q] = m < g.M && n < g.N ? *(const half4*)(g.res + rr * g.ldr + n) : z;
            }
    };
    auto res_f32 = [&](_Float16 h) -> float {
        if constexpr (BF)
            return __builtin_bit_cast(float, (uint32_t)__builtin_bit_cast(uint16_t, h) << 16);
        else
            return (float)h;
    };
    // RES: a residual operand is present.  A kernel of its own, so that calls without one pay nothing for it.
    constexpr bool has_res = RES;

    // The constants of result quad q of channel tile tn: four consecutive channels.
    struct QuadConst {
        float4v mul, add;
        int4v dw, cn;
    };
    auto quad_const = [&](int tn, int q) {
        const int cl = (wn * TN + tn) * 32 + 8 * q + 4 * kb;  // channel inside the workgroup tile
        QuadConst k;
        k.mul = *(const float4v*)(ch_mul + cl);
        k.add = *(const float4v*)(ch_add + cl);
        if constexpr (I8) {
            k.dw = *(const int4v*)(ch_dw + cl);
            k.cn = *(const int4v*)(ch_cn + cl);
        }
        return k;
    };
    // int8 path: the exact integer sums of result quad q of tile (tm, tn) with both zero-point corrections.
    auto int_quad = [&](int tm, int tn, int q, const QuadConst& k) {
        int4v a = {0, 0, 0, 0};
        if constexpr (I8) {
            int4v border = {0, 0, 0, 0};
            if constexpr (MODE == 4) {
                // Convolution: a filter tap outside the image reads zero bytes, which stand for the code
                // 128, not for the value 0 (code z_x).  The constant term cn counts every tap; take back
                // dx * sum_c (q_w - z_w) of the taps this pixel does not have.
                const uint32_t have = tap_mask(m0 + (wm * TM + tm) * 32 + l31);
                if (have != 0x1FFu) {
                    const int n_real = n0 + (wn * TN + tn) * 32 + 8 * q + 4 * kb;
                    const int dxv = 128 - *g.act_zp_p;
                    const int cin = g.conv_cpt * 64;
                    for (int t = 0; t < 9; ++t) {
                        if (have >> t & 1u) continue;
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int n = n_real + r < g.N ? n_real + r : g.N - 1;
                            border[r] += dxv * (g.w_tapsum[t * g.N + n] - cin * (g.w_off - k.dw[r]));
                        }
                    }
                }
            }
#pragma unroll
            for (int r = 0; r < 4; ++r)
                // |dw| <= 255 and |rowsum| <= 128 * K < 2^23: a 24-bit multiply (full rate) is exact
                a[r] = acc[tm][tn][4 * q + r] + __mul24(k.dw[r], rsum[tm]) + k.cn[r] - border[r];
        }
        return a;
    };
    // Finishes result quad q of tile (tm, tn) and writes it into the slab image at `slab`.
    auto finish_quad = [&](uint8_t* slab, int tm, int tn, int q, const QuadConst& k, const half4& rq) {
        float4v add = k.add;
        if constexpr (has_res) {  // joins the bias term
#pragma unroll
            for (int r = 0; r < 4; ++r) add[r] += res_f32(rq[r]);
        }
        half4 o;
        if constexpr (I8) {
            const int4v a = int_quad(tm, tn, q, k);
#pragma unroll
            for (int r = 0; r < 4; ++r) o[r] = (_Float16)((float)a[r] * k.mul[r] + add[r]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float v = acc[tm][tn][4 * q + r] * k.mul[r] + add[r];
                if constexpr (BF)
                    o[r] = __builtin_bit_cast(_Float16, float_to_bf16_bits(v));  // bits only
                else
                    o[r] = (_Float16)v;
            }
        }
        const int chunk = tn * 4 + q;
        *(half4*)(slab + l31 * (CPR * 16) + (((chunk ^ (l31 >> RSH)) & (CPR - 1)) << 4) + kb * 8) = o;
    };
    // The integer sums themselves, for the tests that pin them (a pass of its own: the ordinary epilogue carries no
    // trace of it).
    if constexpr (I8) {
        if (g.acc_debug) {
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                if (KS > 1 && owner(tm) != grp) continue;
                const int m = m0 + (wm * TM + tm) * 32 + l31;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int n_real = n0 + (wn * TN + tn) * 32 + 8 * q + 4 * kb;
                        const int4v a = int_quad(tm, tn, q, quad_const(tn, q));
                        if (m < g.M && n_real < g.N) *(int4v*)(g.acc_debug + (long)m * g.N + n_real) = a;
                    }
            }
        }
    }
    // Reads the slab image back as 16 bytes per lane along rows and stores it: CPR lanes cover one contiguous row
    // segment of TN * 64 bytes.  All reads are requested before the first store (a store that waits for its own read
    // pays the LDS latency every time), and with the identity row map the addresses advance by a constant.
    auto store_slab = [&](const uint8_t* slab, int tm) {
        constexpr int NP = 32 / ROWS_PER_PASS;
        const int r0 = lane / CPR, c = lane % CPR;
        const int m_first = m0 + (wm * TM + tm) * 32 + r0, n = nw0 + c * 8;
        uint4v v[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int row = i * ROWS_PER_PASS + r0;
            v[i] = *(const uint4v*)(slab + row * (CPR * 16) + (((c ^ (row >> RSH)) & (CPR - 1)) << 4));
        }
        if (n >= g.N) return;
        // Streaming stores: the output is not read again by this kernel, and a line that is written through as it is
        // produced does not wait in the XCD's L2 for the write-back at the end of the kernel (worth 7 % of the
        // dominant kernel's time).
        bool identity = true;
        if constexpr (I8) identity = g.out_map.rows_per_group <= 0;
        if (identity) {
            uint16_t* yp = g.y + (long)m_first * g.ldy + n;
            const long step = (long)ROWS_PER_PASS * g.ldy;
#pragma unroll
            for (int i = 0; i < NP; ++i)
                if (m_first + i * ROWS_PER_PASS < g.M) __builtin_nontemporal_store(v[i], (uint4v*)(yp + i * step));
        } else {
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int m = m_first + i * ROWS_PER_PASS;
                if (m < g.M) __builtin_nontemporal_store(v[i], (uint4v*)(g.y + g.out_map.phys(m) * g.ldy + n));
            }
        }
    };
    if constexpr (ALL_SLABS) {
        const half4 none = {0, 0, 0, 0};
        // (the constants of the next quad are requested before the conversions of the current one: the compiler does
        // not move an LDS read above the staging writes by itself)
        QuadConst k = quad_const(0, 0);
#pragma unroll
        for (int i = 0; i < TN * 4; ++i) {
            const QuadConst kn = quad_const((i + 1 < TN * 4 ? i + 1 : i) >> 2, (i + 1 < TN * 4 ? i + 1 : i) & 3);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) finish_quad(ep + tm * EP_BYTES, tm, i >> 2, i & 3, k, none);
            k = kn;
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) store_slab(ep + tm * EP_BYTES, tm);
    } else {
        constexpr bool RES_AHEAD = KS == 1 && TM > 1;
        half4 rs[2][TN][4] = {};
        if constexpr (RES_AHEAD && has_res) load_res(0, rs[0]);
#pragma unroll
        for (int tm = 0; tm < TM; ++tm) {
            if (KS > 1 && owner(tm) != grp) continue;  // the finished sums of this slab live in the other group
            if constexpr (has_res) {
                if constexpr (RES_AHEAD) {
                    if (tm + 1 < TM) load_res(tm + 1, rs[(tm + 1) & 1]);
                } else {
                    load_res(tm, rs[tm & 1]);
                }
            }
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
#pragma unroll
                for (int q = 0; q < 4; ++q) finish_quad(ep, tm, tn, q, quad_const(tn, q), rs[tm & 1][tn][q]);
            __builtin_amdgcn_wave_barrier();
            store_slab(ep, tm);
            __builtin_amdgcn_wave_barrier();
        }
    }
    }
    if (g.phase_clk && threadIdx.x == 0) {
        long long* o = g.phase_clk + (long)blockIdx.x * 4;
        o[0] = t0;
        o[1] = t1;
        o[2] = t2;
        o[3] = clock64();
    }
}

// ---------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------
// Tile table.  index -> workgroup tile (rows x channels), waves, wave tile:
//   0: 128x256, 4 waves (1x4) of 128x64     1: 128x128, 4 waves (2x2) of 64x64     2: 64x64, 4 waves of 32x32
//   3: as 1 and 4: as 2, with a second wave group splitting k inside the workgroup (8 waves)
//   5: 64x128, 4 waves (1x4) of 64x32, two or three LDS stages: the form of tile 1 that puts more workgroups on a
//      compute unit
// A tall wave tile pays: every widened weight fragment then feeds 4 MFMAs (measured: an MFMA hides about five vector
// ALU instructions on its SIMD; what a wave needs beyond that costs time of its own).  256x256 tiles with one wave per
// SIMD and 128x128 tiles with two-wave workgroups were measured slower on every configured shape.
// The number of LDS stages is the largest (<= 4; <= 8 for tile 2, whose problems are latency bound) that lets two
// workgroups share a compute unit and keeps the hand-counted loads within the 6-bit vmcnt.
static int g_force_tile = -1;
static long long* g_phase_clk = nullptr;
static long g_phase_cap = 0;
void set_phase_buffer(long long* p, long workgroups) {
    g_phase_clk = p;
    g_phase_cap = workgroups;
}
void set_force_tile(int t) { g_force_tile = t; }

// ---- reduction split over workgroups ------------------------------------------------------------------------
// Problems with few tiles and a long reduction (K/V projections, a handful of activation rows) are bound by memory
// latency: the only remedy is to have more workgroups request the operands at once.  Their partial sums and one
// arrival counter per tile live in the CALLER's workspace: [counters: tiles x 4 bytes, rounded up to 256]
// [partial sums: tiles x parts x BM x BN x 4 bytes].  The counters are cleared by a small kernel on the same stream
// right before the GEMM (the workspace arrives with unknown contents); whoever owns the workspace owns the hazard,
// as with any workspace: one stream at a time.
static int g_force_splits = 0;  // 0: automatic, 1: never, n > 1: n parts wherever the reduction is long enough
void set_force_splits(int n) { g_force_splits = n < 0 ? 0 : n; }
int forced_splits() { return g_force_splits; }
static int g_force_band = 0;  // 0: automatic, n >= 1: n row blocks per band of the workgroup -> tile map
void set_force_band(int n) { g_force_band = n < 0 ? 0 : n; }

__global__ void split_clear_kernel(uint32_t* counters, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) counters[i] = 0;
}

static inline size_t split_counter_bytes(long tiles) { return ((size_t)tiles * 4 + 255) / 256 * 256; }

// Measured on the SDXL shapes: the large tile wins once it yields two or more workgroups per compute unit; the
// k-split variants only pay where tiles are few and k is long (FF-out at the 640 level, the K/V projections).
static int pick_tile(int M, int N, int K, bool wide_weights = false) {
    if ((g_force_tile >= 0 && g_force_tile <= 4) || g_force_tile == 6) return g_force_tile;
    if (g_force_tile == 5) return 1;  // the half-height form of tile 1: the linear layers' dispatch decides (narrow_tile)
    const long t0 = (long)((M + 127) / 128) * ((N + 255) / 256);
    // One row block of 65 to 96 rows over very many column tiles (one prompt's 77 text tokens through all K/V
    // projections of the UNet, stacked): the 96x256 tile does three quarters of the large tile's MFMA and widening work
    // on the same weight stream (measured at N = 166400: 13 to 18 % faster with 2- and 4-bit weights, equal at 8).
    if (M > 64 && M <= 96 && t0 >= 256) return 6;
    // (8-bit weights of the int8 path: the large tile leaves LDS for one workgroup per compute unit only, and two
    // co-resident 128x128 workgroups were measured faster on every configured shape)
    if (t0 >= 512 && !wide_weights) return 0;
    const long t1 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (t1 >= 128) return (t1 < 256 && K >= 2048) ? 3 : 1;
    return K >= 1024 ? 4 : 2;
}

// Tile 1 or its half-height form (tile 5: 64x128, four waves side by side, two or three LDS stages, three to five
// workgroups per compute unit)?  The 128x128 problems of this path have 160 to 640 tiles, one or two workgroups on
// most compute units, and a wave's LDS reads, code widening and MFMAs run one after the other: what is missing is
// other waves on the SIMD to fill the gaps.  Twice the workgroups at half the height fetch every weight tile twice as
// often (weights are the small operand; halving the width instead doubles the activation traffic and was measured
// slower on the 16-bit-activation path).  Measured on operands that are not cached: 8 to 19 % faster on every such
// shape of both paths, except with unquantised 16-bit weights (4 KB per weight tile), which keep tile 1.  Two
// stages instead of three, and eight waves on 64x256, were measured slower.
// Weights that do not fit an XCD's L2 by a wide margin are streamed from the last-level cache once per row block,
// twice as often with the half height: 8-bit 1280 -> 10240 (13 MB) on the int8 path took 121 us against 88; they
// keep the full height.
template <bool I8, int BITS>
static int narrow_tile(int t, long N, long K) {
    if (g_force_tile == 5) return 5;
    if (g_force_tile >= 0 || (t != 1 && t != 3)) return t;
    if (BITS == 16 || N * K * BITS / 8 > (8L << 20)) return t;
    return 5;  // (also in place of tile 3: 5 to 7 % faster on its one regime, 4096 x 2560 x 640)
}

template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int S, int KS>
constexpr bool stages_fit(int budget) {
    using P = GemmPlan<I8, BITS, WGM, WGN, TM, TN, S, KS>;
    return P::LDS_BYTES <= budget && (S - 2) * P::OPS <= 63;
}

template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int KS>
constexpr int pick_stages(int budget, int max_stages) {
    if (max_stages >= 8 && stages_fit<I8, BITS, WGM, WGN, TM, TN, 8, KS>(budget)) return 8;
    if (max_stages >= 6 && stages_fit<I8, BITS, WGM, WGN, TM, TN, 6, KS>(budget)) return 6;
    if (max_stages >= 4 && stages_fit<I8, BITS, WGM, WGN, TM, TN, 4, KS>(budget)) return 4;
    if (stages_fit<I8, BITS, WGM, WGN, TM, TN, 3, KS>(budget)) return 3;
    return 2;
}

template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int KS, int BUDGET, int MAXS, bool BF, int MODE, bool RES>
static int run_gemm_r(GemmArgs& g, int tile_index, hipStream_t st) {
    constexpr int S = pick_stages<I8, BITS, WGM, WGN, TM, TN, KS>(BUDGET, MAXS);
    using P = GemmPlan<I8, BITS, WGM, WGN, TM, TN, S, KS>;
    static_assert(P::LDS_BYTES <= 160 * 1024, "LDS plan exceeds the compute unit");
    g.tiles_m = (g.M + P::BM - 1) / P::BM;
    g.tiles_n = (g.N + P::BN - 1) / P::BN;
    if (MODE == 1 || MODE == 5 || MODE == 6) g.tiles_n = (int)((g.ld8 + P::BN / 2 - 1) / (P::BN / 2));  // gated columns up to the padded row end
    // Split the reduction over workgroups where the tiles alone would leave most compute units idle and the reduction
    // is long: as many parts as fill about two workgroups per compute unit, each at least four pipeline stages long.
    const long tiles = (long)g.tiles_m * g.tiles_n;
    // Height of the bands of the tile walk, measured on operands that are not cached over 1 to 64 row blocks: the
    // int8 path gains 4 to 23 % at 8 to 16 (every shape of the sweep, most at 16384 x 640 x 640 and with 8-bit
    // weights) and loses again from 32 on; unquantised 16-bit weights (the largest weight tiles) gain up to 15 % at
    // 8; quantised weights under 16-bit activations move by -10 (8-bit, 4096 x 2560 x 640) to +2 % at 8, and every
    // weight tile is then fetched once per eight row blocks instead of once per row block.
    g.band_rows = g_force_band > 0 ? g_force_band : (I8 ? 16 : 8);
    if (g.band_rows > g.tiles_m) g.band_rows = g.tiles_m;
    if (g.band_rows < 1) g.band_rows = 1;
    const int KT = (g.k_stages + KS - 1) / KS;
    int splits = 1;
    if (g_force_splits > 1) {
        splits = g_force_splits < KT ? g_force_splits : KT;
    } else if (g_force_splits == 0 && tiles <= 64 && KT >= 16) {
        // (measured: handing the sums over costs about as much as eight pipeline stages)
        splits = (int)(512 / tiles);
        if (splits > KT / 4) splits = KT / 4;
        if (splits > 16) splits = 16;
    }
    g.splits = 1;
    if (MODE == 0 && TM * TN <= 4 && splits > 1) {
        // as many parts as the caller's workspace holds (forced part counts are for tests: they must fit)
        const size_t cbytes = split_counter_bytes(tiles), part_bytes = (size_t)tiles * P::BM * P::BN * 4;
        const size_t room = g.split_ws && g.split_ws_bytes > cbytes ? (g.split_ws_bytes - cbytes) / part_bytes : 0;
        if (g_force_splits > 1 && room < (size_t)splits) return MQ_ERR_WORKSPACE_TOO_SMALL;
        if (room < (size_t)splits) splits = (int)room;
        if (splits > 1) {
            g.splits = splits;
            g.counters = (uint32_t*)g.split_ws;
            g.partial = (uint32_t*)((uint8_t*)g.split_ws + cbytes);
        }
    }
    g.fd_band_tiles = FastDiv::make((uint32_t)(g.band_rows * g.tiles_n));
    g.fd_band_rows = FastDiv::make((uint32_t)g.band_rows);
    g.fd_last_rows = FastDiv::make((uint32_t)(g.tiles_m % g.band_rows ? g.tiles_m % g.band_rows : g.band_rows));
    g.fd_splits = FastDiv::make((uint32_t)g.splits);
    g.kt_q = KT / g.splits;
    g.kt_r = KT % g.splits;
    g.phase_clk = (tiles * g.splits <= g_phase_cap) ? g_phase_clk : nullptr;
    auto kern = gemm_kernel<I8, BITS, WGM, WGN, TM, TN, S, KS, BF, MODE, RES>;
    // Once per instantiation and device (callers may be on several host threads): allow more than 64 KB of dynamic
    // LDS, name the profiling slot.
    const int slot = prof_gemm_slot(MODE >= 5 ? 3 : (MODE ? 2 + MODE : (I8 ? 1 : (BF ? 2 : 0))), BITS, tile_index);
    static std::mutex prep_mutex;
    static bool prepared[16] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) dev = 0;
    {
        std::lock_guard<std::mutex> lock(prep_mutex);
        if (!prepared[dev]) {
            if (hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, P::LDS_BYTES) !=
                hipSuccess) {
                set_hip_error((int)hipGetLastError());
                return MQ_ERR_HIP;
            }
            // (the residual variant shares the slot of the plain kernel and leaves the slot's name to it)
            char name[112];
            snprintf(name, sizeof name, "mq::gemm_kernel<%s, %d, %d, %d, %d, %d, %d, %d, %s, %d, false>",
                     I8 ? "true" : "false", BITS, WGM, WGN, TM, TN, S, KS, BF ? "true" : "false", MODE);
            prof_name_slot(slot, name);
            prepared[dev] = true;
        }
    }
    // (a convolution reads each input pixel once, not nine times: the whole input tensor)
    const double abytes = MODE == 3 || MODE == 4 ? (double)g.a_bytes
                                    : (I8 ? 1.0 * g.M * g.K + (MODE == 0 ? 4.0 * g.M : 0.0) : 2.0 * g.M * g.K);
    const double ybytes = MODE == 1 || MODE == 6 ? 1.0 * g.M * g.ld8 + (g.y ? 1.0 * g.M * g.N : 0.0)
                                    : (MODE == 5 ? 1.0 * g.M * g.N : 2.0 * g.M * g.N);
    ProfScope prof(st, slot, 2.0 * g.M * g.N * g.K,
                   abytes + (double)g.N * g.K * BITS / 8 + (I8 ? 14.0 : 10.0) * g.N + ybytes);
    if (g.splits > 1) {
        hipLaunchKernelGGL(split_clear_kernel, dim3((unsigned)((tiles + 255) / 256)), dim3(256), 0, st, g.counters, (int)tiles);
        MQ_HIP_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(kern, dim3(g.tiles_m * g.tiles_n * g.splits), dim3(P::NT), P::LDS_BYTES, st, g);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

template <bool I8, int BITS, int WGM, int WGN, int TM, int TN, int KS, int BUDGET, int MAXS, bool BF = false, int MODE = 0>
static int run_gemm(GemmArgs& g, int tile_index, hipStream_t st) {
    if constexpr (MODE != 1 && MODE != 5 && MODE != 6)
        if (g.res) return run_gemm_r<I8, BITS, WGM, WGN, TM, TN, KS, BUDGET, MAXS, BF, MODE, true>(g, tile_index, st);
    return run_gemm_r<I8, BITS, WGM, WGN, TM, TN, KS, BUDGET, MAXS, BF, MODE, false>(g, tile_index, st);
}

template <bool I8, int BITS>
static int dispatch_gemm(GemmArgs& g, hipStream_t st) {
    // 8-bit weights of the int8 path take 2 KB of LDS per 32x64 tile and unquantised 16-bit weights 4 KB: with the
    // large tile two workgroups per compute unit would not fit, so it runs one per compute unit with a deeper
    // pipeline (and is not chosen automatically)
    constexpr bool WIDE = (I8 && BITS == 8) || BITS == 16;
    switch (narrow_tile<I8, BITS>(pick_tile(g.M, g.N, g.K, WIDE), g.N, g.K)) {
        case 0: return run_gemm<I8, BITS, 1, 4, 4, 2, 1, WIDE ? 160 * 1024 : 80 * 1024, 4>(g, 0, st);
        case 1: return run_gemm<I8, BITS, 2, 2, 2, 2, 1, 80 * 1024, 4>(g, 1, st);
        case 2: return run_gemm<I8, BITS, 2, 2, 1, 1, 1, 80 * 1024, 8>(g, 2, st);
        case 3: return run_gemm<I8, BITS, 2, 2, 2, 2, 2, 160 * 1024, 4>(g, 3, st);
        case 5: return run_gemm<I8, BITS, 1, 4, 2, 1, 1, I8 ? 40 * 1024 : 52 * 1024, 3>(g, 5, st);
        case 6: return run_gemm<I8, BITS, 1, 4, 3, 2, 1, WIDE ? 160 * 1024 : 80 * 1024, 4>(g, 6, st);
        default: return run_gemm<I8, BITS, 2, 2, 1, 1, 2, 80 * 1024, 8>(g, 4, st);
    }
}

// bfloat16 activations: the three plain tiles (the k-split variants fall back to their plain counterparts).
template <int BITS>
static int dispatch_gemm_bf16(GemmArgs& g, hipStream_t st) {
    constexpr bool WIDE = BITS == 16;
    int t = pick_tile(g.M, g.N, g.K, WIDE);
    t = narrow_tile<false, BITS>(t == 6 ? 0 : (t >= 3 ? t - 2 : t), g.N, g.K);
    switch (t) {
        case 0: return run_gemm<false, BITS, 1, 4, 4, 2, 1, WIDE ? 160 * 1024 : 80 * 1024, 4, true>(g, 0, st);
        case 1: return run_gemm<false, BITS, 2, 2, 2, 2, 1, 80 * 1024, 4, true>(g, 1, st);
        case 5: return run_gemm<false, BITS, 1, 4, 2, 1, 1, 52 * 1024, 3, true>(g, 5, st);
        default: return run_gemm<false, BITS, 2, 2, 1, 1, 1, 80 * 1024, 8, true>(g, 2, st);
    }
}

int launch_gemm_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, int bits,
                       const float* w_scale, const int32_t* w_zp, const void* bias, void* y, int ldy, int dtype,
                       const void* res, int ldr, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
    GemmArgs g{};
    g.split_ws = split_ws; g.split_ws_bytes = split_ws_bytes;
    g.a = x;
    g.a_row_bytes = (long)ldx * 2;
    g.a_bytes = (uint32_t)(((long)(M - 1) * ldx + K) * 2);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((N + 31) / 32) * (K / 64) * 256 * bits);
    g.M = M; g.N = N; g.K = K;
    g.k_stages = K / 64;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)y; g.ldy = ldy;
    g.res = (const uint16_t*)res; g.ldr = ldr;
    if (dtype == MQ_BF16) {
        switch (bits) {
            case 2: return dispatch_gemm_bf16<2>(g, st);
            case 3: return dispatch_gemm_bf16<3>(g, st);
            case 4: return dispatch_gemm_bf16<4>(g, st);
            case 8: return dispatch_gemm_bf16<8>(g, st);
            case 16: return dispatch_gemm_bf16<16>(g, st);
        }
        return MQ_ERR_UNSUPPORTED_BITS;
    }
    switch (bits) {
        case 2: return dispatch_gemm<false, 2>(g, st);
        case 3: return dispatch_gemm<false, 3>(g, st);
        case 4: return dispatch_gemm<false, 4>(g, st);
        case 8: return dispatch_gemm<false, 8>(g, st);
        case 16: return dispatch_gemm<false, 16>(g, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

int launch_gemm_a8(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                   const void* packed, int N, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                   const int32_t* w_colsum, const void* bias, void* y, int ldy, RowMap out_map, int32_t* acc_debug,
                   const void* res, int ldr, void* split_ws, size_t split_ws_bytes, hipStream_t st) {
    const int Kp = (K + 127) / 128 * 128;
    GemmArgs g{};
    g.split_ws = split_ws; g.split_ws_bytes = split_ws_bytes;
    g.a = a8;
    g.a_row_bytes = Kp;
    g.a_bytes = (uint32_t)((long)M * Kp);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((N + 31) / 32) * (K / 64) * 256 * w_bits);
    g.M = M; g.N = N; g.K = K;
    g.k_stages = Kp / 128;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)y; g.ldy = ldy;
    g.res = (const uint16_t*)res; g.ldr = ldr;
    g.rowsum = rowsum; g.params = params; g.w_colsum = w_colsum;
    g.out_map = out_map; g.acc_debug = acc_debug;
    if (w_bits == 4 || w_bits == 2) {
        g.w_off = 0;
        return w_bits == 4 ? dispatch_gemm<true, 4>(g, st) : dispatch_gemm<true, 2>(g, st);
    }
    if (w_bits == 8) {
        // Unsigned 8-bit codes do not fit a signed MFMA operand: the kernel flips their top bit in registers,
        // which reads them as q - 128 (w_off = 128); signed (symmetric) codes are used as they are.
        g.w_off = w_signed ? 0 : 128;
        return dispatch_gemm<true, 8>(g, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}


// Gated feed-forward projection with 8-bit output (MODE 1).  N = 2H weight rows.
int launch_gemm_a8_geglu(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                         const void* packed, int H, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                         const int32_t* w_colsum, const void* bias, const float* out_scale, const int32_t* out_zp,
                         int8_t* a8_out, void* h16, int ldh, float* mm_out, int* mm_pairs, hipStream_t st) {
    const int Kp = (K + 127) / 128 * 128;
    GemmArgs g{};
    g.mm_out = mm_out;
    g.a = a8;
    g.a_row_bytes = Kp;
    g.a_bytes = (uint32_t)((long)M * Kp);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((2 * H + 31) / 32) * (K / 64) * 256 * w_bits);
    g.M = M; g.N = 2 * H; g.K = K;
    g.k_stages = Kp / 128;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)h16; g.ldy = ldh;
    g.rowsum = rowsum; g.params = params; g.w_colsum = w_colsum;
    g.out_scale_p = out_scale; g.out_zp_p = out_zp;
    g.a8_out = a8_out; g.ld8 = (H + 127) / 128 * 128;
    // the large tile (128 gated columns per workgroup) once it yields two workgroups per compute unit
    const bool big = g_force_tile == 0 || (g_force_tile < 0 && (long)((M + 127) / 128) * ((H + 127) / 128) >= 512);
    int rc = MQ_ERR_UNSUPPORTED_BITS;
    if (mm_out) {  // fp16 product and its range, no codes
        if (w_bits == 4) {
            g.w_off = 0;
            if (big) rc = run_gemm<true, 4, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 5>(g, 0, st);
            else rc = run_gemm<true, 4, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 5>(g, 1, st);
        }
        if (w_bits == 2) {
            g.w_off = 0;
            if (big) rc = run_gemm<true, 2, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 5>(g, 0, st);
            else rc = run_gemm<true, 2, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 5>(g, 1, st);
        }
        if (w_bits == 8) {
            g.w_off = w_signed ? 0 : 128;
            if (g_force_tile == 0) rc = run_gemm<true, 8, 1, 4, 4, 2, 1, 160 * 1024, 4, false, 5>(g, 0, st);
            else rc = run_gemm<true, 8, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 5>(g, 1, st);
        }
    } else {
        if (w_bits == 4) {
            g.w_off = 0;
            if (big) rc = run_gemm<true, 4, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 1>(g, 0, st);
            else rc = run_gemm<true, 4, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 1>(g, 1, st);
        }
        if (w_bits == 2) {
            g.w_off = 0;
            if (big) rc = run_gemm<true, 2, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 1>(g, 0, st);
            else rc = run_gemm<true, 2, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 1>(g, 1, st);
        }
        if (w_bits == 8) {
            g.w_off = w_signed ? 0 : 128;
            if (g_force_tile == 0) rc = run_gemm<true, 8, 1, 4, 4, 2, 1, 160 * 1024, 4, false, 1>(g, 0, st);
            else rc = run_gemm<true, 8, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 1>(g, 1, st);
        }
    }
    if (mm_pairs) *mm_pairs = g.tiles_m * g.tiles_n;  // workgroups of the launch: one pair each
    return rc;
}

template <int BITS>
static int dispatch_w_only_geglu(GemmArgs& g, int H, hipStream_t st) {
    const bool big = g_force_tile == 0 || (g_force_tile < 0 && (long)((g.M + 127) / 128) * ((H + 127) / 128) >= 512);
    if (g.a8_out) {  // 8-bit codes out
        if (big) return run_gemm<false, BITS, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 6>(g, 0, st);
        return run_gemm<false, BITS, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 6>(g, 1, st);
    }
    if (big) return run_gemm<false, BITS, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 1>(g, 0, st);
    return run_gemm<false, BITS, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 1>(g, 1, st);
}

// Weight-only gated projection, fp16 out (MODE 1 on the fp16 path).
int launch_gemm_w_only_geglu(const void* x, int M, int K, int ldx, const void* packed, int H, int bits,
                             const float* w_scale, const int32_t* w_zp, const void* bias, void* h16, int ldh,
                             const float* out_scale, const int32_t* out_zp, int8_t* a8_out, hipStream_t st) {
    GemmArgs g{};
    g.out_scale_p = out_scale; g.out_zp_p = out_zp; g.a8_out = a8_out;
    g.a = x;
    g.a_row_bytes = (long)ldx * 2;
    g.a_bytes = (uint32_t)(((long)(M - 1) * ldx + K) * 2);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((2 * H + 31) / 32) * (K / 64) * 256 * bits);
    g.M = M; g.N = 2 * H; g.K = K;
    g.k_stages = K / 64;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)h16; g.ldy = ldh;
    g.ld8 = a8_out ? (H + 127) / 128 * 128 : H;  // without code output the grid covers the H gated columns only
    switch (bits) {
        case 2: return dispatch_w_only_geglu<2>(g, H, st);
        case 3: return dispatch_w_only_geglu<3>(g, H, st);
        case 4: return dispatch_w_only_geglu<4>(g, H, st);
        case 8: return dispatch_w_only_geglu<8>(g, H, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

// Integer GEMM on activations that arrive as codes in the int8 activation layout (MODE 2).
int launch_gemm_a8_codes(const int8_t* a8, long lda, const float* act_scale, const int32_t* act_zp, int M, int K,
                         const void* packed, int N, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                         const int32_t* w_colsum, const void* bias, void* y, int ldy, int32_t* acc_debug,
                         const void* res, int ldr, hipStream_t st) {
    const int Kp = (K + 127) / 128 * 128;
    GemmArgs g{};
    g.a = a8;
    g.a_row_bytes = lda;
    g.a_bytes = (uint32_t)((long)(M - 1) * lda + Kp);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((N + 31) / 32) * (K / 64) * 256 * w_bits);
    g.M = M; g.N = N; g.K = K;
    g.k_stages = Kp / 128;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)y; g.ldy = ldy;
    g.res = (const uint16_t*)res; g.ldr = ldr;
    g.w_colsum = w_colsum;
    g.act_scale_p = act_scale; g.act_zp_p = act_zp;
    g.acc_debug = acc_debug;
    // no in-workgroup k split here, and not the large tile (no registers to spare for the row sums; the layers this
    // serves, the output linears of feed-forward blocks, are narrow); the half-height tile 5 in place of tile 1
    int t = pick_tile(M, N, K, true);
    t = t == 6 ? 1 : (t >= 3 ? t - 2 : t);
    // (tile 5 doubles the row-sum work per MFMA: measured 8 % faster at K = 1280, 5 % at 2560, 9 % slower at 5120)
    const bool half_height = g_force_tile == 5 || (g_force_tile < 0 && K < 4096);
    if (w_bits == 4) {
        g.w_off = 0;
        switch (t) {
            case 0:
            case 1:
                if (half_height) return run_gemm<true, 4, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 2>(g, 5, st);
                return run_gemm<true, 4, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 2>(g, 1, st);
            default: return run_gemm<true, 4, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 2>(g, 2, st);
        }
    }
    if (w_bits == 2) {
        g.w_off = 0;
        switch (t) {
            case 0:
            case 1:
                if (half_height) return run_gemm<true, 2, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 2>(g, 5, st);
                return run_gemm<true, 2, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 2>(g, 1, st);
            default: return run_gemm<true, 2, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 2>(g, 2, st);
        }
    }
    if (w_bits == 8) {
        g.w_off = w_signed ? 0 : 128;
        switch (t) {
            case 0:
            case 1:
                if (half_height) return run_gemm<true, 8, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 2>(g, 5, st);
                return run_gemm<true, 8, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 2>(g, 1, st);
            default: return run_gemm<true, 8, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 2>(g, 2, st);
        }
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}


// 3x3 convolution, stride 1, zero padding 1, channels-last (MODE 3 weight-only, MODE 4 int8 activations).
static void conv_args(GemmArgs& g, int B, int H, int W, int Cin, int stride, long pix_bytes) {
    g.a_row_bytes = pix_bytes;
    g.a_bytes = (uint32_t)((long)B * H * W * pix_bytes);
    g.conv_stride = stride;
    g.conv_ho = (H - 1) / stride + 1;
    g.conv_wo = (W - 1) / stride + 1;
    g.M = B * g.conv_ho * g.conv_wo;
    g.K = 9 * Cin;
    g.conv_h = H;
    g.conv_w = W;
    g.conv_cpt = Cin / 64;
    g.conv_cpt_inv = g.conv_cpt > 1 ? (uint32_t)(((1ull << 32) + g.conv_cpt - 1) / g.conv_cpt) : 0u;
}

template <int BITS>
static int dispatch_conv_w_only(GemmArgs& g, hipStream_t st) {
    constexpr bool WIDE = BITS == 16;
    int t = pick_tile(g.M, g.N, g.K, WIDE);
    t = t == 6 ? 1 : (t >= 3 ? t - 2 : t);
    // (the large tile only where its 256 channels are filled: the UNet's 320-channel level is better served by 128)
    if (g_force_tile < 0 && t == 0 && g.N < 512) t = 1;
    if (g_force_tile == 5 || (g_force_tile < 0 && t == 1))
        return run_gemm<false, BITS, 1, 4, 2, 1, 1, 52 * 1024, 3, false, 3>(g, 5, st);
    switch (t) {
        case 0: return run_gemm<false, BITS, 1, 4, 4, 2, 1, 80 * 1024, 4, false, 3>(g, 0, st);
        case 1: return run_gemm<false, BITS, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 3>(g, 1, st);
        default: return run_gemm<false, BITS, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 3>(g, 2, st);
    }
}

int launch_conv3x3_w_only(const void* x, int B, int H, int W, int Cin, int stride, const void* packed, int N, int bits,
                          const float* w_scale, const int32_t* w_zp, const void* bias, void* y, const void* res,
                          hipStream_t st) {
    GemmArgs g{};
    g.a = x;
    conv_args(g, B, H, W, Cin, stride, (long)Cin * 2);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((N + 31) / 32) * (g.K / 64) * 256 * bits);
    g.N = N;
    g.k_stages = g.K / 64;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)y; g.ldy = N;
    g.res = (const uint16_t*)res; g.ldr = N;
    switch (bits) {
        case 2: return dispatch_conv_w_only<2>(g, st);
        case 3: return dispatch_conv_w_only<3>(g, st);
        case 4: return dispatch_conv_w_only<4>(g, st);
        case 8: return dispatch_conv_w_only<8>(g, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

int launch_conv3x3_a8(const int8_t* a8, const ActParams* params, int B, int H, int W, int Cin, int stride, const void* packed, int N,
                      int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                      const int32_t* w_tapsum, const void* bias, void* y, int32_t* acc_debug, const void* res,
                      hipStream_t st) {
    GemmArgs g{};
    g.a = a8;
    conv_args(g, B, H, W, Cin, stride, (long)(Cin + 127) / 128 * 128);
    g.packed = (const uint8_t*)packed;
    g.packed_bytes = (uint32_t)((long)((N + 31) / 32) * (g.K / 64) * 256 * w_bits);
    g.N = N;
    g.k_stages = (g.K + 127) / 128;
    g.w_scale = w_scale; g.w_zp = w_zp; g.bias = (const uint16_t*)bias;
    g.y = (uint16_t*)y; g.ldy = N;
    g.res = (const uint16_t*)res; g.ldr = N;
    g.w_colsum = w_colsum; g.w_tapsum = w_tapsum;
    g.act_scale_p = &params->scale; g.act_zp_p = &params->zp;
    g.acc_debug = acc_debug;
    // (not the large tile: no registers to spare for the row sums and the tap masks; tile 5 in place of tile 1)
    int t = pick_tile(g.M, N, g.K, true);
    t = t == 6 ? 1 : (t >= 3 ? t - 2 : t);
    if (w_bits == 4) {
        g.w_off = 0;
        if (t <= 1 && g_force_tile != 1) return run_gemm<true, 4, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 4>(g, 5, st);
        if (t <= 1) return run_gemm<true, 4, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 4>(g, 1, st);
        return run_gemm<true, 4, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 4>(g, 2, st);
    }
    if (w_bits == 2) {
        g.w_off = 0;
        if (t <= 1 && g_force_tile != 1) return run_gemm<true, 2, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 4>(g, 5, st);
        if (t <= 1) return run_gemm<true, 2, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 4>(g, 1, st);
        return run_gemm<true, 2, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 4>(g, 2, st);
    }
    if (w_bits == 8) {
        g.w_off = w_signed ? 0 : 128;
        if (t <= 1 && g_force_tile != 1) return run_gemm<true, 8, 1, 4, 2, 1, 1, 40 * 1024, 3, false, 4>(g, 5, st);
        if (t <= 1) return run_gemm<true, 8, 2, 2, 2, 2, 1, 80 * 1024, 4, false, 4>(g, 1, st);
        return run_gemm<true, 8, 2, 2, 1, 1, 1, 80 * 1024, 8, false, 4>(g, 2, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

}  // namespace mq
