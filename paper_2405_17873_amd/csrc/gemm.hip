// MFMA GEMMs of the quantized-linear hot path for gfx950 (64-wide wavefronts, 32x32 MFMA tiles).
//
//   gemm_w_only : Y = X . dequant(Wq)^T      fp16 MFMA (v_mfma_f32_32x32x16_f16), fp32 accumulate
//                 (paper App. C item 2: weight-only layers keep 16-bit floating-point compute)
//   gemm_a8     : ACC = A8 . W8^T            int8 MFMA (v_mfma_i32_32x32x32_i8), int32 accumulate
//                 (paper Sec. 4.3 / App. C item 4: integer GEMM for W8A8; 4-bit codes widened for W4A8)
//
// Shared structure
//   * One workgroup = 4 waves arranged WGM x WGN; each wave owns TM x TN MFMA tiles of 32x32.
//   * The activation operand goes HBM -> registers -> LDS (double buffered, 128 bytes of K per row per
//     stage, 16-byte pieces XOR-swizzled so that ds_read_b128 of 32 consecutive rows is conflict free).
//   * The weight operand never touches LDS: the packed kernel layout stores, for every 32-channel x 64-k
//     tile, the 64 lane chunks in lane order, so one global_load per 16 bytes of chunk is a fully contiguous
//     wave access and lands directly in the MFMA operand's lane.  Codes are widened in registers.
//   * The MFMA is issued with the weight fragment as the first operand: the 32x32 result then holds, per
//     lane, 4 consecutive output channels of one activation row, i.e. an 8-byte fp16 store.
//   * k-order inside a stage is permuted identically for both operands (a sum does not care), chosen so
//     that every lane's global and LDS accesses are 16 bytes wide.
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
    static constexpr int WORDS = BITS == 8 ? 8 : BITS;  // 32-bit words per lane per 64-k tile
    uint32_t w[WORDS];
};

template <int SHIFT>
__device__ __forceinline__ half2v field_to_h2(uint32_t w, uint32_t mask, int z) {
    // field value sits at bit SHIFT of each half: magic|field = 1024 + 2^SHIFT q
    const half2v v = as_h2((w & mask) | 0x64006400u);
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

template <int BITS>
__device__ __forceinline__ void load_chunk(WChunk<BITS>& c, const uint8_t* tile, int lane) {
    if constexpr (BITS == 4) {
        const uint4v v = *(const uint4v*)(tile + lane * 16);
        c.w[0] = v[0]; c.w[1] = v[1]; c.w[2] = v[2]; c.w[3] = v[3];
    } else if constexpr (BITS == 2) {
        const uint2v v = *(const uint2v*)(tile + lane * 8);
        c.w[0] = v[0]; c.w[1] = v[1];
    } else if constexpr (BITS == 3) {
        const uint32_t* p = (const uint32_t*)(tile + lane * 12);
        c.w[0] = p[0]; c.w[1] = p[1]; c.w[2] = p[2];
    } else {
        const uint4v v0 = *(const uint4v*)(tile + lane * 16);
        const uint4v v1 = *(const uint4v*)(tile + 1024 + lane * 16);
        c.w[0] = v0[0]; c.w[1] = v0[1]; c.w[2] = v0[2]; c.w[3] = v0[3];
        c.w[4] = v1[0]; c.w[5] = v1[1]; c.w[6] = v1[2]; c.w[7] = v1[3];
    }
}

// Chunk of a k range that does not exist: every byte must widen to 0, i.e. hold `fill` = the flip mask.
template <int BITS>
__device__ __forceinline__ void zero_chunk(WChunk<BITS>& c, uint32_t fill) {
#pragma unroll
    for (int i = 0; i < WChunk<BITS>::WORDS; ++i) c.w[i] = fill;
}

// ---------------------------------------------------------------------------------------------
// Activation tile: BM rows x 128 bytes, staged through registers into swizzled LDS.
// ---------------------------------------------------------------------------------------------
template <int BM>
struct AStage {
    static constexpr int LOADS = BM / 32;  // 16-byte loads per thread (256 threads)
    uint4v v[LOADS];
};

// row_bytes: byte stride of a source row; col_byte: byte offset of this stage inside the row;
// valid_bytes: bytes of the row that exist from col_byte on (pieces beyond are re-read from column 0:
// their products meet zero weights).
template <int BM>
__device__ __forceinline__ void a_stage_load(AStage<BM>& st, const uint8_t* src, long row_bytes, int m0, int M,
                                            long col_byte, long row_len_bytes) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int r = 0; r < AStage<BM>::LOADS; ++r) {
        const int q = tid + 256 * r;
        const int row = q >> 3, piece = q & 7;
        int gr = m0 + row;
        gr = gr < M ? gr : M - 1;
        long cb = col_byte + piece * 16;
        cb = cb < row_len_bytes ? cb : 0;
        st.v[r] = *(const uint4v*)(src + (long)gr * row_bytes + cb);
    }
}

template <int BM>
__device__ __forceinline__ void a_stage_store(const AStage<BM>& st, uint8_t* lds) {
    const int tid = threadIdx.x;
#pragma unroll
    for (int r = 0; r < AStage<BM>::LOADS; ++r) {
        const int q = tid + 256 * r;
        const int row = q >> 3, piece = q & 7;
        *(uint4v*)(lds + row * 128 + ((piece ^ swz(row)) << 4)) = st.v[r];
    }
}

// ---------------------------------------------------------------------------------------------
// Weight-only GEMM
// ---------------------------------------------------------------------------------------------
template <int BITS, int WGM, int WGN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_w_only_kernel(const _Float16* __restrict__ x, int M, int K, long ldx,
                                                          const uint8_t* __restrict__ packed, int N,
                                                          const float* __restrict__ w_scale,
                                                          const int32_t* __restrict__ w_zp,
                                                          const _Float16* __restrict__ bias,
                                                          _Float16* __restrict__ y, long ldy, int tiles_n) {
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int bn = blockIdx.x % tiles_n, bm = blockIdx.x / tiles_n;
    const int m0 = bm * BM, n0 = bn * BN;
    const int KC = K >> 6;
    const int G = (N + 31) >> 5;
    const int l31 = lane & 31, kb = lane >> 5;

    // per-lane zero points of the TN weight fragments and their tile pointers
    int zc[TN];
    const uint8_t* wtile[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        int g = (n0 >> 5) + wn * TN + tn;
        g = g < G ? g : G - 1;
        const int n = g * 32 + l31;
        zc[tn] = w_zp[n < N ? n : N - 1];
        wtile[tn] = packed + (size_t)g * KC * kl_tile_bytes(BITS);
    }

    float16v acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0.0f;

    AStage<BM> ast;
    WChunk<BITS> wcur[TN], wnxt[TN];
    const uint8_t* xsrc = (const uint8_t*)x;
    const long row_bytes = ldx * 2, row_len = (long)K * 2;

    a_stage_load<BM>(ast, xsrc, row_bytes, m0, M, 0, row_len);
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) load_chunk<BITS>(wcur[tn], wtile[tn], lane);
    a_stage_store<BM>(ast, lds);
    __syncthreads();

    const int sw = swz(l31);
    int cur = 0;
    for (int kc = 0; kc < KC; ++kc) {
        const bool more = kc + 1 < KC;
        if (more) {
            a_stage_load<BM>(ast, xsrc, row_bytes, m0, M, (long)(kc + 1) * 128, row_len);
#pragma unroll
            for (int tn = 0; tn < TN; ++tn)
                load_chunk<BITS>(wnxt[tn], wtile[tn] + (size_t)(kc + 1) * kl_tile_bytes(BITS), lane);
        }
        const uint8_t* abuf = lds + cur * (BM * 128);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            half8 wf[TN], xf[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) wf[tn] = dequant_step<BITS>(wcur[tn], s, zc[tn]);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = (wm * TM + tm) * 32 + l31;
                xf[tm] = *(const half8*)(abuf + row * 128 + (((kb * 4 + s) ^ sw) << 4));
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_f32_32x32x16_f16(wf[tn], xf[tm], acc[tm][tn], 0, 0, 0);
        }
        if (more) a_stage_store<BM>(ast, lds + (cur ^ 1) * (BM * 128));
        __syncthreads();
        if (more) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) wcur[tn] = wnxt[tn];
        }
        cur ^= 1;
    }

    // epilogue: result element v of a lane is channel 8*(v/4) + 4*kb + v%4 of the tile, row l31
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int nb = n0 + (wn * TN + tn) * 32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = nb + 8 * q + 4 * kb;
            if (n >= N) continue;
            const float4v sc = *(const float4v*)(w_scale + n);
            float4v bs = {0.f, 0.f, 0.f, 0.f};
            if (bias) {
                const half4 b = *(const half4*)(bias + n);
                bs = float4v{(float)b[0], (float)b[1], (float)b[2], (float)b[3]};
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int m = m0 + (wm * TM + tm) * 32 + l31;
                if (m >= M) continue;
                half4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) o[r] = (_Float16)(acc[tm][tn][4 * q + r] * sc[r] + bs[r]);
                *(half4*)(y + (long)m * ldy + n) = o;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// 8-bit-activation GEMM.  A stage is 128 k (128 bytes of int8 per row) = two 64-k weight tiles.
// ---------------------------------------------------------------------------------------------
// xflip = 0x80808080 turns unsigned 8-bit codes q into the signed bytes q - 128 (0 for signed codes).
template <int WBITS>
__device__ __forceinline__ int4v widen_step(const WChunk<WBITS>& c, int s /*0..1 inside the 64-k tile*/,
                                            uint32_t xflip) {
    if constexpr (WBITS == 8) {
        return int4v{(int)(c.w[4 * s] ^ xflip), (int)(c.w[4 * s + 1] ^ xflip), (int)(c.w[4 * s + 2] ^ xflip),
                     (int)(c.w[4 * s + 3] ^ xflip)};
    } else {
        const uint32_t w0 = c.w[2 * s], w1 = c.w[2 * s + 1];
        return int4v{(int)(w0 & 0x0F0F0F0Fu), (int)((w0 >> 4) & 0x0F0F0F0Fu), (int)(w1 & 0x0F0F0F0Fu),
                     (int)((w1 >> 4) & 0x0F0F0F0Fu)};
    }
}

template <int WBITS, int WGM, int WGN, int TM, int TN>
__global__ __launch_bounds__(256) void gemm_a8_kernel(const int8_t* __restrict__ a8,
                                                      const int32_t* __restrict__ rowsum,
                                                      const ActParams* __restrict__ params, int M, int K,
                                                      const uint8_t* __restrict__ packed, int N, int w_off,
                                                      const float* __restrict__ w_scale,
                                                      const int32_t* __restrict__ w_zp,
                                                      const int32_t* __restrict__ w_colsum,
                                                      const _Float16* __restrict__ bias, _Float16* __restrict__ y,
                                                      long ldy, RowMap out_map, int32_t* __restrict__ acc_debug,
                                                      int tiles_n) {
    static_assert(WGM * WGN == 4, "four waves per workgroup");
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int wm = wv / WGN, wn = wv % WGN;
    const int bn = blockIdx.x % tiles_n, bm = blockIdx.x / tiles_n;
    const int m0 = bm * BM, n0 = bn * BN;
    const int KC = K >> 6;
    const int KT = (KC + 1) >> 1;
    const int G = (N + 31) >> 5;
    const int l31 = lane & 31, kb = lane >> 5;
    const uint32_t xflip = w_off ? 0x80808080u : 0u;

    const uint8_t* wtile[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        int g = (n0 >> 5) + wn * TN + tn;
        g = g < G ? g : G - 1;
        wtile[tn] = packed + (size_t)g * KC * kl_tile_bytes(WBITS);
    }

    int16v acc[TM][TN];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm)
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[tm][tn][i] = 0;

    AStage<BM> ast;
    WChunk<WBITS> wcur[TN][2], wnxt[TN][2];
    const uint8_t* asrc = (const uint8_t*)a8;

    auto load_w = [&](WChunk<WBITS>(&dst)[TN][2], int kt) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn)
#pragma unroll
            for (int cc = 0; cc < 2; ++cc) {
                const int ch = 2 * kt + cc;
                if (ch < KC)
                    load_chunk<WBITS>(dst[tn][cc], wtile[tn] + (size_t)ch * kl_tile_bytes(WBITS), lane);
                else
                    zero_chunk<WBITS>(dst[tn][cc], xflip);
            }
    };

    a_stage_load<BM>(ast, asrc, (long)K, m0, M, 0, (long)K);
    load_w(wcur, 0);
    a_stage_store<BM>(ast, lds);
    __syncthreads();

    const int sw = swz(l31);
    int cur = 0;
    for (int kt = 0; kt < KT; ++kt) {
        const bool more = kt + 1 < KT;
        if (more) {
            a_stage_load<BM>(ast, asrc, (long)K, m0, M, (long)(kt + 1) * 128, (long)K);
            load_w(wnxt, kt + 1);
        }
        const uint8_t* abuf = lds + cur * (BM * 128);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int cc = s >> 1, sp = s & 1;
            int4v wf[TN], xf[TM];
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) wf[tn] = widen_step<WBITS>(wcur[tn][cc], sp, xflip);
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int row = (wm * TM + tm) * 32 + l31;
                xf[tm] = *(const int4v*)(abuf + row * 128 + (((cc * 4 + kb * 2 + sp) ^ sw) << 4));
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm)
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    acc[tm][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[tn], xf[tm], acc[tm][tn], 0, 0, 0);
        }
        if (more) a_stage_store<BM>(ast, lds + (cur ^ 1) * (BM * 128));
        __syncthreads();
        if (more) {
#pragma unroll
            for (int tn = 0; tn < TN; ++tn) {
                wcur[tn][0] = wnxt[tn][0];
                wcur[tn][1] = wnxt[tn][1];
            }
        }
        cur ^= 1;
    }

    // epilogue.  Stored operands are a' = qx - 128 and b' = qw - w_off, so with dx = 128 - z_x and
    // dw[n] = w_off - z_w[n]:   ACC = raw + dw[n] * rowsum_a'[m] + dx * (colsum_b'[n] + K * dw[n]),
    // colsum_b'[n] = colsum_code[n] - K * w_off.  Wrap-around int32 arithmetic is exact because ACC fits.
    const float sx = params->scale;
    const int dx = 128 - params->zp;
    int ra[TM];
#pragma unroll
    for (int tm = 0; tm < TM; ++tm) {
        const int m = m0 + (wm * TM + tm) * 32 + l31;
        ra[tm] = rowsum[m < M ? m : M - 1];
    }
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) {
        const int nb = n0 + (wn * TN + tn) * 32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int n = nb + 8 * q + 4 * kb;
            if (n >= N) continue;
            const float4v sc = *(const float4v*)(w_scale + n);
            const int4v zw = *(const int4v*)(w_zp + n);
            const int4v cs = *(const int4v*)(w_colsum + n);
            float4v bs = {0.f, 0.f, 0.f, 0.f};
            if (bias) {
                const half4 b = *(const half4*)(bias + n);
                bs = float4v{(float)b[0], (float)b[1], (float)b[2], (float)b[3]};
            }
            int dw[4], cn[4];
            float sf[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                dw[r] = w_off - zw[r];
                cn[r] = dx * (cs[r] - K * w_off + K * dw[r]);
                sf[r] = sx * sc[r];
            }
#pragma unroll
            for (int tm = 0; tm < TM; ++tm) {
                const int m = m0 + (wm * TM + tm) * 32 + l31;
                if (m >= M) continue;
                int4v a;
                half4 o;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    a[r] = acc[tm][tn][4 * q + r] + dw[r] * ra[tm] + cn[r];
                    o[r] = (_Float16)((float)a[r] * sf[r] + bs[r]);
                }
                const long yr = out_map.phys(m);
                *(half4*)(y + yr * ldy + n) = o;
                if (acc_debug) *(int4v*)(acc_debug + (long)m * N + n) = a;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Launchers
// ---------------------------------------------------------------------------------------------
template <int BITS, int WGM, int WGN, int TM, int TN>
static int run_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, const float* w_scale,
                      const int32_t* w_zp, const void* bias, void* y, int ldy, hipStream_t st) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    auto kern = gemm_w_only_kernel<BITS, WGM, WGN, TM, TN>;
    // algorithmic traffic: X read once, packed W, scale + zp + bias, Y written once
    ProfScope prof(st, prof_gemm_slot(0, BITS, TM == 4 ? 0 : TM == 2 ? 1 : 2), 2.0 * M * N * K,
                   2.0 * M * K + (double)N * K * BITS / 8 + 10.0 * N + 2.0 * M * N);
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), 2 * BM * 128, st, (const _Float16*)x, M, K, (long)ldx,
                       (const uint8_t*)packed, N, w_scale, w_zp, (const _Float16*)bias, (_Float16*)y, (long)ldy,
                       tiles_n);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

// Tile choice: the largest tile that still gives every compute unit about two workgroups.
static int g_force_tile = -1;
void set_force_tile(int t) { g_force_tile = t; }

static int pick_tile(int M, int N) {
    if (g_force_tile >= 0 && g_force_tile <= 2) return g_force_tile;
    const long t128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (t128 >= 256) return 1;
    return 2;
}

template <int BITS>
static int dispatch_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, const float* w_scale,
                           const int32_t* w_zp, const void* bias, void* y, int ldy, hipStream_t st) {
    switch (pick_tile(M, N)) {
        case 0: return run_w_only<BITS, 2, 2, 4, 4>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
        case 1: return run_w_only<BITS, 2, 2, 2, 2>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
        default: return run_w_only<BITS, 2, 2, 1, 1>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
    }
}

int launch_gemm_w_only(const void* x, int M, int K, int ldx, const void* packed, int N, int bits,
                       const float* w_scale, const int32_t* w_zp, const void* bias, void* y, int ldy, int dtype,
                       hipStream_t st) {
    (void)dtype;
    switch (bits) {
        case 2: return dispatch_w_only<2>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
        case 3: return dispatch_w_only<3>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
        case 4: return dispatch_w_only<4>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
        case 8: return dispatch_w_only<8>(x, M, K, ldx, packed, N, w_scale, w_zp, bias, y, ldy, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

template <int WBITS, int WGM, int WGN, int TM, int TN>
static int run_a8(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K, const void* packed,
                  int N, int w_off, const float* w_scale, const int32_t* w_zp, const int32_t* w_colsum,
                  const void* bias, void* y, int ldy, RowMap out_map, int32_t* acc_debug, hipStream_t st) {
    constexpr int BM = WGM * TM * 32, BN = WGN * TN * 32;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    auto kern = gemm_a8_kernel<WBITS, WGM, WGN, TM, TN>;
    // algorithmic traffic of the integer GEMM itself: int8 activations, packed W, per-channel vectors, Y
    ProfScope prof(st, prof_gemm_slot(1, WBITS, TM == 4 ? 0 : TM == 2 ? 1 : 2), 2.0 * M * N * K,
                   1.0 * M * K + 4.0 * M + (double)N * K * WBITS / 8 + 14.0 * N + 2.0 * M * N);
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(256), 2 * BM * 128, st, a8, rowsum, params, M, K,
                       (const uint8_t*)packed, N, w_off, w_scale, w_zp, w_colsum, (const _Float16*)bias, (_Float16*)y,
                       (long)ldy, out_map, acc_debug, tiles_n);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

template <int WBITS>
static int dispatch_a8(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                       const void* packed, int N, int w_off, const float* w_scale, const int32_t* w_zp,
                       const int32_t* w_colsum, const void* bias, void* y, int ldy, RowMap out_map,
                       int32_t* acc_debug, hipStream_t st) {
    switch (pick_tile(M, N)) {
        case 0:
            return run_a8<WBITS, 2, 2, 4, 4>(a8, rowsum, params, M, K, packed, N, w_off, w_scale, w_zp, w_colsum, bias,
                                            y, ldy, out_map, acc_debug, st);
        case 1:
            return run_a8<WBITS, 2, 2, 2, 2>(a8, rowsum, params, M, K, packed, N, w_off, w_scale, w_zp, w_colsum, bias,
                                            y, ldy, out_map, acc_debug, st);
        default:
            return run_a8<WBITS, 2, 2, 1, 1>(a8, rowsum, params, M, K, packed, N, w_off, w_scale, w_zp, w_colsum, bias,
                                            y, ldy, out_map, acc_debug, st);
    }
}

int launch_gemm_a8(const int8_t* a8, const int32_t* rowsum, const ActParams* params, int M, int K,
                   const void* packed, int N, int w_bits, int w_signed, const float* w_scale, const int32_t* w_zp,
                   const int32_t* w_colsum, const void* bias, void* y, int ldy, RowMap out_map, int32_t* acc_debug,
                   hipStream_t st) {
    if (w_bits == 4)
        return dispatch_a8<4>(a8, rowsum, params, M, K, packed, N, 0, w_scale, w_zp, w_colsum, bias, y, ldy, out_map,
                              acc_debug, st);
    if (w_bits == 8) {
        // Unsigned 8-bit codes do not fit a signed MFMA operand: the kernel flips their top bit in registers,
        // which reads them as q - 128 (w_off = 128); signed (symmetric) codes are used as they are.
        return dispatch_a8<8>(a8, rowsum, params, M, K, packed, N, w_signed ? 0 : 128, w_scale, w_zp, w_colsum, bias,
                              y, ldy, out_map, acc_debug, st);
    }
    return MQ_ERR_UNSUPPORTED_BITS;
}

}  // namespace mq
