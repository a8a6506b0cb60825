// Device-side bodies of the BOS rows of the BOS-aware K/V projection (paper Sec. 3.1): token 0 of every prompt is kept
// out of activation quantisation; its to_k/to_v output is the fp16 linear with the unquantised weights (fp32
// accumulation), or a copy of the vector that was pre-computed offline.  They are functions of a block index so that
// they can run as a kernel of their own or as extra workgroups of the activation-quantise launch.
#pragma once
#include "mq_common.h"

namespace mq {

typedef _Float16 bos_half8 __attribute__((ext_vector_type(8)));

// 256 threads: one wave per output channel n = 4 * blk + wave.  The wave walks K in rounds of 4 x 64 sixteen-byte
// pieces: it requests the four weight pieces and the matching pieces of BCHUNK prompts' BOS rows before it multiplies
// any, so that one round trip to memory covers 512 k (latency bound: a few MB of weights, a few KB of activations).
template <int BCHUNK>
__device__ __forceinline__ void bos_rows_block(int blk, int tid, const BosWork& bw) {
    constexpr int U = 4;
    const int lane = tid & 63;
    const int n = blk * 4 + (tid >> 6);
    if (n >= bw.N) return;
    const int K = bw.K, B = bw.B, T = bw.T, N = bw.N;
    const int K8 = K >> 3;
    const bos_half8* wr = (const bos_half8*)(bw.w_f16 + (size_t)n * K);
    for (int b0 = 0; b0 < B; b0 += BCHUNK) {
        float acc[BCHUNK];
#pragma unroll
        for (int i = 0; i < BCHUNK; ++i) acc[i] = 0.0f;
        for (int p0 = 0; p0 < K8; p0 += 64 * U) {
            bos_half8 wv[U], xv[BCHUNK][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = p0 + u * 64 + lane;
                const int pc = p < K8 ? p : K8 - 1;  // clamped piece: its products are dropped below
                wv[u] = wr[pc];
#pragma unroll
                for (int i = 0; i < BCHUNK; ++i) {
                    const int b = b0 + i < B ? b0 + i : B - 1;
                    xv[i][u] = ((const bos_half8*)(bw.ctx + (size_t)b * T * K))[pc];
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (p0 + u * 64 + lane >= K8) continue;
#pragma unroll
                for (int i = 0; i < BCHUNK; ++i)
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i] += (float)xv[i][u][e] * (float)wv[u][e];
            }
        }
#pragma unroll
        for (int i = 0; i < BCHUNK; ++i) {
            float v = acc[i];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
            if (lane == 0 && b0 + i < B) {
                if (bw.bias) v += (float)bw.bias[n];
                bw.y[(size_t)(b0 + i) * T * N + n] = (_Float16)v;
            }
        }
    }
}

// 256 threads copy 256 of the B * N pre-computed values.
__device__ __forceinline__ void bos_copy_block(int blk, int tid, const BosWork& bw) {
    const long idx = (long)blk * 256 + tid;
    if (idx >= (long)bw.B * bw.N) return;
    const int b = (int)(idx / bw.N), n = (int)(idx % bw.N);
    bw.y[(size_t)b * bw.T * bw.N + n] = bw.bos_out[n];
}

// Workgroups (of 256 threads) that the BOS rows take.
inline int bos_blocks(const BosWork& bw) {
    return bw.bos_out ? (int)(((long)bw.B * bw.N + 255) / 256) : (bw.N + 3) / 4;
}

}  // namespace mq
