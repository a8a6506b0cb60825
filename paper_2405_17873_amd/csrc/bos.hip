// BOS rows of the BOS-aware K/V projection (paper Sec. 3.1): token 0 of every prompt is kept out of
// activation quantisation; its to_k/to_v output is the fp16 linear with the unquantised weights (fp32
// accumulation), or a copy of the vector that was pre-computed offline.
#include "mq_common.h"

namespace mq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// One wave per output channel n.  The wave walks K in rounds of 4 x 64 sixteen-byte pieces: it requests the four
// weight pieces and the matching pieces of every prompt's BOS row before it multiplies any, so that one round trip
// to memory covers 512 k (the kernel is latency bound: a few MB of weights, a few KB of activations).
template <int BCHUNK>
__global__ __launch_bounds__(256) void bos_rows_kernel(const _Float16* __restrict__ ctx, int B, int T, int K,
                                                       const _Float16* __restrict__ w, const _Float16* __restrict__ bias,
                                                       _Float16* __restrict__ y, int N) {
    constexpr int U = 4;
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const int K8 = K >> 3;
    const half8* wr = (const half8*)(w + (size_t)n * K);
    for (int b0 = 0; b0 < B; b0 += BCHUNK) {
        float acc[BCHUNK];
#pragma unroll
        for (int i = 0; i < BCHUNK; ++i) acc[i] = 0.0f;
        for (int p0 = 0; p0 < K8; p0 += 64 * U) {
            half8 wv[U], xv[BCHUNK][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int p = p0 + u * 64 + lane;
                const int pc = p < K8 ? p : K8 - 1;  // clamped piece: its products are dropped below
                wv[u] = wr[pc];
#pragma unroll
                for (int i = 0; i < BCHUNK; ++i) {
                    const int b = b0 + i < B ? b0 + i : B - 1;
                    xv[i][u] = ((const half8*)(ctx + (size_t)b * T * K))[pc];
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
                if (bias) v += (float)bias[n];
                y[(size_t)(b0 + i) * T * N + n] = (_Float16)v;
            }
        }
    }
}

__global__ void bos_copy_kernel(const _Float16* __restrict__ bos_out, _Float16* __restrict__ y, int B, int T, int N) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)B * N) return;
    const int b = idx / N, n = idx % N;
    y[(size_t)b * T * N + n] = bos_out[n];
}

int launch_bos_rows(const void* ctx, int B, int T, int K, const void* w_f16, const void* bos_out, const void* bias,
                    void* y, int N, hipStream_t st) {
    if (bos_out) {
        const long total = (long)B * N;
        hipLaunchKernelGGL(bos_copy_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const _Float16*)bos_out, (_Float16*)y, B, T, N);
    } else {
        ProfScope prof(st, PROF_BOS_ROWS, 2.0 * B * N * K, 2.0 * N * K + 2.0 * B * K + 2.0 * B * N);
        hipLaunchKernelGGL(bos_rows_kernel<8>, dim3((N + 3) / 4), dim3(256), 0, st, (const _Float16*)ctx, B, T, K,
                           (const _Float16*)w_f16, (const _Float16*)bias, (_Float16*)y, N);
    }
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

}  // namespace mq
