// BOS rows of the BOS-aware K/V projection (paper Sec. 3.1): token 0 of every prompt is kept out of
// activation quantisation; its to_k/to_v output is the fp16 linear with the unquantised weights (fp32
// accumulation), or a copy of the vector that was pre-computed offline.
#include "mq_common.h"

namespace mq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

// One wave per output channel n; the wave walks K in 16-byte pieces and keeps one accumulator per prompt.
template <int BCHUNK>
__global__ __launch_bounds__(256) void bos_rows_kernel(const _Float16* __restrict__ ctx, int B, int T, int K,
                                                       const _Float16* __restrict__ w, const _Float16* __restrict__ bias,
                                                       _Float16* __restrict__ y, int N) {
    const int lane = threadIdx.x & 63;
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const int K8 = K >> 3;
    const half8* wr = (const half8*)(w + (size_t)n * K);
    for (int b0 = 0; b0 < B; b0 += BCHUNK) {
        float acc[BCHUNK];
#pragma unroll
        for (int i = 0; i < BCHUNK; ++i) acc[i] = 0.0f;
        for (int p = lane; p < K8; p += 64) {
            const half8 wv = wr[p];
#pragma unroll
            for (int i = 0; i < BCHUNK; ++i) {
                if (b0 + i < B) {
                    const half8 xv = ((const half8*)(ctx + (size_t)(b0 + i) * T * K))[p];
#pragma unroll
                    for (int e = 0; e < 8; ++e) acc[i] += (float)xv[e] * (float)wv[e];
                }
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
