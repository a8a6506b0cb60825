// Per-tensor 8-bit activation quantisation (paper Sec. 4.1 "Quantization Scheme": one scale and
// zero point per activation tensor; Sec. 4.3: the FP16->INT8 conversion that precedes the integer GEMM).
//
//   pass 1 (dynamic only): every workgroup reduces the min/max of its rows with wavefront shuffles and
//           writes one partial pair; no atomics, no pre-cleared memory, order independent.
//   pass 2: every workgroup re-reduces the partials (a few KB, L2 resident), derives (scale, zp) with the
//           same fp32 operations as the weight quantiser, then converts its rows:
//               a'[m,k] = clamp(rne(x*inv) + zp, 0, 255) - 128   stored as int8, groups of 8 k in the order
//               0,4,1,5,2,6,3,7, rows padded with zeros to a multiple of 128, and rowsum[m] = sum_k a'[m,k].
//
// Compiled with -ffp-contract=off: each fp32 operation rounds once.
#include "mq_common.h"

namespace mq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));

static constexpr int kPartialSlots = 1024;  // upper bound of pass-1 workgroups
int act_quant_partial_slots() { return kPartialSlots; }

template <typename T, typename Op>
__device__ inline T wave_reduce(T v, Op op) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = op(v, __shfl_xor(v, off, 64));
    return v;
}

// A wave walks RPW rows at a time with 16-byte loads, so that every lane keeps RPW (or more) loads in flight.
static constexpr int RPW = 4;

__global__ __launch_bounds__(256) void act_minmax_kernel(const _Float16* __restrict__ x, int M, int K, long ldx,
                                                         RowMap map, float* __restrict__ partials) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int K8 = K >> 3;
    float mn = INFINITY, mx = -INFINITY;
    for (long r0 = ((long)blockIdx.x * 4 + wv) * RPW; r0 < M; r0 += (long)gridDim.x * 4 * RPW) {
        const half8* row[RPW];
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const long r = r0 + j < M ? r0 + j : M - 1;  // a repeated row does not change a min or a max
            row[j] = (const half8*)(x + map.phys(r) * ldx);
        }
        for (int p = lane; p < K8; p += 64) {
            half8 v[RPW];
#pragma unroll
            for (int j = 0; j < RPW; ++j) v[j] = row[j][p];
#pragma unroll
            for (int j = 0; j < RPW; ++j)
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float f = (float)v[j][e];
                    mn = fminf(mn, f);
                    mx = fmaxf(mx, f);
                }
        }
    }
    mn = wave_reduce(mn, [](float a, float b) { return fminf(a, b); });
    mx = wave_reduce(mx, [](float a, float b) { return fmaxf(a, b); });
    __shared__ float smn[4], smx[4];
    if (lane == 0) {
        smn[wv] = mn;
        smx[wv] = mx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        partials[2 * blockIdx.x] = fminf(fminf(smn[0], smn[1]), fminf(smn[2], smn[3]));
        partials[2 * blockIdx.x + 1] = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
    }
}

__global__ __launch_bounds__(256) void act_quantize_kernel(const _Float16* __restrict__ x, int M, int K, long ldx,
                                                           RowMap map, const float* __restrict__ partials,
                                                           int n_partials, const float* __restrict__ act_scale,
                                                           const int32_t* __restrict__ act_zp,
                                                           int8_t* __restrict__ a8, int32_t* __restrict__ rowsum,
                                                           ActParams* __restrict__ params,
                                                           float* __restrict__ act_scale_out,
                                                           int32_t* __restrict__ act_zp_out) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float s, zf;
    if (partials) {
        float mn = INFINITY, mx = -INFINITY;
        for (int i = threadIdx.x; i < n_partials; i += 256) {
            mn = fminf(mn, partials[2 * i]);
            mx = fmaxf(mx, partials[2 * i + 1]);
        }
        mn = wave_reduce(mn, [](float a, float b) { return fminf(a, b); });
        mx = wave_reduce(mx, [](float a, float b) { return fmaxf(a, b); });
        __shared__ float smn[4], smx[4];
        if (lane == 0) {
            smn[wv] = mn;
            smx[wv] = mx;
        }
        __syncthreads();
        mn = fminf(fminf(smn[0], smn[1]), fminf(smn[2], smn[3]));
        mx = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));
        const float lo = fminf(mn, 0.0f), hi = fmaxf(mx, 0.0f);
        s = 1.0f;
        if (hi != lo) {
            const float range = hi - lo;
            s = range / 255.0f;
        }
        const float inv0 = 1.0f / s;
        zf = rintf((-lo) * inv0);
        zf = fminf(fmaxf(zf, 0.0f), 255.0f);
    } else {
        s = *act_scale;
        zf = (float)*act_zp;
    }
    const float inv = 1.0f / s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        params->scale = s;
        params->zp = (int)zf;
        if (act_scale_out) *act_scale_out = s;
        if (act_zp_out) *act_zp_out = (int)zf;
    }
    const int K8 = K >> 3;
    const int Kp = (K + 127) / 128 * 128;  // row stride of the int8 copy; the padding is zero
    for (long r0 = ((long)blockIdx.x * 4 + wv) * RPW; r0 < M; r0 += (long)gridDim.x * 4 * RPW) {
        const half8* row[RPW];
        int sum[RPW];
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const long r = r0 + j < M ? r0 + j : M - 1;
            row[j] = (const half8*)(x + map.phys(r) * ldx);
            sum[j] = 0;
        }
        for (int p = lane; p < (Kp >> 3); p += 64) {
            half8 v[RPW];
            if (p < K8) {
#pragma unroll
                for (int j = 0; j < RPW; ++j) v[j] = row[j][p];
            }
#pragma unroll
            for (int j = 0; j < RPW; ++j) {
                uint32_t w0 = 0, w1 = 0;
                if (p < K8) {
                    int q[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float t = rintf((float)v[j][e] * inv) + zf;
                        t = fminf(fmaxf(t, 0.0f), 255.0f);
                        q[e] = (int)t - 128;
                        sum[j] += q[e];
                    }
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        w0 |= ((uint32_t)(q[k8_perm(b)] & 255)) << (8 * b);
                        w1 |= ((uint32_t)(q[k8_perm(4 + b)] & 255)) << (8 * b);
                    }
                }
                if (r0 + j < M) ((uint2*)(a8 + (r0 + j) * (long)Kp))[p] = make_uint2(w0, w1);
            }
        }
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int t = wave_reduce(sum[j], [](int a, int b) { return a + b; });
            if (lane == 0 && r0 + j < M) rowsum[r0 + j] = t;
        }
    }
}

int launch_act_quant(const void* x, int M, int K, int ldx, RowMap in_map, const float* act_scale,
                     const int32_t* act_zp, int8_t* a8, int32_t* rowsum, ActParams* params, float* partials,
                     float* act_scale_out, int32_t* act_zp_out, hipStream_t st) {
    int grid = (M + 4 * RPW - 1) / (4 * RPW);
    if (grid > kPartialSlots) grid = kPartialSlots;
    const bool dynamic = act_scale == nullptr;
    if (dynamic) {
        ProfScope prof(st, PROF_ACT_MINMAX, 0.0, 2.0 * M * K);
        hipLaunchKernelGGL(act_minmax_kernel, dim3(grid), dim3(256), 0, st, (const _Float16*)x, M, K, (long)ldx, in_map,
                           partials);
        MQ_HIP_CHECK_LAUNCH();
    }
    int qgrid = (M + 4 * RPW - 1) / (4 * RPW);
    if (qgrid > 4096) qgrid = 4096;
    ProfScope prof(st, PROF_ACT_QUANTIZE, 0.0, 3.0 * M * K + 4.0 * M);
    hipLaunchKernelGGL(act_quantize_kernel, dim3(qgrid), dim3(256), 0, st, (const _Float16*)x, M, K, (long)ldx, in_map,
                       dynamic ? partials : (const float*)nullptr, grid, act_scale, act_zp, a8, rowsum, params,
                       act_scale_out, act_zp_out);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

}  // namespace mq
