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
#include "bos_rows.h"

namespace mq {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

static constexpr int kPartialSlots = 512;  // upper bound of pass-1 workgroups
int act_quant_partial_slots() { return kPartialSlots; }

template <typename T, typename Op>
__device__ inline T wave_reduce(T v, Op op) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = op(v, __shfl_xor(v, off, 64));
    return v;
}

// Both passes are bound by memory latency at the sizes of this path (5 to 80 MB per tensor): what counts is the
// number of bytes requested before the first one arrives.  The tensor is therefore walked as a flat list of 16-byte
// vectors (8 values; vector i is piece i % (K/8) of row i / (K/8)), every lane requests several vectors before it
// touches one, and the grids are sized so that every compute unit holds a few workgroups.
static constexpr int MM_U = 8;  // vectors per lane per round, pass 1
static constexpr int Q_U = 4;   // vectors per lane per round, pass 2

__global__ __launch_bounds__(256) void act_minmax_kernel(const _Float16* __restrict__ x, uint32_t nv, uint32_t K8,
                                                         long ldx, RowMap map, int flat,
                                                         float* __restrict__ partials) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float mn = INFINITY, mx = -INFINITY;
    for (uint32_t base = blockIdx.x * (256u * MM_U); base < nv; base += gridDim.x * (256u * MM_U)) {
        half8 v[MM_U];
#pragma unroll
        for (int u = 0; u < MM_U; ++u) {
            uint32_t i = base + u * 256u + threadIdx.x;
            i = i < nv ? i : nv - 1;  // a repeated vector does not change a min or a max
            if (flat) {
                v[u] = ((const half8*)x)[i];
            } else {
                const uint32_t row = i / K8, p = i - row * K8;
                v[u] = ((const half8*)(x + map.phys(row) * ldx))[p];
            }
        }
#pragma unroll
        for (int u = 0; u < MM_U; ++u)
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float f = (float)v[u][e];
                mn = fminf(mn, f);
                mx = fmaxf(mx, f);
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

static constexpr int Q_MAX_ROWS = 128;  // rows per workgroup, pass 2 (1024 output vectors of at least 8 per row)

// A workgroup converts R whole rows (so that it owns their row sums): R * Kp/8 output vectors, 1024 per round.
// BOS: workgroups from index qgrid on compute the BOS rows of a BOS-aware K/V projection instead (they depend on
// nothing this kernel produces; one launch less on a path whose kernels are all bound by launch latency).
template <bool BOS>
__global__ __launch_bounds__(256) void act_quantize_kernel(const _Float16* __restrict__ x, int M, int K, long ldx,
                                                           RowMap map, int R, const float* __restrict__ partials,
                                                           int n_partials, const float* __restrict__ act_scale,
                                                           const int32_t* __restrict__ act_zp,
                                                           int8_t* __restrict__ a8, int32_t* __restrict__ rowsum,
                                                           ActParams* __restrict__ params,
                                                           float* __restrict__ act_scale_out,
                                                           int32_t* __restrict__ act_zp_out, int qgrid, BosWork bw) {
    if constexpr (BOS) {
        if ((int)blockIdx.x >= qgrid) {  // (whole workgroups: none of them reaches a barrier below)
            if (bw.bos_out)
                bos_copy_block((int)blockIdx.x - qgrid, (int)threadIdx.x, bw);
            else
                bos_rows_block<4>((int)blockIdx.x - qgrid, (int)threadIdx.x, bw);
            return;
        }
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    __shared__ float smn[4], smx[4];
    __shared__ int lsum[Q_MAX_ROWS];
    const int r0 = blockIdx.x * R;
    const int Rr = M - r0 < R ? M - r0 : R;
    if (threadIdx.x < Q_MAX_ROWS) lsum[threadIdx.x] = 0;
    const uint32_t K8 = K >> 3;
    const uint32_t Kp = (K + 127) / 128 * 128;  // row stride of the int8 copy; the padding is zero
    const uint32_t Kp8 = Kp >> 3;               // a multiple of 16: an aligned group of 8 lanes never straddles rows
    const uint32_t nvo = (uint32_t)Rr * Kp8;
    half8 v[Q_U];
    uint32_t lr[Q_U], pp[Q_U];
    auto request = [&](uint32_t base) {
#pragma unroll
        for (int u = 0; u < Q_U; ++u) {
            const uint32_t i = base + u * 256u + threadIdx.x;
            lr[u] = i / Kp8;
            pp[u] = i - lr[u] * Kp8;
            if (i < nvo && pp[u] < K8) v[u] = ((const half8*)(x + map.phys(r0 + lr[u]) * ldx))[pp[u]];
        }
    };
    request(0);  // on its way while the parameters are derived (most workgroups have a single round)
    float s, zf;
    if (partials) {
        float mn = INFINITY, mx = -INFINITY;
        for (int i = threadIdx.x; i < n_partials; i += 256) {
            mn = fminf(mn, partials[2 * i]);
            mx = fmaxf(mx, partials[2 * i + 1]);
        }
        mn = wave_reduce(mn, [](float a, float b) { return fminf(a, b); });
        mx = wave_reduce(mx, [](float a, float b) { return fmaxf(a, b); });
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
        __syncthreads();
    }
    const float inv = 1.0f / s;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        params->scale = s;
        params->zp = (int)zf;
        if (act_scale_out) *act_scale_out = s;
        if (act_zp_out) *act_zp_out = (int)zf;
    }
    for (uint32_t base = 0; base < nvo; base += 256u * Q_U) {
        if (base) request(base);
#pragma unroll
        for (int u = 0; u < Q_U; ++u) {
            const uint32_t i = base + u * 256u + threadIdx.x;
            const bool valid = i < nvo;
            uint32_t w0 = 0, w1 = 0;
            int sum = 0;
            if (valid && pp[u] < K8) {
                int q[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float t = rintf((float)v[u][e] * inv) + zf;
                    t = fminf(fmaxf(t, 0.0f), 255.0f);
                    q[e] = (int)t - 128;
                    sum += q[e];
                }
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    w0 |= ((uint32_t)(q[k8_perm(b)] & 255)) << (8 * b);
                    w1 |= ((uint32_t)(q[k8_perm(4 + b)] & 255)) << (8 * b);
                }
            }
            // (streaming store: read next by another kernel, nothing gained by keeping it in this XCD's L2)
            if (valid) {
                const uint2v out = {w0, w1};
                __builtin_nontemporal_store(out, (uint2v*)(a8 + (long)(r0 + lr[u]) * Kp) + pp[u]);
            }
            sum += __shfl_xor(sum, 1, 64);
            sum += __shfl_xor(sum, 2, 64);
            sum += __shfl_xor(sum, 4, 64);
            if (valid && (lane & 7) == 0) atomicAdd(&lsum[lr[u]], sum);
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < Rr) rowsum[r0 + threadIdx.x] = lsum[threadIdx.x];
}

int launch_act_quant(const void* x, int M, int K, int ldx, RowMap in_map, const float* act_scale,
                     const int32_t* act_zp, int8_t* a8, int32_t* rowsum, ActParams* params, float* partials,
                     float* act_scale_out, int32_t* act_zp_out, const BosWork* bos, hipStream_t st,
                     int given_partials) {
    const uint32_t K8 = (uint32_t)K >> 3;
    const uint32_t nv = (uint32_t)M * K8;  // M * ldx * 2 < 2^31 has been checked: this fits easily
    long g1 = ((long)nv + 256 * MM_U - 1) / (256 * MM_U);
    int grid = (int)(g1 > kPartialSlots ? kPartialSlots : g1);
    const bool dynamic = act_scale == nullptr;
    // given_partials > 0: the producer of x has left that many (min, max) pairs in `partials` already (the gated
    // projection's epilogue does), so the pass over x that would find them is skipped
    if (dynamic && given_partials > 0) {
        grid = given_partials;
    } else if (dynamic) {
        const int flat = in_map.rows_per_group <= 0 && ldx == K;
        ProfScope prof(st, PROF_ACT_MINMAX, 0.0, 2.0 * M * K);
        hipLaunchKernelGGL(act_minmax_kernel, dim3(grid), dim3(256), 0, st, (const _Float16*)x, nv, K8, (long)ldx,
                           in_map, flat, partials);
        MQ_HIP_CHECK_LAUNCH();
    }
    const int Kp8 = (K + 127) / 128 * 16;
    int R = 256 * Q_U / Kp8;
    R = R < 1 ? 1 : (R > Q_MAX_ROWS ? Q_MAX_ROWS : R);
    const int qgrid = (M + R - 1) / R;
    ProfScope prof(st, PROF_ACT_QUANTIZE, 0.0, 3.0 * M * K + 4.0 * M);
    if (bos)
        hipLaunchKernelGGL(act_quantize_kernel<true>, dim3(qgrid + bos_blocks(*bos)), dim3(256), 0, st,
                           (const _Float16*)x, M, K, (long)ldx, in_map, R, dynamic ? partials : (const float*)nullptr,
                           grid, act_scale, act_zp, a8, rowsum, params, act_scale_out, act_zp_out, qgrid, *bos);
    else
        hipLaunchKernelGGL(act_quantize_kernel<false>, dim3(qgrid), dim3(256), 0, st, (const _Float16*)x, M, K,
                           (long)ldx, in_map, R, dynamic ? partials : (const float*)nullptr, grid, act_scale, act_zp,
                           a8, rowsum, params, act_scale_out, act_zp_out, qgrid, BosWork{});
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

}  // namespace mq
