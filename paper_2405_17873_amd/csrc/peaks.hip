// Microbenchmarks of the chip itself: what a kernel of this library could reach at best on the machine it runs on.
// The per-shape report prints its fractions against these measured rates beside the published peaks.  Each kind runs
// one kernel of fixed work between two events on the given stream and returns the elapsed milliseconds of the best of
// five runs; the caller turns that into a rate with the work figures stated per kind below.  Measurement hooks only:
// they synchronise, and nothing in the hot path calls them.
#include "mq_common.h"

namespace mq {

typedef int int16v __attribute__((ext_vector_type(16)));
typedef int int4v __attribute__((ext_vector_type(4)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

static constexpr int kGrid = 512;        // two workgroups per compute unit
static constexpr int kMfmaIters = 4096;  // iterations of 4 independent MFMAs per wave
static constexpr int kValuPerIter = 32;  // vector ALU instructions a VALU wave issues per iteration (4 x 32 = 128 cycles,
                                         // the time of the 4 MFMAs of an MFMA wave's iteration)

// One vector ALU instruction that the compiler can neither remove nor merge.
__device__ __forceinline__ void valu_op(uint32_t& x, uint32_t y) { asm volatile("v_xor_b32 %0, %0, %1" : "+v"(x) : "v"(y)); }

// ROLE of a wave: 1 = MFMA only, 2 = VALU only, 3 = both in one instruction stream (1 MFMA, then NV VALU, ...), 0 = exit.
// Per iteration: 4 independent MFMAs (128 cycles of the matrix pipe) and / or 4 * NV vector ALU instructions (NV = 8:
// 128 cycles).
template <bool I8, int ROLE, int NV = kValuPerIter / 4>
__device__ __forceinline__ void role_loop(int iters, int* out) {
    if constexpr (ROLE == 0) return;
    int4v a = {(int)threadIdx.x, 1, 2, 3}, b = {3, 2, 1, (int)blockIdx.x};
    half8 ha, hb;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        ha[i] = (_Float16)(threadIdx.x * 0.001f + i);
        hb[i] = (_Float16)(i * 0.5f);
    }
    asm volatile("" : "+v"(a), "+v"(b), "+v"(ha), "+v"(hb));  // operands live in vector registers for the whole loop
    int16v acc[4];
    float16v facc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            acc[j][i] = 0;
            facc[j][i] = 0;
        }
    uint32_t x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = threadIdx.x + i;
    uint32_t y = blockIdx.x | 1u;
    asm volatile("" : "+v"(y));
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr ((ROLE & 1) != 0) {
                if constexpr (I8)
                    acc[j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[j], 0, 0, 0);
                else
                    facc[j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(ha, hb, facc[j], 0, 0, 0);
            }
            if constexpr ((ROLE & 2) != 0) {
#pragma unroll
                for (int v = 0; v < NV; ++v) valu_op(x[v], y);
            }
            __builtin_amdgcn_sched_barrier(0);  // keep the order as written: MFMA, its share of the VALU work, next MFMA
        }
    }
    int s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 16; ++i) s += acc[j][i] + (int)facc[j][i];
#pragma unroll
    for (int i = 0; i < 8; ++i) s += (int)x[i];
    if (s == 0x7fffffff) out[0] = s;
}

// Waves 0..3 of the 512-thread workgroup take ROLE_LO, waves 4..7 ROLE_HI; wave w and wave w + 4 share a SIMD.
template <bool I8, int ROLE_LO, int ROLE_HI, int NV = kValuPerIter / 4>
__global__ __launch_bounds__(512) void mfma_valu_kernel(int iters, int* out) {
    if (__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) < 4)
        role_loop<I8, ROLE_LO, NV>(iters, out);
    else
        role_loop<I8, ROLE_HI, NV>(iters, out);
}

// Read-only stream: every lane reads 16 bytes x 8 per round, grid stride, nothing is written.
__global__ __launch_bounds__(256) void read_stream_kernel(const uint4v* __restrict__ p, size_t n16, uint32_t* out) {
    uint4v acc = {0, 0, 0, 0};
    const size_t stride = (size_t)gridDim.x * 256 * 8;
    for (size_t i = (size_t)blockIdx.x * 256 * 8 + threadIdx.x; i + 7 * 256 < n16; i += stride) {
        uint4v v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; ++u) acc ^= v[u];
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;
}

// LDS read rate: every wave reads 8 KB of its workgroup's LDS per iteration with ds_read_b128, in the swizzled row
// pattern the GEMMs use for their activation fragments.
__global__ __launch_bounds__(256) void lds_read_kernel(int iters, uint32_t* out) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[32768];
    for (int i = threadIdx.x; i < 8192; i += 256) ((uint32_t*)lds)[i] = i;
    __syncthreads();
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int row = lane & 31, kb = lane >> 5;
    const int sw = (row & 7) ^ ((row >> 3) & 1);
    uint32_t base[4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
        base[s] = (uint32_t)(uintptr_t)lds + wv * 8192 + row * 128 + ((((s >> 1) * 4 + kb * 2 + (s & 1)) ^ sw) << 4);
    uint32_t sum = 0;
    for (int it = 0; it < iters; ++it) {
        uint4v a0, a1, a2, a3, a4, a5, a6, a7;
        asm volatile(
            "ds_read_b128 %0, %8\n ds_read_b128 %1, %9\n ds_read_b128 %2, %10\n ds_read_b128 %3, %11\n"
            "ds_read_b128 %4, %8 offset:4096\n ds_read_b128 %5, %9 offset:4096\n ds_read_b128 %6, %10 offset:4096\n"
            "ds_read_b128 %7, %11 offset:4096\n s_waitcnt lgkmcnt(0)"
            : "=v"(a0), "=v"(a1), "=v"(a2), "=v"(a3), "=v"(a4), "=v"(a5), "=v"(a6), "=v"(a7)
            : "v"(base[0]), "v"(base[1]), "v"(base[2]), "v"(base[3]));
        sum += a0[0] + a3[1] + a7[3];
    }
    if (sum == 0x12345u) out[0] = sum;
}

static constexpr int kLdsIters = 4000;

// L2 -> LDS rate: what the GEMMs' operand pipeline can draw at best.  Every wave copies 1 KB pieces (16 bytes per
// lane, the LDS-writing buffer load of the GEMMs) from a region small enough to stay in the L2 of every XCD (2 MiB)
// into its workgroup's LDS, 8 loads in flight per wave, three workgroups of 4 waves per compute unit.
static constexpr int kFillIters = 2048;  // rounds of 8 loads per wave
__global__ __launch_bounds__(256) void l2_to_lds_kernel(const uint8_t* __restrict__ src, uint32_t region_bytes, int iters) {
    __shared__ __attribute__((aligned(16))) uint8_t lds[32768];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const uint64_t a = (uint64_t)(uintptr_t)src;
    typedef int int4s __attribute__((ext_vector_type(4)));
    int4s rsrc;
    rsrc[0] = __builtin_amdgcn_readfirstlane((int)(uint32_t)a);
    rsrc[1] = __builtin_amdgcn_readfirstlane((int)(uint32_t)((a >> 32) & 0xFFFFu));
    rsrc[2] = __builtin_amdgcn_readfirstlane((int)region_bytes);
    rsrc[3] = 0x00020000;
    const uint32_t lds_wave = (uint32_t)(uintptr_t)lds + wv * 8192;
    uint32_t off = ((blockIdx.x * 4 + wv) * 8192u) % region_bytes;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t m0 = __builtin_amdgcn_readfirstlane(lds_wave + j * 1024);
            const int voff = (int)((off + j * 1024u) % region_bytes) + lane * 16;
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds" ::"s"(m0), "v"(voff), "s"(rsrc) : "memory");
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        off = (off + 8192u * 4u * 97u) % region_bytes;  // another piece of the region every round
    }
    __syncthreads();
    if (lds[threadIdx.x] == 0xA5 && src[0] == 0x5A) ((volatile uint8_t*)lds)[0] = 1;
}

// kind                           work of the one kernel launch
//  0  int8 MFMA only             512 workgroups x 4 waves x kMfmaIters x 4 MFMAs x 65536 operations
//  1  fp16 MFMA only             ... x 32768 operations
//  2  vector ALU only            512 x 4 waves x kMfmaIters x 32 instructions (as many cycles as the MFMAs of kind 0)
//  3  int8 MFMA and vector ALU work in ONE wave, interleaved (1 MFMA, 8 ALU instructions, ...): the work of 0 plus 2
//  4  int8 MFMA waves and vector ALU waves side by side on every SIMD: the work of 0 plus 2
//  5  read-only stream over buf (buf_bytes, at least 1 GiB to defeat the last-level cache): buf_bytes read
//  6  LDS reads: 1024 workgroups x 4 waves x kLdsIters x 8 KB
//  7  L2 -> LDS: 768 workgroups x 4 waves x kFillIters x 8 KB copied from the first 2 MiB of buf into LDS
//  8  as 3 with 4 instead of 8 vector ALU instructions behind every MFMA: the work of 0 plus half the work of 2
// Returns elapsed milliseconds (best of five) in *ms_host.
int prof_microbench(int kind, void* buf, size_t buf_bytes, double* ms_host, hipStream_t st) {
    if (!ms_host || kind < 0 || kind > 8) return MQ_ERR_BAD_ARG;
    if (kind == 7 && buf_bytes < (2u << 20)) return MQ_ERR_BAD_ARG;
    if (!buf || buf_bytes < 4096 || (uintptr_t)buf % 16) return MQ_ERR_BAD_ARG;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return MQ_ERR_HIP;
    double best = 1e30;
    int rc = MQ_OK;
    for (int rep = 0; rep < 6 && rc == MQ_OK; ++rep) {
        const int it = rep == 0 ? 16 : kMfmaIters;  // (the first run warms up: code fetch, clocks)
        (void)hipEventRecord(a, st);
        switch (kind) {
            case 0: hipLaunchKernelGGL((mfma_valu_kernel<true, 1, 0>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            case 1: hipLaunchKernelGGL((mfma_valu_kernel<false, 1, 0>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            case 2: hipLaunchKernelGGL((mfma_valu_kernel<true, 0, 2>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            case 3: hipLaunchKernelGGL((mfma_valu_kernel<true, 3, 0>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            case 4: hipLaunchKernelGGL((mfma_valu_kernel<true, 1, 2>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            case 5:
                hipLaunchKernelGGL(read_stream_kernel, dim3(4096), dim3(256), 0, st, (const uint4v*)buf + 256,
                                   (buf_bytes - 4096) / 16, (uint32_t*)buf);
                break;
            case 6:
                hipLaunchKernelGGL(lds_read_kernel, dim3(1024), dim3(256), 0, st, rep == 0 ? 16 : kLdsIters, (uint32_t*)buf);
                break;
            case 8: hipLaunchKernelGGL((mfma_valu_kernel<true, 3, 0, 4>), dim3(kGrid), dim3(512), 0, st, it, (int*)buf); break;
            default:
                hipLaunchKernelGGL(l2_to_lds_kernel, dim3(768), dim3(256), 0, st, (const uint8_t*)buf, 2u << 20,
                                   rep == 0 ? 16 : kFillIters);
        }
        if (hipGetLastError() != hipSuccess) rc = MQ_ERR_HIP;
        (void)hipEventRecord(b, st);
        float ms = 0;
        if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) rc = MQ_ERR_HIP;
        if (rep > 0 && ms < best) best = ms;
    }
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (rc != MQ_OK) {
        set_hip_error((int)hipGetLastError());
        return rc;
    }
    *ms_host = best;
    return MQ_OK;
}

}  // namespace mq
