// Offline preparation kernels: per-output-channel min-max weight quantiser (paper Sec. 4.1
// "Quantization Scheme"), bit packers for 2/3/4/8-bit codes in the canonical and the kernel layout,
// the matching unpackers and the per-channel code sums the integer GEMM epilogue needs.
//
// Every floating-point operation that decides an integer code is one IEEE fp32 operation
// (this file is compiled with -ffp-contract=off): subtract, divide, reciprocal, multiply, round-to-nearest-even.
#include "mq_common.h"

namespace mq {

__device__ inline float load16(const uint16_t* p, int dtype) {
    uint16_t b = *p;
    if (dtype == MQ_BF16) return __uint_as_float(((uint32_t)b) << 16);
    return (float)__builtin_bit_cast(_Float16, b);
}

template <typename T, typename Op>
__device__ inline T wave_reduce(T v, Op op) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = op(v, __shfl_xor(v, off, 64));
    return v;
}

// One workgroup per output channel.
__global__ __launch_bounds__(256) void quantize_weights_kernel(const uint16_t* __restrict__ w, int N, int K, int bits,
                                                               int symmetric, int dtype, uint8_t* __restrict__ codes,
                                                               float* __restrict__ scale, int32_t* __restrict__ zp) {
    const int n = blockIdx.x;
    const uint16_t* row = w + (size_t)n * K;
    float mn = INFINITY, mx = -INFINITY;
    for (int k = threadIdx.x; k < K; k += blockDim.x) {
        float v = load16(row + k, dtype);
        mn = fminf(mn, v);
        mx = fmaxf(mx, v);
    }
    mn = wave_reduce(mn, [](float a, float b) { return fminf(a, b); });
    mx = wave_reduce(mx, [](float a, float b) { return fmaxf(a, b); });
    __shared__ float smn[4], smx[4];
    const int wv = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        smn[wv] = mn;
        smx[wv] = mx;
    }
    __syncthreads();
    mn = fminf(fminf(smn[0], smn[1]), fminf(smn[2], smn[3]));
    mx = fmaxf(fmaxf(smx[0], smx[1]), fmaxf(smx[2], smx[3]));

    if (symmetric) {
        const int Q = (1 << (bits - 1)) - 1;
        const float amax = fmaxf(fabsf(mn), fabsf(mx));
        const float s = (amax == 0.0f) ? 1.0f : amax / (float)Q;
        const float inv = 1.0f / s;
        if (threadIdx.x == 0) {
            scale[n] = s;
            zp[n] = 0;
        }
        for (int k = threadIdx.x; k < K; k += blockDim.x) {
            float r = rintf(load16(row + k, dtype) * inv);
            r = fminf(fmaxf(r, (float)-Q), (float)Q);
            codes[(size_t)n * K + k] = (uint8_t)(int8_t)(int)r;
        }
    } else {
        const int qmax = (1 << bits) - 1;
        const float lo = fminf(mn, 0.0f), hi = fmaxf(mx, 0.0f);
        float s = 1.0f;
        if (hi != lo) {
            const float range = hi - lo;
            s = range / (float)qmax;
        }
        const float inv = 1.0f / s;
        float zf = rintf((-lo) * inv);
        zf = fminf(fmaxf(zf, 0.0f), (float)qmax);
        if (threadIdx.x == 0) {
            scale[n] = s;
            zp[n] = (int)zf;
        }
        for (int k = threadIdx.x; k < K; k += blockDim.x) {
            // rne(x*inv) is integer valued; adding the zero point and clamping in float equals the integer
            // formula wherever that one is defined and saturates cleanly elsewhere.
            float r = rintf(load16(row + k, dtype) * inv) + zf;
            r = fminf(fmaxf(r, 0.0f), (float)qmax);
            codes[(size_t)n * K + k] = (uint8_t)(int)r;
        }
    }
}

// ------------------------------------------------------------------------------------------ canonical layout
// One thread per output byte: byte B of a row covers bits [8B, 8B+8) of the row's little-endian bit stream.
__global__ void pack_canonical_kernel(const uint8_t* __restrict__ codes, int N, int K, int bits,
                                      uint8_t* __restrict__ packed) {
    const long rb = (long)K * bits / 8;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= rb * N) return;
    const long n = idx / rb, B = idx % rb;
    const uint8_t* row = codes + n * K;
    const unsigned mask = (1u << bits) - 1u;
    const long bit0 = B * 8;
    const long k0 = bit0 / bits, k1 = (bit0 + 7) / bits;
    unsigned out = 0;
    for (long k = k0; k <= k1 && k < K; ++k) {
        const long pos = k * bits - bit0;  // may be negative: the code started in the previous byte
        const unsigned c = row[k] & mask;
        out |= pos >= 0 ? (c << pos) : (c >> (-pos));
    }
    packed[idx] = (uint8_t)out;
}

__global__ void unpack_canonical_kernel(const uint8_t* __restrict__ packed, int N, int K, int bits,
                                        uint8_t* __restrict__ codes) {
    const long rb = (long)K * bits / 8;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)N * K) return;
    const long n = idx / K, k = idx % K;
    const long bit0 = k * bits;
    const long B = bit0 / 8;
    unsigned v = packed[n * rb + B];
    if (B + 1 < rb) v |= ((unsigned)packed[n * rb + B + 1]) << 8;
    codes[idx] = (uint8_t)((v >> (bit0 % 8)) & ((1u << bits) - 1u));
}

// ------------------------------------------------------------------------------------------ kernel layout
// One thread per lane chunk (32 codes of one channel).  Rows n >= N are padding and hold code 0.
__device__ inline size_t kl_chunk_offset(int g, int c, int KC, int bits, int L) {
    return ((size_t)g * KC + c) * kl_tile_bytes(bits) + (size_t)L * (bits == 8 ? 16 : 4 * bits);
}

__global__ void pack_kernel_layout_kernel(const uint8_t* __restrict__ codes, int N, int K, int bits,
                                          uint8_t* __restrict__ packed) {
    const int KC = K / 64;
    const int Np = (N + 31) / 32 * 32;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)Np * KC * 2) return;
    const int j = idx % 32;
    const int kb = (idx / 32) % 2;
    const int c = (idx / 64) % KC;
    const int g = idx / (64L * KC);
    const int n = g * 32 + j;
    const int L = kb * 32 + j;
    const unsigned mask = (1u << bits) - 1u;
    unsigned cd[32];
#pragma unroll
    for (int e = 0; e < 32; ++e) cd[e] = n < N ? (codes[(size_t)n * K + c * 64 + kb * 32 + e] & mask) : 0u;
    uint32_t* out = (uint32_t*)(packed + kl_chunk_offset(g, c, KC, bits, L));
    if (bits == 4) {
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
            uint32_t w = 0;
#pragma unroll
            for (int p = 0; p < 4; ++p) w |= (cd[8 * wd + 2 * p] << (4 * p)) | (cd[8 * wd + 2 * p + 1] << (16 + 4 * p));
            out[wd] = w;
        }
    } else if (bits == 2) {
#pragma unroll
        for (int wd = 0; wd < 2; ++wd) {
            uint32_t w = 0;
#pragma unroll
            for (int p = 0; p < 8; ++p)
                w |= (cd[16 * wd + 2 * p] << (2 * p)) | (cd[16 * wd + 2 * p + 1] << (16 + 2 * p));
            out[wd] = w;
        }
    } else if (bits == 3) {
        uint32_t W[3] = {0, 0, 0};
#pragma unroll
        for (int p = 0; p < 15; ++p) {
            const int t = p / 5, f = p % 5;
            W[t] |= (cd[2 * p] << (3 * f)) | (cd[2 * p + 1] << (16 + 3 * f));
        }
#pragma unroll
        for (int i = 0; i < 3; ++i) W[i] |= (((cd[30] >> i) & 1u) << 15) | (((cd[31] >> i) & 1u) << 31);
        out[0] = W[0];
        out[1] = W[1];
        out[2] = W[2];
    } else {  // 8 bit: two pieces, groups of 8 in the order c0,c4,c1,c5,c2,c6,c3,c7
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            uint32_t* o = (uint32_t*)((uint8_t*)out + h * 1024);
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                uint32_t w = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b) w |= cd[16 * h + 8 * (wd / 2) + k8_perm(4 * (wd % 2) + b)] << (8 * b);
                o[wd] = w;
            }
        }
    }
}

__global__ void unpack_kernel_layout_kernel(const uint8_t* __restrict__ packed, int N, int K, int bits,
                                            uint8_t* __restrict__ codes) {
    const int KC = K / 64;
    const int Np = (N + 31) / 32 * 32;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)Np * KC * 2) return;
    const int j = idx % 32;
    const int kb = (idx / 32) % 2;
    const int c = (idx / 64) % KC;
    const int g = idx / (64L * KC);
    const int n = g * 32 + j;
    if (n >= N) return;
    const int L = kb * 32 + j;
    const uint32_t* in = (const uint32_t*)(packed + kl_chunk_offset(g, c, KC, bits, L));
    unsigned cd[32];
    if (bits == 4) {
#pragma unroll
        for (int wd = 0; wd < 4; ++wd) {
            const uint32_t w = in[wd];
#pragma unroll
            for (int p = 0; p < 4; ++p) {
                cd[8 * wd + 2 * p] = (w >> (4 * p)) & 15u;
                cd[8 * wd + 2 * p + 1] = (w >> (16 + 4 * p)) & 15u;
            }
        }
    } else if (bits == 2) {
#pragma unroll
        for (int wd = 0; wd < 2; ++wd) {
            const uint32_t w = in[wd];
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                cd[16 * wd + 2 * p] = (w >> (2 * p)) & 3u;
                cd[16 * wd + 2 * p + 1] = (w >> (16 + 2 * p)) & 3u;
            }
        }
    } else if (bits == 3) {
        const uint32_t W[3] = {in[0], in[1], in[2]};
#pragma unroll
        for (int p = 0; p < 15; ++p) {
            const int t = p / 5, f = p % 5;
            cd[2 * p] = (W[t] >> (3 * f)) & 7u;
            cd[2 * p + 1] = (W[t] >> (16 + 3 * f)) & 7u;
        }
        cd[30] = ((W[0] >> 15) & 1u) | (((W[1] >> 15) & 1u) << 1) | (((W[2] >> 15) & 1u) << 2);
        cd[31] = ((W[0] >> 31) & 1u) | (((W[1] >> 31) & 1u) << 1) | (((W[2] >> 31) & 1u) << 2);
    } else {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const uint32_t* i8 = (const uint32_t*)((const uint8_t*)in + h * 1024);
#pragma unroll
            for (int wd = 0; wd < 4; ++wd) {
                const uint32_t w = i8[wd];
#pragma unroll
                for (int b = 0; b < 4; ++b) cd[16 * h + 8 * (wd / 2) + k8_perm(4 * (wd % 2) + b)] = (w >> (8 * b)) & 255u;
            }
        }
    }
#pragma unroll
    for (int e = 0; e < 32; ++e) codes[(size_t)n * K + c * 64 + kb * 32 + e] = (uint8_t)cd[e];
}

// 16-bit weights (the layers a bit-width configuration leaves unquantised): the same 32-channel x 64-k tiles, 4 KB each.
// Lane L = kb * 32 + j owns the 32 values k' = 0..31 of channel j in k-half kb; they are stored as four 16-byte pieces,
// piece s (values 8s .. 8s+7: the lane's MFMA operand of step s) at s * 1024 + L * 16.  One thread per piece.
__global__ void pack16_kernel_layout_kernel(const uint16_t* __restrict__ w, int N, int K, int to_kernel,
                                            uint16_t* __restrict__ out) {
    const int KC = K / 64;
    const int Np = (N + 31) / 32 * 32;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)Np * KC * 8) return;
    const int L = idx % 64;
    const int s = (idx / 64) % 4;
    const int c = (idx / 256) % KC;
    const int g = idx / (256L * KC);
    const int j = L % 32, kb = L / 32;
    const int n = g * 32 + j;
    const size_t tile = ((size_t)g * KC + c) * 2048 + (size_t)s * 512 + (size_t)L * 8;  // in 16-bit units
    const size_t src = (size_t)n * K + c * 64 + kb * 32 + s * 8;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (to_kernel)
            out[tile + e] = n < N ? w[src + e] : (uint16_t)0;
        else if (n < N)
            out[src + e] = w[tile + e];
    }
}

// One wave per channel.
__global__ __launch_bounds__(256) void code_colsum_kernel(const uint8_t* __restrict__ codes, int N, int K, int bits,
                                                          int codes_signed, int32_t* __restrict__ colsum) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;
    const unsigned mask = (1u << bits) - 1u;
    int s = 0;
    for (int k = threadIdx.x & 63; k < K; k += 64) {
        const uint8_t c = codes[(size_t)n * K + k];
        s += codes_signed ? (int)(int8_t)c : (int)(c & mask);
    }
    s = wave_reduce(s, [](int a, int b) { return a + b; });
    if ((threadIdx.x & 63) == 0) colsum[n] = s;
}

// Sums of the weight codes per filter tap of a 3x3 convolution (codes [N, 9 * Cin], k = tap * Cin + c): one wave per
// (channel, tap).  The int8 convolution needs them for output pixels whose filter reaches outside the image.
__global__ __launch_bounds__(256) void tap_sums_kernel(const uint8_t* __restrict__ codes, int N, int Cin, int bits,
                                                       int codes_signed, int32_t* __restrict__ tapsum) {
    const int idx = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (idx >= N * 9) return;
    const int n = idx / 9, t = idx % 9;
    const unsigned mask = (1u << bits) - 1u;
    int s = 0;
    for (int c = threadIdx.x & 63; c < Cin; c += 64) {
        const uint8_t q = codes[(size_t)n * 9 * Cin + (size_t)t * Cin + c];
        s += codes_signed ? (int)(int8_t)q : (int)(q & mask);
    }
    s = wave_reduce(s, [](int a, int b) { return a + b; });
    if ((threadIdx.x & 63) == 0) tapsum[(size_t)t * N + n] = s;
}

int launch_tap_sums(const uint8_t* codes, int N, int Cin, int bits, int codes_signed, int32_t* tapsum, hipStream_t st) {
    hipLaunchKernelGGL(tap_sums_kernel, dim3((N * 9 + 3) / 4), dim3(256), 0, st, codes, N, Cin, bits, codes_signed,
                       tapsum);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

int launch_quantize_weights(const void* w, int N, int K, int bits, int symmetric, int dtype, uint8_t* codes,
                            float* scale, int32_t* zp, hipStream_t st) {
    hipLaunchKernelGGL(quantize_weights_kernel, dim3(N), dim3(256), 0, st, (const uint16_t*)w, N, K, bits, symmetric,
                       dtype, codes, scale, zp);
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

int launch_pack(const uint8_t* codes, int N, int K, int bits, int layout, int codes_signed, void* packed,
                int32_t* colsum, hipStream_t st) {
    if (bits == 16) {  // 16-bit values, not codes: canonical is the matrix itself
        if (layout == MQ_LAYOUT_CANONICAL) {
            if (hipMemcpyAsync(packed, codes, (size_t)N * K * 2, hipMemcpyDeviceToDevice, st) != hipSuccess) {
                set_hip_error((int)hipGetLastError());
                return MQ_ERR_HIP;
            }
            return MQ_OK;
        }
        const long total = (long)((N + 31) / 32 * 32) * (K / 64) * 8;
        hipLaunchKernelGGL(pack16_kernel_layout_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const uint16_t*)codes, N, K, 1, (uint16_t*)packed);
        MQ_HIP_CHECK_LAUNCH();
        return MQ_OK;
    }
    if (layout == MQ_LAYOUT_CANONICAL) {
        const long total = (long)N * ((long)K * bits / 8);
        hipLaunchKernelGGL(pack_canonical_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, codes, N, K,
                           bits, (uint8_t*)packed);
    } else {
        const long total = (long)((N + 31) / 32 * 32) * (K / 64) * 2;
        hipLaunchKernelGGL(pack_kernel_layout_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, codes, N,
                           K, bits, (uint8_t*)packed);
    }
    MQ_HIP_CHECK_LAUNCH();
    if (colsum) {
        hipLaunchKernelGGL(code_colsum_kernel, dim3((N + 3) / 4), dim3(256), 0, st, codes, N, K, bits, codes_signed,
                           colsum);
        MQ_HIP_CHECK_LAUNCH();
    }
    return MQ_OK;
}

int launch_unpack(const void* packed, int N, int K, int bits, int layout, uint8_t* codes, hipStream_t st) {
    if (bits == 16) {
        if (layout == MQ_LAYOUT_CANONICAL) {
            if (hipMemcpyAsync(codes, packed, (size_t)N * K * 2, hipMemcpyDeviceToDevice, st) != hipSuccess) {
                set_hip_error((int)hipGetLastError());
                return MQ_ERR_HIP;
            }
            return MQ_OK;
        }
        const long total = (long)((N + 31) / 32 * 32) * (K / 64) * 8;
        hipLaunchKernelGGL(pack16_kernel_layout_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const uint16_t*)packed, N, K, 0, (uint16_t*)codes);
        MQ_HIP_CHECK_LAUNCH();
        return MQ_OK;
    }
    if (layout == MQ_LAYOUT_CANONICAL) {
        const long total = (long)N * K;
        hipLaunchKernelGGL(unpack_canonical_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const uint8_t*)packed, N, K, bits, codes);
    } else {
        const long total = (long)((N + 31) / 32 * 32) * (K / 64) * 2;
        hipLaunchKernelGGL(unpack_kernel_layout_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st,
                           (const uint8_t*)packed, N, K, bits, codes);
    }
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

}  // namespace mq
