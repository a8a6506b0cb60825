// BOS rows of the BOS-aware K/V projection (paper Sec. 3.1): token 0 of every prompt is kept out of
// activation quantisation; its to_k/to_v output is the fp16 linear with the unquantised weights (fp32
// accumulation), or a copy of the vector that was pre-computed offline.
#include "bos_rows.h"

namespace mq {

template <int BCHUNK>
__global__ __launch_bounds__(256) void bos_rows_kernel(BosWork bw) {
    bos_rows_block<BCHUNK>((int)blockIdx.x, (int)threadIdx.x, bw);
}

__global__ __launch_bounds__(256) void bos_copy_kernel(BosWork bw) {
    bos_copy_block((int)blockIdx.x, (int)threadIdx.x, bw);
}

int launch_bos_rows(const BosWork& bw, hipStream_t st) {
    if (bw.bos_out) {
        hipLaunchKernelGGL(bos_copy_kernel, dim3(bos_blocks(bw)), dim3(256), 0, st, bw);
    } else {
        ProfScope prof(st, PROF_BOS_ROWS, 2.0 * bw.B * bw.N * bw.K, 2.0 * bw.N * bw.K + 2.0 * bw.B * bw.K + 2.0 * bw.B * bw.N);
        hipLaunchKernelGGL(bos_rows_kernel<8>, dim3(bos_blocks(bw)), dim3(256), 0, st, bw);
    }
    MQ_HIP_CHECK_LAUNCH();
    return MQ_OK;
}

}  // namespace mq
