// Worker step on the GPU: forward and backward pass of the paper's CNN (model endnote) for n
// workers x B images in one batch of launches.  Worker w reads the weights of ring slot
// meta[w].slot in place (a stale snapshot costs no copy) and its gradient is written straight into
// queue entry meta[w].q (Section 3.3 worker step: read weights, compute gradient, append).
// This file holds the launch order, the final fixed-order reduction of partial sums, and the debug
// mask kernel; the layers live in ps_conv1.hip, ps_conv2.hip, ps_fc1.hip and ps_fc2.hip.
#include "ps_common.h"
#include "ps_philox.h"

namespace ps {

namespace {

// Sums the partial slots in fixed order into the worker's queue entry: conv1 tensors have one partial
// per (8 images, wavefront) of conv2's input-gradient kernel, conv2 tensors one per (chunk, wavefront) of its
// weight-gradient kernel, fc2 tensors, fc1 bias and the loss one per block of the fc2 kernel.
// Grid (workers, REDUCE_Y) x 256 threads.  The 160 conv1 values have many slots each (128 at 256 images), so
// a block takes 20 of them with 12 threads per value (thread j adds slots j, j + 12, ... in order, thread 0
// then adds the 12 sums in order); everything else is one thread per value over the few slots it has.
constexpr int REDUCE_Y = 8, C1_PER_BLOCK = OFF_W2 / REDUCE_Y, C1_LANES = 12;
static_assert(C1_PER_BLOCK * REDUCE_Y == OFF_W2 && C1_PER_BLOCK * C1_LANES <= 256, "conv1 values over the blocks");

__global__ __launch_bounds__(256) void grad_reduce_kernel(WorkerBuffers wb, int fc2_slots, int c1_slots)
{
    __shared__ float c1_sum[C1_PER_BLOCK][C1_LANES + 1];
    const int w = blockIdx.x;
    float* grad = worker_grad(wb, w);
    {
        const int e = threadIdx.x / C1_LANES, j = threadIdx.x % C1_LANES;
        if (e < C1_PER_BLOCK) {
            const float* p1 = wb.part1 + (size_t)w * c1_slots * OFF_W2 + blockIdx.y * C1_PER_BLOCK + e;
            float sum = 0.f;
            for (int c = j; c < c1_slots; c += C1_LANES) sum += p1[(size_t)c * OFF_W2];
            c1_sum[e][j] = sum;
        }
        __syncthreads();
        if (threadIdx.x < C1_PER_BLOCK) {
            float sum = 0.f;
#pragma unroll
            for (int j2 = 0; j2 < C1_LANES; ++j2) sum += c1_sum[threadIdx.x][j2];
            grad[blockIdx.y * C1_PER_BLOCK + threadIdx.x] = sum;
        }
    }
    const float* part = wb.part + (size_t)w * N_PART * CONV_PART;
    const int tid = blockIdx.y * 256 + threadIdx.x, stride = REDUCE_Y * 256;
    for (int i = OFF_W2 + tid; i < CONV_PART; i += stride) {
        float sum = 0.f;
#pragma unroll
        for (int c = 0; c < N_PART; ++c) sum += part[(size_t)c * CONV_PART + i];
        grad[i] = sum;
    }
    const float* fpart = wb.fpart + (size_t)w * fc2_slots * FC2_PART;
    for (int i = tid; i <= FC2_PART_LOSS; i += stride) {
        float sum = 0.f;
        for (int c = 0; c < fc2_slots; ++c) sum += fpart[(size_t)c * FC2_PART + i];
        if (i < FC2_PART_B4)
            grad[OFF_W4 + i] = sum;
        else if (i < FC2_PART_B3)
            grad[OFF_B4 + i - FC2_PART_B4] = sum;
        else if (i < FC2_PART_LOSS)
            grad[OFF_B3 + i - FC2_PART_B3] = sum;
        else if (wb.loss)
            wb.loss[w] = sum / (float)wb.B;
    }
}

__global__ __launch_bounds__(256) void keep_mask_kernel(uint8_t* keep, int B, uint32_t mb_lo, uint32_t mb_hi,
                                                        uint32_t seed_lo, uint32_t seed_hi, uint32_t threshold)
{
    const int i = blockIdx.x * 256 + threadIdx.x;  // one Philox call = 4 units
    if (i >= B * (FC1 / 4)) return;
    const int s = i / (FC1 / 4), u4 = i % (FC1 / 4);
    const uint4 r = philox4x32_10(make_uint4(mb_lo, mb_hi, (uint32_t)s, (uint32_t)u4), make_uint2(seed_lo, seed_hi));
    uint8_t* k = keep + (size_t)s * FC1 + u4 * 4;
    k[0] = r.x >= threshold;
    k[1] = r.y >= threshold;
    k[2] = r.z >= threshold;
    k[3] = r.w >= threshold;
}

}  // namespace

#define PS_TIMED(id, ...)      \
    do {                       \
        prof.begin(id, s);     \
        __VA_ARGS__;           \
        prof.end(s);           \
    } while (0)

hipError_t launch_worker_forward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof)
{
    if (wb.n * wb.B <= 0) return hipSuccess;
    PS_TIMED(K_CONV1_FWD, launch_conv1_fwd(wb, s));
    PS_TIMED(K_CONV2_FWD, launch_conv2_fwd(wb, s));
    PS_TIMED(K_FC1_FWD, launch_fc1_fwd(wb, s));
    return hipGetLastError();
}

hipError_t launch_worker_backward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof)
{
    if (wb.n * wb.B <= 0) return hipSuccess;
    PS_TIMED(K_FC2, launch_fc2(wb, s));
    PS_TIMED(K_FC1_DW, launch_fc1_dw(wb, s));
    PS_TIMED(K_FC1_DX, launch_fc1_dx(wb, s));
    PS_TIMED(K_CONV2_DW, launch_conv2_dw(wb, s));
    PS_TIMED(K_CONV2_DX, launch_conv2_dx(wb, s));
    PS_TIMED(K_GRAD_REDUCE, hipLaunchKernelGGL(grad_reduce_kernel, dim3(wb.n, REDUCE_Y), dim3(256), 0, s, wb, fc2_split(wb.n),
                                                conv1_part_slots(wb.B)));
    return hipGetLastError();
}

const char* kernel_name(int id)
{
    static const char* const names[K_COUNT] = {
        "conv1_fwd_kernel", "conv2_fwd_kernel", "gemm_f32_mfma<Fc1FwdEpi>", "fc2_kernel",
        "gemm_f32_mfma<Fc1DwEpi>", "gemm_f32_mfma<Fc1DxEpi>", "conv2_dw_kernel",
        "conv2_dx_kernel", "grad_reduce_kernel", "apply_kernel<0>", "apply_kernel<1>", "grad_sqnorm_kernel",
        "apply_kernel<0, clip>", "apply_kernel<1, clip>", "apply_adadelta_kernel", "local_step_kernel",
        "elastic_average_kernel"};
    return id >= 0 && id < K_COUNT ? names[id] : "";
}

hipError_t launch_keep_mask(uint8_t* keep_dev, int B, uint32_t mb_lo, uint32_t mb_hi, uint32_t seed_lo,
                            uint32_t seed_hi, uint32_t threshold, hipStream_t s)
{
    hipLaunchKernelGGL(keep_mask_kernel, dim3((B * (FC1 / 4) + 255) / 256), dim3(256), 0, s, keep_dev, B, mb_lo, mb_hi,
                       seed_lo, seed_hi, threshold);
    return hipGetLastError();
}

}  // namespace ps
