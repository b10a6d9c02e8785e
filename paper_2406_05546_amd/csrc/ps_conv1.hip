// conv1 (1 -> 16 channels, 3x3, pad 1, on the 28x28 input) forward with fused ReLU + 2x2 max pool.
// K = 9 is too short for the matrix cores; it runs on the vector ALU with the zero-padded image in
// LDS.  (Its weight gradient is fused into conv2's input-gradient kernel.)
#include "ps_common.h"

namespace ps {

namespace {

// One (pooled position, output channel) pair: four 3x3 sums over the 4x4 input patch, pool, store.
__device__ __forceinline__ void conv1_pair(const WorkerBuffers& wb, const float* __restrict__ ws, const float (&patch)[4][4],
                                           size_t g, int pos, int o)
{
    float k[9];
#pragma unroll
    for (int i = 0; i < 9; ++i) k[i] = ws[o * 9 + i];
    const float bias = ws[OFF_B1 + o];
    float v[4];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            float acc = bias;
#pragma unroll
            for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                for (int dx = 0; dx < 3; ++dx) acc = fmaf(k[dy * 3 + dx], patch[a + dy][b + dx], acc);
            v[a * 2 + b] = acc;
        }
    int code;
    const float best = pool_first_max(v[0], v[1], v[2], v[3], code);
    const size_t out = g * P1_SIZE + o * P1_POS + pos;
    wb.p1[out] = fmaxf(best, 0.f);
    wb.am1[out] = (uint8_t)(code | (best > 0.f ? 4 : 0));
}

// conv1 (1 -> 16, 3x3, pad 1) + ReLU + 2x2 max pool.  One block per image.  The kernel is bound by
// vector-ALU issue, and 196 pooled positions are three wavefronts plus four lanes: so wavefronts 0-2
// own positions 0..191, a lane walking the 16 output channels with its 4x4 input patch in registers,
// and wavefront 3 only does the 64 (position, channel) pairs of positions 192..195, one per lane.
__global__ __launch_bounds__(256) void conv1_fwd_kernel(WorkerBuffers wb)
{
    __shared__ float xs[30 * 30];
    __shared__ float ws[OFF_W2];  // conv1.W (144) + conv1.b (16)
    const int g = blockIdx.x, w = g / wb.B, t = threadIdx.x;
    const float* theta = worker_theta(wb, w);
    for (int i = t; i < 900; i += 256) {
        const int yy = i / 30 - 1, xx = i % 30 - 1;
        xs[i] = (yy >= 0 && yy < 28 && xx >= 0 && xx < 28) ? wb.x[(size_t)g * IMG_PIX + yy * 28 + xx] : 0.f;
    }
    if (t < OFF_W2) ws[t] = theta[OFF_W1 + t];
    __syncthreads();
    const int pos = t < 192 ? t : 192 + ((t - 192) >> 4);
    const int py = pos / P1_W, px = pos % P1_W;
    float patch[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) patch[a][b] = xs[(2 * py + a) * 30 + 2 * px + b];
    if (t < 192) {
#pragma unroll
        for (int o = 0; o < C1; ++o) conv1_pair(wb, ws, patch, g, pos, o);
    } else {
        conv1_pair(wb, ws, patch, g, pos, t & 15);
    }
}

}  // namespace

void launch_conv1_fwd(const WorkerBuffers& wb, hipStream_t s)
{
    hipLaunchKernelGGL(conv1_fwd_kernel, dim3(wb.n * wb.B), dim3(256), 0, s, wb);
}

}  // namespace ps
