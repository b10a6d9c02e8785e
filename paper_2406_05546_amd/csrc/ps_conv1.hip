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
    // first maximum in scan order; the winner is kept as its offset in a 30-wide padded input image
    float best = v[0];
    int off = 0;
    if (v[1] > best) { best = v[1]; off = 1; }
    if (v[2] > best) { best = v[2]; off = 30; }
    if (v[3] > best) { best = v[3]; off = 31; }
    const size_t out = g * P1_SIZE + o * P1_POS + pos;
    wb.p1[out] = fmaxf(best, 0.f);
    wb.am1[out] = (uint8_t)(off | (best > 0.f ? AM1_GATE : 0));
}

// conv1 (1 -> 16, 3x3, pad 1) + ReLU + 2x2 max pool.  The kernel is bound by vector-ALU issue, and 196
// pooled positions are three wavefronts plus four lanes: so wavefronts 0-2 own positions 0..191, a lane
// walking the 16 output channels with its 4x4 input patch in registers, and wavefront 3 only does the
// 64 (position, channel) pairs of positions 192..195, one per lane: 49 wavefront passes per image, the
// minimum.  A block walks up to CONV1_IPB images of one worker; the next image's pixels are fetched
// into registers while this one is computed and go into the other of two padded LDS images.
constexpr int CONV1_IPB = 4;

__global__ __launch_bounds__(256) void conv1_fwd_kernel(WorkerBuffers wb, int blocks_per_worker)
{
    __shared__ float xs[2][30 * 30];
    __shared__ float ws[OFF_W2];  // conv1.W (144) + conv1.b (16)
    const int t = threadIdx.x, w = blockIdx.x / blocks_per_worker, chunk = blockIdx.x % blocks_per_worker;
    const int s_begin = chunk * CONV1_IPB, s_end = min(wb.B, s_begin + CONV1_IPB);
    const float* theta = worker_theta(wb, w);
    for (int i = t; i < 2 * 900; i += 256) (&xs[0][0])[i] = 0.f;  // the borders stay zero
    if (t < OFF_W2) ws[t] = theta[OFF_W1 + t];
    // pixels t, t + 256, t + 512 and (for t < 16) t + 768 of an image, and where they go in a padded image
    float xv[4];
    int at[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int i = min(t + 256 * k, IMG_PIX - 1);
        at[k] = (i / IMG_W + 1) * 30 + i % IMG_W + 1;
    }
    auto prefetch = [&](size_t g) {
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (t + 256 * k < IMG_PIX) xv[k] = wb.x[g * IMG_PIX + t + 256 * k];
    };
    const int pos = t < 192 ? t : 192 + ((t - 192) >> 4);
    const int py = pos / P1_W, px = pos % P1_W;
    prefetch((size_t)w * wb.B + s_begin);
    __syncthreads();
    for (int s = s_begin; s < s_end; ++s) {
        const size_t g = (size_t)w * wb.B + s;
        float* xcur = xs[(s - s_begin) & 1];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (t + 256 * k < IMG_PIX) xcur[at[k]] = xv[k];
        __syncthreads();  // also: everybody is done with the image before last, whose buffer comes next
        if (s + 1 < s_end) prefetch(g + 1);
        float patch[4][4];
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) patch[a][b] = xcur[(2 * py + a) * 30 + 2 * px + b];
        if (t < 192) {
#pragma unroll
            for (int o = 0; o < C1; ++o) conv1_pair(wb, ws, patch, g, pos, o);
        } else {
            conv1_pair(wb, ws, patch, g, pos, t & 15);
        }
    }
}

}  // namespace

void launch_conv1_fwd(const WorkerBuffers& wb, hipStream_t s)
{
    const int bpw = (wb.B + CONV1_IPB - 1) / CONV1_IPB;
    hipLaunchKernelGGL(conv1_fwd_kernel, dim3(wb.n * bpw), dim3(256), 0, s, wb, bpw);
}

}  // namespace ps
