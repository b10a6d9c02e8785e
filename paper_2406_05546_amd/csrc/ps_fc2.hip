// fc2 (512 -> 10), softmax cross-entropy and everything of their backward pass that does not need
// the matrix cores, in one kernel:
//   z = W4 . h + b4;  loss_i = logsumexp(z) - z[y];  d4 = (softmax(z) - onehot(y)) / B;
//   d3 = (W4^T d4) / (1-p) where the dropped-and-rectified fc1 activation is > 0, else 0;
//   per worker: d W4 += d4 (x) h,  d b4 += d4,  d b3 += d3,  loss += loss_i.
// A wavefront keeps its 10 x 8 slice of W4 and of the d W4 accumulator in registers and walks every
// (4 * split)-th image of one worker; lane l owns fc1 units l, l+64, ..., l+448.  Each wavefront's
// sums go to its own partial slot and are added up in fixed order by the reduction kernel.
#include "ps_common.h"

namespace ps {

namespace {

// Sum over the 64 lanes of a wavefront, the same value returned in every lane.  Data-parallel
// primitives (lane permutes inside the vector ALU) instead of shuffles through the LDS crossbar:
// butterflies inside quads and rows of 16, then the row sums are passed up rows 0 -> 1, {0,1} -> {2,3},
// which leaves the total in lane 63.
__device__ __forceinline__ float wave_sum(float v)
{
    auto dpp_add = [](float x, int ctrl, int row_mask) {
        const int moved = 0;  // rows outside the mask add nothing
        int r;
        switch (ctrl) {
            case 0: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0xB1, 0xF, 0xF, false); break;   // quad_perm [1,0,3,2]
            case 1: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0x4E, 0xF, 0xF, false); break;   // quad_perm [2,3,0,1]
            case 2: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0x141, 0xF, 0xF, false); break;  // row_half_mirror
            case 3: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0x140, 0xF, 0xF, false); break;  // row_mirror
            case 4: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0x142, 0xA, 0xF, false); break;  // row_bcast:15 into rows 1, 3
            default: r = __builtin_amdgcn_update_dpp(moved, __float_as_int(x), 0x143, 0xC, 0xF, false); break; // row_bcast:31 into rows 2, 3
        }
        (void)row_mask;
        return x + __int_as_float(r);
    };
    v = dpp_add(v, 0, 0xF);
    v = dpp_add(v, 1, 0xF);
    v = dpp_add(v, 2, 0xF);
    v = dpp_add(v, 3, 0xF);
    v = dpp_add(v, 4, 0xA);
    v = dpp_add(v, 5, 0xC);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__global__ __launch_bounds__(256, 2) void fc2_kernel(WorkerBuffers wb)
{
    const int lane = threadIdx.x & 63, w = blockIdx.x, B = wb.B;
    const int nsub = 4 * gridDim.y, sub = 4 * blockIdx.y + (threadIdx.x >> 6);
    const float* __restrict__ theta = worker_theta(wb, w);
    float w4[NCLS][8], acc[NCLS][8], accb3[8], accb4[NCLS], b4[NCLS];
#pragma unroll
    for (int c = 0; c < NCLS; ++c) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            w4[c][j] = theta[OFF_W4 + c * FC1 + lane + 64 * j];
            acc[c][j] = 0.f;
        }
        accb4[c] = 0.f;
        b4[c] = theta[OFF_B4 + c];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) accb3[j] = 0.f;
    float loss = 0.f;
    const float inv_b = 1.f / (float)B;

    float hn[8];
    if (sub < B) {
#pragma unroll
        for (int j = 0; j < 8; ++j) hn[j] = wb.ht[((size_t)w * B + sub) * FC1 + lane + 64 * j];
    }
    for (int s = sub; s < B; s += nsub) {
        const size_t g = (size_t)w * B + s;
        float hv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) hv[j] = hn[j];
        if (s + nsub < B) {
#pragma unroll
            for (int j = 0; j < 8; ++j) hn[j] = wb.ht[(g + nsub) * FC1 + lane + 64 * j];
        }
        float z[NCLS];
#pragma unroll
        for (int c = 0; c < NCLS; ++c) {
            float part = 0.f;
#pragma unroll
            for (int j = 0; j < 8; ++j) part = fmaf(hv[j], w4[c][j], part);
            z[c] = wave_sum(part) + b4[c];
        }
        const int label = wb.y[g];
        float zmax = z[0];
        int pred = 0;
#pragma unroll
        for (int c = 1; c < NCLS; ++c)
            if (z[c] > zmax) { zmax = z[c]; pred = c; }
        float e[NCLS], se = 0.f;
#pragma unroll
        for (int c = 0; c < NCLS; ++c) {
            e[c] = expf(z[c] - zmax);
            se += e[c];
        }
        const float lse = zmax + logf(se), inv_se = 1.f / se;
        float d4[NCLS], zy = 0.f;
#pragma unroll
        for (int c = 0; c < NCLS; ++c) {
            d4[c] = (e[c] * inv_se - (c == label ? 1.f : 0.f)) * inv_b;
            if (c == label) zy = z[c];
            accb4[c] += d4[c];
        }
        loss += lse - zy;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float dh = 0.f;
#pragma unroll
            for (int c = 0; c < NCLS; ++c) {
                dh = fmaf(d4[c], w4[c][j], dh);
                acc[c][j] = fmaf(d4[c], hv[j], acc[c][j]);
            }
            const float d3 = hv[j] > 0.f ? dh * wb.drop_scale : 0.f;
            wb.d3[g * FC1 + lane + 64 * j] = d3;
            accb3[j] += d3;
        }
        float zl = 0.f;
#pragma unroll
        for (int c = 0; c < NCLS; ++c)
            if (lane == c) zl = z[c];
        if (lane < NCLS) wb.z[g * NCLS + lane] = zl;
        if (lane == 0) wb.pred[g] = pred;
    }

    float* part = wb.fpart + ((size_t)w * nsub + sub) * FC2_PART;
#pragma unroll
    for (int c = 0; c < NCLS; ++c)
#pragma unroll
        for (int j = 0; j < 8; ++j) part[c * FC1 + lane + 64 * j] = acc[c][j];
#pragma unroll
    for (int j = 0; j < 8; ++j) part[FC2_PART_B3 + lane + 64 * j] = accb3[j];
    if (lane == 0) {
#pragma unroll
        for (int c = 0; c < NCLS; ++c) part[FC2_PART_B4 + c] = accb4[c];
        part[FC2_PART_LOSS] = loss;
    }
}

// Inference head (no dropout, no backward): logits, predicted class (lowest index on ties), per-image
// cross-entropy and whether the prediction equals the label.  One wavefront per image.
__global__ __launch_bounds__(256) void fc2_eval_kernel(WorkerBuffers wb, float* __restrict__ loss_i,
                                                       int32_t* __restrict__ correct)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= wb.n * wb.B) return;
    const float* __restrict__ theta = worker_theta(wb, g / wb.B);
    float hv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) hv[j] = wb.ht[(size_t)g * FC1 + lane + 64 * j];
    float z[NCLS];
#pragma unroll
    for (int c = 0; c < NCLS; ++c) {
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) part = fmaf(hv[j], theta[OFF_W4 + c * FC1 + lane + 64 * j], part);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        z[c] = part + theta[OFF_B4 + c];
    }
    const int label = wb.y[g];
    float zmax = z[0], zy = 0.f, zl = 0.f;
    int pred = 0;
#pragma unroll
    for (int c = 1; c < NCLS; ++c)
        if (z[c] > zmax) { zmax = z[c]; pred = c; }
    float se = 0.f;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) {
        se += expf(z[c] - zmax);
        if (c == label) zy = z[c];
        if (c == lane) zl = z[c];
    }
    if (lane < NCLS) wb.z[(size_t)g * NCLS + lane] = zl;
    if (lane == 0) {
        wb.pred[g] = pred;
        loss_i[g] = zmax + logf(se) - zy;
        correct[g] = pred == label;
    }
}

}  // namespace

void launch_fc2_eval(const WorkerBuffers& wb, float* loss_i, int32_t* correct, hipStream_t s)
{
    hipLaunchKernelGGL(fc2_eval_kernel, dim3((wb.n * wb.B + 3) / 4), dim3(256), 0, s, wb, loss_i, correct);
}

int fc2_split(int n) { return std::min(16, std::max(1, (512 + n - 1) / n)); }

void launch_fc2(const WorkerBuffers& wb, hipStream_t s)
{
    hipLaunchKernelGGL(fc2_kernel, dim3(wb.n, fc2_split(wb.n)), dim3(256), 0, s, wb);
}

}  // namespace ps
