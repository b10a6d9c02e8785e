// fc2 (512 -> 10), softmax cross-entropy and everything of their backward pass that the fc1 GEMMs do
// not do, in one kernel:
//   z = W4 . h + b4;  loss_i = logsumexp(z) - z[y];  d4 = (softmax(z) - onehot(y)) / B;
//   d3 = (W4^T d4) / (1-p) where the dropped-and-rectified fc1 activation is > 0, else 0;
//   per worker: d W4 += d4 (x) h,  d b4 += d4,  d b3 += d3,  loss += loss_i.
// The three contractions run on the matrix cores (v_mfma_f32_16x16x4_f32), 16 images at a time, the
// ten classes padded to 16.  A block stages the 16 x 512 activations of a group in LDS (the next
// group's are on their way into registers meanwhile); wavefront v owns fc1 units 128v .. 128v+127:
//   logits     rows = images, columns = classes, K = this wavefront's 128 units; the four wavefronts'
//              partial sums meet in LDS and every wavefront then does the (cheap) softmax itself, which
//              leaves d4 in MFMA accumulator layout: lane (q, l) holds images 4q..4q+3 of class l;
//   d3         rows = images, columns = this wavefront's units (8 tiles), K = classes; its A operand is
//              d4 transposed through a wavefront-private LDS tile.  Column l of tile (T, e) is unit
//              128v + 64T + 4l + e, so that a lane's values of the four tiles e = 0..3 are four
//              consecutive units: one 16-byte LDS read for the gate, one 16-byte store for d3;
//   d W4       rows = classes, columns = units, K = images; its A operand is d4 exactly as the
//              accumulator layout holds it, its B operand the activations that also gate d3.
// W4 sits in registers in both operand layouts (64 per lane), d W4 in 32 accumulators per lane.  Each
// block's sums go to its own partial slot and are added up in fixed order by the reduction kernel.
#include "ps_common.h"

namespace ps {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

constexpr int FC2_G = 16;                 // images per group
constexpr int FC2_HP = FC1 + 4;           // LDS row pitch of the activation tile (floats)
constexpr int FC2_TP = 20;                // row pitch of the 16 x 16 transpose tiles

// Lane l of a row of 16 gets op over the 16 lanes of its row (data-parallel primitives: swaps inside
// quads, then the two mirrors).
template <class Op>
__device__ __forceinline__ float row16_reduce(float v, Op op)
{
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, false)));   // quad_perm [1,0,3,2]
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, false)));   // quad_perm [2,3,0,1]
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, false)));  // row_half_mirror
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, false)));  // row_mirror
    return v;
}

__global__ __launch_bounds__(256, 2) void fc2_kernel(WorkerBuffers wb)
{
    __shared__ __attribute__((aligned(16))) float hs[2][FC2_G * FC2_HP];     // 66,048 B
    __shared__ __attribute__((aligned(16))) float zpart[4 * 64 * 4];         // the wavefronts' partial logits
    __shared__ __attribute__((aligned(16))) float d4t[4][FC2_G * FC2_TP];    // wavefront-private transposes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane >> 4, l16 = lane & 15;
    const int w = blockIdx.x, B = wb.B, split = gridDim.y, n_groups = (B + FC2_G - 1) / FC2_G;
    const float* __restrict__ theta = worker_theta(wb, w);
    const float* __restrict__ W4 = theta + OFF_W4;
    const bool cls_ok = l16 < NCLS;
    const int u0 = 128 * wave;

    // B operand of the logits: k-step (j, e) pairs lane quarter q with unit u0 + 16j + 4q + e
    float wa[8][4];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) wa[j][e] = cls_ok ? W4[l16 * FC1 + u0 + 16 * j + 4 * q + e] : 0.f;
    // B operand of d3: tile t = 4T + e, k-step i pairs lane quarter q with class 4q + i; column l16 = unit
    // u0 + 64T + 4*l16 + e
    float wbk[8][4];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
            wbk[t][i] = 4 * q + i < NCLS ? W4[(4 * q + i) * FC1 + u0 + 64 * (t >> 2) + 4 * l16 + (t & 3)] : 0.f;
    const float b4 = cls_ok ? theta[OFF_B4 + l16] : 0.f;
    const float inv_b = 1.f / (float)B;

    floatx4 acc_w4[8];  // d W4 tile t = 4T + e: register i = class 4q + i, column l16 = unit u0 + 64T + 4*l16 + e
    float acc_b3[8], acc_b4 = 0.f, acc_loss = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
        acc_w4[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        acc_b3[t] = 0.f;
    }

    // activations of a group: 16 x 128 float4, eight per thread; rows beyond the batch are zero
    float4 hv[8];
    auto prefetch = [&](int grp) {
        const size_t g0 = (size_t)w * B + (size_t)grp * FC2_G;
        const int valid = min(FC2_G, B - grp * FC2_G);
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int f = tid + 256 * k, img = f >> 7, c4 = f & 127;
            hv[k] = img < valid ? *reinterpret_cast<const float4*>(wb.ht + (g0 + img) * FC1 + 4 * c4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    int grp = blockIdx.y, buf = 0;
    if (grp < n_groups) prefetch(grp);
    for (; grp < n_groups; grp += split, buf ^= 1) {
        const size_t g0 = (size_t)w * B + (size_t)grp * FC2_G;
        const int valid = min(FC2_G, B - grp * FC2_G);
        float* __restrict__ hb = hs[buf];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int f = tid + 256 * k, img = f >> 7, c4 = f & 127;
            *reinterpret_cast<float4*>(hb + img * FC2_HP + 4 * c4) = hv[k];
        }
        __syncthreads();  // also: every wavefront is done with the group before last, whose buffer comes next
        if (grp + split < n_groups) prefetch(grp + split);
        int label[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) label[i] = 4 * q + i < valid ? wb.y[g0 + 4 * q + i] : -1;

        // logits, this wavefront's share of K: rows = images (lane row l16), columns = classes
        floatx4 zacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const floatx4 a = *reinterpret_cast<const floatx4*>(hb + l16 * FC2_HP + u0 + 16 * j + 4 * q);
#pragma unroll
            for (int e = 0; e < 4; ++e) zacc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], wa[j][e], zacc, 0, 0, 0);
        }
        *reinterpret_cast<floatx4*>(zpart + (wave * 64 + lane) * 4) = zacc;
        __syncthreads();
        floatx4 z = *reinterpret_cast<const floatx4*>(zpart + lane * 4);
#pragma unroll
        for (int v = 1; v < 4; ++v) z += *reinterpret_cast<const floatx4*>(zpart + (v * 64 + lane) * 4);

        // softmax and d4 for images 4q + i, class l16 (classes 10..15 are padding)
        floatx4 d4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float zi = z[i] + b4;
            const float zmax = row16_reduce(cls_ok ? zi : -INFINITY, [](float a, float b) { return fmaxf(a, b); });
            const float e = cls_ok ? expf(zi - zmax) : 0.f;
            const float se = row16_reduce(e, [](float a, float b) { return a + b; });
            const bool img_ok = label[i] >= 0, mine = l16 == label[i];
            d4[i] = (img_ok && cls_ok) ? (e * (1.f / se) - (mine ? 1.f : 0.f)) * inv_b : 0.f;
            if (wave == 0) {
                if (mine) acc_loss += zmax + logf(se) - zi;
                acc_b4 += d4[i];
                const float first = row16_reduce((cls_ok && zi == zmax) ? (float)l16 : 99.f, [](float a, float b) { return fminf(a, b); });
                if (img_ok && cls_ok) wb.z[(g0 + 4 * q + i) * NCLS + l16] = zi;
                if (img_ok && l16 == 0) wb.pred[g0 + 4 * q + i] = (int)first;
            }
        }

        // d4 with images along the lane rows, for the A operand of d3 (wavefront-private: no barrier)
        float* tp = d4t[wave];
#pragma unroll
        for (int i = 0; i < 4; ++i) tp[(4 * q + i) * FC2_TP + l16] = d4[i];
        const floatx4 d4a = *reinterpret_cast<const floatx4*>(tp + l16 * FC2_TP + 4 * q);

#pragma unroll
        for (int T = 0; T < 2; ++T) {
            // activations of images 4q + i at units u0 + 64T + 4*l16 .. +3: gate of d3 and B operand of d W4
            floatx4 hc[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) hc[i] = *reinterpret_cast<const floatx4*>(hb + (4 * q + i) * FC2_HP + u0 + 64 * T + 4 * l16);
            floatx4 dh[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dh[e] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int i = 0; i < 4; ++i) dh[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(d4a[i], wbk[4 * T + e][i], dh[e], 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    acc_w4[4 * T + e] = __builtin_amdgcn_mfma_f32_16x16x4f32(d4[i], hc[i][e], acc_w4[4 * T + e], 0, 0, 0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                floatx4 d3;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    d3[e] = hc[i][e] > 0.f ? dh[e][i] * wb.drop_scale : 0.f;
                    acc_b3[4 * T + e] += d3[e];
                }
                if (4 * q + i < valid) *reinterpret_cast<floatx4*>(wb.d3 + (g0 + 4 * q + i) * FC1 + u0 + 64 * T + 4 * l16) = d3;
            }
        }
    }

    float* part = wb.fpart + ((size_t)w * split + blockIdx.y) * FC2_PART;
#pragma unroll
    for (int T = 0; T < 2; ++T) {
        const int u = u0 + 64 * T + 4 * l16;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (4 * q + i < NCLS)
                *reinterpret_cast<floatx4*>(part + (4 * q + i) * FC1 + u) =
                    floatx4{acc_w4[4 * T][i], acc_w4[4 * T + 1][i], acc_w4[4 * T + 2][i], acc_w4[4 * T + 3][i]};
        floatx4 b3;  // the four lane quarters hold different images
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float v = acc_b3[4 * T + e];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            b3[e] = v;
        }
        if (q == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e) part[FC2_PART_B3 + u + e] = b3[e];
        }
    }
    if (wave == 0) {
        acc_b4 += __shfl_xor(acc_b4, 16, 64);
        acc_b4 += __shfl_xor(acc_b4, 32, 64);
        if (q == 0 && cls_ok) part[FC2_PART_B4 + l16] = acc_b4;
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) acc_loss += __shfl_xor(acc_loss, off, 64);
        if (lane == 0) part[FC2_PART_LOSS] = acc_loss;
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
