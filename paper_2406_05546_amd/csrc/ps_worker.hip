// Worker step on the GPU: forward and backward pass of the paper's CNN (model endnote) for n
// workers x B images in one batch of launches.  Worker w reads the weights of ring slot
// meta[w].slot in place (a stale snapshot costs no copy) and its gradient is written straight into
// queue entry meta[w].q (Section 3.3 worker step: read weights, compute gradient, append).
#include "ps_common.h"
#include "ps_gemm.h"
#include "ps_philox.h"

namespace ps {

namespace {

// ---------------------------------------------------------------------------------------------
// conv1 (1 -> 16, 3x3, pad 1) + ReLU + 2x2 max pool.  One block per image; a thread owns one
// pooled position and walks the 16 output channels with its 4x4 input patch in registers.
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
    if (t >= P1_POS) return;
    const int py = t / P1_W, px = t % P1_W;
    float patch[4][4];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) patch[a][b] = xs[(2 * py + a) * 30 + 2 * px + b];
    for (int o = 0; o < C1; ++o) {
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
        const size_t out = (size_t)g * P1_SIZE + o * P1_POS + t;
        wb.p1[out] = fmaxf(best, 0.f);
        wb.am1[out] = (uint8_t)(code | (best > 0.f ? 4 : 0));
    }
}

// ---------------------------------------------------------------------------------------------
// fc1 on the matrix cores.  Rows m are fc1 units, columns n are the worker's samples, so that the
// four accumulators a lane holds for one column are four consecutive units of one sample: exactly
// the four words of one Philox call.
struct Fc1FwdEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return worker_theta(wb, z) + OFF_W3; }
    __device__ const float* b_ptr(int z) const { return wb.p2 + (size_t)z * wb.B * P2_SIZE; }
    __device__ void operator()(int z, int m, int n, float4 acc) const
    {
        const float4 b = *reinterpret_cast<const float4*>(worker_theta(wb, z) + OFF_B3 + m);
        const WorkerMeta mt = wb.meta[z];
        const uint4 r = philox4x32_10(make_uint4(mt.mb_lo, mt.mb_hi, (uint32_t)n, (uint32_t)(m >> 2)),
                                      make_uint2(wb.seed_lo, wb.seed_hi));
        float4 o;
        o.x = r.x >= wb.drop_threshold ? fmaxf(acc.x + b.x, 0.f) * wb.drop_scale : 0.f;
        o.y = r.y >= wb.drop_threshold ? fmaxf(acc.y + b.y, 0.f) * wb.drop_scale : 0.f;
        o.z = r.z >= wb.drop_threshold ? fmaxf(acc.z + b.z, 0.f) * wb.drop_scale : 0.f;
        o.w = r.w >= wb.drop_threshold ? fmaxf(acc.w + b.w, 0.f) * wb.drop_scale : 0.f;
        *reinterpret_cast<float4*>(wb.ht + ((size_t)z * wb.B + n) * FC1 + m) = o;
    }
};

// d pool2 = d3 . W3, zeroed where the pooled activation is zero (ReLU gate of conv2).
// Rows m are pool2 features, columns n samples, contraction over the 512 units.
struct Fc1DxEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return worker_theta(wb, z) + OFF_W3; }
    __device__ const float* b_ptr(int z) const { return wb.d3 + (size_t)z * wb.B * FC1; }
    __device__ void operator()(int z, int m, int n, float4 acc) const
    {
        const size_t at = ((size_t)z * wb.B + n) * P2_SIZE + m;
        const float4 a = *reinterpret_cast<const float4*>(wb.p2 + at);
        float4 o;
        o.x = a.x > 0.f ? acc.x : 0.f;
        o.y = a.y > 0.f ? acc.y : 0.f;
        o.z = a.z > 0.f ? acc.z : 0.f;
        o.w = a.w > 0.f ? acc.w : 0.f;
        *reinterpret_cast<float4*>(wb.dp2g + at) = o;
    }
};

// Per-worker d fc1.W[u][i] = sum_s d3[s][u] * pool2[s][i], written into the worker's queue entry.
// Rows m are units, columns n features, so a wavefront's lanes run along contiguous memory.
struct Fc1DwEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return wb.d3 + (size_t)z * wb.B * FC1; }
    __device__ const float* b_ptr(int z) const { return wb.p2 + (size_t)z * wb.B * P2_SIZE; }
    __device__ void operator()(int z, int m, int n, float4 acc) const
    {
        float* g = worker_grad(wb, z) + OFF_W3 + (size_t)m * P2_SIZE + n;
        g[0] = acc.x;
        g[P2_SIZE] = acc.y;
        g[2 * P2_SIZE] = acc.z;
        g[3 * P2_SIZE] = acc.w;
    }
};

// ---------------------------------------------------------------------------------------------
// fc2, softmax cross-entropy and their backward, one wavefront per image:
//   z = W4 . h + b4;  loss_i = logsumexp(z) - z[y];  d4 = (softmax(z) - onehot(y)) / B;
//   d3 = (W4^T d4) * 1/(1-p) where the dropped-and-rectified activation is > 0, else 0.
__global__ __launch_bounds__(256) void fc2_kernel(WorkerBuffers wb)
{
    const int lane = threadIdx.x & 63;
    const int g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= wb.n * wb.B) return;
    const int w = g / wb.B;
    const float* theta = worker_theta(wb, w);
    const float* W4 = theta + OFF_W4;
    float hv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) hv[j] = wb.ht[(size_t)g * FC1 + lane + 64 * j];
    float z[NCLS];
#pragma unroll
    for (int c = 0; c < NCLS; ++c) {
        float part = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) part = fmaf(hv[j], W4[c * FC1 + lane + 64 * j], part);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off, 64);
        z[c] = part + theta[OFF_B4 + c];
    }
    const int label = wb.y[g];
    float zmax = z[0];
    int pred = 0;
#pragma unroll
    for (int c = 1; c < NCLS; ++c)
        if (z[c] > zmax) { zmax = z[c]; pred = c; }
    float se = 0.f;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) se += expf(z[c] - zmax);
    const float lse = zmax + logf(se);
    const float inv_b = 1.f / (float)wb.B;
    float d4[NCLS], zy = 0.f;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) {
        d4[c] = (expf(z[c] - lse) - (c == label ? 1.f : 0.f)) * inv_b;
        if (c == label) zy = z[c];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float dh = 0.f;
#pragma unroll
        for (int c = 0; c < NCLS; ++c) dh = fmaf(d4[c], W4[c * FC1 + lane + 64 * j], dh);
        wb.d3[(size_t)g * FC1 + lane + 64 * j] = hv[j] > 0.f ? dh * wb.drop_scale : 0.f;
    }
    if (lane == 0) {
#pragma unroll
        for (int c = 0; c < NCLS; ++c) {
            wb.z[(size_t)g * NCLS + c] = z[c];
            wb.d4[(size_t)g * NCLS + c] = d4[c];
        }
        wb.pred[g] = pred;
        wb.loss_i[g] = lse - zy;
    }
}

// Per-worker d fc2.W, d fc2.b, d fc1.b and the worker's mean loss.  grid (n, 2): a thread owns
// one fc1 unit and sums over the worker's samples in order.
__global__ __launch_bounds__(256) void fc2_grad_kernel(WorkerBuffers wb)
{
    const int w = blockIdx.x, u = blockIdx.y * 256 + threadIdx.x, B = wb.B;
    float* grad = worker_grad(wb, w);
    float acc[NCLS], accb = 0.f;
#pragma unroll
    for (int c = 0; c < NCLS; ++c) acc[c] = 0.f;
    for (int s = 0; s < B; ++s) {
        const size_t g = (size_t)w * B + s;
        const float hv = wb.ht[g * FC1 + u];
        accb += wb.d3[g * FC1 + u];
#pragma unroll
        for (int c = 0; c < NCLS; ++c) acc[c] = fmaf(wb.d4[g * NCLS + c], hv, acc[c]);
    }
#pragma unroll
    for (int c = 0; c < NCLS; ++c) grad[OFF_W4 + c * FC1 + u] = acc[c];
    grad[OFF_B3 + u] = accb;
    if (blockIdx.y == 0 && threadIdx.x <= NCLS) {
        const int c = threadIdx.x;
        float sum = 0.f;
        if (c < NCLS) {
            for (int s = 0; s < B; ++s) sum += wb.d4[((size_t)w * B + s) * NCLS + c];
            grad[OFF_B4 + c] = sum;
        } else {
            for (int s = 0; s < B; ++s) sum += wb.loss_i[(size_t)w * B + s];
            if (wb.loss) wb.loss[w] = sum / (float)B;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// conv1 weight gradient: d W1[o][dy][dx] = sum over images and pooled positions of
// dpool1g[o][p] * xpad[winner(p) + (dy,dx)].  grid (n, N_CHUNK); 16 lanes share an output channel.
__global__ __launch_bounds__(256) void conv1_dw_kernel(WorkerBuffers wb)
{
    __shared__ float xs[30 * 30];
    const int w = blockIdx.x, chunk = blockIdx.y, t = threadIdx.x, B = wb.B;
    const int per = (B + N_CHUNK - 1) / N_CHUNK;
    const int s0 = chunk * per, s1 = min(B, s0 + per);
    const int o = t >> 4, l16 = t & 15;
    float acc[9], accb = 0.f;
#pragma unroll
    for (int i = 0; i < 9; ++i) acc[i] = 0.f;
    for (int s = s0; s < s1; ++s) {
        const size_t g = (size_t)w * B + s;
        __syncthreads();
        for (int i = t; i < 900; i += 256) {
            const int yy = i / 30 - 1, xx = i % 30 - 1;
            xs[i] = (yy >= 0 && yy < 28 && xx >= 0 && xx < 28) ? wb.x[g * IMG_PIX + yy * 28 + xx] : 0.f;
        }
        __syncthreads();
        for (int p = l16; p < P1_POS; p += 16) {
            const size_t at = g * P1_SIZE + o * P1_POS + p;
            const float v = wb.dp1g[at];
            const int code = wb.am1[at] & 3;
            const int base = (2 * (p / P1_W) + (code >> 1)) * 30 + 2 * (p % P1_W) + (code & 1);
            accb += v;
#pragma unroll
            for (int dy = 0; dy < 3; ++dy)
#pragma unroll
                for (int dx = 0; dx < 3; ++dx) acc[dy * 3 + dx] = fmaf(v, xs[base + dy * 30 + dx], acc[dy * 3 + dx]);
        }
    }
#pragma unroll
    for (int m = 8; m > 0; m >>= 1) {
#pragma unroll
        for (int i = 0; i < 9; ++i) acc[i] += __shfl_xor(acc[i], m, 64);
        accb += __shfl_xor(accb, m, 64);
    }
    if (l16 == 0) {
        float* part = wb.part + ((size_t)w * N_PART + chunk * 4) * CONV_PART;
#pragma unroll
        for (int i = 0; i < 9; ++i) part[OFF_W1 + o * 9 + i] = acc[i];
        part[OFF_B1 + o] = accb;
    }
}

// Sums the partial slots in fixed order into the worker's queue entry: conv1 tensors have one partial
// per chunk (slot 4*chunk), conv2 tensors one per (chunk, wavefront).
__global__ __launch_bounds__(256) void conv_grad_reduce_kernel(WorkerBuffers wb)
{
    const int w = blockIdx.x;
    float* grad = worker_grad(wb, w);
    const float* part = wb.part + (size_t)w * N_PART * CONV_PART;
    for (int i = threadIdx.x; i < CONV_PART; i += 256) {
        float sum = 0.f;
        if (i < OFF_W2) {
#pragma unroll
            for (int c = 0; c < N_CHUNK; ++c) sum += part[(size_t)c * 4 * CONV_PART + i];
        } else {
#pragma unroll
            for (int c = 0; c < N_PART; ++c) sum += part[(size_t)c * CONV_PART + i];
        }
        grad[i] = sum;
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

inline dim3 gemm_grid(int M, int N, int n) { return dim3((M + GEMM_BM - 1) / GEMM_BM, (N + GEMM_BN - 1) / GEMM_BN, n); }

}  // namespace

#define PS_TIMED(id, ...)      \
    do {                       \
        prof.begin(id, s);     \
        __VA_ARGS__;           \
        prof.end(s);           \
    } while (0)

hipError_t launch_worker_forward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof)
{
    const int N = wb.n * wb.B;
    if (N <= 0) return hipSuccess;
    PS_TIMED(K_CONV1_FWD, hipLaunchKernelGGL(conv1_fwd_kernel, dim3(N), dim3(256), 0, s, wb));
    PS_TIMED(K_CONV2_FWD, launch_conv2_fwd(wb, s));
    GemmShape sh{FC1, wb.B, P2_SIZE, P2_SIZE, P2_SIZE};
    PS_TIMED(K_FC1_FWD, hipLaunchKernelGGL((gemm_f32_mfma<true, true, Fc1FwdEpi>), gemm_grid(sh.M, sh.N, wb.n),
                                           dim3(256), 0, s, sh, Fc1FwdEpi{wb}));
    PS_TIMED(K_FC2, hipLaunchKernelGGL(fc2_kernel, dim3((N + 3) / 4), dim3(256), 0, s, wb));
    return hipGetLastError();
}

hipError_t launch_worker_backward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof)
{
    const int N = wb.n * wb.B;
    if (N <= 0) return hipSuccess;
    PS_TIMED(K_FC2_GRAD, hipLaunchKernelGGL(fc2_grad_kernel, dim3(wb.n, 2), dim3(256), 0, s, wb));
    GemmShape dw{FC1, P2_SIZE, wb.B, FC1, P2_SIZE};
    PS_TIMED(K_FC1_DW, hipLaunchKernelGGL((gemm_f32_mfma<false, false, Fc1DwEpi>), gemm_grid(dw.M, dw.N, wb.n),
                                          dim3(256), 0, s, dw, Fc1DwEpi{wb}));
    GemmShape dx{P2_SIZE, wb.B, FC1, P2_SIZE, FC1};
    PS_TIMED(K_FC1_DX, hipLaunchKernelGGL((gemm_f32_mfma<false, true, Fc1DxEpi>), gemm_grid(dx.M, dx.N, wb.n),
                                          dim3(256), 0, s, dx, Fc1DxEpi{wb}));
    PS_TIMED(K_CONV2_DW, launch_conv2_dw(wb, s));
    PS_TIMED(K_CONV2_DX, launch_conv2_dx(wb, s));
    PS_TIMED(K_CONV1_DW, hipLaunchKernelGGL(conv1_dw_kernel, dim3(wb.n, N_CHUNK), dim3(256), 0, s, wb));
    PS_TIMED(K_CONV_REDUCE, hipLaunchKernelGGL(conv_grad_reduce_kernel, dim3(wb.n), dim3(256), 0, s, wb));
    return hipGetLastError();
}

const char* kernel_name(int id)
{
    static const char* const names[K_COUNT] = {
        "conv1_fwd_kernel", "conv2_fwd_kernel", "gemm_f32_mfma<true, true, Fc1FwdEpi>", "fc2_kernel",
        "fc2_grad_kernel", "gemm_f32_mfma<false, false, Fc1DwEpi>", "gemm_f32_mfma<false, true, Fc1DxEpi>",
        "conv2_dw_kernel", "conv2_dx_kernel", "conv1_dw_kernel", "conv_grad_reduce_kernel", "apply_kernel<0>",
        "apply_kernel<1>"};
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
