// Server-side update kernels: the sync / async apply and the buffered drain (Section 2.1 update
// rules; Section 2.3 and the Section 3.3 server pseudo-code for the drain).  One pass over HBM:
// every buffered gradient is read exactly once, the weights are read and written once and stay
// in registers while the K gradients stream past, so the SUM and SEQ forms move the same bytes.
#include "ps_common.h"

namespace ps {

namespace {

constexpr int ROW4 = PSTRIDE / 4;  // float4 per row
constexpr int UNROLL = 8;          // independent 16-byte loads in flight per lane

__device__ __forceinline__ float4 ld_stream(const float4* p)
{
    // The queue is read once and never again: keep it out of the caches' way.
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

template <int MODE>
__global__ __launch_bounds__(256) void apply_kernel(float4* __restrict__ theta, const float4* __restrict__ queue,
                                                     const int32_t* __restrict__ idx, int K, float lr)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= ROW4) return;
    float4 t = theta[i];
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
    const float4* col = queue + i;
    int k = 0;
    for (; k + UNROLL <= K; k += UNROLL) {
        float4 g[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) g[u] = ld_stream(col + (size_t)idx[k + u] * ROW4);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            if (MODE == 0) {
                s.x += g[u].x; s.y += g[u].y; s.z += g[u].z; s.w += g[u].w;
            } else {
                t.x = fmaf(-lr, g[u].x, t.x); t.y = fmaf(-lr, g[u].y, t.y);
                t.z = fmaf(-lr, g[u].z, t.z); t.w = fmaf(-lr, g[u].w, t.w);
            }
        }
    }
    for (; k < K; ++k) {
        float4 g = ld_stream(col + (size_t)idx[k] * ROW4);
        if (MODE == 0) {
            s.x += g.x; s.y += g.y; s.z += g.z; s.w += g.w;
        } else {
            t.x = fmaf(-lr, g.x, t.x); t.y = fmaf(-lr, g.y, t.y);
            t.z = fmaf(-lr, g.z, t.z); t.w = fmaf(-lr, g.w, t.w);
        }
    }
    if (MODE == 0) {
        t.x = fmaf(-lr, s.x, t.x); t.y = fmaf(-lr, s.y, t.y);
        t.z = fmaf(-lr, s.z, t.z); t.w = fmaf(-lr, s.w, t.w);
    }
    theta[i] = t;
}

}  // namespace

hipError_t launch_apply(float* theta, const float* queue, const int32_t* idx_dev, int K, float lr, int mode,
                        hipStream_t s, Profiler& prof)
{
    if (K <= 0) return hipSuccess;
    dim3 grid((ROW4 + 255) / 256), block(256);
    prof.begin(mode == 0 ? K_APPLY_SUM : K_APPLY_SEQ, s);
    if (mode == 0)
        hipLaunchKernelGGL(apply_kernel<0>, grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr);
    else
        hipLaunchKernelGGL(apply_kernel<1>, grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr);
    prof.end(s);
    return hipGetLastError();
}

}  // namespace ps
