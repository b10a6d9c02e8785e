// Server-side update kernels: the sync / async apply and the buffered drain (Section 2.1 update
// rules; Section 2.3 and the Section 3.3 server pseudo-code for the drain).  One pass over HBM:
// every buffered gradient is read exactly once, the weights are read and written once and stay
// in registers while the K gradients stream past, so the SUM and SEQ forms move the same bytes.
#include "../../include/ps_hotpath.h"

#include <cstdio>
#include "ps_common.h"

static_assert(PS_ROW_FLOATS == ps::PSTRIDE, "header and kernels disagree on the row pitch");

// Fixed scratch memory of the drain entry point that allocates nothing (ps_drain_rows_mitigated, at the
// end of this file): row list int32 [rows] | clip factors float [rows] | partial sums of the squared
// norms float [rows][32].  Every GPU the process uses holds its own copy at its own address; in host
// code this name is only a handle for hipGetSymbolAddress, never a device address.
#define PS_STATIC_SCRATCH_BYTES ((size_t)PS_STATIC_DRAIN_MAX_ROWS * (4 + 4 + 4 * 32))  /* 557,056 */
static __device__ __align__(256) unsigned char scratch[PS_STATIC_SCRATCH_BYTES];

namespace ps {

namespace {

constexpr int ROW4 = PSTRIDE / 4;  // float4 per row
constexpr int UNROLL = 8;          // independent 16-byte loads in flight per lane
// Threads per block of the streaming kernels: one wavefront.  The 203,328 float4 columns then make
// 3,177 blocks, which spread over the 256 CUs far more evenly than 795 blocks of 256 threads did
// (3.1 blocks per CU: some CUs had a third more rows to stream); the drain went from 6.3 to 6.9 TB/s.
constexpr int APPLY_BLOCK = 64;

__device__ __forceinline__ float4 ld_stream(const float4* p)
{
    // For data a kernel reads once and never again (queue rows, streamed weight copies): keep it out
    // of the caches' way.
    typedef float v4f __attribute__((ext_vector_type(4)));
    v4f v = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ void st_stream(float4* p, float4 x)
{
    typedef float v4f __attribute__((ext_vector_type(4)));
    const v4f v = {x.x, x.y, x.z, x.w};
    __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p));
}

// SCALED: gradient k is multiplied by scale[k] first (norm clipping of stale gradients).
template <int MODE, bool SCALED>
__global__ __launch_bounds__(APPLY_BLOCK) void apply_kernel(float4* __restrict__ theta, const float4* __restrict__ queue,
                                                     const int32_t* __restrict__ idx, int K, float lr,
                                                     const float* __restrict__ scale,
                                                     const uint32_t* __restrict__ K_dev)
{
    const int i = blockIdx.x * APPLY_BLOCK + threadIdx.x;
    if (i >= ROW4) return;
    if (K_dev) K = (int)*K_dev;  // the consumer of the lock-free store learns the count on the device
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
            const float c = SCALED ? scale[k + u] : 1.f;
            if (MODE == 0) {
                if (SCALED) {
                    s.x = fmaf(c, g[u].x, s.x); s.y = fmaf(c, g[u].y, s.y);
                    s.z = fmaf(c, g[u].z, s.z); s.w = fmaf(c, g[u].w, s.w);
                } else {
                    s.x += g[u].x; s.y += g[u].y; s.z += g[u].z; s.w += g[u].w;
                }
            } else {
                const float a = SCALED ? -lr * c : -lr;
                t.x = fmaf(a, g[u].x, t.x); t.y = fmaf(a, g[u].y, t.y);
                t.z = fmaf(a, g[u].z, t.z); t.w = fmaf(a, g[u].w, t.w);
            }
        }
    }
    for (; k < K; ++k) {
        float4 g = ld_stream(col + (size_t)idx[k] * ROW4);
        const float c = SCALED ? scale[k] : 1.f;
        if (MODE == 0) {
            s.x = fmaf(c, g.x, s.x); s.y = fmaf(c, g.y, s.y);
            s.z = fmaf(c, g.z, s.z); s.w = fmaf(c, g.w, s.w);
        } else {
            const float a = -lr * c;
            t.x = fmaf(a, g.x, t.x); t.y = fmaf(a, g.y, t.y);
            t.z = fmaf(a, g.z, t.z); t.w = fmaf(a, g.w, t.w);
        }
    }
    if (MODE == 0) {
        t.x = fmaf(-lr, s.x, t.x); t.y = fmaf(-lr, s.y, t.y);
        t.z = fmaf(-lr, s.z, t.z); t.w = fmaf(-lr, s.w, t.w);
    }
    theta[i] = t;
}

// Adadelta steps over the K listed rows in order (Zeiler 2012, Algorithm 1), one pass over HBM like the
// plain drain: a lane keeps its four weights and their two accumulators in registers while the rows
// stream past.  The quotient sqrt(E[dx^2] + eps) / sqrt(E[g^2] + eps) is formed with the hardware's
// square root and reciprocal square root (about 1 ulp each), which keeps the kernel bandwidth bound.
__global__ __launch_bounds__(APPLY_BLOCK) void apply_adadelta_kernel(float4* __restrict__ theta, float4* __restrict__ acc_g2,
                                                              float4* __restrict__ acc_dx2, const float4* __restrict__ queue,
                                                              const int32_t* __restrict__ idx, int K, float lr, float rho,
                                                              float eps)
{
    const int i = blockIdx.x * APPLY_BLOCK + threadIdx.x;
    if (i >= ROW4) return;
    float t[4], g2[4], dx2[4];
    {
        const float4 a = theta[i], b = acc_g2[i], c = acc_dx2[i];
        t[0] = a.x; t[1] = a.y; t[2] = a.z; t[3] = a.w;
        g2[0] = b.x; g2[1] = b.y; g2[2] = b.z; g2[3] = b.w;
        dx2[0] = c.x; dx2[1] = c.y; dx2[2] = c.z; dx2[3] = c.w;
    }
    const float one_m_rho = 1.f - rho;
    const float4* col = queue + i;
    auto step = [&](const float4& g4) {
        const float g[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            g2[e] = fmaf(rho, g2[e], one_m_rho * g[e] * g[e]);
            const float dx = -(__builtin_amdgcn_sqrtf(dx2[e] + eps) * __builtin_amdgcn_rsqf(g2[e] + eps)) * g[e];
            dx2[e] = fmaf(rho, dx2[e], one_m_rho * dx * dx);
            t[e] = fmaf(lr, dx, t[e]);
        }
    };
    int k = 0;
    for (; k + UNROLL <= K; k += UNROLL) {
        float4 g[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) g[u] = ld_stream(col + (size_t)idx[k + u] * ROW4);
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) step(g[u]);
    }
    for (; k < K; ++k) step(ld_stream(col + (size_t)idx[k] * ROW4));
    theta[i] = make_float4(t[0], t[1], t[2], t[3]);
    acc_g2[i] = make_float4(g2[0], g2[1], g2[2], g2[3]);
    acc_dx2[i] = make_float4(dx2[0], dx2[1], dx2[2], dx2[3]);
}

// Worker-local SGD steps (elastic averaging SGD: every worker trains on its own copy of the weights):
// block row j does ring[slot_j] -= lr * queue[q_j] for the pair (slot_j, q_j); slots are distinct.
__global__ __launch_bounds__(APPLY_BLOCK) void local_step_kernel(float4* __restrict__ ring, const float4* __restrict__ queue,
                                                          const int2* __restrict__ pairs, float lr)
{
    const int i = blockIdx.x * APPLY_BLOCK + threadIdx.x;
    if (i >= ROW4) return;
    const int2 p = pairs[blockIdx.y];
    float4* x = ring + (size_t)p.x * ROW4 + i;
    const float4 g = ld_stream(queue + (size_t)p.y * ROW4 + i);
    float4 t = ld_stream(x);
    t.x = fmaf(-lr, g.x, t.x); t.y = fmaf(-lr, g.y, t.y); t.z = fmaf(-lr, g.z, t.z); t.w = fmaf(-lr, g.w, t.w);
    st_stream(x, t);
}

// One synchronous elastic-averaging step (Zhang et al. 2015, Section 2): with d_k = ring[slot_k] - theta,
// all against the old theta, ring[slot_k] -= alpha d_k and theta += alpha sum_k d_k (summed in list
// order).  One pass: a lane keeps its four centre weights while the n local copies stream through.
// Unlike the read-only streams above this one writes as much as it reads, and it runs fastest with
// one row per iteration and cache-bypassing loads and stores (6.0 TB/s in a timing probe of this
// access pattern, against 5.0 TB/s with eight loads batched before eight stores and 5.3 TB/s for
// the runtime's device-to-device copy of the same bytes).
__global__ __launch_bounds__(APPLY_BLOCK) void elastic_average_kernel(float4* __restrict__ theta, float4* __restrict__ ring,
                                                               const int32_t* __restrict__ slots, int n, float alpha)
{
    const int i = blockIdx.x * APPLY_BLOCK + threadIdx.x;
    if (i >= ROW4) return;
    const float4 c = theta[i];
    float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll 1
    for (int k = 0; k < n; ++k) {
        float4* px = ring + (size_t)slots[k] * ROW4 + i;
        const float4 x = ld_stream(px);
        const float4 d = make_float4(x.x - c.x, x.y - c.y, x.z - c.z, x.w - c.w);
        s.x += d.x; s.y += d.y; s.z += d.z; s.w += d.w;
        st_stream(px, make_float4(fmaf(-alpha, d.x, x.x), fmaf(-alpha, d.y, x.y), fmaf(-alpha, d.z, x.z), fmaf(-alpha, d.w, x.w)));
    }
    theta[i] = make_float4(fmaf(alpha, s.x, c.x), fmaf(alpha, s.y, c.y), fmaf(alpha, s.z, c.z), fmaf(alpha, s.w, c.w));
}

// Squared 2-norm of queue rows, first pass: block (b, k) sums the squares of slice b of row idx[k]
// (the row padding is zero) and writes one partial; fixed slices and a fixed tree keep it reproducible.
constexpr int NORM_SLICES = 32;

__global__ __launch_bounds__(256) void grad_sqnorm_kernel(const float4* __restrict__ queue, const int32_t* __restrict__ idx,
                                                          float* __restrict__ partial)
{
    __shared__ float red[4];
    const int k = blockIdx.y, b = blockIdx.x;
    constexpr int PER = (ROW4 + NORM_SLICES - 1) / NORM_SLICES;
    const float4* row = queue + (size_t)idx[k] * ROW4;
    const int end = min(ROW4, (b + 1) * PER);
    float acc = 0.f;
    for (int i = b * PER + threadIdx.x; i < end; i += 256) {
        const float4 g = ld_stream(row + i);
        acc = fmaf(g.x, g.x, acc); acc = fmaf(g.y, g.y, acc); acc = fmaf(g.z, g.z, acc); acc = fmaf(g.w, g.w, acc);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) partial[k * NORM_SLICES + b] = (red[0] + red[1]) + (red[2] + red[3]);
}

// Second pass: scale[k] = min(1, clip / ||g_k||_2)  (1 for a zero gradient).
__global__ __launch_bounds__(256) void clip_scale_kernel(const float* __restrict__ partial, float* __restrict__ scale, int K,
                                                         float clip)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k >= K) return;
    float sq = 0.f;
    for (int b = 0; b < NORM_SLICES; ++b) sq += partial[k * NORM_SLICES + b];
    const float norm = sqrtf(sq);
    scale[k] = norm > clip ? clip / norm : 1.f;
}

}  // namespace

hipError_t launch_apply(float* theta, const float* queue, const int32_t* idx_dev, int K, float lr, int mode,
                        hipStream_t s, Profiler& prof, const uint32_t* K_dev)
{
    if (K <= 0) return hipSuccess;
    dim3 grid((ROW4 + APPLY_BLOCK - 1) / APPLY_BLOCK), block(APPLY_BLOCK);
    prof.begin(mode == 0 ? K_APPLY_SUM : K_APPLY_SEQ, s);
    if (mode == 0)
        hipLaunchKernelGGL((apply_kernel<0, false>), grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr,
                           (const float*)nullptr, K_dev);
    else
        hipLaunchKernelGGL((apply_kernel<1, false>), grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr,
                           (const float*)nullptr, K_dev);
    prof.end(s);
    return hipGetLastError();
}

hipError_t launch_apply_clipped(float* theta, const float* queue, const int32_t* idx_dev, int K, float lr, int mode,
                                float clip, float* partial_dev, float* scale_dev, hipStream_t s, Profiler& prof)
{
    if (K <= 0) return hipSuccess;
    prof.begin(K_GRAD_SQNORM, s);
    hipLaunchKernelGGL(grad_sqnorm_kernel, dim3(NORM_SLICES, K), dim3(256), 0, s, (const float4*)queue, idx_dev, partial_dev);
    prof.end(s);
    hipLaunchKernelGGL(clip_scale_kernel, dim3((K + 255) / 256), dim3(256), 0, s, partial_dev, scale_dev, K, clip);
    dim3 grid((ROW4 + APPLY_BLOCK - 1) / APPLY_BLOCK), block(APPLY_BLOCK);
    prof.begin(mode == 0 ? K_APPLY_SUM_CLIP : K_APPLY_SEQ_CLIP, s);
    if (mode == 0)
        hipLaunchKernelGGL((apply_kernel<0, true>), grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr,
                           (const float*)scale_dev, (const uint32_t*)nullptr);
    else
        hipLaunchKernelGGL((apply_kernel<1, true>), grid, block, 0, s, (float4*)theta, (const float4*)queue, idx_dev, K, lr,
                           (const float*)scale_dev, (const uint32_t*)nullptr);
    prof.end(s);
    return hipGetLastError();
}

hipError_t launch_apply_adadelta(float* theta, float* acc_g2, float* acc_dx2, const float* queue, const int32_t* idx_dev,
                                 int K, float lr, float rho, float eps, hipStream_t s, Profiler& prof)
{
    if (K <= 0) return hipSuccess;
    prof.begin(K_APPLY_ADADELTA, s);
    hipLaunchKernelGGL(apply_adadelta_kernel, dim3((ROW4 + APPLY_BLOCK - 1) / APPLY_BLOCK), dim3(APPLY_BLOCK), 0, s, (float4*)theta, (float4*)acc_g2,
                       (float4*)acc_dx2, (const float4*)queue, idx_dev, K, lr, rho, eps);
    prof.end(s);
    return hipGetLastError();
}

hipError_t launch_local_steps(float* ring, const float* queue, const int32_t* pairs_dev, int n, float lr, hipStream_t s,
                              Profiler& prof)
{
    if (n <= 0) return hipSuccess;
    prof.begin(K_LOCAL_STEP, s);
    hipLaunchKernelGGL(local_step_kernel, dim3((ROW4 + APPLY_BLOCK - 1) / APPLY_BLOCK, n), dim3(APPLY_BLOCK), 0, s, (float4*)ring, (const float4*)queue,
                       (const int2*)pairs_dev, lr);
    prof.end(s);
    return hipGetLastError();
}

hipError_t launch_elastic_average(float* theta, float* ring, const int32_t* slots_dev, int n, float alpha, hipStream_t s,
                                  Profiler& prof)
{
    if (n <= 0) return hipSuccess;
    prof.begin(K_ELASTIC, s);
    hipLaunchKernelGGL(elastic_average_kernel, dim3((ROW4 + APPLY_BLOCK - 1) / APPLY_BLOCK), dim3(APPLY_BLOCK), 0, s, (float4*)theta, (float4*)ring,
                       slots_dev, n, alpha);
    prof.end(s);
    return hipGetLastError();
}

int norm_slices() { return NORM_SLICES; }

// ---------------------------------------------------------------------------------------------
// Drain for callers that cannot allocate.  What the context's workspace holds for the mitigated drain
// (the row list, the per-slice partial sums of the squared norms, the clip factors) lives here in a
// fixed array in device memory instead; every GPU of the process has its own copy at its own address.
namespace {

constexpr int STATIC_MAX_ROWS = PS_STATIC_DRAIN_MAX_ROWS;
constexpr size_t STATIC_IDX_OFF = 0;                                                   // int32 [rows]
constexpr size_t STATIC_SCALE_OFF = STATIC_IDX_OFF + sizeof(int32_t) * STATIC_MAX_ROWS;  // float [rows]
constexpr size_t STATIC_PART_OFF = STATIC_SCALE_OFF + sizeof(float) * STATIC_MAX_ROWS;   // float [rows][NORM_SLICES]
static_assert(STATIC_PART_OFF + sizeof(float) * STATIC_MAX_ROWS * NORM_SLICES == PS_STATIC_SCRATCH_BYTES, "scratch array size");

constexpr int MAX_DEVICES = 64;
unsigned char* scratch_of_device[MAX_DEVICES] = {};  // device address of `scratch` on each GPU, once resolved

// rows are taken in the order they lie in memory: idx[k] = k
__global__ __launch_bounds__(256) void row_list_kernel(int32_t* __restrict__ idx, int n)
{
    const int k = blockIdx.x * 256 + threadIdx.x;
    if (k < n) idx[k] = k;
}

thread_local char static_error[160] = "";

ps_status static_fail(ps_status st, const char* msg)
{
    std::snprintf(static_error, sizeof(static_error), "%s", msg);
    return st;
}

}  // namespace

// Device address of this GPU's copy of the array (the array's name is only a host-side handle), looked
// up once per device with that device current.
hipError_t static_scratch(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
    if (!scratch_of_device[dev]) {
        unsigned char* ptr = nullptr;
        e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_of_device[dev] = ptr;
    }
    *out = scratch_of_device[dev];
    return hipSuccess;
}

const char* static_last_error() { return static_error; }

}  // namespace ps

extern "C" ps_status ps_drain_rows_mitigated(float* theta_dev, const float* grads_dev, int32_t n_rows, int32_t mode,
                                             const ps_drain_policy* pol, float* lr_used_host, void* hip_stream)
{
    using namespace ps;
    if (!pol || (mode != PS_DRAIN_SUM && mode != PS_DRAIN_SEQ) || !(pol->lr_backlog_ref >= 0.f) || !(pol->clip_norm >= 0.f))
        return static_fail(PS_EINVAL, "ps_drain_rows_mitigated: bad mode or policy");
    if (n_rows < 0) return static_fail(PS_EINVAL, "ps_drain_rows_mitigated: negative row count");
    if (n_rows > STATIC_MAX_ROWS)
        return static_fail(PS_EINVAL, "ps_drain_rows_mitigated: more than PS_STATIC_DRAIN_MAX_ROWS (4096) rows");
    const float K = (float)n_rows;
    const float lr = (pol->lr_backlog_ref > 0.f && K > pol->lr_backlog_ref) ? pol->lr * (pol->lr_backlog_ref / K) : pol->lr;
    if (lr_used_host) *lr_used_host = lr;
    if (n_rows == 0) return PS_OK;
    if (!theta_dev || !grads_dev || (reinterpret_cast<uintptr_t>(theta_dev) & 15) || (reinterpret_cast<uintptr_t>(grads_dev) & 15))
        return static_fail(PS_EINVAL, "ps_drain_rows_mitigated: null or misaligned device pointer");
    unsigned char* base = nullptr;
    if (static_scratch(&base) != hipSuccess)
        return static_fail(PS_EDEVICE, "ps_drain_rows_mitigated: the address of the static scratch array could not be resolved");
    int32_t* idx = reinterpret_cast<int32_t*>(base + STATIC_IDX_OFF);
    float* scale = reinterpret_cast<float*>(base + STATIC_SCALE_OFF);
    float* partial = reinterpret_cast<float*>(base + STATIC_PART_OFF);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    static Profiler no_timing;  // never enabled
    // Nothing in the array has to start at zero: the row list, every partial sum and every clip factor of
    // the rows in use are written before they are read.
    hipLaunchKernelGGL(row_list_kernel, dim3((n_rows + 255) / 256), dim3(256), 0, s, idx, (int)n_rows);
    hipError_t e = pol->clip_norm > 0.f
                       ? launch_apply_clipped(theta_dev, grads_dev, idx, n_rows, lr, mode, pol->clip_norm, partial, scale, s, no_timing)
                       : launch_apply(theta_dev, grads_dev, idx, n_rows, lr, mode, s, no_timing);
    if (e != hipSuccess) return static_fail(PS_EDEVICE, hipGetErrorString(e));
    return PS_OK;
}
