// What this chip sustains, measured with the same instructions the library's kernels are made of, so
// that every roofline figure can be read against the datasheet and against the achievable rate:
// the two fp32 MFMA shapes alone, MFMAs with vector-ALU instructions between them (do they overlap?),
// MFMA wavefronts and vector-ALU wavefronts sharing a SIMD, and plain HBM streams.  Instrumentation,
// not part of the method.  Every kernel is a fixed-length loop over registers or an in-bounds stream.
#include "../../include/ps_hotpath.h"

#include <algorithm>
#include <vector>

#include "ps_common.h"

namespace ps {

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Two independent accumulator chains per wavefront, eight MFMAs per chain and iteration.
__global__ __launch_bounds__(256) void mfma32_kernel(float* out, int iters, float a, float b)
{
    floatx16 acc[2];
    for (int c = 0; c < 2; ++c)
        for (int v = 0; v < 16; ++v) acc[c][v] = 0.f;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < 2; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[c], 0, 0, 0);
    }
    float s = 0.f;
    for (int c = 0; c < 2; ++c)
        for (int v = 0; v < 16; ++v) s += acc[c][v];
    if (s == 12345.678f) out[threadIdx.x] = s;  // keeps the loop alive; never true for the arguments used
}

// 16x16x4 MFMAs, NV independent vector FMAs after each one (NV = 0: MFMAs alone).  MFMA: 1 = issue MFMAs,
// 0 = only the vector instructions (the same number per iteration as with MFMAs).
template <int NV, int MFMA>
__device__ __forceinline__ void mixed_loop(float* out, int iters, float a, float b)
{
    floatx4 acc[2] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    float x[NV > 0 ? NV : 1];
    for (int j = 0; j < (NV > 0 ? NV : 1); ++j) x[j] = (float)threadIdx.x + j;
    for (int i = 0; i < iters; ++i) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                if (MFMA) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[c], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < NV; ++j) x[j] = __builtin_fmaf(x[j], a, b);
            }
    }
    float s = acc[0][0] + acc[0][1] + acc[0][2] + acc[0][3] + acc[1][0] + acc[1][1] + acc[1][2] + acc[1][3];
    for (int j = 0; j < NV; ++j) s += x[j];
    if (s == 12345.678f) out[threadIdx.x] = s;
}

template <int NV>
__global__ __launch_bounds__(256) void mfma16_valu_kernel(float* out, int iters, float a, float b)
{
    mixed_loop<NV, 1>(out, iters, a, b);
}

// 512 threads = two wavefronts per SIMD: wavefronts 0-3 run `first`, wavefronts 4-7 run `second`
// (0 = nothing, 1 = MFMAs alone, 2 = four vector FMAs per MFMA slot and no MFMA).
__global__ __launch_bounds__(512) void shared_simd_kernel(float* out, int iters, float a, float b, int first, int second)
{
    const int kind = threadIdx.x < 256 ? first : second;  // uniform per wavefront
    if (kind == 1) mixed_loop<0, 1>(out, iters, a, b);
    if (kind == 2) mixed_loop<4, 0>(out, iters, a, b);
}

// 16x16x4 MFMAs whose A operand comes out of LDS: READS values read per MFMA (0: operands from registers;
// 1: one ds_read_b32 per MFMA, consecutive lanes on consecutive banks; 2: a second value read and added up on
// the side).  Two blocks per compute unit, as the conv2 kernels run.
template <int READS>
__global__ __launch_bounds__(256, 2) void mfma16_lds_kernel(float* out, int iters, float b)
{
    __shared__ __attribute__((aligned(16))) float lds[16384];
    for (int i = threadIdx.x; i < 16384; i += 256) lds[i] = (float)(i & 7);
    __syncthreads();
    const float* p = lds + (threadIdx.x & 63) + (threadIdx.x >> 6) * 2048;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    float side = 0.f;
    for (int i = 0; i < iters; ++i) {
        const float* q = p + (i & 3) * 256;  // stays inside the wavefront's 2048 + 1024 + 16 * 272 floats < 16384
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            if (READS >= 2) side += q[u * 272 + 64];
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(READS >= 1 ? q[u * 272] : b, b, acc, 0, 0, 0);
        }
    }
    const float s = acc[0] + acc[1] + acc[2] + acc[3] + side;
    if (s == 12345.678f) out[threadIdx.x] = s;
}

__device__ __forceinline__ floatx4 ld_nt(const floatx4* p) { return __builtin_nontemporal_load(p); }

// Reads `rows` rows of row4 float4 once, in the drain kernel's geometry: one-wavefront blocks, a lane owns
// one float4 column and walks down the rows with eight loads in flight; the sum goes nowhere unless it hits
// a magic value.
__global__ __launch_bounds__(64) void stream_read_kernel(const floatx4* __restrict__ src, int row4, int rows, float* out)
{
    const int i = blockIdx.x * 64 + threadIdx.x;
    if (i >= row4) return;
    const floatx4* col = src + i;
    floatx4 s = {0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (; k + 8 <= rows; k += 8) {
        floatx4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = ld_nt(col + (size_t)(k + u) * row4);
#pragma unroll
        for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; k < rows; ++k) s += ld_nt(col + (size_t)k * row4);
    if (s[0] + s[1] + s[2] + s[3] == 12345.678f) out[threadIdx.x] = s[0];
}

__global__ __launch_bounds__(256) void stream_copy_kernel(const floatx4* __restrict__ src, floatx4* __restrict__ dst, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) __builtin_nontemporal_store(ld_nt(src + i), dst + i);
}

__global__ __launch_bounds__(256) void fill_kernel(floatx4* __restrict__ dst, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) dst[i] = floatx4{1.f, 1.f, 1.f, 1.f};
}

struct Timer {
    hipStream_t s;
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t err = hipSuccess;
    explicit Timer(hipStream_t st) : s(st)
    {
        err = hipEventCreate(&a);
        if (err == hipSuccess) err = hipEventCreate(&b);
    }
    ~Timer()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
    // median duration in ms of `reps` runs of launch()
    template <class F>
    double median(F launch, int reps)
    {
        std::vector<float> ms;
        for (int r = 0; r < reps && err == hipSuccess; ++r) {
            err = hipEventRecord(a, s);
            launch();
            if (err == hipSuccess) err = hipGetLastError();
            if (err == hipSuccess) err = hipEventRecord(b, s);
            if (err == hipSuccess) err = hipEventSynchronize(b);
            float t = 0.f;
            if (err == hipSuccess) err = hipEventElapsedTime(&t, a, b);
            ms.push_back(t);
        }
        if (ms.empty()) return 0.0;
        std::sort(ms.begin(), ms.end());
        return ms[ms.size() / 2];
    }
};

}  // namespace

}  // namespace ps

extern "C" ps_status ps_measure_ceilings(void* workspace_dev, uint64_t workspace_bytes, void* hip_stream, ps_ceilings* out)
{
    using namespace ps;
    if (!out || !workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < (64u << 20)) return PS_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        return PS_EDEVICE;
    *out = ps_ceilings{};
    out->compute_units = cus;
    float* sink = static_cast<float*>(workspace_dev);  // never written: the kernels' guards are never true
    Timer t(s);
    if (t.err != hipSuccess) return PS_EDEVICE;

    // the clock ramps up under load: the first launches run slower than the sustained rate
    const int blocks = 2 * cus, iters32 = 6000;
    const double flop32 = 4.0 * 8 * 2 * (32.0 * 32 * 2 * 2) * iters32 * blocks;
    const double first = t.median([&] { hipLaunchKernelGGL(mfma32_kernel, dim3(blocks), dim3(256), 0, s, sink, iters32, 1.f, 1.f); }, 1);
    out->mfma_32x32x2_first_launch_tflops = flop32 / (first * 1e-3) / 1e12;
    for (int w = 0; w < 8; ++w) hipLaunchKernelGGL(mfma32_kernel, dim3(blocks), dim3(256), 0, s, sink, iters32, 1.f, 1.f);
    out->mfma_32x32x2_tflops =
        flop32 / (t.median([&] { hipLaunchKernelGGL(mfma32_kernel, dim3(blocks), dim3(256), 0, s, sink, iters32, 1.f, 1.f); }, 7) * 1e-3) / 1e12;

    // one wavefront per SIMD: MFMAs with 0, 1, 2, 4 vector FMAs behind each
    const int iters16 = 20000;
    const double flop16 = 4.0 * 8 * 2 * (16.0 * 16 * 4 * 2) * iters16 * cus, mfmas_per_wave = 8.0 * 2 * iters16;
    const double m0 = t.median([&] { hipLaunchKernelGGL(mfma16_valu_kernel<0>, dim3(cus), dim3(256), 0, s, sink, iters16, 1.f, 1.f); }, 5);
    const double m1 = t.median([&] { hipLaunchKernelGGL(mfma16_valu_kernel<1>, dim3(cus), dim3(256), 0, s, sink, iters16, 1.f, 1.f); }, 5);
    const double m2 = t.median([&] { hipLaunchKernelGGL(mfma16_valu_kernel<2>, dim3(cus), dim3(256), 0, s, sink, iters16, 1.f, 1.f); }, 5);
    const double m4 = t.median([&] { hipLaunchKernelGGL(mfma16_valu_kernel<4>, dim3(cus), dim3(256), 0, s, sink, iters16, 1.f, 1.f); }, 5);
    out->mfma_16x16x4_tflops = flop16 / (m0 * 1e-3) / 1e12;
    out->ns_per_mfma_16x16x4 = m0 * 1e6 / mfmas_per_wave;
    out->ns_per_mfma_with_valu[0] = m0 * 1e6 / mfmas_per_wave;
    out->ns_per_mfma_with_valu[1] = m1 * 1e6 / mfmas_per_wave;
    out->ns_per_mfma_with_valu[2] = m2 * 1e6 / mfmas_per_wave;
    out->ns_per_mfma_with_valu[3] = m4 * 1e6 / mfmas_per_wave;

    // an MFMA wavefront and a vector-ALU wavefront on each SIMD: alone, alone, together
    out->shared_simd_ms[0] = t.median([&] { hipLaunchKernelGGL(shared_simd_kernel, dim3(cus), dim3(512), 0, s, sink, iters16, 1.f, 1.f, 1, 0); }, 5);
    out->shared_simd_ms[1] = t.median([&] { hipLaunchKernelGGL(shared_simd_kernel, dim3(cus), dim3(512), 0, s, sink, iters16, 1.f, 1.f, 0, 2); }, 5);
    out->shared_simd_ms[2] = t.median([&] { hipLaunchKernelGGL(shared_simd_kernel, dim3(cus), dim3(512), 0, s, sink, iters16, 1.f, 1.f, 1, 2); }, 5);

    // MFMAs fed from LDS, two blocks of four wavefronts per compute unit
    {
        const int itl = 8000;
        const double per = 1e6 / (itl * 16.0 * 2.0);  // two wavefronts share a SIMD: ns of SIMD time per MFMA
        out->ns_per_mfma_with_lds_reads[0] = per * t.median([&] { hipLaunchKernelGGL(mfma16_lds_kernel<0>, dim3(2 * cus), dim3(256), 0, s, sink, itl, 1.f); }, 5);
        out->ns_per_mfma_with_lds_reads[1] = per * t.median([&] { hipLaunchKernelGGL(mfma16_lds_kernel<1>, dim3(2 * cus), dim3(256), 0, s, sink, itl, 1.f); }, 5);
        out->ns_per_mfma_with_lds_reads[2] = per * t.median([&] { hipLaunchKernelGGL(mfma16_lds_kernel<2>, dim3(2 * cus), dim3(256), 0, s, sink, itl, 1.f); }, 5);
    }

    // HBM streams over the workspace (at most 4 GiB of it): read once; copy first half to second half
    const uint64_t bytes = std::min<uint64_t>(workspace_bytes, 4ull << 30) & ~uint64_t(511);
    const size_t n4 = bytes / 16;
    floatx4* buf = static_cast<floatx4*>(workspace_dev);
    hipLaunchKernelGGL(fill_kernel, dim3(8 * cus), dim3(256), 0, s, buf, n4);
    const int row4 = PSTRIDE / 4, rows = (int)(n4 / row4);  // rows of one P-vector each, as the drain streams them
    const double rd = t.median([&] { hipLaunchKernelGGL(stream_read_kernel, dim3((row4 + 63) / 64), dim3(64), 0, s, buf, row4, rows, sink); }, 7);
    out->hbm_read_bytes = (uint64_t)rows * row4 * 16;
    out->hbm_read_GBps = (double)out->hbm_read_bytes / (rd * 1e-3) / 1e9;
    const double cp = t.median([&] { hipLaunchKernelGGL(stream_copy_kernel, dim3(16 * cus), dim3(256), 0, s, buf, buf + n4 / 2, n4 / 2); }, 7);
    out->hbm_copy_GBps = (double)bytes / (cp * 1e-3) / 1e9;  // half read + half written
    if (t.err != hipSuccess || hipStreamSynchronize(s) != hipSuccess) return PS_EDEVICE;
    return PS_OK;
}
