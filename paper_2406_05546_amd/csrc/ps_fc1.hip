// The three contractions of the 1568 -> 512 fully connected layer on the matrix cores: forward with
// fused bias + ReLU + dropout, input gradient with the conv2 ReLU gate, and the per-worker weight
// gradient written straight into the worker's queue entry.
#include "ps_common.h"
#include "ps_gemm.h"
#include "ps_philox.h"

namespace ps {

namespace {

// fc1 on the matrix cores.  Rows m are fc1 units, columns n are the worker's samples, so that the
// four accumulators a lane holds for one column are four consecutive units of one sample: exactly
// the four words of one Philox call.
struct Fc1FwdEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return worker_theta(wb, z) + OFF_W3; }
    __device__ const float* b_ptr(int z) const { return wb.p2 + (size_t)z * wb.B * P2_SIZE; }
    struct Pre {};
    __device__ Pre prefetch(int, int, int) const { return Pre{}; }
    __device__ void operator()(int z, int m, int n, float4 acc, Pre) const
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
// Rows m are pool2 features, columns n samples, contraction over the 512 units.  The gate is bit 2 of
// the pool2 window bytes (winner > 0, which is the same as pooled activation > 0): four bytes per
// epilogue call, fetched before the contraction starts.
struct Fc1DxEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return worker_theta(wb, z) + OFF_W3; }
    __device__ const float* b_ptr(int z) const { return wb.d3 + (size_t)z * wb.B * FC1; }
    typedef uint32_t Pre;
    __device__ Pre prefetch(int z, int m, int n) const
    {
        return *reinterpret_cast<const uint32_t*>(wb.am2 + ((size_t)z * wb.B + n) * P2_SIZE + m);  // m % 4 == 0
    }
    __device__ void operator()(int z, int m, int n, float4 acc, Pre gate) const
    {
        float4 o;
        o.x = (gate & 0x00000004u) ? acc.x : 0.f;
        o.y = (gate & 0x00000400u) ? acc.y : 0.f;
        o.z = (gate & 0x00040000u) ? acc.z : 0.f;
        o.w = (gate & 0x04000000u) ? acc.w : 0.f;
        *reinterpret_cast<float4*>(wb.dp2g + ((size_t)z * wb.B + n) * P2_SIZE + m) = o;
    }
};

// Per-worker d fc1.W[u][i] = sum_s d3[s][u] * pool2[s][i], written into the worker's queue entry.
// Rows m are units, columns n features, so a wavefront's lanes run along contiguous memory.
struct Fc1DwEpi {
    WorkerBuffers wb;
    __device__ const float* a_ptr(int z) const { return wb.d3 + (size_t)z * wb.B * FC1; }
    __device__ const float* b_ptr(int z) const { return wb.p2 + (size_t)z * wb.B * P2_SIZE; }
    struct Pre {};
    __device__ Pre prefetch(int, int, int) const { return Pre{}; }
    __device__ void operator()(int z, int m, int n, float4 acc, Pre) const
    {
        float* g = worker_grad(wb, z) + OFF_W3 + (size_t)m * P2_SIZE + n;
        g[0] = acc.x;
        g[P2_SIZE] = acc.y;
        g[2 * P2_SIZE] = acc.z;
        g[3 * P2_SIZE] = acc.w;
    }
};

}  // namespace

// All three use 128 x 128 block tiles (four wavefronts of 64 x 64), K stepped 16 at a time.  The 1568
// features are 12 such tiles plus 32: that edge is covered with 32-wide tiles (four wavefronts of
// 32 x 32 side by side) instead of a thirteenth wide tile that would be three quarters empty, by extra
// blocks of the same launch that run next to the last wide tiles.
constexpr int FEAT_WIDE = P2_SIZE / 128 * 128;  // 1536

// forward: rows = 512 units (W3, k-contiguous), columns = the worker's samples (pool2, k-contiguous)
// A launch too small to give every compute unit two 128 x 128 tiles is cut into 64 x 128 tiles instead (the
// order in which a value's products are added up does not depend on the tile shape).
void launch_fc1_fwd(const WorkerBuffers& wb, hipStream_t s)
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
    }
    const int wide_tiles = (FC1 / 128) * ((wb.B + 127) / 128) * wb.n;
    if (wide_tiles >= 2 * cus)
        gemm_launch<GemmCfg<true, true, 2, 2, 2, 2, 16>, 1>(FC1, wb.B, P2_SIZE, P2_SIZE, P2_SIZE, wb.n, Fc1FwdEpi{wb}, s);
    else
        gemm_launch<GemmCfg<true, true, 1, 2, 2, 2, 16>, 1>(FC1, wb.B, P2_SIZE, P2_SIZE, P2_SIZE, wb.n, Fc1FwdEpi{wb}, s);
}

// weight gradient: rows = 512 units (d3, row-contiguous), columns = 1568 features (pool2, row-contiguous),
// contraction over the worker's samples
void launch_fc1_dw(const WorkerBuffers& wb, hipStream_t s)
{
    gemm_launch_edge<GemmCfg<false, false, 2, 2, 2, 2, 16>, GemmCfg<false, false, 1, 1, 4, 1, 16>, 1>(
        FC1, P2_SIZE, wb.B, FC1, P2_SIZE, wb.n, FC1, FEAT_WIDE, Fc1DwEpi{wb}, s);
}

// input gradient: rows = 1568 features (W3, row-contiguous), columns = samples (d3, k-contiguous),
// contraction over the 512 units
void launch_fc1_dx(const WorkerBuffers& wb, hipStream_t s)
{
    gemm_launch_edge<GemmCfg<false, true, 2, 2, 2, 2, 16>, GemmCfg<false, true, 1, 1, 1, 4, 16>, 1>(
        P2_SIZE, wb.B, FC1, P2_SIZE, FC1, wb.n, FEAT_WIDE, wb.B, Fc1DxEpi{wb}, s);
}

}  // namespace ps
