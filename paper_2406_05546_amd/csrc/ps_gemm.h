// Batched fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32), used for the three
// contractions of the 1568 -> 512 fully connected layer (forward, input gradient, per-worker
// weight gradient).
//
//   C[m][n] = sum_k A(m,k) * B(n,k)        one problem per blockIdx.z (= worker)
//
// Either operand may be stored k-contiguous ("KC": element (r,k) at base[r*ld + k]) or
// row-contiguous ("RC": element (r,k) at base[k*ld + r]).  A 256-thread block (4 wavefronts, 2x2)
// owns a 128x128 tile of C; each wavefront owns 64x64 as 2x2 MFMA tiles.  K advances 16 at a time
// through double-buffered LDS.  Within a 16-deep stage the contraction index is consumed in the
// order that lets a lane fetch four consecutive k of a KC operand with one 16-byte LDS read:
// MFMA step (j,i), j<2, i<4, pairs lane half h with k = 8j + 4h + i for both operands.
//
// The epilogue functor receives four consecutive rows m..m+3 of one column n:
//   epi(z, m, n, float4 acc)   with m % 4 == 0.
#pragma once
#include "ps_common.h"

namespace ps {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int GEMM_BM = 128, GEMM_BN = 128, GEMM_KS = 16;
constexpr int GEMM_KC_LD = GEMM_KS + 4;  // padded row of a KC tile in LDS: 16-byte reads hit distinct banks
constexpr int GEMM_TILE_FLOATS = 128 * GEMM_KC_LD;  // >= 16 * 128 (RC tile)

struct GemmShape {
    int M, N, K;     // M % 4 == 0; K % 4 == 0 when an operand is KC
    int lda, ldb;
};

// Global -> registers for one 128 x 16 operand stage (two float4 per thread).
template <bool KC>
__device__ __forceinline__ void gemm_load_stage(const float* __restrict__ base, int ld, int row0, int nrows, int k0,
                                                int K, int tid, float4 (&r)[2])
{
    if (KC) {
        const int kc = (tid & 3) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int row = row0 + (tid >> 2) + 64 * i;
            r[i] = (row < nrows && k0 + kc < K)
                       ? *reinterpret_cast<const float4*>(base + (size_t)row * ld + k0 + kc)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    } else {
        const int r4 = (tid & 31) * 4;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int k = k0 + (tid >> 5) + 8 * i;
            r[i] = (row0 + r4 < nrows && k < K)
                       ? *reinterpret_cast<const float4*>(base + (size_t)k * ld + row0 + r4)
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}

template <bool KC>
__device__ __forceinline__ void gemm_store_stage(float* __restrict__ tile, int tid, const float4 (&r)[2])
{
    if (KC) {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<float4*>(tile + ((tid >> 2) + 64 * i) * GEMM_KC_LD + (tid & 3) * 4) = r[i];
    } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<float4*>(tile + ((tid >> 5) + 8 * i) * 128 + (tid & 31) * 4) = r[i];
    }
}

// The four operand values (i = 0..3) a lane feeds to MFMA steps (j, 0..3) for tile row `row`.
template <bool KC>
__device__ __forceinline__ float4 gemm_fetch(const float* __restrict__ tile, int row, int j, int h)
{
    if (KC) return *reinterpret_cast<const float4*>(tile + row * GEMM_KC_LD + 8 * j + 4 * h);
    const float* p = tile + (8 * j + 4 * h) * 128 + row;
    return make_float4(p[0], p[128], p[256], p[384]);
}

template <bool A_KC, bool B_KC, class Epi>
__global__ __launch_bounds__(256) void gemm_f32_mfma(GemmShape sh, Epi epi)
{
    __shared__ __attribute__((aligned(16))) float lds[2][2][GEMM_TILE_FLOATS];  // [buffer][A|B]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int wm = wave & 1, wn = wave >> 1;
    const int z = blockIdx.z;
    const int m0 = blockIdx.x * GEMM_BM, n0 = blockIdx.y * GEMM_BN;
    const float* __restrict__ A = epi.a_ptr(z);
    const float* __restrict__ B = epi.b_ptr(z);

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

    float4 ra[2], rb[2];
    gemm_load_stage<A_KC>(A, sh.lda, m0, sh.M, 0, sh.K, tid, ra);
    gemm_load_stage<B_KC>(B, sh.ldb, n0, sh.N, 0, sh.K, tid, rb);
    gemm_store_stage<A_KC>(lds[0][0], tid, ra);
    gemm_store_stage<B_KC>(lds[0][1], tid, rb);
    __syncthreads();

    const int nk = (sh.K + GEMM_KS - 1) / GEMM_KS;
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) {
            gemm_load_stage<A_KC>(A, sh.lda, m0, sh.M, (kt + 1) * GEMM_KS, sh.K, tid, ra);
            gemm_load_stage<B_KC>(B, sh.ldb, n0, sh.N, (kt + 1) * GEMM_KS, sh.K, tid, rb);
        }
        const float* ta = lds[cur][0];
        const float* tb = lds[cur][1];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            float4 fa[2], fb[2];
#pragma unroll
            for (int a = 0; a < 2; ++a) fa[a] = gemm_fetch<A_KC>(ta, wm * 64 + a * 32 + l32, j, h);
#pragma unroll
            for (int b = 0; b < 2; ++b) fb[b] = gemm_fetch<B_KC>(tb, wn * 64 + b * 32 + l32, j, h);
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].x, fb[b].x, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].y, fb[b].y, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].z, fb[b].z, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].w, fb[b].w, acc[a][b], 0, 0, 0);
                }
        }
        if (kt + 1 < nk) {
            gemm_store_stage<A_KC>(lds[cur ^ 1][0], tid, ra);
            gemm_store_stage<B_KC>(lds[cur ^ 1][1], tid, rb);
        }
        __syncthreads();
    }

    // Accumulator register v of lane (h, l32) holds C[8*(v/4) + 4*h + v%4][l32] of its 32x32 tile.
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int n = n0 + wn * 64 + b * 32 + l32;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = m0 + wm * 64 + a * 32 + 8 * g + 4 * h;
                if (m < sh.M && n < sh.N)
                    epi(z, m, n,
                        make_float4(acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]));
            }
        }
}

}  // namespace ps
