// Batched fp32 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x2_f32), used for the three
// contractions of the 1568 -> 512 fully connected layer (forward, input gradient, per-worker
// weight gradient).
//
//   C[m][n] = sum_k A(m,k) * B(n,k)        one problem per batch index z (= worker)
//
// Either operand may be stored k-contiguous ("KC": element (r,k) at base[r*ld + k]) or
// row-contiguous ("RC": element (r,k) at base[k*ld + r]).  A 256-thread block (4 wavefronts arranged
// WM x WN) owns a (WM*TM*32) x (WN*TN*32) tile of C; each wavefront owns TM x TN MFMA tiles of 32x32.
// K advances KS at a time through double-buffered LDS, with the global loads running two stages
// ahead and everything inside the loop straight-line code, so that loads, LDS writes and address
// updates issue in the shadow of the 64-cycle MFMAs.  Within a stage the contraction index is
// consumed in the order that lets a lane fetch four consecutive k of a KC operand with one 16-byte
// LDS read: MFMA step (j,i), j < KS/8, i < 4, pairs lane half h with k = 8j + 4h + i for both
// operands.
//
// Blocks are numbered so that the blocks of one batch index run next to each other on one XCD (work
// groups are handed to the 8 XCDs round-robin, each XCD has its own L2): the operand that belongs to
// the batch index is then fetched from HBM once and re-used out of that L2.
//
// The epilogue functor receives four consecutive rows m..m+3 of one column n:
//   epi(z, m, n, float4 acc, pre)   with m % 4 == 0,
// where pre = epi.prefetch(z, m, n) was fetched before the K loop (type Epi::Pre; an empty struct if the
// epilogue needs nothing from memory), so that its latency hides under the whole contraction.
#pragma once
#include "ps_common.h"

namespace ps {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4v __attribute__((ext_vector_type(4)));  // first-class vector: stays in registers

constexpr int GEMM_XCDS = 8;

struct GemmShape {
    int M, N, K;     // M % 4 == 0; K % 4 == 0 when an operand is KC
    int lda, ldb;
    int gx, gy, gz;  // tiles along M, along N, batch size
    int m_base, n_base;  // origin of the tile grid inside C (a launch may cover only part of C)
};

// Operand tiles are read with unconditional loads from addresses that are clamped into the operand,
// so the loop carries no branches and no 64-bit address arithmetic (uniform base + 32-bit offset):
//   KC operand [nrows][ld]: a row >= nrows reads the last row instead.  It only reaches rows/columns
//                           of C that are never stored.  K must be a multiple of KS.
//   RC operand [K][ld]:     four-row groups >= nrows read the last group instead.  If K is not a
//                           multiple of KS (RAGGED), a k >= K reads k = K-1 and is then replaced by
//                           zeros, because it is part of the contraction.
template <int ROWS, int KS, bool KC, bool RAGGED>
struct GemmOperand {
    static constexpr int LD = KC ? KS + 4 : ROWS;           // LDS pitch: padded k-row, or one k-plane of ROWS
    static constexpr int FLOATS = KC ? ROWS * LD : KS * LD;
    static constexpr int N4 = ROWS * KS / 4, NV = (N4 + 255) / 256;  // float4 per stage, per thread

    const float* base;
    uint32_t off[NV];     // float offset of this thread's float4 i in stage 0
    uint32_t last[NV];    // RC only: the same element at k = K-1
    uint32_t stage_step;  // float distance between consecutive stages

    __device__ __forceinline__ void init(const float* b, int ld, int row0, int nrows, int K, int tid)
    {
        base = b;
        stage_step = KC ? KS : KS * ld;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int f = min(tid + 256 * i, N4 - 1);  // threads without an element repeat the last one
            if (KC) {
                off[i] = (uint32_t)min(row0 + f / (KS / 4), nrows - 1) * ld + (f % (KS / 4)) * 4;
                last[i] = 0;
            } else {
                const uint32_t row = min(row0 + (f % (ROWS / 4)) * 4, nrows - 4);
                off[i] = (uint32_t)(f / (ROWS / 4)) * ld + row;
                last[i] = (uint32_t)(K - 1) * ld + row;
            }
        }
    }

    // Global -> registers for stage kt.
    __device__ __forceinline__ void load(int kt, floatx4v (&r)[NV]) const
    {
        const uint32_t so = (uint32_t)kt * stage_step;
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            if (KC || !RAGGED) {
                r[i] = *reinterpret_cast<const floatx4v*>(base + so + off[i]);
            } else {
                const uint32_t o = off[i] + so;
                const floatx4v v = *reinterpret_cast<const floatx4v*>(base + min(o, last[i]));
                r[i] = o > last[i] ? floatx4v{0.f, 0.f, 0.f, 0.f} : v;
            }
        }
    }

    static __device__ __forceinline__ void store(float* __restrict__ tile, int tid, const floatx4v (&r)[NV])
    {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int f = tid + 256 * i;
            const int at = KC ? (f / (KS / 4)) * LD + (f % (KS / 4)) * 4 : (f / (ROWS / 4)) * LD + (f % (ROWS / 4)) * 4;
            if (256 * (i + 1) <= N4 || f < N4) *reinterpret_cast<floatx4v*>(tile + at) = r[i];
        }
    }

    // The four operand values (i = 0..3) a lane feeds to MFMA steps (j, 0..3) for tile row `row`.
    static __device__ __forceinline__ floatx4v fetch(const float* __restrict__ tile, int row, int j, int h)
    {
        if (KC) return *reinterpret_cast<const floatx4v*>(tile + row * LD + 8 * j + 4 * h);
        const float* p = tile + (8 * j + 4 * h) * LD + row;
        return floatx4v{p[0], p[LD], p[2 * LD], p[3 * LD]};
    }
};

// Tile configuration of one launch.
template <bool A_KC_, bool B_KC_, int TM_, int TN_, int WM_, int WN_, int KS_>
struct GemmCfg {
    static constexpr bool A_KC = A_KC_, B_KC = B_KC_;
    static constexpr int TM = TM_, TN = TN_, WM = WM_, WN = WN_, KS = KS_;
    static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    static_assert(WM * WN == 4, "four wavefronts per block");
    template <bool RAGGED>
    static constexpr int lds_floats()  // one of the two stage buffers
    {
        return GemmOperand<BM, KS, A_KC, RAGGED>::FLOATS + GemmOperand<BN, KS, B_KC, RAGGED>::FLOATS;
    }
};

// One block's tile: `block` of `sh.gx * sh.gy * sh.gz` (rounded up to the XCD count), stage buffers in lds.
template <class Cfg, bool RAGGED, class Epi>
__device__ __forceinline__ void gemm_block(const GemmShape& sh, const Epi& epi, int block, float* __restrict__ lds)
{
    constexpr bool A_KC = Cfg::A_KC, B_KC = Cfg::B_KC;
    constexpr int TM = Cfg::TM, TN = Cfg::TN, WM = Cfg::WM, KS = Cfg::KS, BM = Cfg::BM, BN = Cfg::BN;
    using OpA = GemmOperand<BM, KS, A_KC, RAGGED>;
    using OpB = GemmOperand<BN, KS, B_KC, RAGGED>;
    constexpr int STAGE = OpA::FLOATS + OpB::FLOATS;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int wm = wave % WM, wn = wave / WM;

    // XCD-aware numbering: XCD x (= linear id mod 8) walks a contiguous range of (z, y, x) triples.
    const int total = sh.gx * sh.gy * sh.gz, per_xcd = (total + GEMM_XCDS - 1) / GEMM_XCDS;
    const int v = (block % GEMM_XCDS) * per_xcd + block / GEMM_XCDS;
    if (v >= total) return;
    const int m0 = sh.m_base + (v % sh.gx) * BM, n0 = sh.n_base + (v / sh.gx % sh.gy) * BN, z = v / (sh.gx * sh.gy);
    const float* __restrict__ A = epi.a_ptr(z);
    const float* __restrict__ B = epi.b_ptr(z);

    floatx16 acc[TM][TN];
    typename Epi::Pre pre[TM][TN][4];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
            const int n = n0 + (wn * TN + b) * 32 + l32;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = m0 + (wm * TM + a) * 32 + 8 * g + 4 * h;
                pre[a][b][g] = (m < sh.M && n < sh.N) ? epi.prefetch(z, m, n) : typename Epi::Pre{};
            }
        }

    // Three-deep pipeline: while the matrix cores consume stage kt out of one LDS buffer, stage kt+1
    // (loaded from HBM/L2 during the previous iteration) is written into the other buffer half way
    // through, and the loads of stage kt+2 are issued right behind that write.
    floatx4v ra[OpA::NV], rb[OpB::NV];
    const int nk = (sh.K + KS - 1) / KS;
    OpA opa;
    OpB opb;
    opa.init(A, sh.lda, m0, sh.M, sh.K, tid);
    opb.init(B, sh.ldb, n0, sh.N, sh.K, tid);
    {
        floatx4v ra0[OpA::NV], rb0[OpB::NV];  // stages 0 and 1 are in flight together
        opa.load(0, ra0);
        opb.load(0, rb0);
        opa.load(min(1, nk - 1), ra);
        opb.load(min(1, nk - 1), rb);
        OpA::store(lds, tid, ra0);
        OpB::store(lds + OpA::FLOATS, tid, rb0);
    }
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        const float* ta = lds + cur * STAGE;
        const float* tb = ta + OpA::FLOATS;
        float* na = lds + (cur ^ 1) * STAGE;
#pragma unroll
        for (int j = 0; j < KS / 8; ++j) {
            floatx4v fa[TM], fb[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) fa[a] = OpA::fetch(ta, (wm * TM + a) * 32 + l32, j, h);
#pragma unroll
            for (int b = 0; b < TN; ++b) fb[b] = OpB::fetch(tb, (wn * TN + b) * 32 + l32, j, h);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b) {
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].x, fb[b].x, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].y, fb[b].y, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].z, fb[b].z, acc[a][b], 0, 0, 0);
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[a].w, fb[b].w, acc[a][b], 0, 0, 0);
                }
            if (j == KS / 16 - 1) {
                // unconditional on purpose (straight-line code schedules under the MFMAs): past the
                // end the last stage is simply loaded and stored again where nobody reads it
                OpA::store(na, tid, ra);
                OpB::store(na + OpA::FLOATS, tid, rb);
                opa.load(min(kt + 2, nk - 1), ra);
                opb.load(min(kt + 2, nk - 1), rb);
            }
        }
        __syncthreads();
    }

    // Accumulator register i of lane (h, l32) holds C[8*(i/4) + 4*h + i%4][l32] of its 32x32 tile.
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int n = n0 + (wn * TN + b) * 32 + l32;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int m = m0 + (wm * TM + a) * 32 + 8 * g + 4 * h;
                if (m < sh.M && n < sh.N)
                    epi(z, m, n,
                        make_float4(acc[a][b][4 * g], acc[a][b][4 * g + 1], acc[a][b][4 * g + 2], acc[a][b][4 * g + 3]),
                        pre[a][b][g]);
            }
        }
}

constexpr int gemm_grid(const GemmShape& sh) { return (sh.gx * sh.gy * sh.gz + GEMM_XCDS - 1) / GEMM_XCDS * GEMM_XCDS; }

template <class Cfg, bool RAGGED, int MINW, class Epi>
__global__ __launch_bounds__(256, MINW) void gemm_f32_mfma(GemmShape sh, Epi epi)
{
    __shared__ __attribute__((aligned(16))) float lds[2 * Cfg::template lds_floats<RAGGED>()];
    gemm_block<Cfg, RAGGED>(sh, epi, blockIdx.x, lds);
}

// Two tile shapes in one launch: the first `main_blocks` blocks cover the main part of C with Main tiles,
// the rest cover an edge strip with Edge tiles.  The edge blocks are dispatched last and run next to the
// last main blocks instead of as a launch of their own behind them.
template <class Main, class Edge, bool RAGGED, int MINW, class Epi>
__global__ __launch_bounds__(256, MINW) void gemm_f32_mfma_edge(GemmShape sh_main, GemmShape sh_edge, int main_blocks, Epi epi)
{
    constexpr int LDS = Main::template lds_floats<RAGGED>() > Edge::template lds_floats<RAGGED>()
                            ? Main::template lds_floats<RAGGED>()
                            : Edge::template lds_floats<RAGGED>();
    __shared__ __attribute__((aligned(16))) float lds[2 * LDS];
    if ((int)blockIdx.x < main_blocks)  // uniform over the block
        gemm_block<Main, RAGGED>(sh_main, epi, blockIdx.x, lds);
    else
        gemm_block<Edge, RAGGED>(sh_edge, epi, blockIdx.x - main_blocks, lds);
}

template <class Cfg>
GemmShape gemm_shape(int M, int N, int K, int lda, int ldb, int batch, int m_begin, int m_end, int n_begin, int n_end)
{
    return GemmShape{M, N, K, lda, ldb, (m_end - m_begin + Cfg::BM - 1) / Cfg::BM, (n_end - n_begin + Cfg::BN - 1) / Cfg::BN,
                     batch, m_begin, n_begin};
}

// One problem per batch index, all of C covered with Cfg tiles over a 1-D grid padded to a multiple of
// the XCD count.
template <class Cfg, int MINW, class Epi>
void gemm_launch(int M, int N, int K, int lda, int ldb, int batch, const Epi& epi, hipStream_t s)
{
    if (M <= 0 || N <= 0 || batch <= 0) return;
    const GemmShape sh = gemm_shape<Cfg>(M, N, K, lda, ldb, batch, 0, M, 0, N);
    if (K % Cfg::KS == 0)
        hipLaunchKernelGGL((gemm_f32_mfma<Cfg, false, MINW, Epi>), dim3(gemm_grid(sh)), dim3(256), 0, s, sh, epi);
    else
        hipLaunchKernelGGL((gemm_f32_mfma<Cfg, true, MINW, Epi>), dim3(gemm_grid(sh)), dim3(256), 0, s, sh, epi);
}

// Rows [0, m_split) x columns [0, n_split) of C with Main tiles and the rest with Edge tiles, where exactly
// one of the splits is inside C (the other equals M or N) and is a multiple of Main's tile: covering a
// ragged edge with narrow tiles avoids a mostly empty wide tile.
template <class Main, class Edge, int MINW, class Epi>
void gemm_launch_edge(int M, int N, int K, int lda, int ldb, int batch, int m_split, int n_split, const Epi& epi, hipStream_t s)
{
    static_assert(Main::KS == Edge::KS, "one K step for both tile shapes");
    if (M <= 0 || N <= 0 || batch <= 0) return;
    const GemmShape sh_main = gemm_shape<Main>(M, N, K, lda, ldb, batch, 0, m_split, 0, n_split);
    const GemmShape sh_edge = m_split < M ? gemm_shape<Edge>(M, N, K, lda, ldb, batch, m_split, M, 0, N)
                                          : gemm_shape<Edge>(M, N, K, lda, ldb, batch, 0, M, n_split, N);
    const int main_blocks = gemm_grid(sh_main), grid = main_blocks + gemm_grid(sh_edge);
    if (K % Main::KS == 0)
        hipLaunchKernelGGL((gemm_f32_mfma_edge<Main, Edge, false, MINW, Epi>), dim3(grid), dim3(256), 0, s, sh_main, sh_edge,
                           main_blocks, epi);
    else
        hipLaunchKernelGGL((gemm_f32_mfma_edge<Main, Edge, true, MINW, Epi>), dim3(grid), dim3(256), 0, s, sh_main, sh_edge,
                           main_blocks, epi);
}

}  // namespace ps
