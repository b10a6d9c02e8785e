// conv2 (16 -> 32 channels, 3x3, pad 1, on 14x14 maps) as implicit GEMMs on the gfx950 matrix cores
// (v_mfma_f32_16x16x4_f32): forward with fused ReLU + 2x2 max pool, input gradient, and per-worker
// weight gradient.  Zero-padded feature maps are staged in LDS as [channel][16][16] planes (plane
// pitch a little above 256 floats), so that a 3x3 tap is a compile-time address offset (dy*16 + dx)
// from a lane's base address.
// The 32x16x9 filter bank lives in registers for the whole block (72 VGPRs per lane) in exactly the
// layout the MFMA B operand wants; it is read from the worker's ring slot once per block.
#include "ps_common.h"

namespace ps {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// LDS pitch (floats) of one padded 16x16 plane, chosen per kernel so that the 32 lanes an LDS read
// serves per cycle fall into 32 different banks: the lane quarters of the forward A operand are four
// channels over 8+8 window columns (pitch = 8 mod 32), those of the input-gradient A operand two
// channels over 16 consecutive positions (pitch = 16 mod 32), and the weight-gradient operands put 16
// channels on 16 lanes at 2 neighbouring positions (pitch = 2 mod 32).
constexpr int CHS_FWD = 264, CHS_DX = 272, CHS_DW = 258;

__device__ __forceinline__ floatx4 mfma16(float a, float b, floatx4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// Staging is split in two so that the global loads of the next group of images are in flight while
// the matrix cores work on the current one: prefetch_* issues the loads into registers, commit_*
// writes the registers into the padded LDS planes after the barrier that ends the current group.

// pool1 planes of COUNT images (16 channels, 14x14 interiors); NV float4 per thread of a block of NT.
template <int COUNT, int CHS, int NT = 256>
struct Pool1Stage {
    static constexpr int P1_IMS = C1 * CHS;
    static constexpr int N4 = COUNT * (P1_SIZE / 4), NV = (N4 + NT - 1) / NT;
    floatx4 v[NV];
    uint32_t src[NV];  // float offset of this thread's k-th float4 inside a group of COUNT images
    __device__ __forceinline__ void init(int tid)
    {
#pragma unroll
        for (int k = 0; k < NV; ++k) src[k] = (uint32_t)min(tid + NT * k, N4 - 1) * 4;  // threads without an element repeat the last one
    }
    // images [g0, g0 + valid) exist; the rest of the group repeats the last existing image (its
    // results are never stored), so the loads need no branches
    __device__ __forceinline__ void prefetch(const float* __restrict__ p1, size_t g0, int valid, int tid)
    {
        const float* group = p1 + g0 * P1_SIZE;
        if (valid >= COUNT) {  // uniform over the block
#pragma unroll
            for (int k = 0; k < NV; ++k) v[k] = *reinterpret_cast<const floatx4*>(group + src[k]);
        } else {
#pragma unroll
            for (int k = 0; k < NV; ++k) {
                const uint32_t img = min(src[k] / P1_SIZE, (uint32_t)(valid - 1));
                v[k] = *reinterpret_cast<const floatx4*>(group + img * P1_SIZE + src[k] % P1_SIZE);
            }
        }
    }
    // Where the float4s land does not change from group to group: a table (bits 0-14 the offset of
    // the first element, bit 15 set when the four positions run over the end of a 14-wide row after two
    // elements) replaces that arithmetic by one 2-byte LDS read per float4.
    static __device__ __forceinline__ void build_table(uint16_t* __restrict__ tab, int tid)
    {
        static_assert(COUNT * P1_IMS < (1 << 15), "offsets must fit 15 bits");
        for (int i4 = tid; i4 < N4; i4 += NT) {
            const int img = i4 / (P1_SIZE / 4), r = (i4 % (P1_SIZE / 4)) * 4, c = r / P1_POS, pos = r % P1_POS;
            const int base = img * P1_IMS + c * CHS + 17 + (pos / P1_W) * 16 + pos % P1_W;  // interior starts at (1,1)
            tab[i4] = (uint16_t)(base | (pos % P1_W == P1_W - 2 ? 0x8000 : 0));
        }
    }
    __device__ __forceinline__ void commit(float* __restrict__ tile, const uint16_t* __restrict__ tab, int tid) const
    {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int i4 = tid + NT * k;
            if (NT * (k + 1) <= N4 || i4 < N4) {
                const uint32_t e = tab[i4];
                float* dst = tile + (e & 0x7fffu);
                const uint32_t hop = (e >> 15) * 2;  // the next row starts 16 - 14 further on
                dst[0] = v[k][0];
                dst[1] = v[k][1];
                dst[2 + hop] = v[k][2];
                dst[3 + hop] = v[k][3];
            }
        }
    }
};

// Gated pool2 gradient of COUNT images, routed to the window winners of padded planes
// d2[o][16][16] (interior at (1,1)).  A thread moves four consecutive values at a time (one 16-byte load
// of gradients, one 4-byte load of window bytes); where a value lands apart from its winner's place in
// the window never changes, so those offsets are computed once per block (two 16-bit offsets per
// register) and a commit costs a handful of vector instructions per value instead of the divisions by 49
// and 7.  Before the next commit the planes are cleared as a whole with 16-byte stores.
template <int COUNT, int CHS, int NT = 256>
struct D2Stage {
    static constexpr int D2_IMS = C2 * CHS;
    static constexpr int N4 = COUNT * (P2_SIZE / 4), NV = (N4 + NT - 1) / NT;
    static_assert(P2_SIZE % 4 == 0, "a group of four values never straddles two images");
    static_assert(COUNT * D2_IMS < (1 << 16), "offsets must fit 16 bits");
    floatx4 v[NV];
    uint32_t code[NV];
    uint32_t base[NV][2];  // offsets of the four values' windows (winner (0,0)), 16 bits each
    __device__ __forceinline__ void init(int tid)
    {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            uint32_t b[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int e = min(4 * (tid + NT * k), COUNT * P2_SIZE - 4) + j;
                const int img = e / P2_SIZE, r = e % P2_SIZE, o = r / P2_POS, p = r % P2_POS;
                b[j] = (uint32_t)(img * D2_IMS + o * CHS + (2 * (p / P2_W) + 1) * 16 + 2 * (p % P2_W) + 1);
            }
            base[k][0] = b[0] | (b[1] << 16);
            base[k][1] = b[2] | (b[3] << 16);
        }
    }
    __device__ __forceinline__ void prefetch(const WorkerBuffers& wb, size_t g0, int valid, int tid)
    {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            const int i4 = tid + NT * k;
            const bool ok = (NT * (k + 1) <= N4 || i4 < N4) && (4 * i4) / P2_SIZE < valid;
            v[k] = ok ? *reinterpret_cast<const floatx4*>(wb.dp2g + g0 * P2_SIZE + (size_t)i4 * 4) : floatx4{0.f, 0.f, 0.f, 0.f};
            code[k] = ok ? *reinterpret_cast<const uint32_t*>(wb.am2 + g0 * P2_SIZE + (size_t)i4 * 4) : 0u;
        }
    }
    __device__ __forceinline__ void commit(float* __restrict__ d2, int tid) const
    {
#pragma unroll
        for (int k = 0; k < NV; ++k) {
            if (!(NT * (k + 1) <= N4 || tid + NT * k < N4)) break;
            // winner (dy, dx) of every byte -> dy * 16 + dx, four at once
            const uint32_t off = (code[k] & 0x01010101u) | ((code[k] & 0x02020202u) << 3);
            d2[(base[k][0] & 0xffffu) + (off & 0xffu)] = v[k][0];
            d2[(base[k][0] >> 16) + ((off >> 8) & 0xffu)] = v[k][1];
            d2[(base[k][1] & 0xffffu) + ((off >> 16) & 0xffu)] = v[k][2];
            d2[(base[k][1] >> 16) + (off >> 24)] = v[k][3];
        }
    }
    // zeroes all COUNT * D2_IMS floats of the planes
    static __device__ __forceinline__ void clear(float* __restrict__ d2, int tid)
    {
        static_assert(COUNT * D2_IMS % 4 == 0, "16-byte stores");
        constexpr int T4 = COUNT * D2_IMS / 4;
#pragma unroll
        for (int i = 0; i < (T4 + NT - 1) / NT; ++i)
            if (NT * (i + 1) <= T4 || tid + NT * i < T4)
                reinterpret_cast<floatx4*>(d2)[tid + NT * i] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
};

// ---------------------------------------------------------------------------------------------
// Forward.  GEMM rows are conv outputs ordered (pooled position, window element) so that the four
// accumulators of a lane are one 2x2 pool window; columns are the 32 output channels (two 16-wide
// MFMA tiles sharing the A operand); K = (tap, channel).  A block owns up to FWD_IPB images of one
// worker and walks them FWD_G at a time (FWD_G * 49 pooled positions, four per row tile), FWD_NW wavefronts
// per block.
constexpr int FWD_G = 4, FWD_NW = 4, FWD_NT = 64 * FWD_NW, FWD_IPB = 32;
constexpr int FWD_TILES = (FWD_G * P2_POS + 3) / 4;

__global__ __launch_bounds__(FWD_NT, 512 / FWD_NT) void conv2_fwd_kernel(WorkerBuffers wb, int blocks_per_worker, int ipb)
{
    constexpr int CHS = CHS_FWD, P1_IMS = C1 * CHS;
    __shared__ __attribute__((aligned(16))) float tile[FWD_G * P1_IMS];  // 16,896 B per image
    // pooled position of the group -> offset of its window in the planes / of its output.  On this chip
    // fp32 MFMAs and vector-ALU instructions do not overlap, so index arithmetic inside the tile loop
    // is paid for in matrix time: look it up.
    // (entries past the group's last position, in a last tile that is not full, point at position 0: read, never stored)
    __shared__ int win_off[4 * FWD_TILES], out_off[4 * FWD_TILES];
    __shared__ uint16_t stage_tab[Pool1Stage<FWD_G, CHS_FWD, FWD_NT>::N4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane >> 4, l16 = lane & 15;
    const int w = blockIdx.x / blocks_per_worker, chunk = blockIdx.x % blocks_per_worker;
    const int B = wb.B, s_begin = chunk * ipb, s_end = min(B, s_begin + ipb);
    const float* __restrict__ W2 = worker_theta(wb, w) + OFF_W2;
    for (int i = tid; i < 4 * FWD_TILES; i += FWD_NT) {
        const int e = i < FWD_G * P2_POS ? i : 0, img = e / P2_POS, pos = e % P2_POS;
        win_off[i] = img * P1_IMS + 2 * (pos / P2_W) * 16 + 2 * (pos % P2_W);
        out_off[i] = img * P2_SIZE + pos;
    }
    Pool1Stage<FWD_G, CHS, FWD_NT>::build_table(stage_tab, tid);

    // B operand of k-step s (channels 4*(s/9) .. +3, tap = s%9): lane (q, l16) holds W2[o][4*(s/9)+q][tap].
    // Taps innermost: the nine A reads of a channel group then share one LDS base address.
    float wreg[36][2];
#pragma unroll
    for (int s = 0; s < 36; ++s)
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) wreg[s][hf] = W2[((l16 + 16 * hf) * C1 + 4 * (s / 9) + q) * 9 + s % 9];
    const float bias0 = W2[C2 * C1 * 9 + l16], bias1 = W2[C2 * C1 * 9 + 16 + l16];

    for (int i = tid; i < FWD_G * P1_IMS / 4; i += FWD_NT)
        reinterpret_cast<float4*>(tile)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    // this lane's part of the A operand address: channel quarter, window element
    const float* a_lane = tile + q * CHS + ((l16 >> 1) & 1) * 16 + (l16 & 1);
    Pool1Stage<FWD_G, CHS, FWD_NT> stage;
    stage.init(tid);
    stage.prefetch(wb.p1, (size_t)w * B + s_begin, min(FWD_G, s_end - s_begin), tid);
    int rot = 0;
    for (int s0 = s_begin; s0 < s_end; s0 += FWD_G, ++rot) {
        const size_t g0 = (size_t)w * B + s0;
        const int valid = min(FWD_G, s_end - s0);
        stage.commit(tile, stage_tab, tid);
        __syncthreads();
        if (s0 + FWD_G < s_end) stage.prefetch(wb.p1, g0 + FWD_G, min(FWD_G, s_end - s0 - FWD_G), tid);
        for (int t = (wave + rot) % FWD_NW; t < FWD_TILES; t += FWD_NW) {  // which wavefront takes the odd tile rotates
            // A operand: lane row l16 = (pooled position 4t + l16/4, window element l16%4)
            const float* a = a_lane + win_off[4 * t + (l16 >> 2)];
            floatx4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 36; ++s) {
                const float av = a[4 * (s / 9) * CHS + ((s % 9) / 3) * 16 + (s % 9) % 3];
                acc0 = mfma16(av, wreg[s][0], acc0);
                acc1 = mfma16(av, wreg[s][1], acc1);
            }
            // lane (q, l16) now holds the 2x2 window of pooled position 4t + q for channels l16, l16+16
            const int ppo = 4 * t + q;
            if (ppo < valid * P2_POS) {
                const size_t out = g0 * P2_SIZE + out_off[ppo];
                // the four values of a window share their channel's bias: it is added to the winner only
                int code;
                float best = pool_first_max(acc0[0], acc0[1], acc0[2], acc0[3], code) + bias0;
                wb.p2[out + l16 * P2_POS] = fmaxf(best, 0.f);
                wb.am2[out + l16 * P2_POS] = (uint8_t)(code | (best > 0.f ? 4 : 0));
                best = pool_first_max(acc1[0], acc1[1], acc1[2], acc1[3], code) + bias1;
                wb.p2[out + (l16 + 16) * P2_POS] = fmaxf(best, 0.f);
                wb.am2[out + (l16 + 16) * P2_POS] = (uint8_t)(code | (best > 0.f ? 4 : 0));
            }
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Input gradient of conv2 fused with the weight gradient of conv1.
//   d pool1[c][y][x] = sum_{o,dy,dx} d2pad[o][y+2-dy][x+2-dx] * W2[o][c][dy][dx], zeroed where pool1 == 0.
// GEMM rows are the 196 positions of an image (16 per tile), columns the 16 input channels,
// K = (flipped tap, output channel) = 288.  The result never goes to memory: conv1 has no input
// gradient, so each value is routed to its pool1 window's winner and multiplied right away with the
// 3x3 neighbourhood of input pixels there,
//   d W1[c][dy][dx] += d pool1[c][p] * xpad[winner(c,p) + (dy,dx)],   d b1[c] += d pool1[c][p],
// on the vector ALU, which is idle while the matrix cores run.  A block owns up to DX_IPB images of
// one worker and walks them DX_G at a time; each wavefront's conv1 sums go to its own partial slot.
// DX_G images per group (between two block barriers), DX_NW wavefronts per block
constexpr int DX_G = 1, DX_NW = 2, DX_NT = 64 * DX_NW, DX_IPB = 32;
// The conv1 sums leave the registers every DX_FLUSH images, one partial slot per (DX_FLUSH images, wavefront),
// whatever number of images a block owns (a multiple of DX_FLUSH): the order in which a worker's partial sums
// are formed and added up then never depends on how the launch was cut into blocks.
constexpr int DX_FLUSH = 8;

__global__ __launch_bounds__(DX_NT, 512 / DX_NT) void conv2_dx_kernel(WorkerBuffers wb, int blocks_per_worker, int ipb)
{
    constexpr int CHS = CHS_DX, D2_IMS = C2 * CHS;
    __shared__ __attribute__((aligned(16))) float tile[DX_G * D2_IMS];  // 69,632 B
    __shared__ __attribute__((aligned(16))) float xs[DX_G * 900];       // zero-padded 30x30 input images
    // position of the group -> offset in the d2 planes; pooled position -> offset of its 2x2 window in
    // the padded input image (looked up rather than computed: see the forward kernel)
    __shared__ int a_off[DX_G * P1_POS];
    __shared__ __attribute__((aligned(16))) int x_off[P1_POS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane >> 4, l16 = lane & 15;
    const int w = blockIdx.x / blocks_per_worker, chunk = blockIdx.x % blocks_per_worker;
    const int B = wb.B, s_begin = chunk * ipb, s_end = min(B, s_begin + ipb);
    const float* __restrict__ W2 = worker_theta(wb, w) + OFF_W2;

    // K = (output channel o, flipped tap t') = 288, four per MFMA step, one per lane quarter q.  A step's four
    // are chosen so that its LDS reads need no address arithmetic and few bank conflicts: the 32 lanes an LDS
    // read serves per cycle are two quarters, and two quarters that read the same plane in the same row (taps
    // next to each other) touch 17 neighbouring addresses, which is conflict-free, whereas two different planes
    // or two different rows always collide somewhere (16 positions of 14-wide rows in 16-wide planes span up
    // to 20 banks).  Per output channel o:
    //   step X_o: taps (0,0) (0,1) | (1,0) (1,1)     both halves conflict-free
    //   step Y_o: taps (2,0) (2,1) | (0,2) (1,2)     first half conflict-free
    // and per four channels one step Z with tap (2,2) of channels 4g .. 4g+3.  Every read is then
    // lane base + o * plane pitch, an immediate offset, from one of three lane bases per tile.
    // B operand: lane (q, l16) holds W2[o][c = l16][8 - t'] for its quarter's tap t'.
    const int tx = q == 0 ? 0 : q == 1 ? 1 : q == 2 ? 3 : 4;   // flipped taps of step X
    const int ty = q == 0 ? 6 : q == 1 ? 7 : q == 2 ? 2 : 5;   // and of step Y
    float wx[32], wy[32], wz[8];
#pragma unroll
    for (int o = 0; o < 32; ++o) {
        wx[o] = W2[(o * C1 + l16) * 9 + 8 - tx];
        wy[o] = W2[(o * C1 + l16) * 9 + 8 - ty];
    }
#pragma unroll
    for (int g = 0; g < 8; ++g) wz[g] = W2[((4 * g + q) * C1 + l16) * 9];

    for (int i = tid; i < DX_G * D2_IMS / 4; i += DX_NT)
        reinterpret_cast<float4*>(tile)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = tid; i < DX_G * 900; i += DX_NT) xs[i] = 0.f;
    for (int i = tid; i < DX_G * P1_POS; i += DX_NT) {
        const int img = i / P1_POS, pos = i % P1_POS;
        a_off[i] = img * D2_IMS + (pos / P1_W) * 16 + pos % P1_W;
        if (img == 0) x_off[pos] = 2 * (pos / P1_W) * 30 + 2 * (pos % P1_W);
    }
    __syncthreads();

    // input pixels of a group: DX_G * 196 float4
    constexpr int NX4 = DX_G * (IMG_PIX / 4), NXV = (NX4 + DX_NT - 1) / DX_NT;
    float4 xv[NXV];
    auto prefetch_x = [&](size_t g0, int valid) {
#pragma unroll
        for (int k = 0; k < NXV; ++k) {
            const int i4 = tid + DX_NT * k;
            xv[k] = (i4 < NX4 && i4 / (IMG_PIX / 4) < valid)
                        ? *reinterpret_cast<const float4*>(wb.x + g0 * IMG_PIX + (size_t)i4 * 4)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto commit_x = [&]() {
#pragma unroll
        for (int k = 0; k < NXV; ++k) {
            const int i4 = tid + DX_NT * k;
            if (i4 >= NX4) break;
            const int img = i4 / (IMG_PIX / 4), r = (i4 % (IMG_PIX / 4)) * 4;  // 28 % 4 == 0: one image row
            float* dst = xs + img * 900 + (r / IMG_W + 1) * 30 + r % IMG_W + 1;
            dst[0] = xv[k].x; dst[1] = xv[k].y; dst[2] = xv[k].z; dst[3] = xv[k].w;
        }
    };

    float g1[9], gb1 = 0.f;  // this lane's share of d W1[l16][.] and d b1[l16]
#pragma unroll
    for (int i = 0; i < 9; ++i) g1[i] = 0.f;

    // lane parts of the three A-operand bases: tap offset (row * 16 + column) of the lane's quarter
    const float* ax_lane = tile + (tx / 3) * 16 + tx % 3;
    const float* ay_lane = tile + (ty / 3) * 16 + ty % 3;
    const float* az_lane = tile + q * CHS + 2 * 16 + 2;
    D2Stage<DX_G, CHS, DX_NT> stage;
    stage.init(tid);
    stage.prefetch(wb, (size_t)w * B + s_begin, min(DX_G, s_end - s_begin), tid);
    prefetch_x((size_t)w * B + s_begin, min(DX_G, s_end - s_begin));
    for (int s0 = s_begin; s0 < s_end; s0 += DX_G) {
        const size_t g0 = (size_t)w * B + s0;
        const int valid = min(DX_G, s_end - s0);
        const int rot = s0 / DX_G;  // which wavefront takes the odd tile depends on the images, not on the block
        stage.commit(tile, tid);
        commit_x();
        __syncthreads();
        if (s0 + DX_G < s_end) {
            stage.prefetch(wb, g0 + DX_G, min(DX_G, s_end - s0 - DX_G), tid);
            prefetch_x(g0 + DX_G, min(DX_G, s_end - s0 - DX_G));
        }
        // Lane (q, l16) of tile t will hold channel l16 at positions 16t + 4q .. +3 (never straddling an image).
        // Their pool1 window bytes (winner's offset in the padded input image, gate) are fetched one tile ahead;
        // a position beyond the images of the group gets zero bytes, whose gate is shut, so the tile needs no
        // branch.  The 36 input pixels of conv1's weight gradient are read in front of the matrix work and used
        // behind it; the first A-operand values of the next tile are read during the current one, so that the
        // matrix cores do not wait behind those 36 reads at the start of a tile (LDS reads return in order).
        static_assert(DX_G <= 2, "image of a position is found with one comparison");
        constexpr int N_TILES = (DX_G * P1_POS + 15) / 16, AHEAD = 4;  // A values of channels 0 .. AHEAD-1 read ahead
        const uint8_t* am1_lane = wb.am1 + g0 * P1_SIZE + l16 * P1_POS + 4 * q;
        auto window_bytes = [&](int t) -> uint32_t {
            const int mo = 16 * t + 4 * q;  // position in the group; the second image starts P1_SIZE bytes after the first
            return (t < N_TILES && mo < valid * P1_POS)
                       ? *reinterpret_cast<const uint32_t*>(am1_lane + 16 * t + (mo >= P1_POS ? P1_SIZE - P1_POS : 0))
                       : 0u;
        };
        auto a_base = [&](int t) -> int {
            const int m = 16 * t + l16;  // lane row l16 = position 16t + l16 of the group (rows beyond it read position 0)
            return a_off[m < DX_G * P1_POS ? m : 0];
        };
        const int t_first = (wave + rot) % DX_NW;
        uint32_t win_next = window_bytes(t_first);
        int at = a_base(t_first);
        float ax_next[AHEAD], ay_next[AHEAD];
#pragma unroll
        for (int o = 0; o < AHEAD; ++o) {
            ax_next[o] = ax_lane[at + o * CHS];
            ay_next[o] = ay_lane[at + o * CHS];
        }
        for (int t = t_first; t < N_TILES; t += DX_NW) {
            const uint32_t win = win_next;
            // the 3x3 input neighbourhoods at the four winners
            const int mo = min(16 * t + 4 * q, DX_G * P1_POS - 4), img_o = mo >= P1_POS ? 1 : 0, pos_o = mo - img_o * P1_POS;
            const float* ximg = xs + img_o * 900;
            const int4 xo = *reinterpret_cast<const int4*>(x_off + pos_o);  // pos_o is a multiple of 4
            const float* px[4] = {ximg + xo.x + (win & 0x7fu), ximg + xo.y + ((win >> 8) & 0x7fu),
                                  ximg + xo.z + ((win >> 16) & 0x7fu), ximg + xo.w + ((win >> 24) & 0x7fu)};
            float xr[36];
#pragma unroll
            for (int r = 0; r < 36; ++r) xr[r] = px[r / 9][((r % 9) / 3) * 30 + (r % 9) % 3];
            win_next = window_bytes(t + DX_NW);
            const float* ax = ax_lane + at;
            const float* ay = ay_lane + at;
            const float* az = az_lane + at;
            const int at_next = a_base(min(t + DX_NW, N_TILES - 1));
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int g = 0; g < 8; ++g) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int o = 4 * g + j;
                    acc = mfma16(o < AHEAD ? ax_next[o] : ax[o * CHS], wx[o], acc);
                    acc = mfma16(o < AHEAD ? ay_next[o] : ay[o * CHS], wy[o], acc);
                }
                acc = mfma16(az[4 * g * CHS], wz[g], acc);
                if (g == 6) {  // the next tile's first reads: their operands above are consumed by now
#pragma unroll
                    for (int o = 0; o < AHEAD; ++o) {
                        ax_next[o] = ax_lane[at_next + o * CHS];
                        ay_next[o] = ay_lane[at_next + o * CHS];
                    }
                }
            }
            at = at_next;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // gate bit -> all ones or zero
                const uint32_t keep = (uint32_t)((int32_t)(win << (24 - 8 * i)) >> 31);
                const float v = __uint_as_float(__float_as_uint(acc[i]) & keep);
                gb1 += v;
#pragma unroll
                for (int k = 0; k < 9; ++k) g1[k] = fmaf(v, xr[9 * i + k], g1[k]);
            }
        }
        __syncthreads();
        stage.clear(tile, tid);
        if ((s0 + DX_G) % DX_FLUSH == 0 || s0 + DX_G >= s_end) {
            // fold the four lane quarters; lanes of quarter 0 hold the wavefront's sums for channel l16
#pragma unroll
            for (int i = 0; i < 9; ++i) {
                g1[i] += __shfl_xor(g1[i], 16, 64);
                g1[i] += __shfl_xor(g1[i], 32, 64);
            }
            gb1 += __shfl_xor(gb1, 16, 64);
            gb1 += __shfl_xor(gb1, 32, 64);
            if (q == 0) {
                float* part = wb.part1 + ((size_t)w * (DX_NW * ((B + DX_FLUSH - 1) / DX_FLUSH)) + (s0 / DX_FLUSH) * DX_NW + wave) * OFF_W2;
#pragma unroll
                for (int i = 0; i < 9; ++i) part[OFF_W1 + l16 * 9 + i] = g1[i];
                part[OFF_B1 + l16] = gb1;
            }
#pragma unroll
            for (int i = 0; i < 9; ++i) g1[i] = 0.f;
            gb1 = 0.f;
        }
        __syncthreads();  // the planes are cleared by all threads, the next commit scatters into them
    }
}

// ---------------------------------------------------------------------------------------------
// Weight gradient: d W2[o][c][dy][dx] = sum over the worker's images and positions of
// d2[o][y][x] * pool1pad[c][y+dy][x+dx];  d b2[o] = sum d2[o].  GEMM rows are the 32 output channels
// (two tiles), columns (tap, input channel) (nine tiles), K = positions, four per MFMA step.  A block
// owns one chunk of a worker's images; its four wavefronts split every image's 49 k-steps and keep
// their 18 accumulator tiles across images; each wavefront's sum goes to its own partial slot.
__global__ __launch_bounds__(256, 2) void conv2_dw_kernel(WorkerBuffers wb)
{
    constexpr int CHS = CHS_DW, D2_IMS = C2 * CHS, P1_IMS = C1 * CHS;
    __shared__ __attribute__((aligned(16))) float d2[D2_IMS];   // 33,024 B
    __shared__ __attribute__((aligned(16))) float p1t[P1_IMS];  // 16,512 B
    // position -> offset inside a padded plane.  On this chip fp32 MFMAs and vector-ALU instructions do
    // not overlap, so index arithmetic inside the MFMA loops is paid for in matrix time: look it up.
    __shared__ int plane_off[P1_POS];
    __shared__ uint16_t stage_tab[Pool1Stage<1, CHS_DW>::N4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, q = lane >> 4, l16 = lane & 15;
    const int w = blockIdx.x, chunk = blockIdx.y, B = wb.B;
    const int per = (B + N_CHUNK - 1) / N_CHUNK;
    const int s_begin = chunk * per, s_end = min(B, s_begin + per);

    floatx4 acc[2][9];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < 9; ++j) acc[mt][j] = floatx4{0.f, 0.f, 0.f, 0.f};
    float sum0 = 0.f, sum1 = 0.f;

    for (int i = tid; i < D2_IMS / 4; i += 256) reinterpret_cast<float4*>(d2)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int i = tid; i < P1_IMS / 4; i += 256) reinterpret_cast<float4*>(p1t)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tid < P1_POS) plane_off[tid] = (tid / P1_W) * 16 + tid % P1_W;
    Pool1Stage<1, CHS>::build_table(stage_tab, tid);
    __syncthreads();
    const float* d2_lane = d2 + l16 * CHS + 17;
    const float* p1_lane = p1t + l16 * CHS;

    D2Stage<1, CHS> sd;
    sd.init(tid);
    Pool1Stage<1, CHS> sp;
    sp.init(tid);
    if (s_begin < s_end) {
        sd.prefetch(wb, (size_t)w * B + s_begin, 1, tid);
        sp.prefetch(wb.p1, (size_t)w * B + s_begin, 1, tid);
    }
    int rot = 0;
    for (int s = s_begin; s < s_end; ++s, ++rot) {
        const size_t g = (size_t)w * B + s;
        sd.commit(d2, tid);
        sp.commit(p1t, stage_tab, tid);
        __syncthreads();
        if (s + 1 < s_end) {
            sd.prefetch(wb, g + 1, 1, tid);
            sp.prefetch(wb.p1, g + 1, 1, tid);
        }
        for (int pos = 4 * ((wave + rot) & 3) + q; pos < P1_POS; pos += 16) {
            const int off = plane_off[pos];
            const float a0 = d2_lane[off], a1 = d2_lane[16 * CHS + off];
            sum0 += a0;
            sum1 += a1;
            const float* b = p1_lane + off;
#pragma unroll
            for (int j = 0; j < 9; ++j) {
                const float bv = b[(j / 3) * 16 + j % 3];
                acc[0][j] = mfma16(a0, bv, acc[0][j]);
                acc[1][j] = mfma16(a1, bv, acc[1][j]);
            }
        }
        __syncthreads();
        sd.clear(d2, tid);
        __syncthreads();  // cleared by all threads before the next commit scatters into the planes
    }

    // accumulator i of tile (mt, j): output channel 16*mt + 4q + i, input channel l16, tap j
    float* part = wb.part + ((size_t)w * N_PART + chunk * 4 + wave) * CONV_PART;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int j = 0; j < 9; ++j)
#pragma unroll
            for (int i = 0; i < 4; ++i) part[OFF_W2 + ((16 * mt + 4 * q + i) * C1 + l16) * 9 + j] = acc[mt][j][i];
    sum0 += __shfl_xor(sum0, 16, 64);
    sum0 += __shfl_xor(sum0, 32, 64);
    sum1 += __shfl_xor(sum1, 16, 64);
    sum1 += __shfl_xor(sum1, 32, 64);
    if (q == 0) {
        part[OFF_B2 + l16] = sum0;
        part[OFF_B2 + 16 + l16] = sum1;
    }
}

}  // namespace

// Images per block: as many as FWD_IPB / DX_IPB when the launch still gives every compute unit as many blocks
// as fit it, else fewer (16, 8), so that a small launch does not leave part of the chip idle.
static int images_per_block(int n, int batch, int most, int blocks_per_cu)
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
            cus = 256;
    }
    int ipb = most;
    while (ipb > DX_FLUSH && n * ((batch + ipb - 1) / ipb) < blocks_per_cu * cus) ipb /= 2;
    return ipb;
}

void launch_conv2_fwd(const WorkerBuffers& wb, hipStream_t s)
{
    const int ipb = images_per_block(wb.n, wb.B, FWD_IPB, 512 / FWD_NT), bpw = (wb.B + ipb - 1) / ipb;
    hipLaunchKernelGGL(conv2_fwd_kernel, dim3(wb.n * bpw), dim3(FWD_NT), 0, s, wb, bpw, ipb);
}

int conv1_part_slots(int batch) { return DX_NW * ((batch + DX_FLUSH - 1) / DX_FLUSH); }

void launch_conv2_dx(const WorkerBuffers& wb, hipStream_t s)
{
    const int ipb = images_per_block(wb.n, wb.B, DX_IPB, 512 / DX_NT), bpw = (wb.B + ipb - 1) / ipb;
    hipLaunchKernelGGL(conv2_dx_kernel, dim3(wb.n * bpw), dim3(DX_NT), 0, s, wb, bpw, ipb);
}

void launch_conv2_dw(const WorkerBuffers& wb, hipStream_t s)
{
    hipLaunchKernelGGL(conv2_dw_kernel, dim3(wb.n, N_CHUNK), dim3(256), 0, s, wb);
}

}  // namespace ps
