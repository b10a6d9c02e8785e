// Shared declarations of the HIP implementation: network sizes (paper's model endnote), the flat
// parameter layout, per-worker call metadata and the launchers the C ABI drives.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <algorithm>
#include <vector>

namespace ps {

constexpr int IMG_W = 28, IMG_PIX = 784;
constexpr int C1 = 16, C2 = 32;
constexpr int P1_W = 14, P1_POS = 196, P1_SIZE = C1 * P1_POS;  // 3136
constexpr int P2_W = 7, P2_POS = 49, P2_SIZE = C2 * P2_POS;    // 1568
constexpr int FC1 = 512, NCLS = 10;

constexpr int OFF_W1 = 0, OFF_B1 = 144, OFF_W2 = 160, OFF_B2 = 4768, OFF_W3 = 4800, OFF_B3 = 807616,
              OFF_W4 = 808128, OFF_B4 = 813248, P = 813258;
// Row pitch of every P-vector in HBM (weights, ring slots, queue entries): P rounded up to 256 B.
constexpr int PSTRIDE = 813312;
constexpr int CONV_PART = OFF_W3;  // conv1 + conv2 gradient floats (4800), reduced from chunk partials
constexpr int N_CHUNK = 8;         // image chunks per worker in the conv weight-gradient reductions
constexpr int N_PART = 4 * N_CHUNK;  // partial slots per worker: one per (chunk, wavefront) of conv2's kernel

constexpr int AM1_GATE = 0x80;  // pool1 window byte: winner's pre-activation > 0

// One worker of a batched call.
struct WorkerMeta {
    int32_t slot;    // ring slot of the snapshot it reads
    int32_t q;       // queue entry its gradient goes to
    uint32_t mb_lo;  // logical minibatch id (dropout counter words 0, 1)
    uint32_t mb_hi;
};

// Device buffers of one batched worker step; activations are indexed by global image g = w*B + s.
struct WorkerBuffers {
    const float* ring;   // [V][PSTRIDE]
    float* queue;        // [cap][PSTRIDE]
    const WorkerMeta* meta;  // [n]
    const float* x;      // [n*B][784]
    const int32_t* y;    // [n*B]
    float* p1;           // [n*B][16][196]  conv1 -> ReLU -> pool
    uint8_t* am1;        // [n*B][16][196]  bits 0-6 the window winner's offset dy*30 + dx in a 30-wide padded input
                         //                 image (0, 1, 30, 31), bit 7 winner > 0: what conv1's weight gradient needs
    float* p2;           // [n*B][32][49]
    uint8_t* am2;        // [n*B][32][49]
    float* ht;           // [n*B][512]      fc1 -> ReLU -> dropout
    float* z;            // [n*B][10]       logits
    int32_t* pred;       // [n*B]
    float* d3;           // [n*B][512]      d loss / d fc1 pre-activation
    float* dp2g;         // [n*B][1568]     d loss / d pool2, zero where pool2 == 0
    float* part;         // [n][N_PART][4800] partial sums of the conv2 weight gradient (conv1 region unused)
    float* part1;        // [n][conv1_part_slots(B)][160] partial sums of the conv1 weight gradient
    float* fpart;        // [n][split][FC2_PART] partial sums of the fc2 kernel's blocks
    float* loss;         // [n] or nullptr
    int32_t n, B;
    uint32_t seed_lo, seed_hi;
    uint32_t drop_threshold;  // drop iff word < threshold
    float drop_scale;         // 1/(1-p)
};

#if defined(__HIPCC__)
__device__ __forceinline__ const float* worker_theta(const WorkerBuffers& wb, int w)
{
    // slot -1 is the server's current weights, which sit one row before the ring
    return wb.ring + (ptrdiff_t)wb.meta[w].slot * PSTRIDE;
}
__device__ __forceinline__ float* worker_grad(const WorkerBuffers& wb, int w)
{
    return wb.queue + (size_t)wb.meta[w].q * PSTRIDE;
}

// First maximum of a 2x2 window scanned (0,0),(0,1),(1,0),(1,1); returns the winner, sets code.
__device__ __forceinline__ float pool_first_max(float v0, float v1, float v2, float v3, int& code)
{
    float best = v0;
    code = 0;
    if (v1 > best) { best = v1; code = 1; }
    if (v2 > best) { best = v2; code = 2; }
    if (v3 > best) { best = v3; code = 3; }
    return best;
}
#endif

// One partial slot of the fc2 kernel: d W4 [10][512], d b4 [10], d b3 [512], summed loss.
constexpr int FC2_PART_B4 = NCLS * FC1, FC2_PART_B3 = FC2_PART_B4 + NCLS, FC2_PART_LOSS = FC2_PART_B3 + FC1,
              FC2_PART = 5648;
int fc2_split(int n);  // blocks per worker of the fc2 kernel (one partial slot each)
int conv1_part_slots(int batch);  // conv1 partial slots per worker (one per wavefront of conv2's input-gradient kernel)

void launch_conv1_fwd(const WorkerBuffers& wb, hipStream_t s);
void launch_fc1_fwd(const WorkerBuffers& wb, hipStream_t s);
void launch_fc1_dw(const WorkerBuffers& wb, hipStream_t s);
void launch_fc1_dx(const WorkerBuffers& wb, hipStream_t s);
void launch_fc2(const WorkerBuffers& wb, hipStream_t s);
void launch_fc2_eval(const WorkerBuffers& wb, float* loss_i, int32_t* correct, hipStream_t s);
void launch_conv2_fwd(const WorkerBuffers& wb, hipStream_t s);
void launch_conv2_dx(const WorkerBuffers& wb, hipStream_t s);
void launch_conv2_dw(const WorkerBuffers& wb, hipStream_t s);

// Kernels of the path, in launch order; ids index the per-kernel timing table.
enum KernelId {
    K_CONV1_FWD, K_CONV2_FWD, K_FC1_FWD, K_FC2, K_FC1_DW, K_FC1_DX, K_CONV2_DW, K_CONV2_DX,
    K_GRAD_REDUCE, K_APPLY_SUM, K_APPLY_SEQ, K_GRAD_SQNORM, K_APPLY_SUM_CLIP, K_APPLY_SEQ_CLIP, K_APPLY_ADADELTA, K_LOCAL_STEP,
    K_ELASTIC, K_COUNT
};
const char* kernel_name(int id);

// Optional per-kernel timing with HIP events recorded on the stream the kernels run on.
class Profiler {
public:
    bool enabled = false;
    void begin(int id, hipStream_t s);
    void end(hipStream_t s);
    hipError_t collect(hipStream_t s);  // waits for the stream, folds finished pairs into the totals
    void reset();
    void destroy();
    double total_ms[K_COUNT] = {};
    int64_t launches[K_COUNT] = {};

private:
    struct Rec { int id; hipEvent_t a, b; };
    hipEvent_t take();
    std::vector<Rec> recs_;
    std::vector<hipEvent_t> pool_;
    Rec open_{-1, nullptr, nullptr};
};

hipError_t launch_worker_forward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof);
hipError_t launch_worker_backward(const WorkerBuffers& wb, hipStream_t s, Profiler& prof);
hipError_t launch_keep_mask(uint8_t* keep_dev, int B, uint32_t mb_lo, uint32_t mb_hi, uint32_t seed_lo,
                            uint32_t seed_hi, uint32_t threshold, hipStream_t s);

// theta -= lr * (sum of the K listed queue rows) [mode 0] or K successive updates [mode 1].
// With K_dev the number of rows is read from device memory by the kernel (at most K_max).
hipError_t launch_apply(float* theta, const float* queue, const int32_t* idx_dev, int K, float lr, int mode,
                        hipStream_t s, Profiler& prof, const uint32_t* K_dev = nullptr);

// Same with every gradient first scaled by min(1, clip / ||g||_2): a norm pass, then the apply pass.
hipError_t launch_apply_clipped(float* theta, const float* queue, const int32_t* idx_dev, int K, float lr, int mode,
                                float clip, float* partial_dev, float* scale_dev, hipStream_t s, Profiler& prof);
int norm_slices();

// Device address, on the current GPU, of the library's fixed scratch array (used by the drain entry point
// that allocates nothing); resolved on first use per device.
hipError_t static_scratch(unsigned char** out);
const char* static_last_error();

// ring[slot_j] -= lr * queue[q_j] for n (slot, q) pairs with distinct slots (pairs_dev: 2n int32).
hipError_t launch_local_steps(float* ring, const float* queue, const int32_t* pairs_dev, int n, float lr, hipStream_t s,
                              Profiler& prof);
// One elastic-averaging step between theta and the n listed (distinct) ring slots.
hipError_t launch_elastic_average(float* theta, float* ring, const int32_t* slots_dev, int n, float alpha, hipStream_t s,
                                  Profiler& prof);

// K Adadelta steps, one per listed queue row in order; acc_g2 and acc_dx2 are P-vector rows of state.
hipError_t launch_apply_adadelta(float* theta, float* acc_g2, float* acc_dx2, const float* queue, const int32_t* idx_dev,
                                 int K, float lr, float rho, float eps, hipStream_t s, Profiler& prof);

// Lock-free gradient store (Section 3.3, last paragraph: a gradient is written once by its worker,
// read once and then deleted by the server, so the store needs no lock).  Positions count appended
// gradients from 0 and never wrap; position p lives in queue row p % capacity.
struct StoreState {
    unsigned long long tail;     // positions claimed by workers
    unsigned long long head;     // positions consumed (applied and deleted) by the server
    unsigned long long version;  // weight updates applied
    unsigned long long log_n;    // consumer steps recorded
    unsigned long long fault;    // set if an append did not land on the rows the host predicted
};
struct StoreEntryMeta {
    unsigned long long pos, version, mb;  // position, version of the snapshot used, minibatch id
    int32_t worker, pad;
};
struct StoreLogRec {  // one consumer step that applied at least one gradient
    unsigned long long first;
    uint32_t count, mode;
    unsigned long long version_after;
};
struct StoreRange {  // what the consumer step in flight has taken
    unsigned long long first;
    uint32_t count, pad;
};
constexpr int STORE_LOG_CAP = 1024;

struct StoreBuffers {
    StoreState* state;
    unsigned long long* stamp;         // [cap] position + 1 once the row is completely written
    StoreEntryMeta* entry;             // [cap]
    unsigned long long* ring_version;  // [V]
    StoreLogRec* log;                  // [STORE_LOG_CAP], a ring
    StoreRange* range;
    int32_t* idx;                      // [cap] rows taken by the consumer step in flight
    int32_t* worker_id;                // [max_workers] of the append in flight
    int cap;
};

hipError_t launch_store_reset(const StoreBuffers& sb, unsigned long long version, hipStream_t s);
hipError_t launch_store_publish(const StoreBuffers& sb, const WorkerMeta* meta, int n, hipStream_t s);
hipError_t launch_store_take(const StoreBuffers& sb, int max_entries, hipStream_t s);
hipError_t launch_store_release(const StoreBuffers& sb, int mode, hipStream_t s);
hipError_t launch_store_stamp_version(const StoreBuffers& sb, int slot, hipStream_t s);

}  // namespace ps
