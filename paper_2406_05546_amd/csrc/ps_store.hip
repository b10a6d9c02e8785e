// Lock-free gradient store on the device (Section 3.3, last paragraph: gradient accesses can be
// lock-free because each gradient is written once by its worker and read, then deleted, by the
// server; the Future Work section asks for a better locking mechanism).  Workers and the server run
// on two HIP streams and meet only through this state:
//   append   a batch of workers writes its rows, then claims consecutive positions with one atomic add
//            on `tail` and stamps each row with position + 1 (release).  The rows are the ones the
//            host predicted from the appends it has enqueued (one worker stream: enqueue order is
//            position order), so nothing on the device waits for the claim; a claim that does not
//            land on the predicted rows raises `fault` and stamps nothing;
//   consume  the server takes the longest prefix of stamped rows starting at `head` (acquire), applies
//            it, and deletes it by advancing `head` (release).
// A row is reused by position + capacity, whose stamp differs, so stamps are never cleared.  The host
// keeps claimed - consumed <= capacity, so a claimed row is never one the server has yet to read.
#include "ps_common.h"

namespace ps {

namespace {

typedef unsigned long long u64;

__global__ void store_reset_kernel(StoreState* st, u64 version) { st->version = version; }

__global__ __launch_bounds__(256) void store_publish_kernel(StoreBuffers sb, const WorkerMeta* meta, int n)
{
    __shared__ u64 base;
    // everything the worker kernels wrote to the rows precedes this launch in stream order
    if (threadIdx.x == 0) base = atomicAdd(&sb.state->tail, (u64)n);
    __syncthreads();
    for (int i = threadIdx.x; i < n; i += 256) {
        const u64 pos = base + (u64)i;
        const WorkerMeta m = meta[i];
        if ((int)(pos % (u64)sb.cap) != m.q) {
            sb.state->fault = 1;  // same value from every lane that sees it
            continue;
        }
        StoreEntryMeta e;
        e.pos = pos;
        e.version = sb.ring_version[m.slot];
        e.mb = ((u64)m.mb_hi << 32) | m.mb_lo;
        e.worker = sb.worker_id[i];
        e.pad = 0;
        sb.entry[m.q] = e;
        // the release makes row and metadata visible to whoever reads the stamp with acquire
        __hip_atomic_store(&sb.stamp[m.q], pos + 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// One wavefront: 64 stamps are tested per pass; the run of ready rows from lane 0 is taken.
__global__ __launch_bounds__(64) void store_take_kernel(StoreBuffers sb, int max_entries)
{
    const int lane = threadIdx.x;
    const u64 head = __hip_atomic_load(&sb.state->head, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    int count = 0;
    while (count < max_entries) {  // ends: every pass either adds 64 or leaves
        const u64 pos = head + (u64)(count + lane);
        const int q = (int)(pos % (u64)sb.cap);
        bool ready = false;
        if (count + lane < max_entries)
            ready = __hip_atomic_load(&sb.stamp[q], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) == pos + 1;
        const u64 mask = __ballot(ready);
        const int run = (mask == ~0ull) ? 64 : __builtin_ctzll(~mask);
        if (lane < run) sb.idx[count + lane] = q;
        count += run;
        if (run < 64) break;
    }
    if (lane == 0) {
        sb.range->first = head;
        sb.range->count = (uint32_t)count;
        sb.range->pad = 0;
    }
}

__global__ void store_release_kernel(StoreBuffers sb, int mode)
{
    const uint32_t k = sb.range->count;
    if (k == 0) return;
    StoreState* st = sb.state;
    const u64 v = st->version + (mode == 0 ? 1ull : (u64)k);
    st->version = v;
    StoreLogRec r;
    r.first = sb.range->first;
    r.count = k;
    r.mode = (uint32_t)mode;
    r.version_after = v;
    sb.log[st->log_n % STORE_LOG_CAP] = r;
    st->log_n += 1;
    __hip_atomic_store(&st->head, r.first + k, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void store_stamp_version_kernel(StoreBuffers sb, int slot) { sb.ring_version[slot] = sb.state->version; }

}  // namespace

hipError_t launch_store_reset(const StoreBuffers& sb, unsigned long long version, hipStream_t s)
{
    hipLaunchKernelGGL(store_reset_kernel, dim3(1), dim3(1), 0, s, sb.state, version);
    return hipGetLastError();
}

hipError_t launch_store_publish(const StoreBuffers& sb, const WorkerMeta* meta, int n, hipStream_t s)
{
    hipLaunchKernelGGL(store_publish_kernel, dim3(1), dim3(256), 0, s, sb, meta, n);
    return hipGetLastError();
}

hipError_t launch_store_take(const StoreBuffers& sb, int max_entries, hipStream_t s)
{
    hipLaunchKernelGGL(store_take_kernel, dim3(1), dim3(64), 0, s, sb, max_entries);
    return hipGetLastError();
}

hipError_t launch_store_release(const StoreBuffers& sb, int mode, hipStream_t s)
{
    hipLaunchKernelGGL(store_release_kernel, dim3(1), dim3(1), 0, s, sb, mode);
    return hipGetLastError();
}

hipError_t launch_store_stamp_version(const StoreBuffers& sb, int slot, hipStream_t s)
{
    hipLaunchKernelGGL(store_stamp_version_kernel, dim3(1), dim3(1), 0, s, sb, slot);
    return hipGetLastError();
}

}  // namespace ps
