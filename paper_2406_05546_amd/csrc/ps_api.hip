// C ABI of the parameter-server hot path (see include/ps_hotpath.h for the contract) and the host
// side of the pending-gradient queue: which entries are free, which are pending and in what
// arrival order, and which snapshot version each gradient was computed on (Section 3.3: gradients
// are written once by a worker, read once by the server and deleted after they are applied).
#include "../../include/ps_hotpath.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ps_common.h"

using namespace ps;

static_assert(PS_PARAM_COUNT == P, "header and kernels disagree on the parameter count");

namespace {

constexpr int N_STAGE = 4;  // pinned host staging buffers for per-call index / metadata uploads
constexpr int N_HEADRB = 8;  // read-backs of the store's consumed count in flight

struct Entry {
    bool pending = false;
    uint64_t seq = 0, version = 0, mb = 0;
    int32_t worker = 0;
};

struct Stage {
    void* host = nullptr;
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

struct HeadReadback {
    hipEvent_t done = nullptr;
    bool in_flight = false;
};

struct Carve {
    uint64_t off = 0;
    uint64_t take(uint64_t bytes)
    {
        const uint64_t at = off;
        off += (bytes + 255) & ~uint64_t(255);
        return at;
    }
};

struct Layout {
    uint64_t theta, ring, queue, ada_g2, ada_dx2, meta, idx, slotq, st_state, st_stamp, st_entry, st_ringver, st_log, st_range, st_idx, st_wid, p1, am1, p2, am2, ht, z, pred, d3, dp2g, part, part1, fpart, normpart, scale, eval_loss, eval_ok, keep, total;
};

bool config_ok(const ps_config* c)
{
    return c && c->max_workers >= 1 && c->batch >= 1 && c->n_versions >= 1 && c->queue_capacity >= 1 &&
           c->dropout_p >= 0.f && c->dropout_p < 1.f && (int64_t)c->max_workers * c->batch <= (int64_t)1 << 24;
}

Layout make_layout(const ps_config& c)
{
    const uint64_t n = (uint64_t)c.max_workers * c.batch, row = (uint64_t)PSTRIDE * sizeof(float);
    Carve k;
    Layout l;
    l.theta = k.take(row);
    l.ring = k.take(row * c.n_versions);
    l.queue = k.take(row * c.queue_capacity);
    l.ada_g2 = k.take(row);
    l.ada_dx2 = k.take(row);
    l.meta = k.take(sizeof(WorkerMeta) * c.max_workers);
    l.idx = k.take(sizeof(int32_t) * c.queue_capacity);
    l.slotq = k.take(2 * sizeof(int32_t) * c.n_versions);
    l.st_state = k.take(sizeof(StoreState));
    l.st_stamp = k.take(sizeof(unsigned long long) * c.queue_capacity);
    l.st_entry = k.take(sizeof(StoreEntryMeta) * c.queue_capacity);
    l.st_ringver = k.take(sizeof(unsigned long long) * c.n_versions);
    l.st_log = k.take(sizeof(StoreLogRec) * STORE_LOG_CAP);
    l.st_range = k.take(sizeof(StoreRange));
    l.st_idx = k.take(sizeof(int32_t) * c.queue_capacity);
    l.st_wid = k.take(sizeof(int32_t) * c.max_workers);
    l.p1 = k.take(n * P1_SIZE * 4);
    l.am1 = k.take(n * P1_SIZE);
    l.p2 = k.take(n * P2_SIZE * 4);
    l.am2 = k.take(n * P2_SIZE);
    l.ht = k.take(n * FC1 * 4);
    l.z = k.take(n * NCLS * 4);
    l.pred = k.take(n * 4);
    l.d3 = k.take(n * FC1 * 4);
    l.dp2g = k.take(n * P2_SIZE * 4);
    l.part = k.take((uint64_t)c.max_workers * N_PART * CONV_PART * 4);
    l.part1 = k.take((uint64_t)c.max_workers * conv1_part_slots(c.batch) * OFF_W2 * 4);
    l.fpart = k.take((uint64_t)(512 + c.max_workers) * FC2_PART * 4);  // >= n * fc2_split(n) slots
    l.normpart = k.take((uint64_t)c.queue_capacity * norm_slices() * 4);
    l.scale = k.take((uint64_t)c.queue_capacity * 4);
    l.eval_loss = k.take(n * 4);
    l.eval_ok = k.take(n * 4);
    l.keep = k.take((uint64_t)c.batch * FC1);
    l.total = k.off;
    return l;
}

}  // namespace

struct ps_ctx {
    ps_config cfg{};
    hipStream_t stream = nullptr;
    char* ws = nullptr;
    Layout lay{};
    std::vector<Entry> entries;
    std::vector<int32_t> free_list;  // stack; lowest index on top
    std::vector<int32_t> pending;    // queue indices in arrival order
    std::vector<uint64_t> ring_version;
    std::vector<WorkerMeta> last_meta;
    uint64_t version = 0, next_seq = 0;
    Stage stage[N_STAGE];
    int next_stage = 0;
    size_t stage_bytes = 0;
    Profiler prof;
    std::string err;

    // Lock-free store: the server stream, and what the host knows of the device-side counters.
    hipStream_t server = nullptr;
    hipEvent_t ev_join = nullptr, ev_workers = nullptr;
    std::vector<hipEvent_t> ev_slot_read, ev_slot_written;  // last worker read of / server write to a ring slot
    std::vector<char> slot_read_valid, slot_written_valid;
    uint64_t store_claimed = 0, store_confirmed = 0;  // exact; lower bound of the consumed count
    bool store_synced = false;   // device-side version counters hold the host's values
    bool server_dirty = false;   // the server stream was given work the worker stream has not waited for
    unsigned long long* headrb_host = nullptr;  // pinned, [N_HEADRB]
    HeadReadback headrb[N_HEADRB];
    int next_headrb = 0;

    template <class T>
    T* at(uint64_t off) const { return reinterpret_cast<T*>(ws + off); }
    float* theta() const { return at<float>(lay.theta); }
    float* ring(int slot) const { return at<float>(lay.ring) + (size_t)slot * PSTRIDE; }
    float* queue(int q) const { return at<float>(lay.queue) + (size_t)q * PSTRIDE; }
};

namespace {

ps_status fail(ps_ctx* c, ps_status st, const std::string& msg)
{
    if (c) c->err = msg;
    return st;
}

#define PS_HIP(ctx, call)                                                                           \
    do {                                                                                            \
        hipError_t e_ = (call);                                                                     \
        if (e_ != hipSuccess)                                                                       \
            return fail(ctx, PS_EDEVICE, std::string(#call) + ": " + hipGetErrorString(e_));        \
    } while (0)

// Copies `bytes` of host data to `dst_dev` through a pinned staging buffer, asynchronously.
ps_status upload(ps_ctx* c, void* dst_dev, const void* src, size_t bytes)
{
    if (bytes == 0) return PS_OK;
    Stage& s = c->stage[c->next_stage];
    c->next_stage = (c->next_stage + 1) % N_STAGE;
    if (s.in_flight) PS_HIP(c, hipEventSynchronize(s.done));
    std::memcpy(s.host, src, bytes);
    PS_HIP(c, hipMemcpyAsync(dst_dev, s.host, bytes, hipMemcpyHostToDevice, c->stream));
    PS_HIP(c, hipEventRecord(s.done, c->stream));
    s.in_flight = true;
    return PS_OK;
}

ps_status apply_entries(ps_ctx* c, const std::vector<int32_t>& idx, float lr, int mode)
{
    ps_status st = upload(c, c->at<int32_t>(c->lay.idx), idx.data(), idx.size() * sizeof(int32_t));
    if (st != PS_OK) return st;
    PS_HIP(c, launch_apply(c->theta(), c->at<float>(c->lay.queue), c->at<int32_t>(c->lay.idx), (int)idx.size(), lr,
                           mode, c->stream, c->prof));
    return PS_OK;
}

void release_entries(ps_ctx* c, const std::vector<int32_t>& idx)
{
    for (int32_t q : idx) c->entries[q].pending = false;
    std::vector<int32_t> keep;
    keep.reserve(c->pending.size());
    for (int32_t q : c->pending)
        if (c->entries[q].pending) keep.push_back(q);
    c->pending.swap(keep);
    // Freed entries go back so that the lowest index is handed out first.
    for (int32_t q : idx) c->free_list.push_back(q);
    std::sort(c->free_list.begin(), c->free_list.end(), [](int32_t a, int32_t b) { return a > b; });
}

int32_t take_entry(ps_ctx* c, int32_t worker, uint64_t version, uint64_t mb)
{
    const int32_t q = c->free_list.back();
    c->free_list.pop_back();
    Entry& e = c->entries[q];
    e.pending = true;
    e.seq = c->next_seq++;
    e.worker = worker;
    e.version = version;
    e.mb = mb;
    c->pending.push_back(q);
    return q;
}

WorkerBuffers buffers(const ps_ctx* c, int n, const float* x, const int32_t* y, float* loss)
{
    WorkerBuffers wb{};
    wb.ring = c->at<float>(c->lay.ring);
    wb.queue = c->at<float>(c->lay.queue);
    wb.meta = c->at<WorkerMeta>(c->lay.meta);
    wb.x = x;
    wb.y = y;
    wb.p1 = c->at<float>(c->lay.p1);
    wb.am1 = c->at<uint8_t>(c->lay.am1);
    wb.p2 = c->at<float>(c->lay.p2);
    wb.am2 = c->at<uint8_t>(c->lay.am2);
    wb.ht = c->at<float>(c->lay.ht);
    wb.z = c->at<float>(c->lay.z);
    wb.pred = c->at<int32_t>(c->lay.pred);
    wb.d3 = c->at<float>(c->lay.d3);
    wb.dp2g = c->at<float>(c->lay.dp2g);
    wb.part = c->at<float>(c->lay.part);
    wb.part1 = c->at<float>(c->lay.part1);
    wb.fpart = c->at<float>(c->lay.fpart);
    wb.loss = loss;
    wb.n = n;
    wb.B = c->cfg.batch;
    wb.seed_lo = (uint32_t)c->cfg.seed;
    wb.seed_hi = (uint32_t)(c->cfg.seed >> 32);
    wb.drop_threshold = (uint32_t)std::floor((double)c->cfg.dropout_p * 4294967296.0);
    wb.drop_scale = (float)(1.0 / (1.0 - (double)c->cfg.dropout_p));
    return wb;
}

StoreBuffers store_buffers(const ps_ctx* c)
{
    StoreBuffers sb{};
    sb.state = c->at<StoreState>(c->lay.st_state);
    sb.stamp = c->at<unsigned long long>(c->lay.st_stamp);
    sb.entry = c->at<StoreEntryMeta>(c->lay.st_entry);
    sb.ring_version = c->at<unsigned long long>(c->lay.st_ringver);
    sb.log = c->at<StoreLogRec>(c->lay.st_log);
    sb.range = c->at<StoreRange>(c->lay.st_range);
    sb.idx = c->at<int32_t>(c->lay.st_idx);
    sb.worker_id = c->at<int32_t>(c->lay.st_wid);
    sb.cap = c->cfg.queue_capacity;
    return sb;
}

// Whatever the server stream has been given so far precedes what the worker stream is given next.
ps_status workers_wait_server(ps_ctx* c)
{
    if (!c->server_dirty) return PS_OK;
    PS_HIP(c, hipEventRecord(c->ev_join, c->server));
    PS_HIP(c, hipStreamWaitEvent(c->stream, c->ev_join, 0));
    c->server_dirty = false;
    return PS_OK;
}

ps_status server_waits_workers(ps_ctx* c)
{
    PS_HIP(c, hipEventRecord(c->ev_workers, c->stream));
    PS_HIP(c, hipStreamWaitEvent(c->server, c->ev_workers, 0));
    return PS_OK;
}

// Folds finished read-backs of the consumed count into the host's lower bound; never blocks.
void poll_consumed(ps_ctx* c)
{
    for (int i = 0; i < N_HEADRB; ++i) {
        HeadReadback& r = c->headrb[i];
        if (r.in_flight && hipEventQuery(r.done) == hipSuccess) {
            c->store_confirmed = std::max<uint64_t>(c->store_confirmed, c->headrb_host[i]);
            r.in_flight = false;
        }
    }
}

bool store_open(ps_ctx* c)
{
    if (c->store_claimed != c->store_confirmed) poll_consumed(c);
    return c->store_claimed != c->store_confirmed;
}

// Entry check of the calls that work on the ordered queue or the server's weights from the worker
// stream: not while the store holds gradients; ordered after the server stream's work.
ps_status store_read(ps_ctx* c, StoreState* state, std::vector<unsigned long long>* stamps);

ps_status ordered_guard(ps_ctx* c, const char* who)
{
    if (store_open(c))
        return fail(c, PS_ESTATE, std::string(who) + ": the lock-free store holds gradients not yet seen consumed "
                                                     "(consume them, then ps_store_state)");
    if (c->store_synced) {
        // The device holds the authoritative version counters while the store is in use: take them
        // back (update count, snapshot versions) before the host's copies are used again.
        StoreState s{};
        const ps_status st = store_read(c, &s, nullptr);
        if (st != PS_OK) return st;
        if (s.head != s.tail) return fail(c, PS_ESTATE, std::string(who) + ": the lock-free store still holds gradients");
        c->store_synced = false;
    }
    return workers_wait_server(c);
}

// First store call after ordered calls: hand the version counters to the device.
ps_status store_begin(ps_ctx* c, const char* who)
{
    if (c->store_synced) return PS_OK;
    if (!c->pending.empty()) return fail(c, PS_ESTATE, std::string(who) + ": the ordered queue is not empty");
    ps_status st = workers_wait_server(c);
    if (st != PS_OK) return st;
    const StoreBuffers sb = store_buffers(c);
    PS_HIP(c, launch_store_reset(sb, c->version, c->stream));
    st = upload(c, sb.ring_version, c->ring_version.data(), sizeof(uint64_t) * c->ring_version.size());
    if (st != PS_OK) return st;
    st = server_waits_workers(c);
    if (st != PS_OK) return st;
    c->store_synced = true;
    return PS_OK;
}

}  // namespace

extern "C" {

ps_status ps_workspace_bytes(const ps_config* cfg, uint64_t* bytes_out)
{
    if (!bytes_out || !config_ok(cfg)) return PS_EINVAL;
    *bytes_out = make_layout(*cfg).total;
    return PS_OK;
}

ps_status ps_init(ps_ctx** out, const ps_config* cfg, void* workspace_dev, uint64_t workspace_bytes, void* hip_stream)
{
    if (!out) return PS_EINVAL;
    *out = nullptr;
    if (!config_ok(cfg) || !workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255)) return PS_EINVAL;
    const Layout lay = make_layout(*cfg);
    if (workspace_bytes < lay.total) return PS_ENOMEM;
    ps_ctx* c = new (std::nothrow) ps_ctx;
    if (!c) return PS_ENOMEM;
    c->cfg = *cfg;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->ws = static_cast<char*>(workspace_dev);
    c->lay = lay;
    c->entries.assign(cfg->queue_capacity, Entry{});
    for (int32_t q = cfg->queue_capacity - 1; q >= 0; --q) c->free_list.push_back(q);
    c->ring_version.assign(cfg->n_versions, 0);
    c->stage_bytes = std::max({sizeof(WorkerMeta) * (size_t)cfg->max_workers, sizeof(int32_t) * (size_t)cfg->queue_capacity,
                               sizeof(uint64_t) * (size_t)cfg->n_versions});
    c->ev_slot_read.assign(cfg->n_versions, nullptr);
    c->ev_slot_written.assign(cfg->n_versions, nullptr);
    c->slot_read_valid.assign(cfg->n_versions, 0);
    c->slot_written_valid.assign(cfg->n_versions, 0);
    hipError_t e = hipStreamCreateWithFlags(&c->server, hipStreamNonBlocking);  // default priority
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_workers, hipEventDisableTiming);
    for (int i = 0; i < cfg->n_versions && e == hipSuccess; ++i) {
        e = hipEventCreateWithFlags(&c->ev_slot_read[i], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_slot_written[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipHostMalloc((void**)&c->headrb_host, sizeof(unsigned long long) * N_HEADRB, hipHostMallocDefault);
    for (int i = 0; i < N_HEADRB && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&c->headrb[i].done, hipEventDisableTiming);
    for (int i = 0; i < N_STAGE && e == hipSuccess; ++i) {
        e = hipHostMalloc(&c->stage[i].host, c->stage_bytes, hipHostMallocDefault);
        if (e == hipSuccess) e = hipEventCreateWithFlags(&c->stage[i].done, hipEventDisableTiming);
    }
    // the drain entry point that allocates nothing finds its scratch array resolved on this device
    if (e == hipSuccess) {
        unsigned char* unused = nullptr;
        e = static_scratch(&unused);
    }
    // Weights, ring, queue (padding included) and the index arrays start at zero.
    if (e == hipSuccess) e = hipMemsetAsync(c->ws, 0, lay.p1, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) {
        std::fprintf(stderr, "ps_init: %s\n", hipGetErrorString(e));
        ps_destroy(c);
        return PS_EDEVICE;
    }
    *out = c;
    return PS_OK;
}

ps_status ps_destroy(ps_ctx* c)
{
    if (!c) return PS_EINVAL;
    (void)hipStreamSynchronize(c->stream);
    if (c->server) (void)hipStreamSynchronize(c->server);
    c->prof.destroy();
    for (Stage& s : c->stage) {
        if (s.done) (void)hipEventDestroy(s.done);
        if (s.host) (void)hipHostFree(s.host);
    }
    for (HeadReadback& r : c->headrb)
        if (r.done) (void)hipEventDestroy(r.done);
    if (c->headrb_host) (void)hipHostFree(c->headrb_host);
    for (hipEvent_t ev : c->ev_slot_read)
        if (ev) (void)hipEventDestroy(ev);
    for (hipEvent_t ev : c->ev_slot_written)
        if (ev) (void)hipEventDestroy(ev);
    if (c->ev_join) (void)hipEventDestroy(c->ev_join);
    if (c->ev_workers) (void)hipEventDestroy(c->ev_workers);
    if (c->server) (void)hipStreamDestroy(c->server);
    delete c;
    return PS_OK;
}

ps_status ps_sync(ps_ctx* c)
{
    if (!c) return PS_EINVAL;
    PS_HIP(c, hipStreamSynchronize(c->stream));
    PS_HIP(c, hipStreamSynchronize(c->server));
    c->server_dirty = false;
    return PS_OK;
}

ps_status ps_set_weights(ps_ctx* c, const float* theta_host)
{
    if (!c || !theta_host) return fail(c, PS_EINVAL, "ps_set_weights: null argument");
    if (!c->pending.empty()) return fail(c, PS_ESTATE, "ps_set_weights: queue not empty");
    { const ps_status g_ = ordered_guard(c, "ps_set_weights"); if (g_ != PS_OK) return g_; }
    PS_HIP(c, hipMemcpyAsync(c->theta(), theta_host, sizeof(float) * P, hipMemcpyHostToDevice, c->stream));
    for (int s = 0; s < c->cfg.n_versions; ++s) {
        PS_HIP(c, hipMemcpyAsync(c->ring(s), c->theta(), sizeof(float) * PSTRIDE, hipMemcpyDeviceToDevice, c->stream));
        c->ring_version[s] = 0;
    }
    PS_HIP(c, hipMemsetAsync(c->at<float>(c->lay.ada_g2), 0, 2 * sizeof(float) * PSTRIDE, c->stream));  // both accumulators
    PS_HIP(c, hipStreamSynchronize(c->stream));
    c->version = 0;
    return PS_OK;
}

ps_status ps_get_weights(ps_ctx* c, int32_t slot, float* theta_host)
{
    if (!c || !theta_host) return fail(c, PS_EINVAL, "ps_get_weights: null argument");
    if (slot < -1 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_get_weights: slot out of range");
    const float* src = slot < 0 ? c->theta() : c->ring(slot);
    PS_HIP(c, hipStreamSynchronize(c->server));
    PS_HIP(c, hipMemcpyAsync(theta_host, src, sizeof(float) * P, hipMemcpyDeviceToHost, c->stream));
    PS_HIP(c, hipStreamSynchronize(c->stream));
    return PS_OK;
}

ps_status ps_snapshot_weights(ps_ctx* c, int32_t slot, uint64_t* version_out)
{
    if (!c) return PS_EINVAL;
    if (slot < 0 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_snapshot_weights: slot out of range");
    { const ps_status g_ = ordered_guard(c, "ps_snapshot_weights"); if (g_ != PS_OK) return g_; }
    PS_HIP(c, hipMemcpyAsync(c->ring(slot), c->theta(), sizeof(float) * PSTRIDE, hipMemcpyDeviceToDevice, c->stream));
    c->ring_version[slot] = c->version;
    if (version_out) *version_out = c->version;
    return PS_OK;
}

ps_status worker_grads_batched(ps_ctx* c, int32_t n, const int32_t* worker_id_host, const int32_t* version_slot_host,
                               const uint64_t* minibatch_id_host, const float* x_dev, const int32_t* y_dev,
                               int32_t* queue_index_host, float* loss_dev)
{
    if (!c) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (n < 0 || n > c->cfg.max_workers) return fail(c, PS_EINVAL, "worker_grads_batched: n outside [0, max_workers]");
    if (!worker_id_host || !version_slot_host || !minibatch_id_host || !x_dev || !y_dev || !queue_index_host)
        return fail(c, PS_EINVAL, "worker_grads_batched: null argument");
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15) || (reinterpret_cast<uintptr_t>(y_dev) & 3))
        return fail(c, PS_EINVAL, "worker_grads_batched: x_dev must be 16-byte and y_dev 4-byte aligned");
    for (int i = 0; i < n; ++i)
        if (version_slot_host[i] < 0 || version_slot_host[i] >= c->cfg.n_versions)
            return fail(c, PS_EINVAL, "worker_grads_batched: version slot out of range");
    if ((size_t)n > c->free_list.size()) return fail(c, PS_EFULL, "worker_grads_batched: gradient queue full");
    { const ps_status g_ = ordered_guard(c, "worker_grads_batched"); if (g_ != PS_OK) return g_; }

    c->last_meta.resize(n);
    for (int i = 0; i < n; ++i) {
        const int32_t slot = version_slot_host[i];
        const uint64_t mb = minibatch_id_host[i];
        const int32_t q = take_entry(c, worker_id_host[i], c->ring_version[slot], mb);
        queue_index_host[i] = q;
        c->last_meta[i] = WorkerMeta{slot, q, (uint32_t)mb, (uint32_t)(mb >> 32)};
    }
    ps_status st = upload(c, c->at<WorkerMeta>(c->lay.meta), c->last_meta.data(), sizeof(WorkerMeta) * n);
    if (st != PS_OK) return st;
    const WorkerBuffers wb = buffers(c, n, x_dev, y_dev, loss_dev);
    PS_HIP(c, launch_worker_forward(wb, c->stream, c->prof));
    PS_HIP(c, launch_worker_backward(wb, c->stream, c->prof));
    return PS_OK;
}

ps_status ps_queue_push_host(ps_ctx* c, const float* grad_host, int32_t worker_id, uint64_t version,
                             uint64_t minibatch_id, int32_t* queue_index_host)
{
    if (!c || !grad_host || !queue_index_host) return fail(c, PS_EINVAL, "ps_queue_push_host: null argument");
    if (c->free_list.empty()) return fail(c, PS_EFULL, "ps_queue_push_host: gradient queue full");
    { const ps_status g_ = ordered_guard(c, "ps_queue_push_host"); if (g_ != PS_OK) return g_; }
    const int32_t q = take_entry(c, worker_id, version, minibatch_id);
    *queue_index_host = q;
    PS_HIP(c, hipMemcpyAsync(c->queue(q), grad_host, sizeof(float) * P, hipMemcpyHostToDevice, c->stream));
    PS_HIP(c, hipStreamSynchronize(c->stream));
    return PS_OK;
}

ps_status ps_apply_sync(ps_ctx* c, const int32_t* queue_index_host, int32_t n, float lr)
{
    if (!c) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (n < 0 || !queue_index_host) return fail(c, PS_EINVAL, "ps_apply_sync: bad arguments");
    { const ps_status g_ = ordered_guard(c, "ps_apply_sync"); if (g_ != PS_OK) return g_; }
    std::vector<int32_t> idx(queue_index_host, queue_index_host + n);
    std::vector<char> seen(c->cfg.queue_capacity, 0);
    for (int32_t q : idx) {
        if (q < 0 || q >= c->cfg.queue_capacity) return fail(c, PS_EINVAL, "ps_apply_sync: queue index out of range");
        if (!c->entries[q].pending || seen[q]) return fail(c, PS_ESTATE, "ps_apply_sync: entry not pending or listed twice");
        seen[q] = 1;
    }
    ps_status st = apply_entries(c, idx, lr, PS_DRAIN_SUM);
    if (st != PS_OK) return st;
    release_entries(c, idx);
    c->version += 1;
    return PS_OK;
}

ps_status ps_apply_async(ps_ctx* c, int32_t q, float lr)
{
    if (!c) return PS_EINVAL;
    if (q < 0 || q >= c->cfg.queue_capacity) return fail(c, PS_EINVAL, "ps_apply_async: queue index out of range");
    if (!c->entries[q].pending) return fail(c, PS_ESTATE, "ps_apply_async: entry not pending");
    { const ps_status g_ = ordered_guard(c, "ps_apply_async"); if (g_ != PS_OK) return g_; }
    const std::vector<int32_t> idx{q};
    ps_status st = apply_entries(c, idx, lr, PS_DRAIN_SEQ);
    if (st != PS_OK) return st;
    release_entries(c, idx);
    c->version += 1;
    return PS_OK;
}

ps_status ps_drain_buffered(ps_ctx* c, int32_t mode, float lr, int32_t* n_applied_host)
{
    if (!c) return PS_EINVAL;
    if (mode != PS_DRAIN_SUM && mode != PS_DRAIN_SEQ) return fail(c, PS_EINVAL, "ps_drain_buffered: unknown mode");
    { const ps_status g_ = ordered_guard(c, "ps_drain_buffered"); if (g_ != PS_OK) return g_; }
    const std::vector<int32_t> idx = c->pending;
    if (n_applied_host) *n_applied_host = (int32_t)idx.size();
    if (idx.empty()) return PS_OK;
    ps_status st = apply_entries(c, idx, lr, mode);
    if (st != PS_OK) return st;
    release_entries(c, idx);
    c->version += mode == PS_DRAIN_SUM ? 1 : idx.size();
    return PS_OK;
}

ps_status ps_drain_buffered_mitigated(ps_ctx* c, int32_t mode, const ps_drain_policy* pol, int32_t* n_applied_host,
                                      float* lr_used_host)
{
    if (!c) return PS_EINVAL;
    if (!pol || (mode != PS_DRAIN_SUM && mode != PS_DRAIN_SEQ) || !(pol->lr_backlog_ref >= 0.f) || !(pol->clip_norm >= 0.f))
        return fail(c, PS_EINVAL, "ps_drain_buffered_mitigated: bad mode or policy");
    { const ps_status g_ = ordered_guard(c, "ps_drain_buffered_mitigated"); if (g_ != PS_OK) return g_; }
    const std::vector<int32_t> idx = c->pending;
    const float K = (float)idx.size();
    const float lr = (pol->lr_backlog_ref > 0.f && K > pol->lr_backlog_ref) ? pol->lr * (pol->lr_backlog_ref / K) : pol->lr;
    if (n_applied_host) *n_applied_host = (int32_t)idx.size();
    if (lr_used_host) *lr_used_host = lr;
    if (idx.empty()) return PS_OK;
    if (pol->clip_norm > 0.f) {
        ps_status st = upload(c, c->at<int32_t>(c->lay.idx), idx.data(), idx.size() * sizeof(int32_t));
        if (st != PS_OK) return st;
        PS_HIP(c, launch_apply_clipped(c->theta(), c->at<float>(c->lay.queue), c->at<int32_t>(c->lay.idx), (int)idx.size(),
                                       lr, mode, pol->clip_norm, c->at<float>(c->lay.normpart), c->at<float>(c->lay.scale),
                                       c->stream, c->prof));
    } else {
        ps_status st = apply_entries(c, idx, lr, mode);
        if (st != PS_OK) return st;
    }
    release_entries(c, idx);
    c->version += mode == PS_DRAIN_SUM ? 1 : idx.size();
    return PS_OK;
}

ps_status worker_grads_append(ps_ctx* c, int32_t n, const int32_t* worker_id_host, const int32_t* version_slot_host,
                              const uint64_t* minibatch_id_host, const float* x_dev, const int32_t* y_dev, float* loss_dev)
{
    if (!c) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (n < 0 || n > c->cfg.max_workers) return fail(c, PS_EINVAL, "worker_grads_append: n outside [0, max_workers]");
    if (!worker_id_host || !version_slot_host || !minibatch_id_host || !x_dev || !y_dev)
        return fail(c, PS_EINVAL, "worker_grads_append: null argument");
    if ((reinterpret_cast<uintptr_t>(x_dev) & 15) || (reinterpret_cast<uintptr_t>(y_dev) & 3))
        return fail(c, PS_EINVAL, "worker_grads_append: x_dev must be 16-byte and y_dev 4-byte aligned");
    for (int i = 0; i < n; ++i)
        if (version_slot_host[i] < 0 || version_slot_host[i] >= c->cfg.n_versions)
            return fail(c, PS_EINVAL, "worker_grads_append: version slot out of range");
    ps_status st = store_begin(c, "worker_grads_append");
    if (st != PS_OK) return st;
    const uint64_t cap = (uint64_t)c->cfg.queue_capacity;
    poll_consumed(c);
    if (c->store_claimed + (uint64_t)n - c->store_confirmed > cap) {
        PS_HIP(c, hipStreamSynchronize(c->server));  // let enqueued server steps finish, then look again
        poll_consumed(c);
        if (c->store_claimed + (uint64_t)n - c->store_confirmed > cap)
            return fail(c, PS_EFULL, "worker_grads_append: gradient store full");
    }

    std::vector<int32_t> slots(version_slot_host, version_slot_host + n);
    std::sort(slots.begin(), slots.end());
    slots.erase(std::unique(slots.begin(), slots.end()), slots.end());
    for (int32_t s : slots)
        if (c->slot_written_valid[s]) PS_HIP(c, hipStreamWaitEvent(c->stream, c->ev_slot_written[s], 0));

    c->last_meta.resize(n);
    for (int i = 0; i < n; ++i) {
        const uint64_t mb = minibatch_id_host[i];
        const int32_t row = (int32_t)((c->store_claimed + (uint64_t)i) % cap);  // the position this append will claim
        c->last_meta[i] = WorkerMeta{version_slot_host[i], row, (uint32_t)mb, (uint32_t)(mb >> 32)};
    }
    const StoreBuffers sb = store_buffers(c);
    WorkerMeta* meta_dev = c->at<WorkerMeta>(c->lay.meta);
    st = upload(c, meta_dev, c->last_meta.data(), sizeof(WorkerMeta) * n);
    if (st != PS_OK) return st;
    st = upload(c, sb.worker_id, worker_id_host, sizeof(int32_t) * n);
    if (st != PS_OK) return st;
    c->store_claimed += (uint64_t)n;
    const WorkerBuffers wb = buffers(c, n, x_dev, y_dev, loss_dev);
    PS_HIP(c, launch_worker_forward(wb, c->stream, c->prof));
    PS_HIP(c, launch_worker_backward(wb, c->stream, c->prof));
    PS_HIP(c, launch_store_publish(sb, meta_dev, n, c->stream));
    for (int32_t s : slots) {
        PS_HIP(c, hipEventRecord(c->ev_slot_read[s], c->stream));
        c->slot_read_valid[s] = 1;
    }
    return PS_OK;
}

ps_status ps_store_consume(ps_ctx* c, int32_t mode, float lr, int32_t max_entries, int32_t wait_for_workers)
{
    if (!c) return PS_EINVAL;
    if ((mode != PS_DRAIN_SUM && mode != PS_DRAIN_SEQ) || max_entries < 0)
        return fail(c, PS_EINVAL, "ps_store_consume: unknown mode or negative limit");
    ps_status st = store_begin(c, "ps_store_consume");
    if (st != PS_OK) return st;
    const int cap = c->cfg.queue_capacity;
    const int limit = (max_entries == 0 || max_entries > cap) ? cap : max_entries;
    if (wait_for_workers) {
        st = server_waits_workers(c);
        if (st != PS_OK) return st;
    }
    const StoreBuffers sb = store_buffers(c);
    PS_HIP(c, launch_store_take(sb, limit, c->server));
    PS_HIP(c, launch_apply(c->theta(), c->at<float>(c->lay.queue), sb.idx, limit, lr, mode, c->server, c->prof, &sb.range->count));
    PS_HIP(c, launch_store_release(sb, mode, c->server));
    HeadReadback& r = c->headrb[c->next_headrb];
    unsigned long long* dst = c->headrb_host + c->next_headrb;
    c->next_headrb = (c->next_headrb + 1) % N_HEADRB;
    if (r.in_flight) {
        PS_HIP(c, hipEventSynchronize(r.done));
        c->store_confirmed = std::max<uint64_t>(c->store_confirmed, *dst);
        r.in_flight = false;
    }
    PS_HIP(c, hipMemcpyAsync(dst, &sb.state->head, sizeof(unsigned long long), hipMemcpyDeviceToHost, c->server));
    PS_HIP(c, hipEventRecord(r.done, c->server));
    r.in_flight = true;
    c->server_dirty = true;
    return PS_OK;
}

ps_status ps_store_publish(ps_ctx* c, int32_t slot)
{
    if (!c) return PS_EINVAL;
    if (slot < 0 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_store_publish: slot out of range");
    ps_status st = store_begin(c, "ps_store_publish");
    if (st != PS_OK) return st;
    if (c->slot_read_valid[slot]) PS_HIP(c, hipStreamWaitEvent(c->server, c->ev_slot_read[slot], 0));
    PS_HIP(c, hipMemcpyAsync(c->ring(slot), c->theta(), sizeof(float) * PSTRIDE, hipMemcpyDeviceToDevice, c->server));
    PS_HIP(c, launch_store_stamp_version(store_buffers(c), slot, c->server));
    PS_HIP(c, hipEventRecord(c->ev_slot_written[slot], c->server));
    c->slot_written_valid[slot] = 1;
    c->server_dirty = true;
    return PS_OK;
}

namespace {

// Both streams idle; device counters, stamps and snapshot versions on the host.
ps_status store_read(ps_ctx* c, StoreState* state, std::vector<unsigned long long>* stamps)
{
    PS_HIP(c, hipStreamSynchronize(c->stream));
    PS_HIP(c, hipStreamSynchronize(c->server));
    c->server_dirty = false;
    const StoreBuffers sb = store_buffers(c);
    PS_HIP(c, hipMemcpy(state, sb.state, sizeof(StoreState), hipMemcpyDeviceToHost));
    if (stamps) {
        stamps->resize(sb.cap);
        PS_HIP(c, hipMemcpy(stamps->data(), sb.stamp, sizeof(unsigned long long) * sb.cap, hipMemcpyDeviceToHost));
    }
    if (state->fault) return fail(c, PS_EDEVICE, "lock-free store: an append claimed positions other than the rows it had written");
    for (HeadReadback& r : c->headrb) r.in_flight = false;  // all finished; superseded by the value just read
    if (c->store_synced) {  // the device holds the authoritative counters
        c->store_confirmed = state->head;
        c->version = state->version;
        std::vector<unsigned long long> rv(c->cfg.n_versions);
        PS_HIP(c, hipMemcpy(rv.data(), sb.ring_version, sizeof(unsigned long long) * rv.size(), hipMemcpyDeviceToHost));
        for (size_t i = 0; i < rv.size(); ++i) c->ring_version[i] = rv[i];
    }
    return PS_OK;
}

uint64_t published_prefix(const ps_ctx* c, const StoreState& s, const std::vector<unsigned long long>& stamps)
{
    uint64_t p = s.head;
    while (p < s.tail && stamps[p % (uint64_t)c->cfg.queue_capacity] == p + 1) ++p;
    return p;
}

}  // namespace

ps_status ps_store_state(ps_ctx* c, ps_store_counters* out)
{
    if (!c || !out) return fail(c, PS_EINVAL, "ps_store_state: null argument");
    StoreState s{};
    std::vector<unsigned long long> stamps;
    ps_status st = store_read(c, &s, &stamps);
    if (st != PS_OK) return st;
    out->claimed = s.tail;
    out->published = published_prefix(c, s, stamps);
    out->consumed = s.head;
    out->version = c->store_synced ? s.version : c->version;
    out->steps = s.log_n;
    return PS_OK;
}

ps_status ps_store_steps(ps_ctx* c, int32_t capacity, int32_t* n_host, ps_store_step* steps_host)
{
    if (!c || !n_host || capacity < 0 || (capacity > 0 && !steps_host)) return fail(c, PS_EINVAL, "ps_store_steps: bad arguments");
    StoreState s{};
    ps_status st = store_read(c, &s, nullptr);
    if (st != PS_OK) return st;
    const uint64_t m = std::min<uint64_t>({s.log_n, (uint64_t)STORE_LOG_CAP, (uint64_t)capacity});
    std::vector<StoreLogRec> log(STORE_LOG_CAP);
    PS_HIP(c, hipMemcpy(log.data(), store_buffers(c).log, sizeof(StoreLogRec) * STORE_LOG_CAP, hipMemcpyDeviceToHost));
    for (uint64_t i = 0; i < m; ++i) {
        const StoreLogRec& r = log[(s.log_n - m + i) % STORE_LOG_CAP];
        steps_host[i] = ps_store_step{r.first, r.count, r.mode, r.version_after};
    }
    *n_host = (int32_t)m;
    return PS_OK;
}

ps_status ps_store_entry(ps_ctx* c, uint64_t position, float* grad_host, int32_t* worker_host, uint64_t* version_host,
                         uint64_t* minibatch_host)
{
    if (!c) return PS_EINVAL;
    StoreState s{};
    std::vector<unsigned long long> stamps;
    ps_status st = store_read(c, &s, &stamps);
    if (st != PS_OK) return st;
    if (position < s.head || position >= published_prefix(c, s, stamps))
        return fail(c, PS_ESTATE, "ps_store_entry: position already consumed or not yet published");
    const int q = (int)(position % (uint64_t)c->cfg.queue_capacity);
    StoreEntryMeta e{};
    PS_HIP(c, hipMemcpy(&e, store_buffers(c).entry + q, sizeof(e), hipMemcpyDeviceToHost));
    if (grad_host) PS_HIP(c, hipMemcpy(grad_host, c->queue(q), sizeof(float) * P, hipMemcpyDeviceToHost));
    if (worker_host) *worker_host = e.worker;
    if (version_host) *version_host = e.version;
    if (minibatch_host) *minibatch_host = e.mb;
    return PS_OK;
}

ps_status ps_apply_local(ps_ctx* c, int32_t n, const int32_t* slot_host, const int32_t* queue_index_host, float lr)
{
    if (!c) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (n < 0 || !slot_host || !queue_index_host) return fail(c, PS_EINVAL, "ps_apply_local: bad arguments");
    std::vector<char> slot_seen(c->cfg.n_versions, 0), q_seen(c->cfg.queue_capacity, 0);
    std::vector<int32_t> pairs(2 * (size_t)n), idx(n);
    for (int i = 0; i < n; ++i) {
        const int32_t s = slot_host[i], q = queue_index_host[i];
        if (s < 0 || s >= c->cfg.n_versions || slot_seen[s]) return fail(c, PS_EINVAL, "ps_apply_local: slot out of range or listed twice");
        if (q < 0 || q >= c->cfg.queue_capacity) return fail(c, PS_EINVAL, "ps_apply_local: queue index out of range");
        if (!c->entries[q].pending || q_seen[q]) return fail(c, PS_ESTATE, "ps_apply_local: entry not pending or listed twice");
        slot_seen[s] = q_seen[q] = 1;
        pairs[2 * i] = s;
        pairs[2 * i + 1] = q;
        idx[i] = q;
    }
    { const ps_status g_ = ordered_guard(c, "ps_apply_local"); if (g_ != PS_OK) return g_; }
    ps_status st = upload(c, c->at<int32_t>(c->lay.slotq), pairs.data(), pairs.size() * sizeof(int32_t));
    if (st != PS_OK) return st;
    PS_HIP(c, launch_local_steps(c->at<float>(c->lay.ring), c->at<float>(c->lay.queue), c->at<int32_t>(c->lay.slotq), n, lr,
                                 c->stream, c->prof));
    release_entries(c, idx);
    return PS_OK;
}

ps_status ps_elastic_average(ps_ctx* c, const int32_t* slot_host, int32_t n, float alpha)
{
    if (!c) return PS_EINVAL;
    if (n == 0) return PS_OK;
    if (n < 0 || !slot_host || !(alpha >= 0.f)) return fail(c, PS_EINVAL, "ps_elastic_average: bad arguments");
    std::vector<char> seen(c->cfg.n_versions, 0);
    for (int i = 0; i < n; ++i) {
        const int32_t s = slot_host[i];
        if (s < 0 || s >= c->cfg.n_versions || seen[s]) return fail(c, PS_EINVAL, "ps_elastic_average: slot out of range or listed twice");
        seen[s] = 1;
    }
    { const ps_status g_ = ordered_guard(c, "ps_elastic_average"); if (g_ != PS_OK) return g_; }
    ps_status st = upload(c, c->at<int32_t>(c->lay.slotq), slot_host, (size_t)n * sizeof(int32_t));
    if (st != PS_OK) return st;
    PS_HIP(c, launch_elastic_average(c->theta(), c->at<float>(c->lay.ring), c->at<int32_t>(c->lay.slotq), n, alpha, c->stream,
                                     c->prof));
    c->version += 1;
    return PS_OK;
}

ps_status ps_drain_buffered_adadelta(ps_ctx* c, float lr, float rho, float eps, int32_t* n_applied_host)
{
    if (!c) return PS_EINVAL;
    if (!(rho >= 0.f && rho < 1.f) || !(eps > 0.f)) return fail(c, PS_EINVAL, "ps_drain_buffered_adadelta: rho must be in [0, 1), eps > 0");
    { const ps_status g_ = ordered_guard(c, "ps_drain_buffered_adadelta"); if (g_ != PS_OK) return g_; }
    const std::vector<int32_t> idx = c->pending;
    if (n_applied_host) *n_applied_host = (int32_t)idx.size();
    if (idx.empty()) return PS_OK;
    ps_status st = upload(c, c->at<int32_t>(c->lay.idx), idx.data(), idx.size() * sizeof(int32_t));
    if (st != PS_OK) return st;
    PS_HIP(c, launch_apply_adadelta(c->theta(), c->at<float>(c->lay.ada_g2), c->at<float>(c->lay.ada_dx2),
                                    c->at<float>(c->lay.queue), c->at<int32_t>(c->lay.idx), (int)idx.size(), lr, rho, eps,
                                    c->stream, c->prof));
    release_entries(c, idx);
    c->version += idx.size();
    return PS_OK;
}

ps_status ps_get_grad(ps_ctx* c, int32_t q, float* grad_host)
{
    if (!c || !grad_host) return fail(c, PS_EINVAL, "ps_get_grad: null argument");
    if (q < 0 || q >= c->cfg.queue_capacity) return fail(c, PS_EINVAL, "ps_get_grad: queue index out of range");
    if (!c->entries[q].pending) return fail(c, PS_ESTATE, "ps_get_grad: entry not pending");
    PS_HIP(c, hipMemcpyAsync(grad_host, c->queue(q), sizeof(float) * P, hipMemcpyDeviceToHost, c->stream));
    PS_HIP(c, hipStreamSynchronize(c->stream));
    return PS_OK;
}

ps_status ps_queue_meta(ps_ctx* c, int32_t capacity, int32_t* n_host, uint64_t* seq_host, int32_t* worker_host,
                        uint64_t* version_host, uint64_t* minibatch_host, int32_t* queue_index_host)
{
    if (!c || !n_host || capacity < 0) return fail(c, PS_EINVAL, "ps_queue_meta: bad arguments");
    *n_host = (int32_t)c->pending.size();
    const int m = std::min<int>(capacity, (int)c->pending.size());
    for (int i = 0; i < m; ++i) {
        const int32_t q = c->pending[i];
        const Entry& e = c->entries[q];
        if (seq_host) seq_host[i] = e.seq;
        if (worker_host) worker_host[i] = e.worker;
        if (version_host) version_host[i] = e.version;
        if (minibatch_host) minibatch_host[i] = e.mb;
        if (queue_index_host) queue_index_host[i] = q;
    }
    return PS_OK;
}

ps_status ps_restore_weights(ps_ctx* c, int32_t slot, int32_t* n_dropped_host)
{
    if (!c) return PS_EINVAL;
    if (slot < 0 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_restore_weights: slot out of range");
    { const ps_status g_ = ordered_guard(c, "ps_restore_weights"); if (g_ != PS_OK) return g_; }
    PS_HIP(c, hipMemcpyAsync(c->theta(), c->ring(slot), sizeof(float) * PSTRIDE, hipMemcpyDeviceToDevice, c->stream));
    if (n_dropped_host) *n_dropped_host = (int32_t)c->pending.size();
    const std::vector<int32_t> idx = c->pending;
    release_entries(c, idx);
    c->version = c->ring_version[slot];
    return PS_OK;
}

ps_status ps_load_snapshot(ps_ctx* c, int32_t slot, const float* theta_host, uint64_t version)
{
    if (!c || !theta_host) return fail(c, PS_EINVAL, "ps_load_snapshot: null argument");
    if (slot < 0 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_load_snapshot: slot out of range");
    { const ps_status g_ = ordered_guard(c, "ps_load_snapshot"); if (g_ != PS_OK) return g_; }
    // the row's padding beyond P stays zero: it was zero after ps_init and every copy into it carries zeros there
    PS_HIP(c, hipMemcpyAsync(c->ring(slot), theta_host, sizeof(float) * P, hipMemcpyHostToDevice, c->stream));
    PS_HIP(c, hipStreamSynchronize(c->stream));
    c->ring_version[slot] = version;
    return PS_OK;
}

ps_status ps_evaluate(ps_ctx* c, int32_t slot, int32_t n_images, const float* x_dev, const int32_t* y_dev,
                      double* loss_host, double* accuracy_host, int32_t* pred_host)
{
    if (!c) return PS_EINVAL;
    const int B = c->cfg.batch;
    if (slot < -1 || slot >= c->cfg.n_versions) return fail(c, PS_EINVAL, "ps_evaluate: slot out of range");
    if (n_images <= 0 || n_images % B != 0 || n_images / B > c->cfg.max_workers)
        return fail(c, PS_EINVAL, "ps_evaluate: n_images must be a positive multiple of batch, at most max_workers * batch");
    if (!x_dev || !y_dev || (reinterpret_cast<uintptr_t>(x_dev) & 15) || (reinterpret_cast<uintptr_t>(y_dev) & 3))
        return fail(c, PS_EINVAL, "ps_evaluate: null or misaligned input");
    const int n = n_images / B;
    PS_HIP(c, hipStreamSynchronize(c->server));
    std::vector<WorkerMeta> meta(n, WorkerMeta{slot, 0, 0, 0});
    c->last_meta.clear();  // the activations of the last worker call are overwritten
    ps_status st = upload(c, c->at<WorkerMeta>(c->lay.meta), meta.data(), sizeof(WorkerMeta) * n);
    if (st != PS_OK) return st;
    WorkerBuffers wb = buffers(c, n, x_dev, y_dev, nullptr);
    wb.drop_threshold = 0;  // inference: nothing is dropped, nothing is rescaled
    wb.drop_scale = 1.f;
    launch_conv1_fwd(wb, c->stream);
    launch_conv2_fwd(wb, c->stream);
    launch_fc1_fwd(wb, c->stream);
    launch_fc2_eval(wb, c->at<float>(c->lay.eval_loss), c->at<int32_t>(c->lay.eval_ok), c->stream);
    PS_HIP(c, hipGetLastError());
    std::vector<float> loss(n_images);
    std::vector<int32_t> ok(n_images);
    PS_HIP(c, hipMemcpyAsync(loss.data(), c->at<float>(c->lay.eval_loss), sizeof(float) * n_images, hipMemcpyDeviceToHost, c->stream));
    PS_HIP(c, hipMemcpyAsync(ok.data(), c->at<int32_t>(c->lay.eval_ok), sizeof(int32_t) * n_images, hipMemcpyDeviceToHost, c->stream));
    if (pred_host) PS_HIP(c, hipMemcpyAsync(pred_host, c->at<int32_t>(c->lay.pred), sizeof(int32_t) * n_images, hipMemcpyDeviceToHost, c->stream));
    PS_HIP(c, hipStreamSynchronize(c->stream));
    double ls = 0.0;
    int64_t hits = 0;
    for (int i = 0; i < n_images; ++i) {
        ls += loss[i];
        hits += ok[i];
    }
    if (loss_host) *loss_host = ls / n_images;
    if (accuracy_host) *accuracy_host = (double)hits / n_images;
    return PS_OK;
}

ps_status ps_version(ps_ctx* c, uint64_t* version_host)
{
    if (!c || !version_host) return PS_EINVAL;
    if (c->store_synced) {  // the count lives on the device while the store is in use
        StoreState s{};
        const ps_status st = store_read(c, &s, nullptr);
        if (st != PS_OK) return st;
    }
    *version_host = c->version;
    return PS_OK;
}

ps_status ps_debug_last_batch(ps_ctx* c, int32_t i, uint8_t* pool1_host, uint8_t* pool2_host, uint8_t* keep_host,
                              float* hdrop_host, float* z_host, int32_t* pred_host)
{
    if (!c) return PS_EINVAL;
    if (i < 0 || i >= (int32_t)c->last_meta.size()) return fail(c, PS_EINVAL, "ps_debug_last_batch: no such worker in the last call");
    const size_t B = c->cfg.batch, g0 = (size_t)i * B;
    hipStream_t s = c->stream;
    if (pool1_host) PS_HIP(c, hipMemcpyAsync(pool1_host, c->at<uint8_t>(c->lay.am1) + g0 * P1_SIZE, B * P1_SIZE, hipMemcpyDeviceToHost, s));
    if (pool2_host) PS_HIP(c, hipMemcpyAsync(pool2_host, c->at<uint8_t>(c->lay.am2) + g0 * P2_SIZE, B * P2_SIZE, hipMemcpyDeviceToHost, s));
    if (hdrop_host) PS_HIP(c, hipMemcpyAsync(hdrop_host, c->at<float>(c->lay.ht) + g0 * FC1, B * FC1 * 4, hipMemcpyDeviceToHost, s));
    if (z_host) PS_HIP(c, hipMemcpyAsync(z_host, c->at<float>(c->lay.z) + g0 * NCLS, B * NCLS * 4, hipMemcpyDeviceToHost, s));
    if (pred_host) PS_HIP(c, hipMemcpyAsync(pred_host, c->at<int32_t>(c->lay.pred) + g0, B * 4, hipMemcpyDeviceToHost, s));
    if (keep_host) {
        const WorkerMeta& m = c->last_meta[i];
        const WorkerBuffers wb = buffers(c, 0, nullptr, nullptr, nullptr);
        PS_HIP(c, launch_keep_mask(c->at<uint8_t>(c->lay.keep), (int)B, m.mb_lo, m.mb_hi, wb.seed_lo, wb.seed_hi,
                                   wb.drop_threshold, s));
        PS_HIP(c, hipMemcpyAsync(keep_host, c->at<uint8_t>(c->lay.keep), B * FC1, hipMemcpyDeviceToHost, s));
    }
    PS_HIP(c, hipStreamSynchronize(s));
    if (pool1_host) {
        // pool1 window bytes are kept as (winner's offset in a 30-wide image, gate in bit 7); the caller gets
        // the documented form: bits 0-1 winner dy*2+dx, bit 2 gate
        for (size_t i = 0; i < B * P1_SIZE; ++i) {
            const uint8_t b = pool1_host[i], off = b & 0x7f;
            pool1_host[i] = (uint8_t)((off & 1) | (off >= 30 ? 2 : 0) | ((b & AM1_GATE) ? 4 : 0));
        }
    }
    return PS_OK;
}

ps_status ps_debug_last_activations(ps_ctx* c, int32_t i, float* pool1_val_host, float* pool2_val_host, float* d3_host,
                                    float* dpool2_host)
{
    if (!c) return PS_EINVAL;
    if (i < 0 || i >= (int32_t)c->last_meta.size())
        return fail(c, PS_EINVAL, "ps_debug_last_activations: no such worker in the last call");
    const size_t B = c->cfg.batch, g0 = (size_t)i * B;
    hipStream_t s = c->stream;
    if (pool1_val_host) PS_HIP(c, hipMemcpyAsync(pool1_val_host, c->at<float>(c->lay.p1) + g0 * P1_SIZE, B * P1_SIZE * 4, hipMemcpyDeviceToHost, s));
    if (pool2_val_host) PS_HIP(c, hipMemcpyAsync(pool2_val_host, c->at<float>(c->lay.p2) + g0 * P2_SIZE, B * P2_SIZE * 4, hipMemcpyDeviceToHost, s));
    if (d3_host) PS_HIP(c, hipMemcpyAsync(d3_host, c->at<float>(c->lay.d3) + g0 * FC1, B * FC1 * 4, hipMemcpyDeviceToHost, s));
    if (dpool2_host) PS_HIP(c, hipMemcpyAsync(dpool2_host, c->at<float>(c->lay.dp2g) + g0 * P2_SIZE, B * P2_SIZE * 4, hipMemcpyDeviceToHost, s));
    PS_HIP(c, hipStreamSynchronize(s));
    return PS_OK;
}

ps_status ps_profile_enable(ps_ctx* c, int32_t enable)
{
    if (!c) return PS_EINVAL;
    PS_HIP(c, hipStreamSynchronize(c->server));
    PS_HIP(c, c->prof.collect(c->stream));
    c->prof.reset();
    c->prof.enabled = enable != 0;
    return PS_OK;
}

ps_status ps_profile_read(ps_ctx* c, int32_t kernel_id, double* total_ms_host, int64_t* launches_host)
{
    if (!c || kernel_id < 0 || kernel_id >= K_COUNT) return fail(c, PS_EINVAL, "ps_profile_read: no such kernel");
    PS_HIP(c, hipStreamSynchronize(c->server));
    PS_HIP(c, c->prof.collect(c->stream));
    if (total_ms_host) *total_ms_host = c->prof.total_ms[kernel_id];
    if (launches_host) *launches_host = c->prof.launches[kernel_id];
    return PS_OK;
}

int32_t ps_profile_kernel_count(void) { return K_COUNT; }

const char* ps_profile_kernel_name(int32_t kernel_id) { return kernel_name(kernel_id); }

const char* ps_last_error(const ps_ctx* c) { return c ? c->err.c_str() : static_last_error(); }

}  // extern "C"
