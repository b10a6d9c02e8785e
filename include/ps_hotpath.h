/*
 * ps_hotpath.h -- C ABI of the parameter-server hot path of "Training Through
 * Failure: Effects of Data Consistency in Parallel Machine Learning Training"
 * (arxiv 2406.05546) for one AMD MI355X (gfx950).
 *
 * W simulated workers are a batch dimension on one GPU.  Each worker runs the
 * forward/backward pass of the paper's CNN (model endnote: conv 16, ReLU, max
 * pool, conv 32, ReLU, max pool, FC 512, ReLU, dropout 25 %, FC 10) on its own
 * minibatch against the weight snapshot it last pulled, which may be stale.
 * The server applies the resulting gradients by the paper's three rules:
 *   sync      (Section 2.1, Section 3.1)  wait for all, one update with all
 *   async     (Section 2.1, Section 3.1)  one update per arriving gradient
 *   stateless (Section 2.3, Section 3.3)  gradients are appended to a pending
 *             list; a server step applies ALL pending ones and publishes; while
 *             the server is down the list only grows and is applied on recovery
 * "Server down" is not library state: the caller simply stops calling apply.
 *
 * Conventions
 *   - Every function returns a ps_status and never throws across the ABI.
 *     ps_last_error() gives a message for the last failing call on a context.
 *   - Pointers named *_dev are DEVICE pointers borrowed for the duration of the
 *     enqueued work; pointers named *_host are HOST pointers owned by the caller.
 *   - All GPU work is enqueued on the HIP stream given to ps_init and is
 *     asynchronous; the ps_get_*, ps_debug_* and ps_sync calls wait for it.
 *     Only the server side of the lock-free store (below) runs on a second
 *     stream, which the context creates at default priority.
 *   - The library allocates no device memory: the caller hands ps_init one
 *     device workspace of ps_workspace_bytes() bytes, which the context carves
 *     into weights, snapshot ring, gradient queue and activations, and which
 *     must outlive the context.
 *   - Not thread-safe per context.
 *
 * Flat parameter vector, P = 813,258 floats, offsets in floats:
 *   conv1.W[16][1][3][3] @0, conv1.b[16] @144, conv2.W[32][16][3][3] @160,
 *   conv2.b[32] @4768, fc1.W[512][1568] @4800 (input index = c*49 + y*7 + x),
 *   fc1.b[512] @807616, fc2.W[10][512] @808128, fc2.b[10] @813248.
 * Readings where the paper is silent (kernel 3x3 pad 1, pool 2x2, softmax
 * cross-entropy, inverted dropout, SUM aggregation, plain SGD) are listed in
 * the design notes.
 */
#ifndef PS_HOTPATH_H
#define PS_HOTPATH_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PS_API __attribute__((visibility("default")))

#define PS_PARAM_COUNT 813258
#define PS_IMAGE_PIXELS 784
#define PS_N_CLASSES 10
#define PS_FC1_UNITS 512
#define PS_POOL1_SIZE 3136 /* 16 x 14 x 14 */
#define PS_POOL2_SIZE 1568 /* 32 x 7 x 7   */
#define PS_ROW_FLOATS 813312 /* pitch, in floats, of every P-vector row in device memory: P rounded up to 256 B */
#define PS_STATIC_DRAIN_MAX_ROWS 4096 /* most rows one ps_drain_rows_mitigated call takes */

typedef struct ps_ctx ps_ctx;

typedef enum {
    PS_OK = 0,
    PS_EINVAL = 1,  /* bad argument: null pointer, index or size out of range        */
    PS_ENOMEM = 2,  /* workspace too small                                           */
    PS_ESTATE = 3,  /* queue entry not pending (already applied or never written)    */
    PS_EFULL = 4,   /* gradient queue has too few free entries; nothing was appended */
    PS_EDEVICE = 5  /* a HIP call failed                                             */
} ps_status;

typedef struct {
    int32_t max_workers;    /* largest n accepted by one worker_grads_batched call, >= 1 */
    int32_t batch;          /* B, images per worker minibatch, >= 1                      */
    int32_t n_versions;     /* V, snapshot ring slots, >= 1                              */
    int32_t queue_capacity; /* most gradients pending at once, >= 1                      */
    uint64_t seed;          /* key of the dropout generator                              */
    float dropout_p;        /* in [0, 1); the paper's model uses 0.25                    */
} ps_config;

typedef enum { PS_DRAIN_SUM = 0, PS_DRAIN_SEQ = 1 } ps_drain_mode;

/* Device bytes ps_init needs for this configuration. */
PS_API ps_status ps_workspace_bytes(const ps_config* cfg, uint64_t* bytes_out);

/* Creates a context over the caller's device workspace (256-byte aligned,
 * >= ps_workspace_bytes()) on `hip_stream` (a hipStream_t, or NULL for the
 * default stream) of the current device.  Weights, ring and queue start zeroed,
 * version 0, queue empty.  On failure *out is NULL. */
PS_API ps_status ps_init(ps_ctx** out, const ps_config* cfg, void* workspace_dev, uint64_t workspace_bytes,
                  void* hip_stream);

/* Waits for enqueued work, releases host resources.  The workspace stays the caller's. */
PS_API ps_status ps_destroy(ps_ctx* ctx);

/* Blocks until everything enqueued on the context's stream has finished. */
PS_API ps_status ps_sync(ps_ctx* ctx);

/* theta := theta_host[P]; every ring slot := theta; version := 0.  Queue must be empty (else PS_ESTATE). */
PS_API ps_status ps_set_weights(ps_ctx* ctx, const float* theta_host);

/* Copies P floats to the host: the server's current weights (slot = -1) or ring slot `slot`. */
PS_API ps_status ps_get_weights(ps_ctx* ctx, int32_t slot, float* theta_host);

/* A worker pulls the weights (Section 2.1: workers pull a snapshot; Section 3.3 worker step:
 * read the stored weights): ring[slot] := theta.  *version_out (may be NULL) receives the
 * number of weight updates applied so far, which is the snapshot's version. */
PS_API ps_status ps_snapshot_weights(ps_ctx* ctx, int32_t slot, uint64_t* version_out);

/* Worker step, batched (Section 3.3 worker pseudo-code; Section 2.3 for the outage case):
 * for i in [0, n): worker worker_id_host[i] computes the gradient of its mean minibatch loss
 * (softmax cross-entropy) at the snapshot in ring slot version_slot_host[i], on images
 * x_dev[i][B][784] (fp32) with labels y_dev[i][B] (int32 in [0,10)), and appends it to the
 * pending queue.  Entries are appended in array order, which is their arrival order.
 * minibatch_id_host[i] is the minibatch's logical 64-bit id; with the seed it keys the
 * dropout mask: unit u of sample s is dropped iff word u%4 of
 * Philox4x32-10(counter {id_lo, id_hi, s, u/4}, key {seed_lo, seed_hi}) < floor(p * 2^32);
 * kept units are scaled by 1/(1-p).
 * queue_index_host[i] receives the queue entry holding gradient i.  loss_dev (device, [n], may
 * be NULL) receives each worker's mean loss.  n = 0 is a no-op.  n > max_workers, a slot outside
 * the ring or a null array give PS_EINVAL; fewer than n free entries give PS_EFULL. */
PS_API ps_status worker_grads_batched(ps_ctx* ctx, int32_t n, const int32_t* worker_id_host,
                               const int32_t* version_slot_host, const uint64_t* minibatch_id_host,
                               const float* x_dev, const int32_t* y_dev, int32_t* queue_index_host,
                               float* loss_dev);

/* Appends a gradient produced elsewhere (the worker-side append of the stateless pseudo-code,
 * Section 3.3): grad_host[P] is copied into a free queue entry with the given metadata. */
PS_API ps_status ps_queue_push_host(ps_ctx* ctx, const float* grad_host, int32_t worker_id, uint64_t version,
                             uint64_t minibatch_id, int32_t* queue_index_host);

/* Synchronous rule (Section 2.1, Section 3.1): one update with all n listed pending gradients,
 * theta := theta - lr * (g_0 + ... + g_{n-1}) summed in list order; the entries are then freed.
 * Version += 1.  n = 0 is a no-op.  A listed entry that is not pending, or listed twice, gives
 * PS_ESTATE and nothing is applied. */
PS_API ps_status ps_apply_sync(ps_ctx* ctx, const int32_t* queue_index_host, int32_t n, float lr);

/* Asynchronous rule (Section 2.1, Section 3.1): theta := theta - lr * g for one arrived
 * gradient; the entry is freed.  Version += 1. */
PS_API ps_status ps_apply_async(ps_ctx* ctx, int32_t queue_index, float lr);

/* Stateless server step / recovery (Section 2.3; Section 3.3 server pseudo-code): applies every
 * pending gradient in arrival order, either as one update with their sum (PS_DRAIN_SUM,
 * version += 1) or as one update per gradient (PS_DRAIN_SEQ, version += K), then empties the
 * queue.  *n_applied_host (may be NULL) receives K; K = 0 changes nothing. */
PS_API ps_status ps_drain_buffered(ps_ctx* ctx, int32_t mode, float lr, int32_t* n_applied_host);

/* Recovery with the mitigations the paper reports or suggests for large backlogs of stale gradients
 * (Section 2.3, last paragraph): the learning rate is turned down with the number K of pending
 * gradients, lr_used = lr * min(1, lr_backlog_ref / K) (lr_backlog_ref = 0 switches this off), and
 * every gradient is clipped to 2-norm clip_norm, g := g * min(1, clip_norm / ||g||_2) (clip_norm = 0
 * switches this off; the norm costs one extra pass over the queue).  Otherwise as ps_drain_buffered.
 * *lr_used_host (may be NULL) receives the learning rate applied.  The paper gives no formula for
 * either; these are this library's readings. */
typedef struct {
    float lr;
    float lr_backlog_ref; /* >= 0 */
    float clip_norm;      /* >= 0 */
} ps_drain_policy;
PS_API ps_status ps_drain_buffered_mitigated(ps_ctx* ctx, int32_t mode, const ps_drain_policy* policy,
                                      int32_t* n_applied_host, float* lr_used_host);

/* ps_drain_buffered_mitigated for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid allocation.  No context: the
 * caller owns the weights and the buffered gradients and passes them as rows of PS_ROW_FLOATS floats
 * (16-byte aligned; the floats beyond PS_PARAM_COUNT in a row are padding and must be zero in the
 * gradient rows): theta_dev is one row, updated in place; grads_dev holds n_rows rows back to back, in
 * arrival order.  Mode, policy and *lr_used_host (host, may be NULL) are those of
 * ps_drain_buffered_mitigated, and the same kernels run, on `hip_stream` (a hipStream_t, NULL for the
 * default stream), asynchronously.  The row list, the partial sums of the squared norms and the clip
 * factors, which the context-based call keeps in its workspace, live in a fixed array of 557,056 bytes
 * in the library's device image (each GPU the process uses holds one copy until the process ends); the
 * call allocates and frees nothing, on the host or on the device, and clears nothing (every element it
 * reads it has written first).  n_rows > PS_STATIC_DRAIN_MAX_ROWS gives PS_EINVAL and nothing runs;
 * n_rows = 0 changes nothing.  All calls on one GPU share that GPU's array: two calls whose kernels may
 * overlap (different streams, or threads) race.  The address of the array is looked up on the first call
 * on a device, or by ps_init on that device, whichever comes first; make one of them before a capture
 * starts.  ps_last_error(NULL) gives the message of the calling thread's last failing call. */
PS_API ps_status ps_drain_rows_mitigated(float* theta_dev, const float* grads_dev, int32_t n_rows, int32_t mode,
                                         const ps_drain_policy* policy, float* lr_used_host, void* hip_stream);

/* Recovery with an adaptive learning rate, which Section 2.3 (last paragraph) names, as Adadelta, among
 * the methods for applying the stale gradients; the paper gives no details, so this is the method as
 * published (Zeiler 2012, Algorithm 1).  Every pending gradient g, in arrival order, is one step; per
 * parameter:  E[g^2] := rho E[g^2] + (1-rho) g^2;  dx := -sqrt(E[dx^2] + eps) / sqrt(E[g^2] + eps) * g;
 * E[dx^2] := rho E[dx^2] + (1-rho) dx^2;  theta := theta + lr * dx.   Version += K, queue emptied.
 * The two accumulators are state of the context: zero after ps_init and ps_set_weights, carried from
 * one call to the next, not part of a snapshot.  rho in [0, 1), eps > 0, else PS_EINVAL. */
PS_API ps_status ps_drain_buffered_adadelta(ps_ctx* ctx, float lr, float rho, float eps, int32_t* n_applied_host);

/* Elastic averaging SGD (Zhang, Choromanska, LeCun 2015), which Section 2.3 (last paragraph) names
 * among the methods to try for the work workers do while the server is away.  Here a worker's local
 * weights are a ring slot of its own: it computes its gradient there (worker_grads_batched with that
 * slot) and takes a plain SGD step on its own copy,
 *   ps_apply_local:      ring[slot_i] := ring[slot_i] - lr * g(queue_index_i)   for i in [0, n)
 * (distinct slots, pending entries, which are then freed; the server's weights and the version do not
 * change), and from time to time, or when the server is back, one synchronous elastic step couples
 * the n listed local copies to the server's weights (the centre), every difference taken first:
 *   ps_elastic_average:  d_i = ring[slot_i] - theta;  ring[slot_i] := ring[slot_i] - alpha * d_i;
 *                        theta := theta + alpha * (d_0 + ... + d_{n-1});  version += 1
 * (alpha = the paper's eta * rho; distinct slots; alpha >= 0).  n = 0 is a no-op in both. */
PS_API ps_status ps_apply_local(ps_ctx* ctx, int32_t n, const int32_t* slot_host, const int32_t* queue_index_host, float lr);
PS_API ps_status ps_elastic_average(ps_ctx* ctx, const int32_t* slot_host, int32_t n, float alpha);

/* Recovery of the checkpointing and chain-replication arms (Section 2.1: the resurrected server
 * rehydrates the latest checkpoint and continues from that older state; Section 2.2: a backup server
 * with periodically replicated weights takes over): theta := ring[slot], version := the version that
 * snapshot was taken at, and every pending gradient is dropped (*n_dropped_host, may be NULL,
 * receives how many).  A checkpoint / replica is a ring slot refreshed with ps_snapshot_weights every
 * N updates by the caller. */
PS_API ps_status ps_restore_weights(ps_ctx* ctx, int32_t slot, int32_t* n_dropped_host);

/* Loads a ring slot from host memory: ring[slot] := theta_host[P], recorded as the snapshot taken at
 * `version` (Section 2.1: a restarted server rehydrates the latest checkpoint from persistent storage;
 * followed by ps_restore_weights(slot) this is that path, and it also restores a worker-local copy).
 * The server's weights and version do not change.  Waits for the copy. */
PS_API ps_status ps_load_snapshot(ps_ctx* ctx, int32_t slot, const float* theta_host, uint64_t version);

/* Periodic evaluation (Section 3.1: accuracy and loss are collected periodically): inference forward
 * pass without dropout on n_images images x_dev[n_images][784] with labels y_dev[n_images], using the
 * server's current weights (slot = -1) or ring slot `slot`.  n_images must be a positive multiple
 * of batch and at most max_workers * batch.  *loss_host = mean cross-entropy, *accuracy_host =
 * fraction of images whose arg-max class (lowest index on ties) equals the label, pred_host[n_images]
 * the predicted classes (each may be NULL).  Waits for the result; overwrites the activations that
 * ps_debug_last_batch reads. */
PS_API ps_status ps_evaluate(ps_ctx* ctx, int32_t slot, int32_t n_images, const float* x_dev, const int32_t* y_dev,
                      double* loss_host, double* accuracy_host, int32_t* pred_host);

/* ---- Lock-free gradient store: workers and server on two streams -------------------------------
 *
 * Section 3.3 (last paragraph) observes that accesses to the gradient store can be lock-free, since a
 * gradient is written once by its worker and read, then deleted, by the server; the implementation
 * measured in the paper takes a lock instead, and the Future Work section lists a better mechanism.
 * Here the store's state lives in device memory.  Workers (the stream given to ps_init) and the
 * server (a second stream the context creates, same priority) run concurrently and meet only there:
 * a batch of workers writes its gradient rows, then claims consecutive positions with one atomic add
 * and stamps the rows as complete; a server step takes the longest prefix of complete rows not yet
 * consumed, applies it in position order and deletes it by advancing the consumed count.  Positions
 * count appended gradients from 0 and never wrap; position p uses queue row p % queue_capacity (the
 * host, which enqueues all appends on the one worker stream, knows the rows in advance; the device
 * checks that the claim lands on them).
 *
 * While the store holds gradients that the host has not yet seen consumed (ps_store_state tells),
 * the calls above that touch the queue or the server's weights return PS_ESTATE; the store calls in
 * turn need the pending queue of those calls to be empty.  Version counts and snapshot versions carry
 * over in both directions: the first store call hands them to the device, and the first of the calls
 * above after store calls waits for both streams and takes them back (no ps_store_state needed in
 * between).  ps_get_weights, ps_evaluate and ps_sync wait for both streams. */

typedef struct {
    uint64_t claimed;   /* gradients ever appended (positions handed out)               */
    uint64_t published; /* length of the prefix of them whose rows are completely written */
    uint64_t consumed;  /* gradients ever applied and deleted                            */
    uint64_t version;   /* weight updates applied so far                                 */
    uint64_t steps;     /* server steps so far that applied at least one gradient        */
} ps_store_counters;

typedef struct {
    uint64_t first;         /* first position the step consumed */
    uint32_t count;         /* how many, consecutive            */
    uint32_t mode;          /* ps_drain_mode                    */
    uint64_t version_after; /* version once it was applied      */
} ps_store_step;

/* Worker step as worker_grads_batched, but into the store: the n gradients take positions
 * claimed .. claimed + n - 1 in array order, claimed and stamped on the device when their rows are
 * complete; no queue index comes back.  Waits (on the device, not the host) for the last ps_store_publish into each ring slot
 * it reads.  PS_EFULL if claimed + n - consumed could exceed queue_capacity by what the host has seen
 * so far (it looks again, waiting for the server stream, before giving up); PS_ESTATE if the ordered
 * queue above is not empty. */
PS_API ps_status worker_grads_append(ps_ctx* ctx, int32_t n, const int32_t* worker_id_host,
                                     const int32_t* version_slot_host, const uint64_t* minibatch_id_host,
                                     const float* x_dev, const int32_t* y_dev, float* loss_dev);

/* Server step on the server stream: takes the rows that are complete when the step runs, at most
 * max_entries of them (0 = no limit), applies them as one update with their sum (PS_DRAIN_SUM,
 * version += 1) or one update each in position order (PS_DRAIN_SEQ, version += count), and deletes
 * them.  Nothing complete: nothing changes.  With wait_for_workers != 0 the step first waits, on the
 * device, for every worker_grads_append enqueued so far, so that it takes all of those (up to the
 * limit); with 0 it races the workers and how many it takes depends on timing (ps_store_steps
 * tells afterwards). */
PS_API ps_status ps_store_consume(ps_ctx* ctx, int32_t mode, float lr, int32_t max_entries, int32_t wait_for_workers);

/* ring[slot] := the server's weights, on the server stream, after the server steps enqueued so far
 * and after every enqueued worker step that reads the slot; the slot's version is recorded on the
 * device.  The lock-free counterpart of ps_snapshot_weights. */
PS_API ps_status ps_store_publish(ps_ctx* ctx, int32_t slot);

/* Waits for both streams and reads the counters.  Once consumed == claimed the ordered calls above
 * are available again. */
PS_API ps_status ps_store_state(ps_ctx* ctx, ps_store_counters* counters_host);

/* Waits for both streams; the most recent server steps that applied something, oldest first: *n_host
 * receives how many are returned (at most `capacity`, at most the 1024 the device keeps). */
PS_API ps_status ps_store_steps(ps_ctx* ctx, int32_t capacity, int32_t* n_host, ps_store_step* steps_host);

/* Waits for both streams; copies the gradient at `position` (P floats) and its metadata (each pointer
 * may be NULL).  PS_ESTATE unless consumed <= position < published. */
PS_API ps_status ps_store_entry(ps_ctx* ctx, uint64_t position, float* grad_host, int32_t* worker_host,
                                uint64_t* version_host, uint64_t* minibatch_host);

/* Copies pending gradient `queue_index` (P floats) to the host. */
PS_API ps_status ps_get_grad(ps_ctx* ctx, int32_t queue_index, float* grad_host);

/* Pending entries in arrival order.  *n_host receives their number K; each array (may be NULL)
 * must hold `capacity` items and receives min(K, capacity): arrival sequence number, worker id,
 * version of the snapshot used, minibatch id, queue entry index. */
PS_API ps_status ps_queue_meta(ps_ctx* ctx, int32_t capacity, int32_t* n_host, uint64_t* seq_host,
                        int32_t* worker_host, uint64_t* version_host, uint64_t* minibatch_host,
                        int32_t* queue_index_host);

/* Number of weight updates applied so far.  After lock-free store calls this waits for both streams. */
PS_API ps_status ps_version(ps_ctx* ctx, uint64_t* version_host);

/* Decisions taken for worker i of the most recent worker_grads_batched call (any pointer may be
 * NULL): pool1_host[B][3136] and pool2_host[B][1568] hold, per pooled output, bits 0-1 = winner
 * of the 2x2 window (dy*2+dx, first maximum wins) and bit 2 = 1 iff the winner's pre-activation
 * is > 0; keep_host[B][512] the dropout keep mask (1 = kept); hdrop_host[B][512] the fc1
 * activation after ReLU and dropout; z_host[B][10] the logits; pred_host[B] the arg-max class
 * (lowest index on ties). */
PS_API ps_status ps_debug_last_batch(ps_ctx* ctx, int32_t i, uint8_t* pool1_host, uint8_t* pool2_host,
                              uint8_t* keep_host, float* hdrop_host, float* z_host, int32_t* pred_host);

/* Values behind those decisions, for the same worker of the same call (any pointer may be NULL):
 * pool1_val_host[B][3136] and pool2_val_host[B][1568] the pooled activations after ReLU (model
 * endnote: conv, ReLU, max pool), d3_host[B][512] the gradient of the worker's mean loss with
 * respect to the fc1 pre-activations (zero exactly where the unit was dropped or its ReLU was
 * off), dpool2_host[B][1568] the gradient with respect to the pool2 outputs, zero where the pooled
 * activation is zero.  Tests measure the fp32 rounding of each layer from these and check that the
 * backward pass used the same dropout mask as the forward pass. */
PS_API ps_status ps_debug_last_activations(ps_ctx* ctx, int32_t i, float* pool1_val_host, float* pool2_val_host,
                                           float* d3_host, float* dpool2_host);

/* Per-kernel timing (instrumentation, not part of the method).  While enabled, every kernel launch
 * of this context is bracketed by two HIP events on the context's stream.  ps_profile_enable waits
 * for the stream, clears the totals and switches timing on (enable != 0) or off.  ps_profile_read
 * waits for the stream and reports the summed duration and number of launches of kernel
 * `kernel_id` in [0, ps_profile_kernel_count()); ps_profile_kernel_name gives the kernel's function
 * name, template arguments abbreviated to the distinguishing one ("" for an unknown id). */
PS_API ps_status ps_profile_enable(ps_ctx* ctx, int32_t enable);
PS_API ps_status ps_profile_read(ps_ctx* ctx, int32_t kernel_id, double* total_ms_host, int64_t* launches_host);
PS_API int32_t ps_profile_kernel_count(void);
PS_API const char* ps_profile_kernel_name(int32_t kernel_id);

/* What the chip sustains with the instructions this library's kernels are made of (instrumentation for
 * the roofline figures, not part of the method).  Runs short timing kernels on `hip_stream` over the
 * caller's device buffer (256-byte aligned, at least 64 MiB, up to 4 GiB of it are streamed; its contents
 * are overwritten) and waits for them:
 *   mfma_32x32x2_tflops / mfma_16x16x4_tflops   fp32 MFMA rate over all compute units, nothing else issued
 *                                               (first_launch: before the clock has ramped up under load)
 *   ns_per_mfma_with_valu[i]                    time per 16x16x4 MFMA of a wavefront that issues 0, 1, 2, 4
 *                                               independent vector FMAs behind every MFMA (one wavefront per SIMD)
 *   shared_simd_ms[0..2]                        the same MFMA loop alone, a vector-FMA loop alone, and both as
 *                                               two wavefronts sharing every SIMD: [2] near max([0], [1]) means
 *                                               the two kinds overlap, near [0] + [1] that they do not
 *   ns_per_mfma_with_lds_reads[i]               SIMD time per 16x16x4 MFMA when i = 0, 1, 2 values per MFMA and lane
 *                                               come out of LDS (ds_read_b32, no bank conflicts; two blocks of four
 *                                               wavefronts per compute unit)
 *   hbm_read_GBps / hbm_copy_GBps               one pass of 16-byte loads over the buffer / copy of one half to
 *                                               the other (bytes read + bytes written) */
typedef struct {
    int32_t compute_units;
    double mfma_32x32x2_tflops, mfma_32x32x2_first_launch_tflops, mfma_16x16x4_tflops;
    double ns_per_mfma_16x16x4;
    double ns_per_mfma_with_valu[4];
    double shared_simd_ms[3];
    double ns_per_mfma_with_lds_reads[3];
    double hbm_read_GBps, hbm_copy_GBps;
    uint64_t hbm_read_bytes;
} ps_ceilings;
PS_API ps_status ps_measure_ceilings(void* workspace_dev, uint64_t workspace_bytes, void* hip_stream, ps_ceilings* out_host);

/* Message of the last failing call on this context ("" if none); valid until the next call.  With
 * ctx = NULL: of the calling thread's last failing ps_drain_rows_mitigated call. */
PS_API const char* ps_last_error(const ps_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* PS_HOTPATH_H */
