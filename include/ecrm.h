/*
 * ecrm.h -- C ABI of the MI355X (gfx950) implementation of the ECRM parameter-server update path.
 *
 * ECRM (arXiv 2104.01981) keeps, for every group of k embedding entries, one parity entry
 * p = e_0 + ... + e_{k-1} (and one parity row of optimizer state), and keeps the parities current
 * by "difference propagation": after the optimizer has been applied to an entry, the differences
 * in entry and optimizer state are added to the parity (Sec. 3.2, 3.3).  This library performs
 * that work for a batch of sparse updates on ONE GPU that holds all S servers' shards.
 *
 * Data model (all DEVICE memory, caller-owned, fp32, row-major, 16-byte aligned):
 *   E [R][D]    embedding entries            A [R][D]    Adagrad accumulators (optimizer state)
 *   PE[R/k][D]  parity entries               PA[R/k][D]  parity accumulators
 *   load_data[S], load_parity[S]  u64: number of entry / parity updates that fell on each server
 * Stripe g consists of rows k*g .. k*g+k-1; its parity lives on server g mod S and member j on
 * server (g+1+j) mod S (rotating placement, Sec. 3.2).
 *
 * Every entry point returns ECRM_OK (0) or a negative error code; nothing throws, logs, or
 * allocates device memory.  encode/route/update only ENQUEUE work on the caller's HIP stream
 * (pass the hipStream_t as void*; NULL is the default stream) and never synchronise: operations
 * take effect in stream order, which is also what guarantees that every difference of an earlier
 * update has reached its parity before later work reads it (Sec. 3.5).  A context is not
 * thread-safe; different contexts are independent.
 */
#ifndef ECRM_H
#define ECRM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ecrm_ctx ecrm_ctx; /* opaque; host memory only */

enum {
    ECRM_OK = 0,
    ECRM_EINVAL = -1,    /* bad argument or configuration                                  */
    ECRM_ENOTBOUND = -2, /* tables not bound yet                                           */
    ECRM_ESCRATCH = -3,  /* scratch buffer missing, misaligned or too small                */
    ECRM_EBATCH = -4,    /* n exceeds config.max_batch                                     */
    ECRM_EKEYRANGE = -5, /* a key >= rows was seen on the device (reported by ecrm_status) */
    ECRM_EHIP = -6,      /* a HIP runtime call failed                                      */
    ECRM_EBUFFER = -7,   /* recovery buffer full on the device (reported by ecrm_status)   */
    ECRM_ESTATE = -8     /* call not allowed in the current recovery state                 */
};

enum { ECRM_OPT_ADAGRAD = 0, ECRM_OPT_MOMENTUM = 1 };

/* How the parities follow the entries. */
enum {
    ECRM_PROP_DIFFERENCE = 0, /* difference propagation, the paper's method (Sec. 3.3.2)               */
    ECRM_PROP_GRADIENT = 1,   /* the strawman of Sec. 3.3.1: the gradient itself goes to the parity,
                                 which applies the optimizer with its own state.  With Adagrad the
                                 parities stop being the sums of their entries -- kept to show that,
                                 and what the second pass over the gradients costs (Sec. 4.3
                                 "Benefit of difference propagation")                                */
    ECRM_PROP_NONE = 2        /* parities left alone: training without fault tolerance, the baseline
                                 the overheads of Sec. 4.3 are quoted against                        */
};

typedef struct {
    uint64_t rows;      /* R: k <= R <= 2^32 - 4096, multiple of k                              */
    uint32_t dim;       /* D: floats per entry, multiple of 4, 4..1024 (the paper uses 128, 256) */
    uint32_t k;         /* data entries per parity, 1..64 (paper: 2, 4, 10); r is fixed to 1     */
    uint32_t servers;   /* S: k+1 <= S <= 1024 (paper: 5)                                        */
    uint32_t optimizer; /* ECRM_OPT_ADAGRAD: the update rule printed in Sec. 3.3.1;
                           ECRM_OPT_MOMENTUM: SGD with momentum, the optimizer of the paper's evaluation
                           (Sec. 4.1; the paper prints no formula): v <- momentum*v + g, e <- e - lr*v,
                           with A holding v                                                       */
    float lr;           /* learning rate, used as its exact fp32 value                           */
    float eps;          /* Adagrad epsilon (under the square root), >= 0                         */
    uint64_t max_batch; /* largest n ever passed to ecrm_update, 1 .. 2^31 (sizes the scratch)   */
    float momentum;     /* ECRM_OPT_MOMENTUM only: coefficient in [0, 1)                          */
    uint32_t combine;   /* 0: several updates to one entry inside a call are applied one after the
                           other in arrival order (asynchronous training, Sec. 2.1).
                           1: their gradients are summed and applied as ONE update per modified entry,
                           and the load counters count one update per modified entry (the synchronous
                           variant of Sec. 4.4 "Synchronous training")                             */
    uint32_t propagation; /* ECRM_PROP_*; GRADIENT needs combine = 0.  With GRADIENT the load counters are
                           those of DIFFERENCE (one entry and one parity update per item); with NONE
                           load_parity is not touched.  The recovery-under-load calls need DIFFERENCE. */
} ecrm_config;

/* Validates the configuration and creates a host-side context.  No device memory is touched. */
int ecrm_create(const ecrm_config *cfg, ecrm_ctx **out);

/* Frees the host-side context only; bound device buffers are never touched. NULL is allowed. */
void ecrm_destroy(ecrm_ctx *ctx);

/* Sizes in bytes: one data table (R*D*4), one parity table (R/k*D*4; the memory overhead of the
 * code is therefore (k+1)/k, Sec. 2.4 / 3.1), and the scratch buffer ecrm_bind needs. */
size_t ecrm_data_bytes(const ecrm_ctx *ctx);
size_t ecrm_parity_bytes(const ecrm_ctx *ctx);
size_t ecrm_scratch_bytes(const ecrm_ctx *ctx);

/* Attaches caller-owned device buffers.  scratch must be 256-byte aligned and at least
 * ecrm_scratch_bytes() long; its contents are private to the library while bound.  The load
 * counters are accumulated into, never cleared.  Returns EINVAL for a NULL / misaligned table,
 * ESCRATCH for the scratch buffer, ESTATE while a recovery is in progress (the updates waiting in its
 * buffer would be lost), EHIP if the device cannot be queried.  Call it outside a stream capture. */
int ecrm_bind(ecrm_ctx *ctx, float *E, float *A, float *PE, float *PA,
              uint64_t *load_data, uint64_t *load_parity, void *scratch, size_t scratch_bytes);

/* Sum encoder with r = 1 (Sec. 3.2 "Encoder and decoder"): PE[g] = sum_j E[k*g+j], PA likewise,
 * accumulated in fp64 and rounded once.  Run once before training (Sec. 3.1).  ESTATE while a
 * recovery (ecrm_recovery_begin) is in progress. */
int ecrm_encode(ecrm_ctx *ctx, void *hip_stream);

/* Rotating parity placement (Sec. 3.2) for n keys: stripe = key / k, member = key % k,
 * data_srv = (stripe+1+member) % S, parity_srv = stripe % S.  All pointers are device memory of
 * n elements; any output pointer may be NULL.  Keys >= rows raise the sticky EKEYRANGE status and
 * leave their outputs unwritten. */
int ecrm_route(ecrm_ctx *ctx, const uint64_t *keys, uint64_t n, uint64_t *stripe, uint32_t *member,
               uint32_t *data_srv, uint32_t *parity_srv, void *hip_stream);

/* One batch of n sparse updates (keys[i] = dense row id, grads[i][0..D) = its gradient), device
 * pointers, read-only.  Per entry, updates are applied in arrival (index) order:
 *     A[x] += g*g ;  E[x] -= lr / sqrt(A[x] + eps) * g            (Adagrad, Sec. 3.3.1)
 * and the resulting differences in E[x] and A[x] are added to PE[x/k] and PA[x/k]
 * (difference propagation, Sec. 3.3.2); load_data / load_parity count one update per item on the
 * entry's and the parity's server (Sec. 3.6).  Arithmetic inside the call is carried in fp64 and
 * every touched element is rounded to fp32 once.  If any key >= rows, NOTHING of this batch is
 * applied and the sticky status becomes EKEYRANGE.  n = 0 is a no-op; n > max_batch is EBATCH.
 * keys/grads may be reused once the stream has passed the call. */
int ecrm_update(ecrm_ctx *ctx, const uint64_t *keys, const float *grads, uint64_t n, void *hip_stream);

/* For callers that cannot allocate device memory or hand over a workspace -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: ecrm_update with the library's own
 * scratch buffer, a fixed array of ECRM_STATIC_SCRATCH_BYTES in the library's image (every GPU the
 * library runs on holds its copy until the process ends).  The call allocates and frees nothing.
 * The context supplies the configuration only (ecrm_bind is not needed and bound buffers are not
 * touched); tables, counters, keys and gradients are passed here, with the meaning, layout and
 * alignment they have in ecrm_bind / ecrm_update.  With ECRM_PROP_NONE, PE, PA and load_parity may be
 * NULL.  Limits: n <= ECRM_STATIC_MAX_BATCH (else EBATCH), and a configuration whose scratch layout
 * for that batch size exceeds the array (large dim with momentum SGD) is refused with ESCRATCH; no
 * recovery may be in progress on the context (ESTATE).
 * The array has no sticky status: every call starts from a cleared header.  *rejected (DEVICE memory, 4
 * bytes, may be NULL) receives 1 if the batch carried a key >= rows -- then nothing of it was applied --
 * and 0 otherwise, in stream order.  All calls on one GPU share the one array: calls that overlap in
 * time on the same GPU (two streams, two contexts, two threads) race; serialise them.
 * The first call of a context, and the first on each device, do one-time host-side set-up (occupancy
 * queries, the array's address): make that call outside a stream capture. */
enum { ECRM_STATIC_MAX_BATCH = 1 << 16, ECRM_STATIC_SCRATCH_BYTES = 8 << 20 };
int ecrm_update_static(ecrm_ctx *ctx, float *E, float *A, float *PE, float *PA, uint64_t *load_data,
                       uint64_t *load_parity, const uint64_t *keys, const float *grads, uint64_t n,
                       uint32_t *rejected, void *hip_stream);

/* Recovery from the loss of one server (Sec. 3.4), with the subtraction decoder of Sec. 3.2:
 * a lost entry is e_j = p - sum_{i != j} e_i (same for its accumulator), a lost parity is re-encoded.
 * Server s holds member j of stripe g when (g+1+j) mod S == s and the parity of g when g mod S == s;
 * the k+1 units of a stripe are on k+1 different servers, so at most one unit per stripe is lost.
 * Sums are carried in fp64 in the order p, then minus the members by increasing j, and rounded once.
 *
 * ecrm_fail_server    test aid: overwrites every unit (rows of E and A, or of PE and PA) held by
 *                     `server` with NaN, as if its memory were gone.
 * ecrm_recover_server rebuilds every unit held by `server` from the k surviving units of its stripe
 *                     ("full recovery").  Work enqueued earlier on the stream -- every difference of
 *                     every earlier update -- is complete before it reads anything (Sec. 3.5).
 * ecrm_degraded_read  reads the entries of n keys into out_E[n][D] (and their accumulators into
 *                     out_A[n][D] if not NULL) while `lost_server` is down: rows it held are decoded on
 *                     the fly from the parity and the other members, all others are copied.  Pass
 *                     ECRM_NO_SERVER for a plain gather.  Keys >= rows raise the sticky EKEYRANGE
 *                     status and leave their output rows unwritten.
 * server >= S (other than ECRM_NO_SERVER for the read) is EINVAL; ecrm_fail_server and
 * ecrm_recover_server return ESTATE while a chunked recovery (ecrm_recovery_begin) is in progress. */
#define ECRM_NO_SERVER 0xFFFFFFFFu
int ecrm_fail_server(ecrm_ctx *ctx, uint32_t server, void *hip_stream);
int ecrm_recover_server(ecrm_ctx *ctx, uint32_t server, void *hip_stream);
int ecrm_degraded_read(ecrm_ctx *ctx, const uint64_t *keys, uint64_t n, uint32_t lost_server,
                       float *out_E, float *out_A, void *hip_stream);

/* Training while a failed server is being rebuilt (Sec. 3.4 "Training during recovery").  The
 * stripes are split into `chunks` equal ranges that are rebuilt one after the other; while a chunk
 * is "locked", every update that touches one of its stripes is buffered instead of applied, and it
 * is applied when the chunk is released -- so the decoder never sees an entry and a parity at
 * different versions, and training never pauses.  Independently of the lock, an update to an entry
 * that the failed server held is buffered until that entry has been rebuilt.  More chunks mean a
 * smaller buffer and more switches (the paper's 1 lock vs 10 locks).  Buffered updates keep their
 * arrival order per entry; their load is counted when they are applied.
 *
 *   ecrm_recovery_begin   declares `server` lost (its rows are NOT overwritten; use ecrm_fail_server
 *                         in tests) and hands over the buffer: device memory for 2*capacity keys
 *                         (u64) and 2*capacity gradient rows, capacity <= max_batch = the largest number
 *                         of updates that can wait at one time.  (The library keeps two lists of
 *                         (key, row slot) entries in buf_keys, a pool of `capacity` gradient rows in the
 *                         first half of buf_grads and its bookkeeping in the second half: a gradient row
 *                         is copied once, when its update is first held back, however long it waits.)  EINVAL with
 *                         combine = 1: synchronous training takes one step per entry and training step,
 *                         and a buffer replayed in one go would merge the waiting updates of several
 *                         steps into one.
 *   ecrm_recovery_lock    host-side only: from now on ecrm_update buffers what touches the next chunk.
 *   ecrm_recovery_decode  enqueues the reconstruction of the locked chunk.  It may run on another
 *                         stream than the updates, provided it starts after every ecrm_update that was
 *                         enqueued BEFORE the lock has finished (an event from that stream).
 *   ecrm_recovery_unlock  call on the update stream once the decode has finished (wait for its event
 *                         first; ESTATE if no decode was enqueued under this lock).  Releases the chunk
 *                         and enqueues the replay of the buffer (what must keep waiting stays in the
 *                         buffer); like ecrm_update it only enqueues.  After the last chunk the
 *                         recovery ends.
 *   ecrm_recovery_state   waits for the stream; reports whether a recovery is active, the number of
 *                         chunks rebuilt, the number of chunks, and how many updates are waiting.
 * A batch whose held-back items do not fit the buffer is rejected as a whole (sticky EBUFFER).
 * ecrm_degraded_read returns entries whose updates are waiting without them; ecrm_recovery_read
 * (below) returns them with the waiting updates applied. */
int ecrm_recovery_begin(ecrm_ctx *ctx, uint32_t server, uint32_t chunks, uint64_t *buf_keys, float *buf_grads,
                        uint64_t capacity, void *hip_stream);
int ecrm_recovery_lock(ecrm_ctx *ctx);
int ecrm_recovery_decode(ecrm_ctx *ctx, void *hip_stream);
int ecrm_recovery_unlock(ecrm_ctx *ctx, void *hip_stream);
int ecrm_recovery_state(ecrm_ctx *ctx, void *hip_stream, uint32_t *active, uint32_t *next_chunk, uint32_t *chunks,
                        uint64_t *buffered);

/* What a worker reads while a recovery is in progress (Sec. 3.4 has workers take a locked entry that
 * has been updated meanwhile out of the buffer): out_E[i][0..D) (and out_A[i] if not NULL) receive
 * entry keys[i] with its waiting updates applied in arrival order -- the value it will have once they
 * are replayed; an entry that the failed server held and that is not rebuilt yet is decoded from its
 * stripe first.  Nothing is modified, so the read may be repeated.  Call it on the update stream.
 * While a recovery is active the call uses the scratch buffer to group the waiting updates by entry
 * (sized by the buffer's capacity: how many are waiting is read on the device); without one it is a plain
 * gather.  Either way it only enqueues.  Keys >= rows raise the sticky EKEYRANGE status and leave their rows unwritten. */
int ecrm_recovery_read(ecrm_ctx *ctx, const uint64_t *keys, uint64_t n, float *out_E, float *out_A,
                       void *hip_stream);

/* Waits for the stream, then returns ECRM_OK, or EKEYRANGE if any batch since the last
 * ecrm_clear_status (or bind) carried a bad key, EBUFFER if one overflowed the recovery buffer, or
 * EHIP if the runtime reports an error. */
int ecrm_status(ecrm_ctx *ctx, void *hip_stream);
int ecrm_clear_status(ecrm_ctx *ctx, void *hip_stream);

/* Measurement aids (not part of the method).
 * ecrm_profile(ctx, 1) makes every later ecrm_update record HIP events around its three phases on
 * the stream it is enqueued on; ecrm_profile_read waits for them, adds up the elapsed time of the
 * calls recorded since the last read into ms[ECRM_PHASES] and returns the number of calls in
 * *calls (at most ECRM_PROFILE_MAX_CALLS are kept between reads).
 * ecrm_batch_stats waits for the stream and reports what the LAST ecrm_update found:
 *   out[0] = entries updated through the split-chain path (more than ECRM_LONG_RUN updates)
 *   out[1] = chain pieces those were cut into,  out[2] = items in those entries,
 *   out[3] = 1 if the batch was rejected for a bad key,
 *   out[4] = how many of the out[0] entries were walked by one workgroup each, with one read of their
 *            gradients (see ecrm_tune), instead of being cut into pieces.
 * ecrm_tune sets a tuning knob of the context (tests and measurements; the library is measured with the
 * defaults).  ECRM_TUNE_MID_MIN_ROWS: on the Adagrad rule an entry with more than ECRM_LONG_RUN and at most
 * ECRM_MID_RUN updates in a call is walked by one workgroup -- one read of its gradients instead of two --
 * but only in calls with at least this many such long entries, since one workgroup is slow and pays only
 * when all of them are busy.  Default (value 0): four per workgroup the device holds at once.  EINVAL for
 * an unknown knob or a value above 2^32-1.
 * ecrm_host_placement runs on the HOST only (no GPU needed): it evaluates, with the very 32-bit
 * arithmetic the kernels use, where `key` lies -- out[0] = stripe, out[1] = member, out[2] = data
 * server, out[3] = parity server (Sec. 3.2) -- and, for a recovery of `failed_server` in `chunks`
 * chunks of which `next_chunk` are rebuilt and the next one is locked or not, out[4] = 1 if an update
 * to `key` would be held back (Sec. 3.4) and out[5] = the unit of its stripe that the failed server
 * holds (member index, k for the parity, 0xFFFFFFFF for none).  EINVAL for key >= rows, a bad server
 * or chunk count.
 * ecrm_probe_row_traffic needs no context: it enqueues one kernel that reads `n` rows of 128 floats, alternately
 * from table_a and table_b (device, 8-byte aligned, table_rows rows each), at the row numbers rows[i] (device;
 * the caller keeps them below table_rows -- they are not checked), eight rows in flight per wavefront, and, if
 * `write` is not 0, writes every row back with 1 added -- the access pattern of the update path's tables, for a
 * benchmark that wants to know what the device's memory delivers for it depending on where two tables lie.
 * sink: one device float (only ever written if a sum of loaded values hits a magic number).  A tail of n mod 8
 * rows is left out.  EINVAL for null pointers, n = 0 or n >= 2^32. */
enum { ECRM_PHASE_GROUP = 0, ECRM_PHASE_CHAINS = 1, ECRM_PHASE_APPLY = 2, ECRM_PHASES = 3 };
enum { ECRM_PROFILE_MAX_CALLS = 256, ECRM_LONG_RUN = 1024, ECRM_MID_RUN = 32768 };
enum { ECRM_TUNE_MID_MIN_ROWS = 1 };
int ecrm_tune(ecrm_ctx *ctx, int what, uint64_t value);
int ecrm_probe_row_traffic(float *table_a, float *table_b, uint64_t table_rows, const uint32_t *rows, uint64_t n,
                           int write, float *sink, void *hip_stream);
int ecrm_profile(ecrm_ctx *ctx, int enable);
int ecrm_profile_read(ecrm_ctx *ctx, double *ms, uint64_t *calls);
int ecrm_batch_stats(ecrm_ctx *ctx, void *hip_stream, uint64_t *out);
int ecrm_host_placement(const ecrm_ctx *ctx, uint64_t key, uint32_t failed_server, uint32_t chunks,
                        uint32_t next_chunk, uint32_t locked, uint32_t *out /*[6]*/);

const char *ecrm_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* ECRM_H */
