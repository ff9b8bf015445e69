// C ABI of libecrm: argument validation, scratch layout, and the order in which the kernels of one
// call are enqueued.  No device memory is allocated here; everything lives in caller buffers.
#include <math.h>
#include <mutex>
#include <new>
#include <string.h>

#include "ecrm_internal.h"

using namespace ecrm;

// Where everything lies inside a scratch buffer that serves batches of up to max_batch items.
struct Layout {
    uint32_t max_batch, max_slots, max_pieces, max_blocks;
    size_t bytes;
    size_t off_cnt, off_keys[2], off_vals[2], off_hist, off_bintotal, off_long_slot, off_long_meta,
        off_piece_slot, off_partial, off_partial2, off_long_res, off_active;
};

// The caller's device arrays one update works on.
struct Tables {
    float *E, *A, *PE, *PA;
    unsigned long long *load_data, *load_parity;
};

struct ecrm_ctx {
    ecrm_config cfg;
    Geometry geo;
    int key_bits;
    Layout lay;               // of the scratch buffer the caller binds (sized by cfg.max_batch)
    Layout slay;              // of the library's own fixed scratch array (ecrm_update_static)
    bool has_partial2;
    // bound state
    bool bound, need_init;
    Tables t;
    Scratch s;
    bool have_device;         // cus, grid sizes known (ecrm_bind, or the first ecrm_update_static)
    int grid_blocks;          // 8 blocks of 256 threads per CU, for the streaming kernels
    int cus;
    LaunchGrids lg;           // resident grids of the grid-stride kernels (filled by ecrm_bind)
    uint32_t tune_mid_min_rows;   // ecrm_tune: replaces lg.mid_min_rows when not 0
    // recovery in progress (host-side state machine; the device sees it as a RecoveryView per call)
    RecoveryView rv;
    uint32_t rec_chunks;
    bool rec_decoded;         // the locked chunk's reconstruction has been enqueued
    HoldBuffer hb;            // the caller's recovery buffer, carved
    uint32_t buf_cur;         // which of its two lists is in use
    // profiling
    bool profiling;
    hipEvent_t ev[ECRM_PROFILE_MAX_CALLS][2 * ECRM_PHASES + 1];   // a call with gradient propagation has the phases twice
    bool ev_made;
    uint32_t ev_calls;
};

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// The multiply-and-shift division against the real one, around every place where it could go wrong
// (multiples of the divisor at both ends of the range) and on a spread of other values.
static bool divider_ok(const Divider &v)
{
    const uint32_t d = v.d;
    uint64_t probe = 0x9E3779B97F4A7C15ull;
    for (uint32_t i = 0; i < 4096; ++i) {
        probe = probe * 6364136223846793005ull + 1442695040888963407ull;
        const uint32_t base = i < 64 ? i * d : i < 128 ? 0xFFFFFFFFu - (i - 64) * d : (uint32_t)(probe >> 32);
        for (int delta = -1; delta <= 1; ++delta) {
            const uint32_t n = base + (uint32_t)delta;
            if (v.div(n) != n / d || v.mod(n) != n % d) return false;
        }
    }
    return true;
}

static Layout make_layout(uint32_t max_batch, uint32_t D, uint32_t S, bool has_partial2)
{
    Layout l;
    l.max_batch = max_batch;
    // blocks of a sort launch: large tiles, or small ones for a batch of at most kSmallSortBatch items
    const uint32_t small_tile = kSortThreads * kSmallSortIpt;
    const uint32_t small_blocks = max_batch >= kSmallSortBatch ? kSmallSortBlocks : (max_batch + small_tile - 1) / small_tile;
    l.max_blocks = (max_batch + kSortTile - 1) / kSortTile;
    if (l.max_blocks < small_blocks) l.max_blocks = small_blocks;
    l.max_slots = max_batch / kLongRun + 1;
    l.max_pieces = max_batch / kPieceMin + l.max_slots + 1;
    const size_t n = max_batch;
    size_t off = sizeof(Header);
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    l.off_cnt = take(2 * (size_t)S * sizeof(unsigned long long));
    for (int i = 0; i < 2; ++i) l.off_keys[i] = take(n * 4);
    for (int i = 0; i < 2; ++i) l.off_vals[i] = take(n * 4);
    l.off_hist = take((size_t)kMaxBins * l.max_blocks * 4);
    l.off_bintotal = take(kMaxBins * 4);
    l.off_long_slot = take(n * 4);
    l.off_active = take((n + kChunk - 1) / kChunk * 4);
    l.off_long_meta = take((size_t)(5 + kMidClasses) * l.max_slots * 4);
    l.off_piece_slot = take((size_t)l.max_pieces * 4);
    l.off_partial = take((size_t)l.max_pieces * D * sizeof(double));
    l.off_partial2 = take(has_partial2 ? (size_t)l.max_pieces * D * sizeof(double) : 0);
    l.off_long_res = take((size_t)l.max_slots * 2 * D * sizeof(double));
    l.bytes = off;
    return l;
}

static Scratch carve(const Layout &l, void *base, bool has_partial2)
{
    char *b = (char *)base;
    Scratch s;
    s.hdr = (Header *)b;
    s.cnt = (unsigned long long *)(b + l.off_cnt);
    for (int i = 0; i < 2; ++i) {
        s.keys[i] = (uint32_t *)(b + l.off_keys[i]);
        s.vals[i] = (uint32_t *)(b + l.off_vals[i]);
    }
    s.block_hist = (uint32_t *)(b + l.off_hist);
    s.bin_total = (uint32_t *)(b + l.off_bintotal);
    s.long_slot = (uint32_t *)(b + l.off_long_slot);
    s.active = (uint32_t *)(b + l.off_active);
    uint32_t *meta = (uint32_t *)(b + l.off_long_meta);
    s.long_head = meta;
    s.long_len = meta + (size_t)l.max_slots;
    s.long_piece = meta + (size_t)2 * l.max_slots;
    s.long_count = meta + (size_t)3 * l.max_slots;
    s.long_base = meta + (size_t)4 * l.max_slots;
    s.mid_list = meta + (size_t)5 * l.max_slots;
    s.piece_slot = (uint32_t *)(b + l.off_piece_slot);
    s.partial = (double *)(b + l.off_partial);
    s.partial2 = has_partial2 ? (double *)(b + l.off_partial2) : nullptr;
    s.long_res = (double *)(b + l.off_long_res);
    return s;
}

extern "C" {

const char *ecrm_strerror(int code)
{
    switch (code) {
        case ECRM_OK: return "ok";
        case ECRM_EINVAL: return "invalid argument or configuration";
        case ECRM_ENOTBOUND: return "no device buffers bound";
        case ECRM_ESCRATCH: return "scratch buffer missing, misaligned or too small";
        case ECRM_EBATCH: return "batch larger than max_batch";
        case ECRM_EKEYRANGE: return "a key was >= rows; that batch was not applied";
        case ECRM_EHIP: return "HIP runtime error";
        case ECRM_EBUFFER: return "recovery buffer full; that batch was not applied";
        case ECRM_ESTATE: return "call not allowed in the current recovery state";
        default: return "unknown error";
    }
}

int ecrm_create(const ecrm_config *cfg, ecrm_ctx **out)
{
    if (!cfg || !out) return ECRM_EINVAL;
    *out = nullptr;
    if (cfg->k < 1 || cfg->k > 64) return ECRM_EINVAL;
    if (cfg->rows < cfg->k || cfg->rows % cfg->k != 0 || cfg->rows > 0x100000000ull - 4096) return ECRM_EINVAL;
    if (cfg->dim < 4 || cfg->dim > 1024 || cfg->dim % 4 != 0) return ECRM_EINVAL;
    if (cfg->servers < cfg->k + 1 || cfg->servers > 1024) return ECRM_EINVAL;
    if (cfg->optimizer != ECRM_OPT_ADAGRAD && cfg->optimizer != ECRM_OPT_MOMENTUM) return ECRM_EINVAL;
    if (cfg->combine > 1) return ECRM_EINVAL;
    if (cfg->propagation > ECRM_PROP_NONE) return ECRM_EINVAL;
    if (cfg->propagation == ECRM_PROP_GRADIENT && cfg->combine) return ECRM_EINVAL;
    if (!isfinite(cfg->lr) || !isfinite(cfg->eps) || cfg->eps < 0.0f) return ECRM_EINVAL;
    if (cfg->optimizer == ECRM_OPT_MOMENTUM && !(cfg->momentum >= 0.0f && cfg->momentum < 1.0f)) return ECRM_EINVAL;
    if (cfg->max_batch < 1 || cfg->max_batch > (1ull << 31)) return ECRM_EINVAL;

    ecrm_ctx *c = new (std::nothrow) ecrm_ctx;
    if (!c) return ECRM_EINVAL;
    memset(c, 0, sizeof(*c));
    c->cfg = *cfg;
    c->geo.D = cfg->dim;
    c->geo.k = cfg->k;
    c->geo.S = cfg->servers;
    c->geo.rows = (uint32_t)cfg->rows;
    c->geo.nc = cfg->dim <= 128 ? 1 : 2;
    c->geo.ncb = (cfg->dim + c->geo.nc * 128 - 1) / (c->geo.nc * 128);
    c->geo.lr = cfg->lr;
    c->geo.eps = cfg->eps;
    c->geo.mu = cfg->optimizer == ECRM_OPT_MOMENTUM ? cfg->momentum : 0.0f;
    c->geo.mode = cfg->optimizer + 2u * cfg->combine;
    c->geo.dk = make_divider(cfg->k);
    c->geo.dS = make_divider(cfg->servers);
    if (!divider_ok(c->geo.dk) || !divider_ok(c->geo.dS)) {
        delete c;
        return ECRM_EINVAL;
    }
    c->key_bits = 1;
    while (c->key_bits < 32 && (1ull << c->key_bits) < cfg->rows) ++c->key_bits;
    c->has_partial2 = cfg->optimizer == ECRM_OPT_MOMENTUM && !cfg->combine;
    c->lay = make_layout((uint32_t)cfg->max_batch, cfg->dim, cfg->servers, c->has_partial2);
    c->slay = make_layout(ECRM_STATIC_MAX_BATCH, cfg->dim, cfg->servers, c->has_partial2);
    *out = c;
    return ECRM_OK;
}

void ecrm_destroy(ecrm_ctx *c)
{
    if (!c) return;
    if (c->ev_made)
        for (int i = 0; i < ECRM_PROFILE_MAX_CALLS; ++i)
            for (int j = 0; j <= 2 * ECRM_PHASES; ++j) (void)hipEventDestroy(c->ev[i][j]);
    delete c;
}

size_t ecrm_data_bytes(const ecrm_ctx *c) { return c ? (size_t)c->cfg.rows * c->cfg.dim * 4 : 0; }
size_t ecrm_parity_bytes(const ecrm_ctx *c) { return c ? (size_t)(c->cfg.rows / c->cfg.k) * c->cfg.dim * 4 : 0; }
size_t ecrm_scratch_bytes(const ecrm_ctx *c) { return c ? c->lay.bytes : 0; }

static bool aligned(const void *p, size_t a) { return p && ((uintptr_t)p % a) == 0; }

// Learns the device the context runs on (compute units, resident grid sizes), once.  Host-side queries
// only; nothing is enqueued.
static int learn_device(ecrm_ctx *c)
{
    if (c->have_device) return ECRM_OK;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ECRM_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return ECRM_EHIP;
    LaunchGrids lg;
    if (!query_launch_grids(c->geo, cus, &lg)) return ECRM_EHIP;
    c->lg = lg;
    c->cus = cus;
    c->grid_blocks = cus * 8;     // 8 x 256 threads = the 2048 threads a CU can hold
    c->have_device = true;
    return ECRM_OK;
}

int ecrm_bind(ecrm_ctx *c, float *E, float *A, float *PE, float *PA, uint64_t *load_data,
              uint64_t *load_parity, void *scratch, size_t scratch_bytes)
{
    if (!c) return ECRM_EINVAL;
    if (c->rv.active) return ECRM_ESTATE;      // updates are waiting in the recovery buffer: binding would drop them
    if (!aligned(E, 16) || !aligned(A, 16) || !aligned(PE, 16) || !aligned(PA, 16)) return ECRM_EINVAL;
    if (!aligned(load_data, 8) || !aligned(load_parity, 8)) return ECRM_EINVAL;
    if (!aligned(scratch, 256) || scratch_bytes < c->lay.bytes) return ECRM_ESCRATCH;
    const int rc = learn_device(c);
    if (rc != ECRM_OK) return rc;

    c->s = carve(c->lay, scratch, c->has_partial2);
    c->t.E = E; c->t.A = A; c->t.PE = PE; c->t.PA = PA;
    c->t.load_data = (unsigned long long *)load_data;
    c->t.load_parity = (unsigned long long *)load_parity;
    c->bound = true;
    c->need_init = true;      // the first enqueue clears the header on its stream
    return ECRM_OK;
}

static int check_launch()
{
    return hipGetLastError() == hipSuccess ? ECRM_OK : ECRM_EHIP;
}

static void init_if_needed(ecrm_ctx *c, hipStream_t st)
{
    if (c->need_init) {
        launch_reset(c->s, c->geo.S, 0, true, kCallerBatch, st);
        c->need_init = false;
    }
}

int ecrm_encode(ecrm_ctx *c, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (c->rv.active) return ECRM_ESTATE;      // rows of the lost server are not there to be summed
    launch_encode(c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, c->grid_blocks, (hipStream_t)stream);
    return check_launch();
}

int ecrm_route(ecrm_ctx *c, const uint64_t *keys, uint64_t n, uint64_t *stripe, uint32_t *member,
               uint32_t *data_srv, uint32_t *parity_srv, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (n == 0) return ECRM_OK;
    if (!aligned(keys, 8)) return ECRM_EINVAL;
    init_if_needed(c, (hipStream_t)stream);
    launch_route(c->s, c->geo, keys, n, stripe, member, data_srv, parity_srv, (hipStream_t)stream);
    return check_launch();
}

// One batch through the whole pipeline, on tables t with scratch s (laid out by l).  During a recovery,
// held-back items are appended to buf[target] (and the key space gets one more value, `rows`, for them
// to sort behind the rest).
static int run_update(ecrm_ctx *c, const Tables &t, const Scratch &s, const Layout &l, const RecoveryView &rv,
                      bool clear_sticky, BatchSource src, const uint64_t *keys, const float *grads, uint32_t n32,
                      hipStream_t st)
{
    // a replay of the waiting updates: n32 only bounds their number, the kernels read the count on the device
    const uint32_t *n_dev = src == kWaitingUpdates ? &s.hdr->n_batch : nullptr;
    hipEvent_t *ev = nullptr;
    if (c->profiling && c->ev_calls < ECRM_PROFILE_MAX_CALLS) ev = c->ev[c->ev_calls++];

    launch_reset(s, c->geo.S, n32, clear_sticky, src, st);
    if (ev) (void)hipEventRecord(ev[0], st);
    int key_bits = c->key_bits;
    if (rv.active)
        while (key_bits < 32 && (1ull << key_bits) <= c->cfg.rows) ++key_bits;
    const uint32_t prop = c->cfg.propagation;
    LaunchGrids lg = c->lg;
    if (c->tune_mid_min_rows) lg.mid_min_rows = c->tune_mid_min_rows;
    uint32_t *sk = nullptr, *si = nullptr;
    launch_sort(s, c->geo, rv, keys, n32, n_dev, src, key_bits, false, true, &sk, &si, st);
    if (rv.active || src == kWaitingUpdates)
        launch_hold_back(s, c->geo, rv, keys, grads, n32, src, c->hb, c->buf_cur, st);
    if (ev) (void)hipEventRecord(ev[1], st);
    launch_chains(s, c->geo, lg, t.A, grads, sk, si, n32, l.max_slots, l.max_pieces, c->cus, st);
    launch_active_groups(s, c->geo, sk, n32, st);
    if (ev) (void)hipEventRecord(ev[2], st);
    const bool diff = prop == ECRM_PROP_DIFFERENCE;
    launch_apply(s, c->geo, lg, t.E, t.A, diff ? t.PE : nullptr, diff ? t.PA : nullptr, t.load_data,
                 prop == ECRM_PROP_NONE ? nullptr : t.load_parity, grads, sk, si, n32, c->cus, st);
    if (prop == ECRM_PROP_GRADIENT) {
        // The strawman of Sec. 3.3.1: the parity server receives the gradient itself and applies the
        // optimizer to the parity entry with the parity's own state.  The same pipeline once more,
        // with the parity tables as the tables, grouped by stripe, every update of a stripe in
        // arrival order.
        Geometry gp = c->geo;
        gp.k = 1;
        int bits = 1;
        while (bits < 32 && (1ull << bits) < c->cfg.rows / c->cfg.k) ++bits;
        if (ev) (void)hipEventRecord(ev[3], st);
        launch_reset(s, c->geo.S, n32, false, kCallerBatch, st);
        launch_sort(s, c->geo, rv, keys, n32, nullptr, kCallerBatch, bits, true, false, &sk, &si, st);
        if (ev) (void)hipEventRecord(ev[4], st);
        launch_chains(s, gp, lg, t.PA, grads, sk, si, n32, l.max_slots, l.max_pieces, c->cus, st);
        launch_active_groups(s, gp, sk, n32, st);
        if (ev) (void)hipEventRecord(ev[5], st);
        launch_apply(s, gp, lg, t.PE, t.PA, nullptr, nullptr, nullptr, nullptr, grads, sk, si, n32, c->cus, st);
        if (ev) (void)hipEventRecord(ev[6], st);
    } else if (ev) {
        (void)hipEventRecord(ev[3], st);
    }
    return check_launch();
}

static int run_bound_update(ecrm_ctx *c, BatchSource src, const uint64_t *keys, const float *grads, uint32_t n32,
                            hipStream_t st)
{
    const bool clear = c->need_init;
    c->need_init = false;
    return run_update(c, c->t, c->s, c->lay, c->rv, clear, src, keys, grads, n32, st);
}

int ecrm_update(ecrm_ctx *c, const uint64_t *keys, const float *grads, uint64_t n, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (n > c->lay.max_batch) return ECRM_EBATCH;
    if (n == 0) return ECRM_OK;
    if (!aligned(keys, 8) || !aligned(grads, 16)) return ECRM_EINVAL;
    return run_bound_update(c, kCallerBatch, keys, grads, (uint32_t)n, (hipStream_t)stream);
}

// ---- ecrm_update for callers that cannot provide a scratch buffer --------------------------------
// The scratch buffer of this entry point lives in the library's image: one copy per GPU, held until the
// process ends.  In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char g_static_scratch[ECRM_STATIC_SCRATCH_BYTES];

enum { kMaxDevices = 64 };
static void *g_static_ptr[kMaxDevices];          // device address of g_static_scratch on each device
static std::mutex g_static_mutex;

static int static_scratch_of_current_device(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ECRM_EHIP;
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_static_scratch)) != hipSuccess || !p) return ECRM_EHIP;
        g_static_ptr[dev] = p;
    }
    *out = g_static_ptr[dev];
    return ECRM_OK;
}

// h == nullptr: an empty batch, nothing can have been rejected
__global__ void publish_rejected_kernel(const Header *h, uint32_t *rejected)
{
    if (threadIdx.x == 0) *rejected = h ? h->batch_bad : 0u;
}

int ecrm_update_static(ecrm_ctx *c, float *E, float *A, float *PE, float *PA, uint64_t *load_data,
                       uint64_t *load_parity, const uint64_t *keys, const float *grads, uint64_t n,
                       uint32_t *rejected, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (c->rv.active) return ECRM_ESTATE;              // the recovery protocol lives in the bound scratch buffer
    if (n > ECRM_STATIC_MAX_BATCH) return ECRM_EBATCH;
    if (c->slay.bytes > ECRM_STATIC_SCRATCH_BYTES) return ECRM_ESCRATCH;   // this geometry needs more than the fixed array
    if (!aligned(E, 16) || !aligned(A, 16) || !aligned(load_data, 8)) return ECRM_EINVAL;
    if (c->cfg.propagation != ECRM_PROP_NONE && (!aligned(PE, 16) || !aligned(PA, 16) || !aligned(load_parity, 8)))
        return ECRM_EINVAL;
    if (rejected && !aligned(rejected, 4)) return ECRM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    if (n == 0) {
        if (!rejected) return ECRM_OK;
        hipLaunchKernelGGL(publish_rejected_kernel, dim3(1), dim3(64), 0, st, (const Header *)nullptr, rejected);
        return check_launch();
    }
    if (!aligned(keys, 8) || !aligned(grads, 16)) return ECRM_EINVAL;
    int rc = learn_device(c);
    if (rc != ECRM_OK) return rc;
    void *base = nullptr;
    rc = static_scratch_of_current_device(&base);
    if (rc != ECRM_OK) return rc;
    const Scratch s = carve(c->slay, base, c->has_partial2);
    Tables t;
    t.E = E; t.A = A; t.PE = PE; t.PA = PA;
    t.load_data = (unsigned long long *)load_data;
    t.load_parity = (unsigned long long *)load_parity;
    RecoveryView none;
    memset(&none, 0, sizeof(none));
    // the array keeps the last call's contents: the reset kernel clears every field of the header,
    // the per-server counts and (clear_sticky) the status word; everything else is written before it is read
    rc = run_update(c, t, s, c->slay, none, true, kCallerBatch, keys, grads, (uint32_t)n, st);
    if (rc == ECRM_OK && rejected) {
        hipLaunchKernelGGL(publish_rejected_kernel, dim3(1), dim3(64), 0, st, s.hdr, rejected);
        rc = check_launch();
    }
    return rc;
}

int ecrm_recovery_begin(ecrm_ctx *c, uint32_t server, uint32_t chunks, uint64_t *buf_keys, float *buf_grads,
                        uint64_t capacity, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (c->rv.active) return ECRM_ESTATE;
    if (c->cfg.propagation != ECRM_PROP_DIFFERENCE) return ECRM_EINVAL;   // no parities a decoder could trust
    // Synchronous (combined) training takes ONE step per modified entry and training step; replaying
    // the waiting updates of several steps in one call would merge them into a single step.
    if (c->cfg.combine) return ECRM_EINVAL;
    const uint32_t stripes = c->geo.rows / c->geo.k;
    if (server >= c->geo.S || chunks < 1 || chunks > stripes) return ECRM_EINVAL;
    if (capacity < 1 || capacity > c->lay.max_batch || !aligned(buf_keys, 8) || !aligned(buf_grads, 16)) return ECRM_EINVAL;
    const uint32_t spc = (uint32_t)(((uint64_t)stripes + chunks - 1) / chunks);   // 64-bit: the sum can pass 2^32
    const Divider spc_div = make_divider(spc);
    if (!divider_ok(spc_div)) return ECRM_EINVAL;
    c->rv.active = 1;
    c->rv.server = server;
    c->rv.next = 0;
    c->rv.locked = 0;
    c->rv.stripes_per_chunk = spc;
    c->rv.dspc = spc_div;
    c->rec_chunks = (uint32_t)(((uint64_t)stripes + spc - 1) / spc);
    // The caller's buffer: two lists of `capacity` entries (key and row-pool slot in 64 bits); a pool of
    // `capacity` gradient rows; and, in the memory behind the pool, the released slots.
    c->hb.cap = (uint32_t)capacity;
    c->hb.list[0] = (unsigned long long *)buf_keys;
    c->hb.list[1] = (unsigned long long *)buf_keys + capacity;
    c->hb.rows = buf_grads;
    c->hb.free_list = (uint32_t *)(buf_grads + capacity * c->geo.D);
    c->buf_cur = 0;
    init_if_needed(c, (hipStream_t)stream);
    launch_clear_buffer(c->s, (hipStream_t)stream);
    return check_launch();
}

int ecrm_recovery_lock(ecrm_ctx *c)
{
    if (!c) return ECRM_EINVAL;
    if (!c->rv.active || c->rv.locked || c->rv.next >= c->rec_chunks) return ECRM_ESTATE;
    c->rv.locked = 1;
    c->rec_decoded = false;
    return ECRM_OK;
}

int ecrm_recovery_decode(ecrm_ctx *c, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->rv.active || !c->rv.locked) return ECRM_ESTATE;
    const uint64_t stripes = c->geo.rows / c->geo.k;
    const uint64_t lo = (uint64_t)c->rv.next * c->rv.stripes_per_chunk;
    const uint64_t hi = lo + c->rv.stripes_per_chunk < stripes ? lo + c->rv.stripes_per_chunk : stripes;
    // a grid sized to the chunk, not a resident one: the decoder is meant to run beside the updates of
    // another stream, which must be able to get onto the device while it runs
    launch_recover_range(c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, c->rv.server, (uint32_t)lo, (uint32_t)hi, 0,
                         (hipStream_t)stream);
    const int rc = check_launch();
    if (rc == ECRM_OK) c->rec_decoded = true;
    return rc;
}

int ecrm_recovery_unlock(ecrm_ctx *c, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->rv.active || !c->rv.locked || !c->rec_decoded) return ECRM_ESTATE;   // nothing rebuilt: lost rows would be trained on
    hipStream_t st = (hipStream_t)stream;
    c->rv.locked = 0;
    c->rv.next += 1;
    // Replay of everything that is waiting, under the new state of the recovery: what the released chunk
    // held is applied, what must go on waiting moves to the other list (its gradient row stays where it
    // is).  How many updates are waiting is known on the device only: the launches are sized by the
    // buffer's capacity and the kernels read the count there -- nothing here waits for the stream.
    const int rc = run_bound_update(c, kWaitingUpdates, (const uint64_t *)c->hb.list[c->buf_cur], c->hb.rows, c->hb.cap, st);
    c->buf_cur ^= 1u;
    if (c->rv.next >= c->rec_chunks) c->rv.active = 0;       // every chunk is rebuilt, nothing can be waiting any more
    return rc;
}

int ecrm_recovery_state(ecrm_ctx *c, void *stream, uint32_t *active, uint32_t *next_chunk, uint32_t *chunks,
                        uint64_t *buffered)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ECRM_EHIP;
    Header h;
    memset(&h, 0, sizeof(h));
    if (!c->need_init && hipMemcpy(&h, c->s.hdr, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return ECRM_EHIP;
    if (active) *active = c->rv.active;
    if (next_chunk) *next_chunk = c->rv.next;
    if (chunks) *chunks = c->rec_chunks;
    if (buffered) *buffered = h.buf_count;
    return ECRM_OK;
}

int ecrm_recovery_read(ecrm_ctx *c, const uint64_t *keys, uint64_t n, float *out_E, float *out_A, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (n == 0) return ECRM_OK;
    if (!aligned(keys, 8) || !aligned(out_E, 16) || (out_A && !aligned(out_A, 16))) return ECRM_EINVAL;
    hipStream_t st = (hipStream_t)stream;
    init_if_needed(c, st);
    if (!c->rv.active) {                       // no recovery in progress: a plain gather
        launch_degraded_read(c->s, c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, keys, n, ECRM_NO_SERVER, out_E, out_A,
                             c->grid_blocks, st);
        return check_launch();
    }
    // The waiting updates, grouped by entry with the update path's own sort on the list's keys.  How
    // many there are is known on the device only: the launches are sized by the buffer's capacity.
    uint32_t *bk = nullptr, *bi = nullptr;
    RecoveryView none;
    memset(&none, 0, sizeof(none));
    launch_sort(c->s, c->geo, none, (const uint64_t *)c->hb.list[c->buf_cur], c->hb.cap, &c->s.hdr->buf_count, kWaitingUpdates,
                c->key_bits, false, false, &bk, &bi, st);
    launch_recovery_read(c->s, c->geo, c->rv, c->t.E, c->t.A, c->t.PE, c->t.PA, keys, n, bk, bi, &c->s.hdr->buf_count,
                         c->hb.rows, out_E, out_A, c->grid_blocks, st);
    return check_launch();
}

int ecrm_fail_server(ecrm_ctx *c, uint32_t server, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (server >= c->geo.S) return ECRM_EINVAL;
    if (c->rv.active) return ECRM_ESTATE;      // a second loss during a recovery is more than r = 1 tolerates
    launch_fail_server(c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, server, c->grid_blocks, (hipStream_t)stream);
    return check_launch();
}

int ecrm_recover_server(ecrm_ctx *c, uint32_t server, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (server >= c->geo.S) return ECRM_EINVAL;
    if (c->rv.active) return ECRM_ESTATE;      // the chunked protocol is rebuilding; updates are waiting for it
    launch_recover_server(c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, server, c->grid_blocks, (hipStream_t)stream);
    return check_launch();
}

int ecrm_degraded_read(ecrm_ctx *c, const uint64_t *keys, uint64_t n, uint32_t lost_server, float *out_E,
                       float *out_A, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (lost_server != ECRM_NO_SERVER && lost_server >= c->geo.S) return ECRM_EINVAL;
    if (n == 0) return ECRM_OK;
    if (!aligned(keys, 8) || !aligned(out_E, 16) || (out_A && !aligned(out_A, 16))) return ECRM_EINVAL;
    init_if_needed(c, (hipStream_t)stream);
    launch_degraded_read(c->s, c->geo, c->t.E, c->t.A, c->t.PE, c->t.PA, keys, n, lost_server, out_E, out_A,
                         c->grid_blocks, (hipStream_t)stream);
    return check_launch();
}

int ecrm_status(ecrm_ctx *c, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ECRM_EHIP;
    if (c->need_init) return ECRM_OK;      // nothing was ever enqueued
    Header h;
    if (hipMemcpy(&h, c->s.hdr, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return ECRM_EHIP;
    if (hipGetLastError() != hipSuccess) return ECRM_EHIP;
    if (h.err_sticky & 1u) return ECRM_EKEYRANGE;
    return (h.err_sticky & 2u) ? ECRM_EBUFFER : ECRM_OK;
}

int ecrm_clear_status(ecrm_ctx *c, void *stream)
{
    if (!c) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (c->need_init) return ECRM_OK;
    launch_clear_status(c->s, (hipStream_t)stream);
    return check_launch();
}

int ecrm_batch_stats(ecrm_ctx *c, void *stream, uint64_t *out)
{
    if (!c || !out) return ECRM_EINVAL;
    if (!c->bound) return ECRM_ENOTBOUND;
    if (hipStreamSynchronize((hipStream_t)stream) != hipSuccess) return ECRM_EHIP;
    Header h;
    memset(&h, 0, sizeof(h));
    if (!c->need_init && hipMemcpy(&h, c->s.hdr, sizeof(h), hipMemcpyDeviceToHost) != hipSuccess) return ECRM_EHIP;
    out[0] = h.n_long;
    out[1] = h.n_pieces;
    out[2] = h.n_long_items;
    out[3] = h.batch_bad;
    out[4] = 0;
    for (uint32_t cl = 0; cl < kMidClasses; ++cl) out[4] += h.n_mid[cl];
    return ECRM_OK;
}

// Host-side evaluation of the 32-bit index arithmetic the kernels use (the multiply-and-shift
// divisions, the hold-back rule, the unit a server holds): the same inline functions, compiled for
// the host, so that a test can compare them with plain 64-bit arithmetic over the whole row range.
int ecrm_host_placement(const ecrm_ctx *c, uint64_t key, uint32_t failed_server, uint32_t chunks,
                        uint32_t next_chunk, uint32_t locked, uint32_t *out)
{
    if (!c || !out || key >= c->cfg.rows || failed_server >= c->geo.S) return ECRM_EINVAL;
    const uint32_t stripes = c->geo.rows / c->geo.k;
    if (chunks < 1 || chunks > stripes) return ECRM_EINVAL;
    const uint32_t x = (uint32_t)key, k = c->geo.k;
    const uint32_t g = c->geo.dk.div(x), j = x - g * k;
    out[0] = g;
    out[1] = j;
    out[2] = c->geo.dS.mod(g + 1 + j);
    out[3] = c->geo.dS.mod(g);
    RecoveryView rv;
    memset(&rv, 0, sizeof(rv));
    rv.active = 1;
    rv.server = failed_server;
    rv.next = next_chunk;
    rv.locked = locked ? 1u : 0u;
    rv.stripes_per_chunk = (uint32_t)(((uint64_t)stripes + chunks - 1) / chunks);
    rv.dspc = make_divider(rv.stripes_per_chunk);
    if (!divider_ok(rv.dspc)) return ECRM_EINVAL;
    out[4] = held_back(rv, x, c->geo.dk, c->geo.dS) ? 1u : 0u;
    out[5] = (uint32_t)unit_on_server(g, k, c->geo.S, failed_server);
    return ECRM_OK;
}

int ecrm_tune(ecrm_ctx *c, int what, uint64_t value)
{
    if (!c) return ECRM_EINVAL;
    if (what != ECRM_TUNE_MID_MIN_ROWS || value > 0xFFFFFFFFull) return ECRM_EINVAL;
    c->tune_mid_min_rows = (uint32_t)value;
    return ECRM_OK;
}

int ecrm_profile(ecrm_ctx *c, int enable)
{
    if (!c) return ECRM_EINVAL;
    if (enable && !c->ev_made) {
        const int per_call = 2 * ECRM_PHASES + 1;
        for (int e = 0; e < ECRM_PROFILE_MAX_CALLS * per_call; ++e) {
            if (hipEventCreate(&c->ev[e / per_call][e % per_call]) != hipSuccess) {
                while (--e >= 0) (void)hipEventDestroy(c->ev[e / per_call][e % per_call]);
                return ECRM_EHIP;
            }
        }
        c->ev_made = true;
    }
    c->profiling = enable != 0;
    return ECRM_OK;
}

int ecrm_profile_read(ecrm_ctx *c, double *ms, uint64_t *calls)
{
    if (!c || !ms || !calls) return ECRM_EINVAL;
    for (int j = 0; j < ECRM_PHASES; ++j) ms[j] = 0.0;
    *calls = c->ev_calls;
    for (uint32_t i = 0; i < c->ev_calls; ++i) {
        const int sets = c->cfg.propagation == ECRM_PROP_GRADIENT ? 2 : 1;
        if (hipEventSynchronize(c->ev[i][sets * ECRM_PHASES]) != hipSuccess) return ECRM_EHIP;
        for (int j = 0; j < sets * ECRM_PHASES; ++j) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, c->ev[i][j], c->ev[i][j + 1]) != hipSuccess) return ECRM_EHIP;
            ms[j % ECRM_PHASES] += (double)t;
        }
    }
    c->ev_calls = 0;
    return ECRM_OK;
}

}  // extern "C"
