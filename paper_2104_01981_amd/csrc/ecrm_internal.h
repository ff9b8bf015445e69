// Internal declarations shared by the HIP sources of libecrm (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ecrm.h"

namespace ecrm {

// ---- tuning constants -------------------------------------------------------------------------
constexpr int kWave = 64;            // CDNA wavefront

constexpr int kSortThreads = 512;    // 8 waves per sort block
constexpr int kSortWaves = kSortThreads / kWave;
#ifndef ECRM_SORT_IPT
#define ECRM_SORT_IPT 12
#endif
constexpr int kSortIpt = ECRM_SORT_IPT;   // items per thread
constexpr int kSortTile = kSortThreads * kSortIpt;   // 6144 items per block: 68 KB of LDS, two blocks per CU
// Batches of at most kSmallSortBatch items are sorted in tiles of kSortThreads * kSmallSortIpt items instead: with
// the large tile a 2^16-item batch would occupy 11 of the compute units.
constexpr int kSmallSortIpt = 2;
constexpr uint32_t kSmallSortBatch = 1u << 19;
constexpr uint32_t kSmallSortBlocks = kSmallSortBatch / (kSortThreads * kSmallSortIpt);
constexpr int kMaxRadixBits = 9;
constexpr int kMaxBins = 1 << kMaxRadixBits;
// Rows with more updates than this use the split-chain path (their gradients are read twice there);
// shorter runs are walked by one wave inside the apply kernel (read once, but at one wave's pace).
// Measured: 256 -> 1024 takes 6 % off the Zipf-only workload and 0.5 % off the mixed one; 2048 loses.
constexpr uint32_t kLongRun = ECRM_LONG_RUN;
constexpr uint32_t kPieceMin = 128;  // smallest chain piece (what the scratch buffer is sized for) ...
constexpr uint32_t kPieceMinCap = 2048;   // ... and the largest value the plan kernel raises that minimum to
constexpr uint32_t kLongRowGuess = 6144;  // updates a long row is taken to have when the piece size is chosen
constexpr uint32_t kPieceMaxCount = 1024;     // a chain is cut into at most this many pieces
// Adagrad runs of more than kLongRun and at most kMidMax updates are walked by ONE workgroup that keeps the
// gradients in registers between the sum of squares and the steps (one read); only longer runs, which need
// many workgroups, go through the pieces and read their gradients twice.  0 = no such tier.  One workgroup
// takes ~0.5 ms over 32768 updates, so this pays only when there are enough such runs to keep every
// workgroup busy meanwhile: with fewer than kMidMinRowsPerBlock long rows per resident workgroup all runs
// go through the pieces (measured: 3801 long rows, 49 % of 2^26 updates -- chains 6.8 -> 5.2 ms; 420 long
// rows in 2^24 updates -- 0.66 -> 1.1 ms if the tier were used there).
constexpr uint32_t kMidMax = ECRM_MID_RUN;
constexpr uint32_t kMidMinRowsPerBlock = 4;
constexpr int kMidWaves = 8;         // waves of the workgroup that walks such a run
constexpr uint32_t kMidClasses = 7;  // the runs are listed by length (x2 per class) and taken longest first
#ifndef ECRM_CHUNK
#define ECRM_CHUNK 16
#endif
constexpr uint32_t kChunk = ECRM_CHUNK;   // sorted positions whose stripes one wave owns per grid-stride step (<= 63)
constexpr uint32_t kNoKey = 0xFFFFFFFFu;

// ---- device-side header at the start of the scratch buffer --------------------------------------
struct Header {
    uint32_t err_sticky;   // set once any batch carried a key >= rows
    uint32_t batch_bad;    // same, for the batch in flight (cleared by reset)
    uint32_t n_long;       // rows on the split-chain path in this batch
    uint32_t n_pieces;     // chain pieces in this batch
    unsigned long long n_long_items;
    uint32_t n_valid;      // items of the batch that are applied now; the rest (held back during a recovery)
                           // carry the row id `rows` and sort behind them
    uint32_t n_held;       // items of the batch held back
    uint32_t buf_count;    // held-back items waiting in the buffer (all batches)
    uint32_t apply_ticket; // next group of sorted positions the apply kernel hands out (cleared by reset)
    uint32_t n_batch;      // items of the batch in flight: the caller's n, or -- when the waiting updates are
                           // replayed -- what buf_count was when the replay started (set by reset)
    uint32_t free_count;   // slots of the recovery buffer's row pool that were released and can be reused
    uint32_t bump;         // slots of the row pool that have ever been handed out
    uint32_t n_mid[kMidClasses];   // long rows of this batch that one workgroup walks, by length class
    uint32_t mid_ticket;   // next of them to be handed out (cleared by reset)
    uint32_t n_active;     // groups of sorted positions the apply kernel has work for (cleared by reset)
    uint32_t pad[42];
};
static_assert(sizeof(Header) == 256, "header is one 256-byte block");

struct Scratch {           // device pointers carved out of the caller's scratch buffer
    Header *hdr;
    unsigned long long *cnt;       // [2*S] per-batch server counters (data, then parity)
    uint32_t *keys[2];             // ping-pong sort buffers (row ids)
    uint32_t *vals[2];             // ping-pong sort buffers (item indices)
    uint32_t *block_hist;          // [bins][nblocks]
    uint32_t *bin_total;           // [bins]
    uint32_t *long_slot;           // [n] slot id, valid at heads of long rows only
    uint32_t *active;              // [ceil(n / kChunk)] groups of sorted positions in which a stripe begins
    uint32_t *long_head, *long_len, *long_piece, *long_count, *long_base;   // [max_slots]
    uint32_t *mid_list;            // [kMidClasses][max_slots] slots of the rows one workgroup walks
    uint32_t *piece_slot;          // [max_pieces]
    double *partial;               // [max_pieces][D]
    double *partial2;              // [max_pieces][D], momentum SGD only (else null)
    double *long_res;              // [max_slots][2][D]: sum of steps, final accumulator
};

// Division of 32-bit numbers by a divisor fixed for the life of a context (k, S, stripes per chunk):
// multiply-high and two shifts instead of the long sequence a division by a run-time value costs --
// the placement arithmetic runs once per item in four kernels while a recovery is in progress.
// q = (t + ((n - t) >> s1)) >> s2 with t = hi32(m * n), m = floor(2^32 (2^l - d) / d) + 1,
// l = ceil(log2 d), s1 = min(l, 1), s2 = max(l - 1, 0): exact for every 32-bit n.
struct Divider {
    uint32_t d, m, s1, s2;
    __host__ __device__ __forceinline__ uint32_t div(uint32_t n) const
    {
#ifdef __HIP_DEVICE_COMPILE__
        const uint32_t t = __umulhi(m, n);
#else
        const uint32_t t = (uint32_t)(((unsigned long long)m * n) >> 32);
#endif
        return (t + ((n - t) >> s1)) >> s2;
    }
    __host__ __device__ __forceinline__ uint32_t mod(uint32_t n) const { return n - div(n) * d; }
};
inline Divider make_divider(uint32_t d)
{
    uint32_t l = 0;
    while (l < 32 && (1ull << l) < d) ++l;
    Divider r;
    r.d = d;
    r.m = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
    r.s1 = l < 1 ? l : 1;
    r.s2 = l ? l - 1 : 0;
    return r;
}

// What an update has to know about a recovery in progress (Sec. 3.4): stripes are split into
// `chunks` equal ranges; chunks below `next` are rebuilt, chunk `next` is being rebuilt if `locked`.
// An update is held back (buffered) if its stripe is in the locked chunk, or if its own entry is
// the unit the failed server held and has not been rebuilt yet.
struct RecoveryView {
    uint32_t active, server, next, locked;
    uint32_t stripes_per_chunk;
    Divider dspc;          // by stripes_per_chunk
};
__host__ __device__ __forceinline__ bool held_back(const RecoveryView &r, uint32_t x, const Divider &dk, const Divider &dS)
{
    if (!r.active) return false;
    const uint32_t k = dk.d, S = dS.d;
    const uint32_t g = dk.div(x), j = x - g * k;
    const uint32_t p = dS.mod(g);
    uint32_t lost = k;                                // unit of stripe g on the failed server: k = its parity
    if (p != r.server) {
        const uint32_t q = p + 1u == S ? 0u : p + 1u; // (g+1) mod S
        lost = r.server + S - q;                      // in [1, 2S): (g+1+lost) mod S == server
        if (lost >= S) lost -= S;
        if (lost >= k) return false;                  // the stripe has nothing on the failed server
    }
    const uint32_t c = r.dspc.div(g);
    if (c < r.next) return false;                     // already rebuilt
    if (c == r.next && r.locked) return true;         // being rebuilt right now
    return lost == j;                                 // not rebuilt yet: only the lost entry itself waits
}

// which unit of stripe g does `server` hold: -1 none, k the parity, j < k member j
__host__ __device__ __forceinline__ int unit_on_server(uint32_t g, uint32_t k, uint32_t S, uint32_t server)
{
    const uint32_t p = g % S;
    if (p == server) return (int)k;
    const uint32_t j = (server + S - (p + 1u) % S) % S;      // (g+1+j) mod S == server  <=>  j == server - (p+1) mod S
    return j < k ? (int)j : -1;
}

struct Geometry {
    uint32_t D, k, S;
    uint32_t rows;         // R (< 2^32)
    uint32_t nc;           // 128-float chunks a lane holds at once (1 or 2)
    uint32_t ncb;          // column blocks of nc*128 floats that cover D
    float lr, eps;
    float mu;              // momentum coefficient (momentum SGD only)
    uint32_t mode;         // optimizer + 2 * combine: which update rule the kernels are instantiated for
    Divider dk, dS;        // by k and by S
};

// Grid sizes of the grid-stride kernels for one geometry: exactly the blocks that are resident at
// once.  Filled once per context when it learns its device (never inside a stream capture).
struct LaunchGrids {
    int p1, p3;            // chain pieces: summaries, steps
    int mid;               // runs walked by one workgroup
    uint32_t mid_min_rows; // ... which is done only in batches with at least this many long rows
    int apply, rows;       // apply with / without the parity rows
};
bool query_launch_grids(const Geometry &g, int cus, LaunchGrids *out);   // false: an occupancy query failed
bool query_chain_grids(const Geometry &g, int cus, LaunchGrids *out);    // its p1, p3, mid, mid_min_rows part

// ---- launchers (each checks nothing: the API layer validates shapes before calling) -------------
// Where a batch comes from.  kCallerBatch: n keys of the caller with gradient row i for item i.
// kWaitingUpdates: the entries of the recovery buffer's list -- (key, row-pool slot) packed into 64 bits --
// of which only the device knows how many there are (n is then an upper bound that sizes the grids).
enum BatchSource { kCallerBatch = 0, kWaitingUpdates = 1 };
// The buffer of a recovery in progress (Sec. 3.4): a pool of gradient rows addressed by slot, two lists
// of waiting updates (the one in use and the one the next replay builds), and the released slots.
struct HoldBuffer {
    unsigned long long *list[2];   // [cap] each: key | slot << 32, in arrival order
    float *rows;                   // [cap][D]
    uint32_t *free_list;           // [cap]
    uint32_t cap;
};
void launch_reset(const Scratch &s, uint32_t S, uint32_t n, bool clear_sticky, BatchSource src, hipStream_t st);
// n_dev (may be null): device word holding the true item count when n is only its upper bound
void launch_sort(const Scratch &s, const Geometry &g, const RecoveryView &rv, const uint64_t *keys, uint32_t n,
                 const uint32_t *n_dev, BatchSource src, int key_bits, bool by_stripe, bool count_servers,
                 uint32_t **sorted_keys, uint32_t **sorted_vals, hipStream_t st);
void launch_hold_back(const Scratch &s, const Geometry &g, const RecoveryView &rv, const uint64_t *keys,
                      const float *grads, uint32_t n, BatchSource src, const HoldBuffer &hb, uint32_t cur,
                      hipStream_t st);
void launch_recover_range(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                          uint32_t g_lo, uint32_t g_hi, int grid_blocks, hipStream_t st);
void launch_clear_buffer(const Scratch &s, hipStream_t st);
void launch_active_groups(const Scratch &s, const Geometry &g, const uint32_t *sk, uint32_t n, hipStream_t st);
void launch_chains(const Scratch &s, const Geometry &g, const LaunchGrids &lg, const float *A, const float *grads,
                   const uint32_t *sk, const uint32_t *si, uint32_t n, uint32_t max_slots,
                   uint32_t max_pieces, int cus, hipStream_t st);
void launch_apply(const Scratch &s, const Geometry &g, const LaunchGrids &lg, float *E, float *A, float *PE, float *PA,
                  unsigned long long *load_data, unsigned long long *load_parity, const float *grads,
                  const uint32_t *sk, const uint32_t *si, uint32_t n, int cus, hipStream_t st);
void launch_encode(const Geometry &g, const float *E, const float *A, float *PE, float *PA,
                   int grid_blocks, hipStream_t st);
void launch_route(const Scratch &s, const Geometry &g, const uint64_t *keys, uint64_t n, uint64_t *stripe,
                  uint32_t *member, uint32_t *data_srv, uint32_t *parity_srv, hipStream_t st);
void launch_recovery_read(const Scratch &s, const Geometry &g, const RecoveryView &rv, const float *E, const float *A,
                          const float *PE, const float *PA, const uint64_t *keys, uint64_t n, const uint32_t *bk,
                          const uint32_t *bi, const uint32_t *m_dev, const float *buf_grads, float *out_E, float *out_A,
                          int grid_blocks, hipStream_t st);
void launch_clear_status(const Scratch &s, hipStream_t st);
void launch_fail_server(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                        int grid_blocks, hipStream_t st);
void launch_recover_server(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                           int grid_blocks, hipStream_t st);
void launch_degraded_read(const Scratch &s, const Geometry &g, const float *E, const float *A, const float *PE,
                          const float *PA, const uint64_t *keys, uint64_t n, uint32_t lost, float *out_E,
                          float *out_A, int grid_blocks, hipStream_t st);

// ---- small device helpers ------------------------------------------------------------------------
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & (kWave - 1); }

// One Adagrad step of the printed rule on one parameter, carried in fp64:
//   G += g^2 ; acc += lr * g / sqrt(G + eps)
// 1/sqrt comes from the fp32 hardware estimate refined by one Newton step in fp64 (relative error
// about 1e-13, far below the fp32 rounding of the stored result).
__device__ __forceinline__ void adagrad_step(double &G, double &acc, float gf, double lr, double eps)
{
    const double g = (double)gf;
    G = fma(g, g, G);
    const double x = G + eps;
    double y = (double)__builtin_amdgcn_rsqf((float)x);
    const double h = 0.5 * x * y;
    const double t = fma(-h, y, 0.5);
    y = fma(y, t, y);
    acc = fma(lr * g, y, acc);
}

}  // namespace ecrm
