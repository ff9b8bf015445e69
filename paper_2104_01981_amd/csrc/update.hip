// The floating-point side of the ECRM update, on items already grouped by row (sort.hip):
//
//   apply_stripes   for each touched entry walk its updates in arrival order (Adagrad, Sec. 3.3.1),
//                   store the entry and its accumulator once, and add the entry's total difference in
//                   value and in accumulator to the stripe's parity rows (difference propagation,
//                   Sec. 3.3.2), which are read and written once per call.  The differences of one
//                   call telescope, so adding their sum is the same as adding them one by one.
//                   Entries that receive more than kLongRun updates in one call (the head of a skewed
//                   key distribution) are not walked here: their totals come from chains.hip.
//
//   recovery_read, route, count_rows: the smaller kernels of the path.
//
// One wavefront works on one row at a time: 64 lanes x float2 = a 128-float slice, so a load
// instruction of the wave moves 512 contiguous bytes from a wave-uniform (scalar) row address, and
// all control flow is wave-uniform.  All chain arithmetic is carried in fp64.  The kernels are
// templated on the update rule (struct Rule in rows.h): Adagrad or momentum SGD, updates of an entry
// applied one by one or combined; the description above is the Adagrad, one-by-one case.
#include "rows.h"

namespace ecrm {

// ================================================================================================
// apply
// ================================================================================================

constexpr uint32_t kGroupsPerTicket = 8;
constexpr int kListThreads = 256;
constexpr uint32_t kListMaxTiles = 4;

// Lists the groups of kChunk sorted positions in which a stripe begins: the groups the apply kernel has work
// for.  All others lie inside runs -- every group of a long row's positions but its first -- and while
// they were handed out like the rest, the waves went through such a stretch at the pace of the ticket counter,
// a few nanoseconds per ticket with nothing done (1.2 of 8.4 ms on a Zipf batch).  A block looks at `tiles`
// tiles of kListThreads groups: a tile's positions are read coalesced, all loads of a thread in flight
// together, and their stripe numbers staged in LDS; a position whose stripe differs from its left neighbour's
// marks its group; the marked groups are appended to the list with one counter update per block (the list
// ascends inside a block's part; the order of the parts does not matter).
__global__ __launch_bounds__(kListThreads) void active_groups_kernel(const uint32_t *sk, uint32_t n, Header *hdr,
                                                                     Divider dk, uint32_t tiles, uint32_t *active)
{
    constexpr uint32_t kTilePos = kListThreads * kChunk;                   // positions of a tile
    constexpr uint32_t kNone = 0xFFFFFFFFu, kEdge = 0xFFFFFFFEu;           // no stripe has these numbers
    __shared__ uint32_t s_q[1 + kTilePos];                                 // [0]: the position left of the tile
    __shared__ uint32_t s_mark[kListMaxTiles][kListThreads];
    __shared__ uint32_t s_cnt[kListMaxTiles][kListThreads / kWave];
    __shared__ uint32_t s_base;
    if (hdr->batch_bad) return;
    n = min(n, hdr->n_valid);
    const uint32_t tid = threadIdx.x, lane = lane_id(), w = tid / kWave;
    const uint32_t g0 = blockIdx.x * tiles * (uint32_t)kListThreads;       // the block's first group
    for (uint32_t t = 0; t < tiles; ++t) {
        const uint32_t p_lo = (g0 + t * (uint32_t)kListThreads) * kChunk;  // < n + 2^16: no overflow, n <= 2^31
        uint32_t key[kChunk];
#pragma unroll
        for (uint32_t i = 0; i < kChunk; ++i) {
            const uint32_t p = p_lo + i * (uint32_t)kListThreads + tid;
            key[i] = p < n ? sk[p] : kNone;
        }
        if (tid == 0) s_q[0] = (p_lo > 0 && p_lo <= n) ? dk.div(sk[p_lo - 1]) : kEdge;
#pragma unroll
        for (uint32_t i = 0; i < kChunk; ++i)
            s_q[1 + i * (uint32_t)kListThreads + tid] = key[i] == kNone ? kNone : dk.div(key[i]);
        s_mark[t][tid] = 0;
        __syncthreads();
#pragma unroll
        for (uint32_t i = 0; i < kChunk; ++i) {
            const uint32_t rel = i * (uint32_t)kListThreads + tid;
            const uint32_t q = s_q[1 + rel];
            if (q != kNone && q != s_q[rel]) s_mark[t][rel / kChunk] = 1u;  // every writer writes 1
        }
        __syncthreads();                                                   // s_q is free for the next tile
    }
    // compaction of the block's marks: per wave and tile a count, then one place in the list for the block
    uint32_t mine_mask = 0;                                                // bit t: group (t, tid) is marked
    for (uint32_t t = 0; t < tiles; ++t) {
        const bool mine = s_mark[t][tid] != 0;
        const unsigned long long bal = __ballot(mine);
        if (mine) mine_mask |= 1u << t;
        if (lane == 0) s_cnt[t][w] = (uint32_t)__popcll(bal);
    }
    __syncthreads();
    uint32_t total = 0, before[kListMaxTiles];
#pragma unroll
    for (uint32_t t = 0; t < kListMaxTiles; ++t) {
        before[t] = 0;
        if (t < tiles) {
#pragma unroll
            for (int v = 0; v < kListThreads / kWave; ++v) {
                const uint32_t c = s_cnt[t][v];
                if ((uint32_t)v == w) before[t] = total;
                total += c;
            }
        }
    }
    if (tid == 0) s_base = total ? atomicAdd(&hdr->n_active, total) : 0u;
    __syncthreads();
#pragma unroll
    for (uint32_t t = 0; t < kListMaxTiles; ++t) {
        const bool mine = (mine_mask >> t) & 1u;                           // never set for t >= tiles
        const unsigned long long bal = __ballot(mine);
        if (mine) active[s_base + before[t] + (uint32_t)__popcll(bal & bits_below(lane))] = g0 + t * (uint32_t)kListThreads + tid;
    }
}

struct ApplyArgs {
    float *E, *A, *PE, *PA;
    const float *grads;
    const uint32_t *sk, *si;
    const uint32_t *active;      // groups of kChunk sorted positions in which a stripe begins (hdr->n_active of them);
                                 // null: no list was made, every group is looked at
    const uint32_t *long_slot, *long_len;
    const double *long_res;
    Header *hdr;
    const unsigned long long *cnt;
    unsigned long long *load_data, *load_parity;
    uint32_t n;
    Geometry geo;
};

// General path: the stripe whose first item sits at sorted position `pos` (wave-uniform), walked
// through memory.  Used when the stripe does not fit the wave's window: runs of more than a few
// dozen updates, and entries whose totals come from the split-chain path.
template <int NC, int MODE, bool PARITY>
__device__ __forceinline__ void apply_stripe_general(const ApplyArgs &a, uint32_t n, uint32_t pos, uint32_t cb)
{
    const uint32_t D = a.geo.D, k = a.geo.k;
    const RuleParams rp = rule_params(a.geo);
    const uint32_t col0 = cb * NC * 128u;
    uint32_t key = uniform(a.sk[pos]);
    const uint32_t g = key / k;
    const rsrc_t perow = row_f32(a.PE, g, D, col0), parow = row_f32(a.PA, g, D, col0);

    D2 pe[NC], pa[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        pe[i] = PARITY ? widen2(ld2(perow, i)) : D2{0, 0};
        pa[i] = PARITY ? widen2(ld2(parow, i)) : D2{0, 0};
    }
    uint32_t cur = pos;
    do {
        const uint32_t x = key;                      // a new entry of this stripe starts at cur
        const bool is_long = (cur + kLongRun < n) && (uniform(a.sk[cur + kLongRun]) == x);
        const rsrc_t erow = row_f32(a.E, x, D, col0), arow = row_f32(a.A, x, D, col0);
        float2 e[NC], a0[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            e[i] = ld2(erow, i);
            a0[i] = ld2(arow, i);
        }
        D2 G[NC], acc[NC];
        if (is_long) {
            const uint32_t slot = uniform(a.long_slot[cur]);
            const rsrc_t r0 = row_f64(a.long_res, (size_t)slot * 2 + 0, D, col0);
            const rsrc_t r1 = row_f64(a.long_res, (size_t)slot * 2 + 1, D, col0);
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                if (Rule<MODE>::combine) {           // slot 0 holds the sum of the run's gradients
                    G[i] = ldd2(r0, i);
                    acc[i] = D2{0, 0};
                } else {                             // slot 0: sum of the steps, slot 1: state after the run
                    acc[i] = ldd2(r0, i);
                    G[i] = ldd2(r1, i);
                }
            }
            cur += uniform(a.long_len[slot]);
        } else {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                G[i] = start2<MODE>(widen2(a0[i]));
                acc[i] = D2{0, 0};
            }
            // the run is at most kLongRun long: walk it 64 positions at a time, U gradients in flight
            constexpr int U = 8;
            bool done = false;
            while (!done) {
                const uint32_t lane = lane_id();
                const uint32_t wk = cur + lane < n ? a.sk[cur + lane] : kNoKey;
                const uint32_t wi = cur + lane < n ? a.si[cur + lane] : 0u;
                const unsigned long long other = ~__ballot(wk == x);
                const uint32_t cnt = other ? lowest_bit(other) : (uint32_t)kWave;   // leading run of x
                done = cnt < kWave;
                for (uint32_t u0 = 0; u0 < cnt; u0 += U) {
                    float2 gr[U][NC];
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const uint32_t idx = from_lane(wi, min(u0 + u, cnt - 1));
                        const rsrc_t r = row_f32(a.grads, idx, D, col0);
#pragma unroll
                        for (int i = 0; i < NC; ++i) gr[u][i] = ldg2(r, i);
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (u0 + u < cnt) {
#pragma unroll
                            for (int i = 0; i < NC; ++i) item2<MODE>(G[i], acc[i], gr[u][i], rp);
                        }
                }
                cur += cnt;
            }
        }
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const D2 e64 = widen2(e[i]), a64 = widen2(a0[i]);
            finish2<MODE>(G[i], acc[i], a64, rp);
            st2(erow, i, narrow2(D2{e64.x - acc[i].x, e64.y - acc[i].y}));
            st2(arow, i, narrow2(G[i]));
            pe[i].x -= acc[i].x;
            pe[i].y -= acc[i].y;
            pa[i].x += G[i].x - a64.x;
            pa[i].y += G[i].y - a64.y;
        }
        key = cur < n ? uniform(a.sk[cur]) : kNoKey;
    } while (cur < n && key / k == g);

    if (PARITY) {
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            st2(perow, i, narrow2(pe[i]));
            st2(parow, i, narrow2(pa[i]));
        }
    }
}

#ifndef ECRM_PREFETCH
#define ECRM_PREFETCH 1
#endif
constexpr int kPrefetch = ECRM_PREFETCH;   // entries whose loads are issued ahead of the one being computed

// Loads of one entry's work: its row of E and A, its first gradient, and -- when it opens a
// stripe -- the stripe's parity rows.
template <int NC>
struct RowLoads {
    float2 e[NC], a[NC], g[NC], pe[NC], pa[NC];
    uint32_t x, j;
    bool opens;
};

template <int NC, bool PARITY>
__device__ __forceinline__ void issue_row(RowLoads<NC> &r, const ApplyArgs &a, uint32_t col0, uint32_t wkey,
                                          uint32_t widx, unsigned long long stripeheads, uint32_t j)
{
    const uint32_t D = a.geo.D;
    r.j = j;
    r.x = from_lane(wkey, j);
    r.opens = (stripeheads >> j) & 1ull;
    const uint32_t idx = from_lane(widx, j);
    const rsrc_t arow = row_f32(a.A, r.x, D, col0), grow = row_f32(a.grads, idx, D, col0),
                 erow = row_f32(a.E, r.x, D, col0);
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        r.a[i] = ld2(arow, i);
        r.g[i] = ldg2(grow, i);
        r.e[i] = ld2(erow, i);
        r.pe[i] = r.pa[i] = float2{0, 0};
    }
    if (PARITY && r.opens) {
        const uint32_t g = r.x / a.geo.k;
        const rsrc_t perow = row_f32(a.PE, g, D, col0), parow = row_f32(a.PA, g, D, col0);
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            r.pe[i] = ld2(perow, i);
            r.pa[i] = ld2(parow, i);
        }
    }
}

// Window path: every stripe that opens in the first kChunk lanes of the wave's 64-position window
// and ends inside the window.  Entries are taken one after the other; the loads of the next entry
// are issued before the current one is computed, so two entries' rows are in flight per wave.
template <int NC, int MODE, bool PARITY>
__device__ __forceinline__ void apply_window(const ApplyArgs &a, uint32_t wkey, uint32_t widx,
                                             unsigned long long rowheads, unsigned long long stripeheads,
                                             uint32_t first, uint32_t end, uint32_t cb)
{
    const uint32_t D = a.geo.D, k = a.geo.k;
    const RuleParams rp = rule_params(a.geo);
    const uint32_t col0 = cb * NC * 128u;
    unsigned long long todo = rowheads & bits_below(end) & ~bits_below(first);
    if (!todo) return;
    RowLoads<NC> q[kPrefetch];                        // entries whose loads are in flight, in order
    int qn = 0;
#pragma unroll
    for (int s = 0; s < kPrefetch; ++s) {
        if (todo) {
            issue_row<NC, PARITY>(q[s], a, col0, wkey, widx, stripeheads, lowest_bit(todo));
            todo &= todo - 1ull;
            qn = s + 1;
        }
    }
    D2 pe[NC], pa[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) pe[i] = pa[i] = D2{0, 0};
    while (true) {
        const RowLoads<NC> cur = q[0];
#pragma unroll
        for (int s = 0; s + 1 < kPrefetch; ++s) q[s] = q[s + 1];
        --qn;
        if (todo) {
            issue_row<NC, PARITY>(q[kPrefetch - 1], a, col0, wkey, widx, stripeheads, lowest_bit(todo));
            todo &= todo - 1ull;
            ++qn;                                     // the queue was full before the pop: slot kPrefetch-1 is free
        }
        const bool has_next = qn > 0;
        const uint32_t rend = has_next ? q[0].j : end;
        const bool next_opens = has_next && q[0].opens;
        D2 G[NC], acc[NC];
        float2 gr[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            G[i] = start2<MODE>(widen2(cur.a[i]));
            acc[i] = D2{0, 0};
            gr[i] = cur.g[i];
        }
#ifndef ECRM_ITEM_AHEAD
#define ECRM_ITEM_AHEAD 4
#endif
        // The entry's updates, in arrival order.  The gradients of the next few updates are in flight
        // while one is applied: with one in flight a run of m updates cost m memory latencies, which
        // is what bounded the workloads with several updates per entry (4 in flight: -3 % and -5 % on
        // large_uniform and medium; two for D > 128, where more would cost a wave per SIMD).
        constexpr int AH = (NC == 1 ? ECRM_ITEM_AHEAD : 2) - 1;
        float2 nx[AH][NC];
#pragma unroll
        for (int q = 0; q < AH; ++q) {
#pragma unroll
            for (int i = 0; i < NC; ++i) nx[q][i] = float2{0, 0};
            if (cur.j + 1 + q < rend) {
                const rsrc_t r = row_f32(a.grads, from_lane(widx, cur.j + 1 + q), D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) nx[q][i] = ldg2(r, i);
            }
        }
        for (uint32_t t = cur.j;;) {
            float2 in[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) in[i] = float2{0, 0};
            if (t + 1 + AH < rend) {
                const rsrc_t r = row_f32(a.grads, from_lane(widx, t + 1 + AH), D, col0);
#pragma unroll
                for (int i = 0; i < NC; ++i) in[i] = ldg2(r, i);
            }
#pragma unroll
            for (int i = 0; i < NC; ++i) item2<MODE>(G[i], acc[i], gr[i], rp);
            if (t + 1 >= rend) break;
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                gr[i] = nx[0][i];
#pragma unroll
                for (int q = 0; q + 1 < AH; ++q) nx[q][i] = nx[q + 1][i];
                nx[AH - 1][i] = in[i];
            }
            ++t;
        }
        if (cur.opens) {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                pe[i] = widen2(cur.pe[i]);
                pa[i] = widen2(cur.pa[i]);
            }
        }
        const rsrc_t erow = row_f32(a.E, cur.x, D, col0), arow = row_f32(a.A, cur.x, D, col0);
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            const D2 e64 = widen2(cur.e[i]), a64 = widen2(cur.a[i]);
            finish2<MODE>(G[i], acc[i], a64, rp);
            st2(erow, i, narrow2(D2{e64.x - acc[i].x, e64.y - acc[i].y}));
            st2(arow, i, narrow2(G[i]));
            pe[i].x -= acc[i].x;
            pe[i].y -= acc[i].y;
            pa[i].x += G[i].x - a64.x;
            pa[i].y += G[i].y - a64.y;
        }
        if (PARITY && (!has_next || next_opens)) {    // last entry of its stripe: the parity rows are complete
            const uint32_t g = cur.x / k;
            const rsrc_t perow = row_f32(a.PE, g, D, col0), parow = row_f32(a.PA, g, D, col0);
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                st2(perow, i, narrow2(pe[i]));
                st2(parow, i, narrow2(pa[i]));
            }
        }
        if (!has_next) break;
    }
}

template <int NC, int MODE, bool PARITY>
__device__ __forceinline__ void apply_stripes_body(const ApplyArgs &a)
{
    if (a.hdr->batch_bad) return;
    // the batch is valid: publish its per-server counts
    if (blockIdx.x == 0) {
        const uint32_t S = a.geo.S;
        for (uint32_t i = threadIdx.x; i < S; i += blockDim.x) {
            if (a.load_data) a.load_data[i] += a.cnt[i];
            if (a.load_parity) a.load_parity[i] += a.cnt[S + i];
        }
    }
    const uint32_t n = min(a.n, a.hdr->n_valid), k = a.geo.k, lane = lane_id();
    // The groups of kChunk sorted positions in which a stripe begins (active_groups_kernel lists them) are handed
    // out through a counter instead of by a fixed stride: the work per group varies (runs, long stripes), and
    // with a fixed stride the slowest wave set the kernel's time (6.50 -> 6.22 ms).  One ticket covers
    // kGroupsPerTicket listed groups: one group per ticket made the counter itself the bottleneck (12.5 ms), 64
    // per ticket is too coarse again.  A wave's first ticket is its own number (no counter traffic at start-up,
    // which is all a small batch consists of); later ones come from the counter.  Small batches get smaller
    // tickets, so that every wave has work.
    const uint32_t ngroups = (n + kChunk - 1) / kChunk;
    const uint32_t nact = a.active ? min(a.hdr->n_active, ngroups) : ngroups;   // no list (a small batch): every group
    const uint32_t per_ticket = min(kGroupsPerTicket, max(1u, nact / (4u * wave_count())));
    const bool one_ticket_each = (nact + per_ticket - 1) / per_ticket <= wave_count();
    uint32_t at = wave_id() * per_ticket;              // the ticket's place in the list
    uint32_t left = 0, taken = 0, listed = 0;          // groups left in the ticket, taken from it; lane i: its group i
    uint32_t pf_ch = 0xFFFFFFFFu, pf_key = 0, pf_idx = 0, pf_prev = 0;
    for (bool first_ticket = true;;) {
        if (left == 0) {
            if (!first_ticket) {
                if (one_ticket_each) break;
                uint32_t t = 0;
                if (lane == 0) t = atomicAdd(&a.hdr->apply_ticket, 1u);
                at = (wave_count() + uniform(t)) * per_ticket;
            }
            first_ticket = false;
            if (at >= nact) break;
            left = min(per_ticket, nact - at);
            listed = lane < left ? (a.active ? a.active[at + lane] : at + lane) : 0u;
            taken = 0;
        }
        const uint32_t ch = from_lane(listed, taken);
        ++taken;
        --left;
        const uint32_t p0 = ch * kChunk;
        uint32_t wkey, widx, prevk;
        // The group's 64 (row, index) pairs were asked for while the previous group was being worked on;
        // only a ticket's first group has to wait for them.
        if (pf_ch == ch) {
            wkey = pf_key;
            widx = pf_idx;
            prevk = uniform(pf_prev);
        } else {
            wkey = p0 + lane < n ? a.sk[p0 + lane] : kNoKey;
            widx = p0 + lane < n ? a.si[p0 + lane] : 0u;
            prevk = p0 ? uniform(a.sk[p0 - 1]) : kNoKey;
        }
        if (left > 0) {
            pf_ch = from_lane(listed, taken);
            const uint32_t q0 = pf_ch * kChunk;
            pf_key = q0 + lane < n ? a.sk[q0 + lane] : kNoKey;
            pf_idx = q0 + lane < n ? a.si[q0 + lane] : 0u;
            pf_prev = q0 ? a.sk[q0 - 1] : kNoKey;
        }
        uint32_t leftk = __shfl_up(wkey, 1, kWave);
        if (lane == 0) leftk = prevk;
        const bool valid = wkey != kNoKey;
        const bool rh = !valid || leftk == kNoKey || leftk != wkey;    // lanes past n end the last run
        const bool sh = valid && (leftk == kNoKey || leftk / k != wkey / k);
        const unsigned long long rowheads = __ballot(rh);
        const unsigned long long stripeheads = __ballot(sh);
        const uint32_t vend = min((uint32_t)kWave, n - p0);
        const unsigned long long owned = stripeheads & bits_below(kChunk);
        if (!owned) continue;
        const uint32_t first = lowest_bit(owned);
        const uint32_t last = 63u - (uint32_t)__builtin_clzll(owned);
        const unsigned long long after = stripeheads & ~bits_below(last + 1);
        const bool last_inside = after != 0ull || p0 + kWave >= n;
        const uint32_t end = last_inside ? (after ? lowest_bit(after) : vend) : last;
        for (uint32_t cb = 0; cb < a.geo.ncb; ++cb) {
            apply_window<NC, MODE, PARITY>(a, wkey, widx, rowheads, stripeheads, first, end, cb);
            if (!last_inside) apply_stripe_general<NC, MODE, PARITY>(a, n, p0 + last, cb);
        }
    }
}

// D <= 128: one 128-float slice per lane pair; D > 128: two slices per lane.
template <int MODE>
__global__ __launch_bounds__(256) void apply_stripes_kernel_d128(ApplyArgs a)
{
    apply_stripes_body<1, MODE, true>(a);
}
template <int MODE>
__global__ __launch_bounds__(256) void apply_stripes_kernel_d256(ApplyArgs a)
{
    apply_stripes_body<2, MODE, true>(a);
}
// The same walk with the parity rows left alone: entries and their state only.  This is the update
// of a system without redundancy (the baseline the overheads of Sec. 4.3 are quoted against), and
// each of the two halves of the gradient-propagation strawman of Sec. 3.3.1.
template <int MODE>
__global__ __launch_bounds__(256) void apply_rows_kernel_d128(ApplyArgs a)
{
    apply_stripes_body<1, MODE, false>(a);
}
template <int MODE>
__global__ __launch_bounds__(256) void apply_rows_kernel_d256(ApplyArgs a)
{
    apply_stripes_body<2, MODE, false>(a);
}

// Combined (synchronous) rule: one update per modified entry, so the per-server load counts one per
// distinct row of the batch and one parity update for each (Sec. 3.6, Sec. 4.4).
__global__ __launch_bounds__(256) void count_rows_kernel(const uint32_t *sk, uint32_t n, Header *hdr,
                                                         unsigned long long *cnt, uint32_t k, uint32_t S)
{
    __shared__ uint32_t s_cnt[2 * 1024];
    if (hdr->batch_bad) return;
    n = min(n, hdr->n_valid);
    for (uint32_t i = threadIdx.x; i < 2 * S; i += blockDim.x) s_cnt[i] = 0;
    __syncthreads();
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p < n; p += stride) {
        const uint32_t x = sk[p];
        if (p == 0 || sk[p - 1] != x) {
            const uint32_t g = x / k, j = x - g * k;
            atomicAdd(&s_cnt[(g + 1 + j) % S], 1u);
            atomicAdd(&s_cnt[S + g % S], 1u);
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < 2 * S; i += blockDim.x)
        if (s_cnt[i]) atomicAdd(&cnt[i], (unsigned long long)s_cnt[i]);
}

// ================================================================================================
// reads while a server is being recovered
// ================================================================================================

// Sec. 3.4 "Training during recovery" serves a locked entry that has been updated meanwhile out of
// the buffer.  The buffer here holds updates, not entries, so the read applies them: the value
// returned is the stored entry with its waiting updates applied in arrival order -- what the entry
// will be once they have been replayed -- and an entry the failed server held that is not rebuilt
// yet is first decoded from its stripe (parity minus the other members, by increasing member, rounded
// to fp32 as the decoder stores it).  The waiting updates come grouped by entry (bk sorted, bi their
// positions in the buffer).  One wave per requested key; nothing is modified.
struct ReadArgs {
    const float *E, *A, *PE, *PA;
    const uint64_t *keys;
    uint64_t n;
    const uint32_t *bk, *bi;
    const uint32_t *m_dev;   // how many updates are waiting (device word)
    const float *buf_grads;
    float *out_E, *out_A;
    Header *hdr;
    RecoveryView rv;
    Geometry geo;
};

template <int MODE>
__global__ __launch_bounds__(256) void recovery_read_kernel(ReadArgs a)
{
    const uint32_t D = a.geo.D, k = a.geo.k, S = a.geo.S, lane = lane_id();
    const RuleParams rp = rule_params(a.geo);
    const uint64_t nw = wave_count();
    const uint32_t m = uniform(*a.m_dev);
    for (uint64_t i = wave_id(); i < a.n; i += nw) {
        const uint64_t key = a.keys[i];
        const uint32_t khi = uniform((uint32_t)(key >> 32)), x = uniform((uint32_t)key);
        if (khi != 0 || x >= a.geo.rows) {
            if (lane == 0) atomicOr(&a.hdr->err_sticky, 1u);
            continue;
        }
        const uint32_t g = x / k, j = x - g * k;
        bool decode = false;                      // the entry the failed server held, not rebuilt yet
        if (a.rv.active) {
            const uint32_t p = g % S;
            if (p != a.rv.server) {
                const uint32_t lost = (a.rv.server + S - (p + 1u) % S) % S;
                decode = lost == j && g / a.rv.stripes_per_chunk >= a.rv.next;
            }
        }
        uint32_t lo = m;                          // first waiting update of x, if it can have any
        if (m && held_back(a.rv, x, a.geo.dk, a.geo.dS)) {
            uint32_t l = 0, h = m;
            while (l < h) {
                const uint32_t mid = l + (h - l) / 2;
                if (uniform(a.bk[mid]) < x) l = mid + 1; else h = mid;
            }
            lo = l;
        }
        for (uint32_t col0 = 0; col0 < D; col0 += 128u) {
            D2 e, s0;
            if (decode) {
                e = widen2(ld2<0>(row_f32(a.PE, g, D, col0), 0));
                s0 = widen2(ld2<0>(row_f32(a.PA, g, D, col0), 0));
                for (uint32_t mth = 0; mth < k; ++mth) {
                    if (mth == j) continue;
                    const D2 ve = widen2(ld2<0>(row_f32(a.E, g * k + mth, D, col0), 0));
                    const D2 vs = widen2(ld2<0>(row_f32(a.A, g * k + mth, D, col0), 0));
                    e.x -= ve.x; e.y -= ve.y;
                    s0.x -= vs.x; s0.y -= vs.y;
                }
                e = widen2(narrow2(e));
                s0 = widen2(narrow2(s0));
            } else {
                e = widen2(ld2<0>(row_f32(a.E, x, D, col0), 0));
                s0 = widen2(ld2<0>(row_f32(a.A, x, D, col0), 0));
            }
            D2 G = start2<MODE>(s0), acc = D2{0, 0};
            bool any = false;
            for (uint32_t pos = lo; pos < m; ++pos) {
                if (uniform(a.bk[pos]) != x) break;
                const float2 gr = ld2<0>(row_f32(a.buf_grads, uniform(a.bi[pos]), D, col0), 0);
                item2<MODE>(G, acc, gr, rp);
                any = true;
            }
            if (any) finish2<MODE>(G, acc, s0, rp); else G = s0;
            const rsrc_t oe = __builtin_amdgcn_make_buffer_rsrc(a.out_E + (size_t)i * D + col0, 0, (int)((D - col0) * 4u), kRsrcFlags);
            st2(oe, 0, narrow2(D2{e.x - acc.x, e.y - acc.y}));
            if (a.out_A) {
                const rsrc_t oa = __builtin_amdgcn_make_buffer_rsrc(a.out_A + (size_t)i * D + col0, 0, (int)((D - col0) * 4u), kRsrcFlags);
                st2(oa, 0, narrow2(G));
            }
        }
    }
}

// ================================================================================================
// route
// ================================================================================================

__global__ __launch_bounds__(256) void route_kernel(const uint64_t *keys, uint64_t n, uint64_t rows, uint32_t k,
                                                    uint32_t S, uint64_t *stripe, uint32_t *member,
                                                    uint32_t *data_srv, uint32_t *parity_srv, Header *hdr)
{
    const uint64_t stride = (uint64_t)gridDim.x * blockDim.x;
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        const uint64_t x = keys[i];
        if (x >= rows) {
            atomicOr(&hdr->err_sticky, 1u);
            continue;
        }
        const uint64_t g = x / k;
        const uint32_t j = (uint32_t)(x - g * k);
        if (stripe) stripe[i] = g;
        if (member) member[i] = j;
        if (data_srv) data_srv[i] = (uint32_t)((g + 1 + j) % S);
        if (parity_srv) parity_srv[i] = (uint32_t)(g % S);
    }
}

// ================================================================================================
// host side
// ================================================================================================

template <int NC, int MODE>
static bool apply_grids_for(int cus, LaunchGrids *out)
{
    if (NC == 1) {
        out->apply = resident_grid(apply_stripes_kernel_d128<MODE>, cus);
        out->rows = resident_grid(apply_rows_kernel_d128<MODE>, cus);
    } else {
        out->apply = resident_grid(apply_stripes_kernel_d256<MODE>, cus);
        out->rows = resident_grid(apply_rows_kernel_d256<MODE>, cus);
    }
    return out->apply > 0 && out->rows > 0;
}

template <int NC, int MODE>
static void apply_for(const ApplyArgs &a, const LaunchGrids &lg, bool parity, hipStream_t st)
{
    if (parity) {
        if (NC == 1) hipLaunchKernelGGL(apply_stripes_kernel_d128<MODE>, dim3(lg.apply), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(apply_stripes_kernel_d256<MODE>, dim3(lg.apply), dim3(256), 0, st, a);
    } else {
        if (NC == 1) hipLaunchKernelGGL(apply_rows_kernel_d128<MODE>, dim3(lg.rows), dim3(256), 0, st, a);
        else hipLaunchKernelGGL(apply_rows_kernel_d256<MODE>, dim3(lg.rows), dim3(256), 0, st, a);
    }
}

bool query_launch_grids(const Geometry &g, int cus, LaunchGrids *out)
{
    bool ok = false;
    ECRM_DISPATCH(ok = apply_grids_for, cus, out);
    return ok && query_chain_grids(g, cus, out);
}

// A batch this small is one wave's ticket or two per wave anyway: the list would cost a launch and save nothing.
static bool lists_groups(uint32_t n) { return n > (1u << 18); }

// the list of groups launch_apply works from; n > 0
void launch_active_groups(const Scratch &s, const Geometry &g, const uint32_t *sk, uint32_t n, hipStream_t st)
{
    if (!lists_groups(n)) return;
    const uint32_t groups = (n + kChunk - 1) / kChunk;
    // a large batch: several tiles per block, so that the list's counter is not updated at its own pace
    const uint32_t tiles = groups > 64u * kListThreads ? kListMaxTiles : 1u;
    const uint32_t per_block = tiles * kListThreads;
    hipLaunchKernelGGL(active_groups_kernel, dim3((groups + per_block - 1) / per_block), dim3(kListThreads), 0, st, sk, n,
                       s.hdr, make_divider(g.k), tiles, s.active);
}

void launch_apply(const Scratch &s, const Geometry &g, const LaunchGrids &lg, float *E, float *A, float *PE, float *PA,
                  unsigned long long *load_data, unsigned long long *load_parity, const float *grads,
                  const uint32_t *sk, const uint32_t *si, uint32_t n, int cus, hipStream_t st)
{
    const bool parity = PE != nullptr;      // no parity tables: entries and state only
    ApplyArgs a;
    a.E = E; a.A = A; a.PE = PE; a.PA = PA;
    a.grads = grads; a.sk = sk; a.si = si;
    a.long_slot = s.long_slot; a.long_len = s.long_len; a.long_res = s.long_res;
    a.active = lists_groups(n) ? s.active : nullptr;
    a.hdr = s.hdr; a.cnt = s.cnt;
    a.load_data = load_data; a.load_parity = load_parity;
    a.n = n; a.geo = g;
    if ((g.mode == kAdagradCombine || g.mode == kMomentumCombine) && load_data)      // one load count per modified entry
        hipLaunchKernelGGL(count_rows_kernel, dim3(cus * 8), dim3(256), 0, st, sk, n, s.hdr, s.cnt, g.k, g.S);
    ECRM_DISPATCH(apply_for, a, lg, parity, st);
}
#undef ECRM_DISPATCH

void launch_recovery_read(const Scratch &s, const Geometry &g, const RecoveryView &rv, const float *E, const float *A,
                          const float *PE, const float *PA, const uint64_t *keys, uint64_t n, const uint32_t *bk,
                          const uint32_t *bi, const uint32_t *m_dev, const float *buf_grads, float *out_E, float *out_A,
                          int grid_blocks, hipStream_t st)
{
    ReadArgs a;
    a.E = E; a.A = A; a.PE = PE; a.PA = PA;
    a.keys = keys; a.n = n; a.bk = bk; a.bi = bi; a.m_dev = m_dev; a.buf_grads = buf_grads;
    a.out_E = out_E; a.out_A = out_A; a.hdr = s.hdr; a.rv = rv; a.geo = g;
    const dim3 grid(grid_blocks), block(256);
    switch (g.mode) {
        case kAdagradSeq: hipLaunchKernelGGL(recovery_read_kernel<kAdagradSeq>, grid, block, 0, st, a); break;
        case kMomentumSeq: hipLaunchKernelGGL(recovery_read_kernel<kMomentumSeq>, grid, block, 0, st, a); break;
        case kAdagradCombine: hipLaunchKernelGGL(recovery_read_kernel<kAdagradCombine>, grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL(recovery_read_kernel<kMomentumCombine>, grid, block, 0, st, a); break;
    }
}

void launch_route(const Scratch &s, const Geometry &g, const uint64_t *keys, uint64_t n, uint64_t *stripe,
                  uint32_t *member, uint32_t *data_srv, uint32_t *parity_srv, hipStream_t st)
{
    uint64_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(route_kernel, dim3((uint32_t)blocks), dim3(256), 0, st, keys, n, (uint64_t)g.rows, g.k, g.S,
                       stripe, member, data_srv, parity_srv, s.hdr);
}

}  // namespace ecrm
