// Grouping pass of the ECRM update: a stable LSD radix sort of (row id, item index) pairs, so that
// all updates of an entry -- and, since stripe = row / k, all updates of a stripe -- become
// contiguous while every entry keeps its arrival order (the per-entry order is what the Adagrad
// rule of Sec. 3.3.1 depends on).  The first pass also does the integer side of the path: the
// key-range check, and the per-server load counts of the rotating placement (Sec. 3.2, Sec. 3.6).
//
// Three kernels per digit: per-block digit histogram -> per-digit scan over blocks -> stable
// scatter that ranks items with wave ballots, orders the tile in LDS and writes it out in runs.
// The scatter is latency bound (load, rank, order, write, with barriers in between): its tile is
// sized so that two blocks share a CU and overlap each other's phases (0.52 -> 0.41 ms per 2^24 items).
#include "ecrm_internal.h"

namespace ecrm {

__device__ __forceinline__ uint32_t wave_incl_scan(uint32_t v)
{
    const uint32_t lane = lane_id();
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        uint32_t t = __shfl_up(v, d, kWave);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}

// exclusive scan of one value per thread over a block of kSortThreads; total returned to all
__device__ __forceinline__ uint32_t block_excl_scan(uint32_t v, uint32_t *s_wave /*[kSortWaves+1]*/,
                                                    uint32_t &total)
{
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    const uint32_t incl = wave_incl_scan(v);
    if (lane == kWave - 1) s_wave[wave] = incl;
    __syncthreads();
    uint32_t off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSortWaves; ++w) {
        const uint32_t t = s_wave[w];
        if ((uint32_t)w < wave) off += t;
        tot += t;
    }
    __syncthreads();
    total = tot;
    return off + incl - v;
}

__global__ void reset_kernel(Header *h, unsigned long long *cnt, uint32_t S, uint32_t n, int clear_sticky, int from_buffer)
{
    const uint32_t t = threadIdx.x;
    if (t == 0) {
        if (clear_sticky) {
            h->err_sticky = 0;
            h->buf_count = 0;
            h->free_count = 0;
            h->bump = 0;
        }
        if (from_buffer) n = min(n, h->buf_count);     // a replay: everything that is waiting right now
        h->batch_bad = 0;
        h->n_long = 0;
        h->n_pieces = 0;
        h->n_long_items = 0;
        h->n_batch = n;
        h->n_valid = n;
        h->n_held = 0;
        h->apply_ticket = 0;
        for (uint32_t c = 0; c < kMidClasses; ++c) h->n_mid[c] = 0;
        h->mid_ticket = 0;
        h->n_active = 0;
    }
    for (uint32_t i = t; i < 2 * S; i += blockDim.x) cnt[i] = 0;
}

__global__ void clear_status_kernel(Header *h)
{
    if (threadIdx.x == 0) h->err_sticky = 0;
}

__global__ void clear_buffer_kernel(Header *h)
{
    if (threadIdx.x == 0) {
        h->buf_count = 0;
        h->free_count = 0;
        h->bump = 0;
    }
}

// Tile a block works on.  Workgroups go to the 8 XCDs (each with its own L2) round-robin by block id;
// with this map every XCD gets a contiguous range of tiles, so the short runs that neighbouring
// tiles write next to each other in a digit's output range meet in one L2 instead of in memory.
#ifndef ECRM_XCD_TILES
#define ECRM_XCD_TILES 1
#endif
__device__ __forceinline__ uint32_t tile_of_block(uint32_t b, uint32_t nblocks)
{
#if ECRM_XCD_TILES
    constexpr uint32_t X = 8;
    const uint32_t q = nblocks / X, r = nblocks % X, xcd = b % X, i = b / X;
    return xcd < r ? xcd * (q + 1u) + i : r * (q + 1u) + (xcd - r) * q + i;
#else
    return b;
#endif
}

// Sort key of one caller key in the first pass, the same in the histogram and in the scatter:
// out-of-range keys keep their low bits (the batch is rejected anyway), held-back items get `rows`.
__device__ __forceinline__ uint32_t first_pass_key(uint64_t k64, uint32_t rows, const Divider &dk, const Divider &dS,
                                                   const RecoveryView &rv, bool by_stripe, bool packed, bool &bad, bool &held)
{
    const uint32_t key = (uint32_t)k64;
    bad = !packed && k64 >= (uint64_t)rows;           // a waiting update's key was checked when it arrived
    held = !bad && held_back(rv, key, dk, dS);
    if (held) return rows;
    return by_stripe ? dk.div(key) : key;
}

// ---- histogram ---------------------------------------------------------------------------------
// FIRST: keys are the caller's u64 row ids; also range check + load accounting (count != 0).  by_stripe
// groups by row id / k instead (for the parity half of gradient propagation).
template <bool FIRST, int IPT>
__global__ __launch_bounds__(kSortThreads) void sort_hist_kernel(
    const void *keys_in, uint32_t n, const uint32_t *n_dev, uint32_t nblocks, int shift, int bits, uint32_t *block_hist,
    Header *hdr, unsigned long long *cnt, uint32_t rows, Divider dk, Divider dS, uint32_t count, RecoveryView rv,
    uint32_t by_stripe, uint32_t packed)
{
    __shared__ uint32_t s_hist[kMaxBins];
    if (n_dev) n = min(n, *n_dev);
    __shared__ uint32_t s_cnt[2 * 1024];
    __shared__ uint32_t s_bad;
    const uint32_t tid = threadIdx.x;
    const uint32_t bins = 1u << bits, mask = bins - 1;
    const uint32_t S = count ? dS.d : 0u;             // 0: the caller counts per distinct row later
    for (uint32_t i = tid; i < bins; i += kSortThreads) s_hist[i] = 0;
    if (FIRST) {
        for (uint32_t i = tid; i < 2 * S; i += kSortThreads) s_cnt[i] = 0;
        if (tid == 0) s_bad = 0;
    }
    __syncthreads();
    const uint32_t tile = tile_of_block(blockIdx.x, nblocks), tile0 = tile * (uint32_t)(kSortThreads * IPT);
    const uint32_t wave = tid / kWave, lane = lane_id();
    bool bad = false;
    constexpr int kUnroll = IPT < 4 ? IPT : 4;
#pragma unroll kUnroll
    for (int r = 0; r < IPT; ++r) {
        const uint32_t i = tile0 + wave * (kWave * IPT) + r * kWave + lane;
        if (i < n) {
            uint32_t key;
            if (FIRST) {
                const uint64_t k64 = ((const uint64_t *)keys_in)[i];
                bool oob, held;                                   // held back: sorts behind every row, not applied
                key = first_pass_key(k64, rows, dk, dS, rv, by_stripe != 0, packed != 0, oob, held);
                bad |= oob;
                if (!oob && !held && S) {
                    const uint32_t x = (uint32_t)k64, g = dk.div(x), j = x - g * dk.d;
                    atomicAdd(&s_cnt[dS.mod(g + 1 + j)], 1u);     // server of the entry
                    atomicAdd(&s_cnt[S + dS.mod(g)], 1u);         // server of its parity
                }
            } else {
                key = ((const uint32_t *)keys_in)[i];
            }
            atomicAdd(&s_hist[(key >> shift) & mask], 1u);
        }
    }
    if (FIRST && bad) s_bad = 1;
    __syncthreads();
    for (uint32_t b = tid; b < bins; b += kSortThreads) block_hist[(size_t)b * nblocks + tile] = s_hist[b];
    if (FIRST) {
        for (uint32_t i = tid; i < 2 * S; i += kSortThreads)
            if (s_cnt[i]) atomicAdd(&cnt[i], (unsigned long long)s_cnt[i]);
        if (tid == 0 && s_bad) {
            atomicOr(&hdr->batch_bad, 1u);
            atomicOr(&hdr->err_sticky, 1u);
        }
    }
}

// ---- per-digit exclusive scan over blocks ----------------------------------------------------------
__global__ __launch_bounds__(kSortThreads) void sort_scan_kernel(uint32_t *block_hist, uint32_t *bin_total,
                                                                 uint32_t nblocks)
{
    __shared__ uint32_t s_wave[kSortWaves + 1];
    uint32_t *row = block_hist + (size_t)blockIdx.x * nblocks;
    uint32_t carry = 0;
    for (uint32_t base = 0; base < nblocks; base += kSortThreads) {
        const uint32_t i = base + threadIdx.x;
        const uint32_t v = i < nblocks ? row[i] : 0;
        uint32_t total;
        const uint32_t ex = block_excl_scan(v, s_wave, total);
        if (i < nblocks) row[i] = carry + ex;
        carry += total;
    }
    if (threadIdx.x == 0) bin_total[blockIdx.x] = carry;
}

// ---- stable scatter ------------------------------------------------------------------------------
#ifndef ECRM_SORT_WAVES
#define ECRM_SORT_WAVES 4
#endif
template <bool FIRST, int IPT>
__global__ __launch_bounds__(kSortThreads, ECRM_SORT_WAVES) void sort_scatter_kernel(
    const void *keys_in, const uint32_t *vals_in, uint32_t *keys_out, uint32_t *vals_out,
    const uint32_t *block_hist, const uint32_t *bin_total, uint32_t n, const uint32_t *n_dev, uint32_t nblocks, int shift,
    int bits, uint32_t rows, Divider dk, Divider dS, RecoveryView rv, uint32_t by_stripe, uint32_t packed)
{
    constexpr uint32_t kTile = kSortThreads * IPT;
    __shared__ uint32_t s_keys[kTile];
    __shared__ uint32_t s_vals[kTile];
    __shared__ uint32_t s_wcnt[kSortWaves][kMaxBins];   // per-wave digit counts, then wave offsets
    __shared__ uint32_t s_binstart[kMaxBins];           // start of the digit inside the sorted tile
    __shared__ uint32_t s_gbase[kMaxBins];              // global position of sorted-tile slot 0 of the digit
    __shared__ uint32_t s_wave[kSortWaves + 1];

    const uint32_t tid = threadIdx.x, wave = tid / kWave, lane = lane_id();
    const uint32_t bins = 1u << bits, mask = bins - 1;
    if (n_dev) n = min(n, *n_dev);
    for (uint32_t i = tid; i < kSortWaves * kMaxBins; i += kSortThreads) (&s_wcnt[0][0])[i] = 0;
    __syncthreads();

    const uint32_t tile = tile_of_block(blockIdx.x, nblocks), tile0 = tile * kTile;
    uint32_t key[IPT], val[IPT], rank[IPT];
#pragma unroll
    for (int r = 0; r < IPT; ++r) {
        const uint32_t i = tile0 + wave * (kWave * IPT) + r * kWave + lane;
        key[r] = 0;
        val[r] = 0;
        if (i < n) {
            if (FIRST) {
                bool oob, held;
                const uint64_t k64 = ((const uint64_t *)keys_in)[i];
                key[r] = first_pass_key(k64, rows, dk, dS, rv, by_stripe != 0, packed != 0, oob, held);
                val[r] = packed ? (uint32_t)(k64 >> 32) : i;        // where the item's gradient row is: slot, or item index
            } else {
                key[r] = ((const uint32_t *)keys_in)[i];
                val[r] = vals_in[i];
            }
        }
    }

    // rank inside the wave: items are ordered (r, lane); equal digits are matched with ballots
    const unsigned long long lt = (1ull << lane) - 1ull;
#pragma unroll
    for (int r = 0; r < IPT; ++r) {
        const uint32_t i = tile0 + wave * (kWave * IPT) + r * kWave + lane;
        const bool valid = i < n;
        const uint32_t digit = (key[r] >> shift) & mask;
        unsigned long long peers = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (digit >> b) & 1u;
            const unsigned long long bal = __ballot(bit);
            peers &= bit ? bal : ~bal;
        }
        const uint32_t below = __popcll(peers & lt);
        const uint32_t old = s_wcnt[wave][digit];
        __builtin_amdgcn_wave_barrier();
        if (valid && below == 0) s_wcnt[wave][digit] = old + (uint32_t)__popcll(peers);
        __builtin_amdgcn_wave_barrier();
        rank[r] = old + below;
    }
    __syncthreads();

    // per digit: exclusive scan over the waves, total of the block
    uint32_t my_total = 0;
    if (tid < bins) {
        uint32_t run = 0;
#pragma unroll
        for (int w = 0; w < kSortWaves; ++w) {
            const uint32_t t = s_wcnt[w][tid];
            s_wcnt[w][tid] = run;
            run += t;
        }
        my_total = run;
    }
    uint32_t dummy;
    const uint32_t binstart = block_excl_scan(my_total, s_wave, dummy);
    const uint32_t gtot = tid < bins ? bin_total[tid] : 0;
    const uint32_t gstart = block_excl_scan(gtot, s_wave, dummy);
    if (tid < bins) {
        s_binstart[tid] = binstart;
        s_gbase[tid] = gstart + block_hist[(size_t)tid * nblocks + tile] - binstart;
    }
    __syncthreads();

#pragma unroll
    for (int r = 0; r < IPT; ++r) {
        const uint32_t i = tile0 + wave * (kWave * IPT) + r * kWave + lane;
        if (i < n) {
            const uint32_t digit = (key[r] >> shift) & mask;
            const uint32_t pos = s_binstart[digit] + s_wcnt[wave][digit] + rank[r];
            s_keys[pos] = key[r];
            s_vals[pos] = val[r];
        }
    }
    __syncthreads();

    const uint32_t count = tile0 < n ? min(kTile, n - tile0) : 0u;
    for (uint32_t i = tid; i < count; i += kSortThreads) {
        const uint32_t kk = s_keys[i];
        const uint32_t gpos = s_gbase[(kk >> shift) & mask] + i;
        keys_out[gpos] = kk;
        vals_out[gpos] = s_vals[i];
    }
}

// ---- host side -------------------------------------------------------------------------------------
void launch_reset(const Scratch &s, uint32_t S, uint32_t n, bool clear_sticky, BatchSource src, hipStream_t st)
{
    hipLaunchKernelGGL(reset_kernel, dim3(1), dim3(256), 0, st, s.hdr, s.cnt, S, n, clear_sticky ? 1 : 0,
                       src == kWaitingUpdates ? 1 : 0);
}

void launch_clear_buffer(const Scratch &s, hipStream_t st)
{
    hipLaunchKernelGGL(clear_buffer_kernel, dim3(1), dim3(64), 0, st, s.hdr);
}

void launch_clear_status(const Scratch &s, hipStream_t st)
{
    hipLaunchKernelGGL(clear_status_kernel, dim3(1), dim3(64), 0, st, s.hdr);
}

// One digit of the sort with tiles of kSortThreads * IPT items.
template <int IPT>
static void launch_sort_pass(const Scratch &s, const Geometry &g, const RecoveryView &rv, bool first, const void *keys_in,
                             const uint32_t *vals_in, uint32_t *keys_out, uint32_t *vals_out, uint32_t n,
                             const uint32_t *n_dev, int shift, int bits, uint32_t count, uint32_t by_stripe,
                             uint32_t packed, hipStream_t st)
{
    const uint32_t tile = kSortThreads * IPT, nblocks = (n + tile - 1) / tile, bins = 1u << bits;
    if (first)
        hipLaunchKernelGGL((sort_hist_kernel<true, IPT>), dim3(nblocks), dim3(kSortThreads), 0, st, keys_in, n, n_dev,
                           nblocks, shift, bits, s.block_hist, s.hdr, s.cnt, g.rows, g.dk, g.dS, count, rv, by_stripe, packed);
    else
        hipLaunchKernelGGL((sort_hist_kernel<false, IPT>), dim3(nblocks), dim3(kSortThreads), 0, st, keys_in, n, n_dev,
                           nblocks, shift, bits, s.block_hist, s.hdr, s.cnt, g.rows, g.dk, g.dS, 0u, rv, 0u, 0u);
    hipLaunchKernelGGL(sort_scan_kernel, dim3(bins), dim3(kSortThreads), 0, st, s.block_hist, s.bin_total, nblocks);
    if (first)
        hipLaunchKernelGGL((sort_scatter_kernel<true, IPT>), dim3(nblocks), dim3(kSortThreads), 0, st, keys_in, vals_in,
                           keys_out, vals_out, s.block_hist, s.bin_total, n, n_dev, nblocks, shift, bits, g.rows, g.dk,
                           g.dS, rv, by_stripe, packed);
    else
        hipLaunchKernelGGL((sort_scatter_kernel<false, IPT>), dim3(nblocks), dim3(kSortThreads), 0, st, keys_in, vals_in,
                           keys_out, vals_out, s.block_hist, s.bin_total, n, n_dev, nblocks, shift, bits, g.rows, g.dk,
                           g.dS, rv, 0u, 0u);
}

void launch_sort(const Scratch &s, const Geometry &g, const RecoveryView &rv, const uint64_t *keys, uint32_t n,
                 const uint32_t *n_dev, BatchSource src, int key_bits, bool by_stripe, bool count_servers,
                 uint32_t **sorted_keys, uint32_t **sorted_vals, hipStream_t st)
{
    const uint32_t count = (count_servers && !(g.mode & 2u)) ? 1u : 0u, bs = by_stripe ? 1u : 0u;
    const uint32_t packed = src == kWaitingUpdates ? 1u : 0u;
    // a small batch is cut into small tiles, so that it still spreads over the compute units
    const bool small = n <= kSmallSortBatch;
    int passes = (key_bits + kMaxRadixBits - 1) / kMaxRadixBits;
    if (passes < 1) passes = 1;
    int shift = 0, cur = 0;
    for (int p = 0; p < passes; ++p) {
        // spread the bits as evenly as possible, wider digits first
        const int left = key_bits - shift;
        int bits = (left + (passes - p) - 1) / (passes - p);
        if (bits < 1) bits = 1;
        const void *kin = p == 0 ? (const void *)keys : (const void *)s.keys[cur];
        const uint32_t *vin = p == 0 ? nullptr : s.vals[cur];
        const int out = p == 0 ? 0 : cur ^ 1;
        if (small)
            launch_sort_pass<kSmallSortIpt>(s, g, rv, p == 0, kin, vin, s.keys[out], s.vals[out], n, n_dev, shift, bits,
                                            count, bs, packed, st);
        else
            launch_sort_pass<kSortIpt>(s, g, rv, p == 0, kin, vin, s.keys[out], s.vals[out], n, n_dev, shift, bits, count,
                                       bs, packed, st);
        cur = out;
        shift += bits;
    }
    *sorted_keys = s.keys[cur];
    *sorted_vals = s.vals[cur];
}

}  // namespace ecrm
