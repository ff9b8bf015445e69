// Training while a server is being recovered (Sec. 3.4 "Training during recovery"): updates that
// touch the chunk of stripes under reconstruction, and updates to lost entries that are not rebuilt
// yet, are not applied but appended -- in arrival order -- to a buffer of (key, gradient row) pairs,
// and replayed when their chunk is released.  The buffer is a pool of gradient rows addressed by
// slot plus a list of (key, slot) entries: a row is copied once, when its update is first held back;
// a replay only rewrites the list (what must go on waiting keeps its row) and releases the slots of
// what it applies.  This file holds the order-preserving append and replay bookkeeping (flag, block
// counts, scan, scatter).
#include "ecrm_internal.h"

namespace ecrm {

constexpr int kHoldThreads = 256;
constexpr int kHoldIpt = 8;                        // items per thread
constexpr int kHoldTile = kHoldThreads * kHoldIpt;

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t block_sum(uint32_t v, uint32_t *s_w)
{
#pragma unroll
    for (int d = kWave / 2; d > 0; d >>= 1) v += __shfl_xor(v, d, kWave);
    if (lane_id() == 0) s_w[threadIdx.x / kWave] = v;
    __syncthreads();
    uint32_t t = 0;
    for (int w = 0; w < kHoldThreads / kWave; ++w) t += s_w[w];
    __syncthreads();
    return t;
}

// Is item i of the batch held back?  A caller's key is checked for range here as well (the first sort
// pass rejects the batch for it); a waiting update's key sits in the low half of its list entry.
__device__ __forceinline__ bool item_held(const uint64_t *keys, uint32_t i, uint32_t rows, const Divider &dk, const Divider &dS,
                                          const RecoveryView &rv, bool packed)
{
    const uint64_t x = keys[i];
    if (!packed && x >= (uint64_t)rows) return false;
    return held_back(rv, (uint32_t)x, dk, dS);
}

// pass 1: how many items of each tile are held back
__global__ __launch_bounds__(kHoldThreads) void hold_count_kernel(const uint64_t *keys, uint32_t n, const uint32_t *n_dev,
                                                                  uint32_t rows, Divider dk, Divider dS, RecoveryView rv,
                                                                  uint32_t packed, uint32_t *tile_count)
{
    __shared__ uint32_t s_w[kHoldThreads / kWave];
    if (n_dev) n = min(n, *n_dev);
    uint32_t c = 0;
    const uint32_t base = blockIdx.x * kHoldTile;
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        const uint32_t i = base + r * kHoldThreads + threadIdx.x;
        if (i < n && item_held(keys, i, rows, dk, dS, rv, packed != 0)) ++c;
    }
    const uint32_t t = block_sum(c, s_w);
    if (threadIdx.x == 0) tile_count[blockIdx.x] = t;
}

// pass 2 (one block): exclusive scan of the tile counts; totals and the capacity check
__global__ __launch_bounds__(1024) void hold_scan_kernel(uint32_t *tile_count, uint32_t ntiles, Header *hdr, uint32_t n,
                                                         const uint32_t *n_dev, uint32_t packed, uint32_t buf_cap)
{
    __shared__ uint32_t s_w[16];
    __shared__ uint32_t s_carry;
    if (n_dev) n = min(n, *n_dev);
    if (threadIdx.x == 0) s_carry = 0;
    __syncthreads();
    for (uint32_t b0 = 0; b0 < ntiles; b0 += 1024) {
        const uint32_t i = b0 + threadIdx.x;
        const uint32_t v = i < ntiles ? tile_count[i] : 0;
        uint32_t incl = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const uint32_t t = __shfl_up(incl, d, kWave);
            if (lane_id() >= (uint32_t)d) incl += t;
        }
        if (lane_id() == kWave - 1) s_w[threadIdx.x / kWave] = incl;
        __syncthreads();
        uint32_t off = s_carry, tot = 0;
        for (uint32_t w = 0; w < 16; ++w) {
            if (w < threadIdx.x / kWave) off += s_w[w];
            tot += s_w[w];
        }
        if (i < ntiles) tile_count[i] = off + incl - v;
        __syncthreads();
        if (threadIdx.x == 0) s_carry += tot;
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const uint32_t held = s_carry;
        hdr->n_held = held;
        hdr->n_valid = n - held;
        // no room: the batch is rejected as a whole (a replay only ever shrinks the list)
        if (!packed && (unsigned long long)hdr->buf_count + held > buf_cap) {
            hdr->batch_bad = 1;
            hdr->err_sticky |= 2u;
        }
    }
}

// pass 3, a caller's batch: every held-back item gets a slot of the row pool -- released slots first,
// last released first, then slots never used -- its gradient row is copied there, and (key, slot) is
// appended to the list in arrival order.
// pass 3, a replay of the list: what must go on waiting is appended to the other list as it is (its row
// stays where it is); the slots of what is applied now are released, in list order.
__global__ __launch_bounds__(kHoldThreads) void hold_scatter_kernel(const uint64_t *keys, const float *grads, uint32_t n,
                                                                    const uint32_t *n_dev, uint32_t rows, uint32_t D,
                                                                    Divider dk, Divider dS, RecoveryView rv, uint32_t packed,
                                                                    const uint32_t *tile_offset, Header *hdr,
                                                                    unsigned long long *list_out, float *pool,
                                                                    uint32_t *free_list)
{
    __shared__ uint32_t s_src[kHoldTile];          // item index of the tile's held-back items, in order
    __shared__ uint32_t s_wcount[kHoldThreads / kWave][kHoldIpt];
    if (hdr->batch_bad) return;
    if (n_dev) n = min(n, *n_dev);
    const uint32_t base = blockIdx.x * kHoldTile;
    if (base >= n) return;
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    // tile order is (r, thread): ballots give each item its rank among the held-back ones
    bool held[kHoldIpt];
    uint32_t below[kHoldIpt];
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        const uint32_t i = base + r * kHoldThreads + threadIdx.x;
        held[r] = i < n && item_held(keys, i, rows, dk, dS, rv, packed != 0);
        const unsigned long long m = __ballot(held[r]);
        below[r] = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) s_wcount[wave][r] = (uint32_t)__popcll(m);
    }
    __syncthreads();
    const uint32_t held_before_tile = tile_offset[blockIdx.x];
    const uint32_t free0 = hdr->free_count, bump0 = hdr->bump;
    uint32_t total = 0;
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        uint32_t before = total;                   // held-back items of earlier (r, wave) groups
        for (uint32_t w = 0; w < kHoldThreads / kWave; ++w) {
            if (w < wave) before += s_wcount[w][r];
            total += s_wcount[w][r];
        }
        const uint32_t pos = r * kHoldThreads + threadIdx.x;          // place in the tile
        const uint32_t i = base + pos;
        const uint32_t hrank = before + below[r];                     // held-back items of the tile before this one
        if (held[r]) s_src[hrank] = i;
        if (packed && i < n) {
            if (held[r]) list_out[held_before_tile + hrank] = keys[i];                    // goes on waiting, row in place
            else free_list[free0 + (base - held_before_tile) + (pos - hrank)] = (uint32_t)(keys[i] >> 32);   // slot released
        }
    }
    if (packed) return;
    __syncthreads();
    const uint32_t first = held_before_tile;       // rank of the tile's first held-back item in this batch
    const uint32_t list0 = hdr->buf_count;
    // row copies: U rows in flight per wave (one at a time the copy ran at 2 TB/s)
    constexpr uint32_t U = 8, W = kHoldThreads / kWave;
    for (uint32_t t0 = wave * U; t0 < total; t0 += W * U) {
        uint32_t slot[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t rk = first + min(t0 + u, total - 1);       // rank among the batch's held-back items
            slot[u] = rk < free0 ? free_list[free0 - 1u - rk] : bump0 + (rk - free0);
            slot[u] = (uint32_t)__builtin_amdgcn_readfirstlane((int)slot[u]);
        }
        for (uint32_t off = lane * 16u; off < D * 4u; off += kWave * 16u) {
            u32x4 v[U];
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                const uint32_t i = (uint32_t)__builtin_amdgcn_readfirstlane((int)s_src[min(t0 + u, total - 1)]);
                const rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(grads + (size_t)i * D), 0, (int)(D * 4u), 0x00020000);
                v[u] = __builtin_amdgcn_raw_buffer_load_b128(src, (int)off, 0, 2);
            }
#pragma unroll
            for (uint32_t u = 0; u < U; ++u) {
                if (t0 + u < total) {
                    const rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(pool + (size_t)slot[u] * D, 0, (int)(D * 4u), 0x00020000);
                    __builtin_amdgcn_raw_buffer_store_b128(v[u], out, (int)off, 0, 0);
                }
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u)
            if (lane == u && t0 + u < total)
                list_out[(size_t)list0 + first + t0 + u] = keys[s_src[t0 + u]] | ((unsigned long long)slot[u] << 32);
    }
}

__global__ void hold_commit_kernel(Header *hdr, uint32_t packed)
{
    if (threadIdx.x != 0 || hdr->batch_bad) return;
    const uint32_t held = hdr->n_held;
    if (packed) {                                  // after a replay: the other list, and the released slots
        hdr->free_count += hdr->n_batch - held;
        hdr->buf_count = held;
    } else {
        const uint32_t reused = min(held, hdr->free_count);
        hdr->free_count -= reused;
        hdr->bump += held - reused;
        hdr->buf_count += held;
    }
}

void launch_hold_back(const Scratch &s, const Geometry &g, const RecoveryView &rv, const uint64_t *keys,
                      const float *grads, uint32_t n, BatchSource src, const HoldBuffer &hb, uint32_t cur,
                      hipStream_t st)
{
    const uint32_t packed = src == kWaitingUpdates ? 1u : 0u;
    const uint32_t *n_dev = packed ? &s.hdr->n_batch : nullptr;
    const uint32_t ntiles = (n + kHoldTile - 1) / kHoldTile;
    uint32_t *tile_count = s.long_slot;            // free until the chain kernels run
    // a caller's batch appends to the list in use; a replay reads it and builds the other one
    unsigned long long *list_out = packed ? hb.list[cur ^ 1u] : hb.list[cur];
    hipLaunchKernelGGL(hold_count_kernel, dim3(ntiles), dim3(kHoldThreads), 0, st, keys, n, n_dev, g.rows, g.dk, g.dS, rv,
                       packed, tile_count);
    hipLaunchKernelGGL(hold_scan_kernel, dim3(1), dim3(1024), 0, st, tile_count, ntiles, s.hdr, n, n_dev, packed, hb.cap);
    hipLaunchKernelGGL(hold_scatter_kernel, dim3(ntiles), dim3(kHoldThreads), 0, st, keys, grads, n, n_dev, g.rows, g.D, g.dk,
                       g.dS, rv, packed, tile_count, s.hdr, list_out, hb.rows, hb.free_list);
    hipLaunchKernelGGL(hold_commit_kernel, dim3(1), dim3(64), 0, st, s.hdr, packed);
}

}  // namespace ecrm
