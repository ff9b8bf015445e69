// Training while a server is being recovered (Sec. 3.4 "Training during recovery"): updates that
// touch the chunk of stripes under reconstruction, and updates to lost entries that are not rebuilt
// yet, are not applied but appended -- in arrival order -- to a buffer of (key, gradient row) pairs,
// and replayed when their chunk is released.  This file holds the order-preserving append (flag,
// block counts, scan, scatter with row copies) and the range form of the decoder.
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

// pass 1: how many items of each tile are held back
__global__ __launch_bounds__(kHoldThreads) void hold_count_kernel(const uint64_t *keys, uint32_t n, uint32_t rows, Divider dk,
                                                                  Divider dS, RecoveryView rv, uint32_t *tile_count)
{
    __shared__ uint32_t s_w[kHoldThreads / kWave];
    uint32_t c = 0;
    const uint32_t base = blockIdx.x * kHoldTile;
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        const uint32_t i = base + r * kHoldThreads + threadIdx.x;
        if (i < n) {
            const uint64_t x = keys[i];
            if (x < (uint64_t)rows && held_back(rv, (uint32_t)x, dk, dS)) ++c;
        }
    }
    const uint32_t t = block_sum(c, s_w);
    if (threadIdx.x == 0) tile_count[blockIdx.x] = t;
}

// pass 2 (one block): exclusive scan of the tile counts; totals and the capacity check
__global__ __launch_bounds__(1024) void hold_scan_kernel(uint32_t *tile_count, uint32_t ntiles, Header *hdr, uint32_t n,
                                                         uint32_t buf_cap)
{
    __shared__ uint32_t s_w[16];
    __shared__ uint32_t s_carry;
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
        if ((unsigned long long)hdr->buf_count + held > buf_cap) {      // no room: the batch is rejected as a whole
            hdr->batch_bad = 1;
            hdr->err_sticky |= 2u;
        }
    }
}

// pass 3: position of every held-back item in the buffer (arrival order), its key, and the copy of
// its gradient row (eight held-back items of the tile per wave and step, 16 bytes per lane)
__global__ __launch_bounds__(kHoldThreads) void hold_scatter_kernel(const uint64_t *keys, const float *grads, uint32_t n,
                                                                    uint32_t rows, uint32_t D, Divider dk, Divider dS,
                                                                    RecoveryView rv, const uint32_t *tile_offset,
                                                                    Header *hdr, unsigned long long *buf_keys,
                                                                    float *buf_grads)
{
    __shared__ uint32_t s_src[kHoldTile];          // item index of the tile's held-back items, in order
    __shared__ uint32_t s_wcount[kHoldThreads / kWave][kHoldIpt];
    if (hdr->batch_bad) return;
    const uint32_t base = blockIdx.x * kHoldTile;
    const uint32_t lane = lane_id(), wave = threadIdx.x / kWave;
    // tile order is (r, thread): ballots give each item its rank among the held-back ones
    bool held[kHoldIpt];
    uint32_t below[kHoldIpt];
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        const uint32_t i = base + r * kHoldThreads + threadIdx.x;
        held[r] = false;
        if (i < n) {
            const uint64_t x = keys[i];
            held[r] = x < (uint64_t)rows && held_back(rv, (uint32_t)x, dk, dS);
        }
        const unsigned long long m = __ballot(held[r]);
        below[r] = (uint32_t)__popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) s_wcount[wave][r] = (uint32_t)__popcll(m);
    }
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int r = 0; r < kHoldIpt; ++r) {
        uint32_t before = total;                   // held-back items of earlier (r, wave) groups
        for (uint32_t w = 0; w < kHoldThreads / kWave; ++w) {
            if (w < wave) before += s_wcount[w][r];
            total += s_wcount[w][r];
        }
        if (held[r]) s_src[before + below[r]] = base + r * kHoldThreads + threadIdx.x;
    }
    __syncthreads();
    const uint32_t first = hdr->buf_count + tile_offset[blockIdx.x];
    // row copies: U rows in flight per wave (one at a time the copy ran at 2 TB/s)
    constexpr uint32_t U = 8, W = kHoldThreads / kWave;
    for (uint32_t t0 = wave * U; t0 < total; t0 += W * U) {
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
                    const rsrc_t out = __builtin_amdgcn_make_buffer_rsrc(buf_grads + ((size_t)first + t0 + u) * D, 0, (int)(D * 4u), 0x00020000);
                    __builtin_amdgcn_raw_buffer_store_b128(v[u], out, (int)off, 0, 0);
                }
            }
        }
        if (lane < U && t0 + lane < total) buf_keys[(size_t)first + t0 + lane] = keys[s_src[t0 + lane]];
    }
}

__global__ void hold_commit_kernel(Header *hdr)
{
    if (threadIdx.x == 0 && !hdr->batch_bad) hdr->buf_count += hdr->n_held;
}

void launch_hold_back(const Scratch &s, const Geometry &g, const RecoveryView &rv, const uint64_t *keys,
                      const float *grads, uint32_t n, unsigned long long *buf_keys, float *buf_grads,
                      uint32_t buf_cap, hipStream_t st)
{
    const uint32_t ntiles = (n + kHoldTile - 1) / kHoldTile;
    uint32_t *tile_count = s.long_slot;            // free until the chain kernels run
    hipLaunchKernelGGL(hold_count_kernel, dim3(ntiles), dim3(kHoldThreads), 0, st, keys, n, g.rows, g.dk, g.dS, rv, tile_count);
    hipLaunchKernelGGL(hold_scan_kernel, dim3(1), dim3(1024), 0, st, tile_count, ntiles, s.hdr, n, buf_cap);
    hipLaunchKernelGGL(hold_scatter_kernel, dim3(ntiles), dim3(kHoldThreads), 0, st, keys, grads, n, g.rows, g.D, g.dk, g.dS,
                       rv, tile_count, s.hdr, buf_keys, buf_grads);
    hipLaunchKernelGGL(hold_commit_kernel, dim3(1), dim3(64), 0, st, s.hdr);
}

}  // namespace ecrm
