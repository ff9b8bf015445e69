// The floating-point side of the ECRM update, on items already grouped by row (sort.hip):
//
//   apply_stripes   one 32-lane group per stripe: for each touched entry walk its updates in arrival
//                   order (Adagrad, Sec. 3.3.1), store the entry and its accumulator once, and add
//                   the entry's total difference in value and in accumulator to the stripe's parity
//                   rows (difference propagation, Sec. 3.3.2), which are read and written once.
//                   The differences of one call telescope, so adding their sum is the same as adding
//                   them one by one.
//
//   chains          entries that receive more than kLongRun updates in one call (the head of a
//                   skewed key distribution) are not walked by one group.  For a run g_1..g_m on one
//                   parameter, G_t = G_0 + sum_{s<=t} g_s^2 is a prefix sum and the entry moves by
//                   -lr * sum_t g_t / sqrt(G_t + eps); so the run is cut into pieces: (1) each piece
//                   sums its g^2, (2) a scan over the pieces gives every piece its starting
//                   accumulator, (3) each piece sums its steps, (4) the pieces' sums are added in
//                   order.  apply_stripes then takes the entry's totals from there.
//
// A "group" is half a wavefront: 32 lanes x float4 = one 128-float slice of a row, so one load
// instruction of a group moves 512 contiguous bytes.  All chain arithmetic is carried in fp64.
#include "ecrm_internal.h"

namespace ecrm {

struct Cols {                 // which floats of a row this lane holds in column block cb
    uint32_t col[2];
    bool on[2];
};

template <int NC>
__device__ __forceinline__ Cols lane_cols(uint32_t D, uint32_t cb)
{
    Cols c;
    const uint32_t gl = threadIdx.x & (kGroup - 1);
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        c.col[i] = (cb * NC + i) * 128u + gl * 4u;
        c.on[i] = c.col[i] < D;
    }
    return c;
}

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ double2 ldd2(const double *p) { return *reinterpret_cast<const double2 *>(p); }
__device__ __forceinline__ void std2(double *p, double2 v) { *reinterpret_cast<double2 *>(p) = v; }

struct D4 { double v[4]; };

__device__ __forceinline__ D4 ldd4(const double *p)
{
    const double2 a = ldd2(p), b = ldd2(p + 2);
    return D4{{a.x, a.y, b.x, b.y}};
}
__device__ __forceinline__ void std4(double *p, const D4 &d)
{
    std2(p, double2{d.v[0], d.v[1]});
    std2(p + 2, double2{d.v[2], d.v[3]});
}
__device__ __forceinline__ D4 widen4(float4 f) { return D4{{(double)f.x, (double)f.y, (double)f.z, (double)f.w}}; }
__device__ __forceinline__ float4 narrow4(const D4 &d)
{
    return float4{(float)d.v[0], (float)d.v[1], (float)d.v[2], (float)d.v[3]};
}
__device__ __forceinline__ void step4(D4 &G, D4 &acc, float4 g, double lr, double eps)
{
    adagrad_step(G.v[0], acc.v[0], g.x, lr, eps);
    adagrad_step(G.v[1], acc.v[1], g.y, lr, eps);
    adagrad_step(G.v[2], acc.v[2], g.z, lr, eps);
    adagrad_step(G.v[3], acc.v[3], g.w, lr, eps);
}
__device__ __forceinline__ void sumsq4(D4 &s, float4 g)
{
    s.v[0] = fma((double)g.x, (double)g.x, s.v[0]);
    s.v[1] = fma((double)g.y, (double)g.y, s.v[1]);
    s.v[2] = fma((double)g.z, (double)g.z, s.v[2]);
    s.v[3] = fma((double)g.w, (double)g.w, s.v[3]);
}

__device__ __forceinline__ uint32_t group_id() { return (blockIdx.x * blockDim.x + threadIdx.x) / kGroup; }
__device__ __forceinline__ uint32_t group_count() { return (gridDim.x * blockDim.x) / kGroup; }

// ================================================================================================
// split-chain path
// ================================================================================================

// Marks the heads of rows with more than kLongRun updates and gives each a slot.
__global__ __launch_bounds__(256) void long_find_kernel(const uint32_t *sk, uint32_t n, Header *hdr,
                                                        uint32_t *long_slot, uint32_t *long_head,
                                                        uint32_t max_slots)
{
    if (hdr->batch_bad) return;
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t p = blockIdx.x * blockDim.x + threadIdx.x; p + kLongRun < n; p += stride) {
        const uint32_t x = sk[p];
        if ((p == 0 || sk[p - 1] != x) && sk[p + kLongRun] == x) {
            const uint32_t slot = atomicAdd(&hdr->n_long, 1u);
            if (slot < max_slots) {          // always true: at most n / (kLongRun+1) such rows exist
                long_head[slot] = p;
                long_slot[p] = slot;
            }
        }
    }
}

// Length of each long run (binary search for its end) and its cut into pieces.
__global__ __launch_bounds__(256) void long_plan_kernel(const uint32_t *sk, uint32_t n, Header *hdr,
                                                        const uint32_t *long_head, uint32_t *long_len,
                                                        uint32_t *long_piece, uint32_t *long_count,
                                                        uint32_t *long_base, uint32_t *piece_slot,
                                                        uint32_t max_slots, uint32_t max_pieces)
{
    if (hdr->batch_bad) return;
    const uint32_t nl = min(hdr->n_long, max_slots);
    const uint32_t stride = gridDim.x * blockDim.x;
    for (uint32_t slot = blockIdx.x * blockDim.x + threadIdx.x; slot < nl; slot += stride) {
        const uint32_t p = long_head[slot];
        const uint32_t x = sk[p];
        uint32_t lo = p + kLongRun, hi = n;            // sk[lo] == x, sk[hi] != x (hi == n: past the end)
        while (hi - lo > 1) {
            const uint32_t mid = lo + (hi - lo) / 2;
            if (sk[mid] == x) lo = mid; else hi = mid;
        }
        const uint32_t L = hi - p;
        uint32_t C = (L + kPieceMaxCount - 1) / kPieceMaxCount;
        if (C < kPieceMin) C = kPieceMin;
        const uint32_t P = (L + C - 1) / C;
        const uint32_t base = atomicAdd(&hdr->n_pieces, P);
        atomicAdd(&hdr->n_long_items, (unsigned long long)L);
        long_len[slot] = L;
        long_piece[slot] = C;
        long_count[slot] = P;
        long_base[slot] = base;
        for (uint32_t j = 0; j < P; ++j)
            if (base + j < max_pieces) piece_slot[base + j] = slot;   // always true by the bound on pieces
    }
}

// Phase 1 (STEPS == false): partial[piece] = sum of g^2 over the piece.
// Phase 3 (STEPS == true):  partial[piece] holds the piece's starting accumulator on entry and the
//                           sum of its steps lr * g_t / sqrt(G_t + eps) on exit.
template <int NC, bool STEPS>
__global__ __launch_bounds__(256) void long_piece_kernel(const uint32_t *si, const float *grads, Header *hdr,
                                                         const uint32_t *long_head, const uint32_t *long_len,
                                                         const uint32_t *long_piece, const uint32_t *long_base,
                                                         const uint32_t *piece_slot, double *partial,
                                                         uint32_t max_pieces, Geometry geo)
{
    if (hdr->batch_bad) return;
    const uint32_t np = min(hdr->n_pieces, max_pieces);
    const uint32_t D = geo.D;
    const double lr = (double)geo.lr, eps = (double)geo.eps;
    constexpr int U = 8;
    for (uint32_t pc = group_id(); pc < np; pc += group_count()) {
        const uint32_t slot = piece_slot[pc];
        const uint32_t j = pc - long_base[slot];
        const uint32_t head = long_head[slot], L = long_len[slot], C = long_piece[slot];
        const uint32_t start = head + j * C;
        const uint32_t end = min(start + C, head + L);
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const Cols c = lane_cols<NC>(D, cb);
            D4 G[NC], acc[NC];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                acc[i] = D4{{0, 0, 0, 0}};
                G[i] = D4{{0, 0, 0, 0}};
                if (STEPS && c.on[i]) G[i] = ldd4(partial + (size_t)pc * D + c.col[i]);
            }
            for (uint32_t cur = start; cur < end; cur += U) {
                float4 g[U][NC];
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const bool live = cur + u < end;
                    const uint32_t idx = live ? si[cur + u] : 0;
#pragma unroll
                    for (int i = 0; i < NC; ++i) {
                        g[u][i] = float4{0, 0, 0, 0};
                        if (live && c.on[i]) g[u][i] = ld4(grads + (size_t)idx * D + c.col[i]);
                    }
                }
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    if (cur + u < end) {
#pragma unroll
                        for (int i = 0; i < NC; ++i) {
                            if (STEPS) step4(G[i], acc[i], g[u][i], lr, eps);
                            else sumsq4(acc[i], g[u][i]);
                        }
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < NC; ++i)
                if (c.on[i]) std4(partial + (size_t)pc * D + c.col[i], acc[i]);
        }
    }
}

// Phase 2: exclusive scan of the pieces' sums of squares, seeded with the stored accumulator;
// long_res[slot][1] receives the accumulator after the whole run.
template <int NC>
__global__ __launch_bounds__(256) void long_scan_kernel(const uint32_t *sk, const float *A, Header *hdr,
                                                        const uint32_t *long_head, const uint32_t *long_count,
                                                        const uint32_t *long_base, double *partial,
                                                        double *long_res, uint32_t max_slots, Geometry geo)
{
    if (hdr->batch_bad) return;
    const uint32_t nl = min(hdr->n_long, max_slots);
    const uint32_t D = geo.D;
    for (uint32_t slot = group_id(); slot < nl; slot += group_count()) {
        const uint32_t x = sk[long_head[slot]];
        const uint32_t P = long_count[slot], base = long_base[slot];
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const Cols c = lane_cols<NC>(D, cb);
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                if (!c.on[i]) continue;
                D4 G = widen4(ld4(A + (size_t)x * D + c.col[i]));
                double *p = partial + (size_t)base * D + c.col[i];
                for (uint32_t j = 0; j < P; ++j, p += D) {
                    const D4 t = ldd4(p);
                    std4(p, G);
#pragma unroll
                    for (int q = 0; q < 4; ++q) G.v[q] += t.v[q];
                }
                std4(long_res + ((size_t)slot * 2 + 1) * D + c.col[i], G);
            }
        }
    }
}

// Phase 4: long_res[slot][0] = sum over the pieces, in order, of their step sums.
template <int NC>
__global__ __launch_bounds__(256) void long_reduce_kernel(Header *hdr, const uint32_t *long_count,
                                                          const uint32_t *long_base, const double *partial,
                                                          double *long_res, uint32_t max_slots, Geometry geo)
{
    if (hdr->batch_bad) return;
    const uint32_t nl = min(hdr->n_long, max_slots);
    const uint32_t D = geo.D;
    for (uint32_t slot = group_id(); slot < nl; slot += group_count()) {
        const uint32_t P = long_count[slot], base = long_base[slot];
        for (uint32_t cb = 0; cb < geo.ncb; ++cb) {
            const Cols c = lane_cols<NC>(D, cb);
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                if (!c.on[i]) continue;
                D4 s = D4{{0, 0, 0, 0}};
                const double *p = partial + (size_t)base * D + c.col[i];
                for (uint32_t j = 0; j < P; ++j, p += D) {
                    const D4 t = ldd4(p);
#pragma unroll
                    for (int q = 0; q < 4; ++q) s.v[q] += t.v[q];
                }
                std4(long_res + ((size_t)slot * 2 + 0) * D + c.col[i], s);
            }
        }
    }
}

// ================================================================================================
// apply
// ================================================================================================

struct ApplyArgs {
    float *E, *A, *PE, *PA;
    const float *grads;
    const uint32_t *sk, *si;
    const uint32_t *long_slot, *long_len;
    const double *long_res;
    Header *hdr;
    const unsigned long long *cnt;
    unsigned long long *load_data, *load_parity;
    uint32_t n;
    Geometry geo;
};

// Processes the stripe whose first item sits at sorted position `pos`, for column block cb.
// Returns the position of the first item of the next stripe.
template <int NC>
__device__ __forceinline__ uint32_t apply_one_stripe(const ApplyArgs &a, uint32_t pos, uint32_t cb)
{
    const uint32_t D = a.geo.D, k = a.geo.k, n = a.n;
    const double lr = (double)a.geo.lr, eps = (double)a.geo.eps;
    const Cols c = lane_cols<NC>(D, cb);
    uint32_t key = a.sk[pos];
    const uint32_t g = key / k;

    D4 pe[NC], pa[NC];
#pragma unroll
    for (int i = 0; i < NC; ++i) {
        pe[i] = D4{{0, 0, 0, 0}};
        pa[i] = D4{{0, 0, 0, 0}};
        if (c.on[i]) {
            pe[i] = widen4(ld4(a.PE + (size_t)g * D + c.col[i]));
            pa[i] = widen4(ld4(a.PA + (size_t)g * D + c.col[i]));
        }
    }

    uint32_t cur = pos;
    do {
        const uint32_t x = key;                      // a new entry of this stripe starts at cur
        const bool is_long = (cur + kLongRun < n) && (a.sk[cur + kLongRun] == x);
        float4 e[NC], a0[NC];
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            e[i] = float4{0, 0, 0, 0};
            a0[i] = float4{0, 0, 0, 0};
            if (c.on[i]) {
                e[i] = ld4(a.E + (size_t)x * D + c.col[i]);
                a0[i] = ld4(a.A + (size_t)x * D + c.col[i]);
            }
        }
        D4 G[NC], acc[NC];
        if (is_long) {
            const uint32_t slot = a.long_slot[cur];
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                acc[i] = D4{{0, 0, 0, 0}};
                G[i] = D4{{0, 0, 0, 0}};
                if (c.on[i]) {
                    acc[i] = ldd4(a.long_res + ((size_t)slot * 2 + 0) * D + c.col[i]);
                    G[i] = ldd4(a.long_res + ((size_t)slot * 2 + 1) * D + c.col[i]);
                }
            }
            cur += a.long_len[slot];
        } else {
#pragma unroll
            for (int i = 0; i < NC; ++i) {
                G[i] = widen4(a0[i]);
                acc[i] = D4{{0, 0, 0, 0}};
            }
            float4 gr[NC];
            {
                const uint32_t idx = a.si[cur];
#pragma unroll
                for (int i = 0; i < NC; ++i) {
                    gr[i] = float4{0, 0, 0, 0};
                    if (c.on[i]) gr[i] = ld4(a.grads + (size_t)idx * D + c.col[i]);
                }
            }
            while (true) {
                ++cur;
                const bool same = (cur < n) && (a.sk[cur] == x);
                float4 nx[NC];
#pragma unroll
                for (int i = 0; i < NC; ++i) nx[i] = float4{0, 0, 0, 0};
                if (same) {                           // next gradient in flight while this one is used
                    const uint32_t idx = a.si[cur];
#pragma unroll
                    for (int i = 0; i < NC; ++i)
                        if (c.on[i]) nx[i] = ld4(a.grads + (size_t)idx * D + c.col[i]);
                }
#pragma unroll
                for (int i = 0; i < NC; ++i) step4(G[i], acc[i], gr[i], lr, eps);
                if (!same) break;
#pragma unroll
                for (int i = 0; i < NC; ++i) gr[i] = nx[i];
            }
        }
        // entry and accumulator: one rounding each; parity: add the differences
#pragma unroll
        for (int i = 0; i < NC; ++i) {
            if (!c.on[i]) continue;
            const D4 e64 = widen4(e[i]), a64 = widen4(a0[i]);
            D4 en;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                en.v[q] = e64.v[q] - acc[i].v[q];
                pe[i].v[q] -= acc[i].v[q];
                pa[i].v[q] += G[i].v[q] - a64.v[q];
            }
            st4(a.E + (size_t)x * D + c.col[i], narrow4(en));
            st4(a.A + (size_t)x * D + c.col[i], narrow4(G[i]));
        }
        key = cur < n ? a.sk[cur] : kNoKey;
    } while (cur < n && key / k == g);

#pragma unroll
    for (int i = 0; i < NC; ++i) {
        if (!c.on[i]) continue;
        st4(a.PE + (size_t)g * D + c.col[i], narrow4(pe[i]));
        st4(a.PA + (size_t)g * D + c.col[i], narrow4(pa[i]));
    }
    return cur;
}

template <int NC>
__global__ __launch_bounds__(256) void apply_stripes_kernel(ApplyArgs a)
{
    if (a.hdr->batch_bad) return;
    // the batch is valid: publish its per-server counts
    if (blockIdx.x == 0) {
        const uint32_t S = a.geo.S;
        for (uint32_t i = threadIdx.x; i < S; i += blockDim.x) {
            a.load_data[i] += a.cnt[i];
            a.load_parity[i] += a.cnt[S + i];
        }
    }
    const uint32_t n = a.n, k = a.geo.k;
    const uint32_t nchunks = (n + kChunk - 1) / kChunk;
    for (uint32_t ch = group_id(); ch < nchunks; ch += group_count()) {
        uint32_t pos = ch * kChunk;
        const uint32_t own_end = min(pos + kChunk, n);
        if (pos > 0) {
            // items at the front that belong to a stripe that started in an earlier chunk
            const uint32_t gprev = a.sk[pos - 1] / k;
            while (pos < own_end && a.sk[pos] / k == gprev) ++pos;
        }
        while (pos < own_end) {
            uint32_t next = pos;
            for (uint32_t cb = 0; cb < a.geo.ncb; ++cb) next = apply_one_stripe<NC>(a, pos, cb);
            pos = next;
        }
    }
}

// ================================================================================================
// encode and route
// ================================================================================================

__global__ __launch_bounds__(256) void encode_kernel(const float *E, const float *A, float *PE, float *PA,
                                                     uint32_t stripes, uint32_t D, uint32_t k)
{
    const uint32_t d4 = D / 4;
    const size_t total = (size_t)stripes * d4;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x; t < total; t += stride) {
        const size_t g = t / d4;
        const uint32_t col = (uint32_t)(t - g * d4) * 4u;
        D4 se = D4{{0, 0, 0, 0}}, sa = D4{{0, 0, 0, 0}};
        for (uint32_t j = 0; j < k; ++j) {
            const D4 e = widen4(ld4(E + (g * k + j) * D + col));
            const D4 s = widen4(ld4(A + (g * k + j) * D + col));
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                se.v[q] += e.v[q];
                sa.v[q] += s.v[q];
            }
        }
        st4(PE + g * D + col, narrow4(se));
        st4(PA + g * D + col, narrow4(sa));
    }
}

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

void launch_chains(const Scratch &s, const Geometry &g, const float *A, const float *grads,
                   const uint32_t *sk, const uint32_t *si, uint32_t n, uint32_t max_slots,
                   uint32_t max_pieces, int grid_blocks, hipStream_t st)
{
    if (n <= kLongRun) return;    // no row can have more than kLongRun updates
    const dim3 grid(grid_blocks), block(256);
    hipLaunchKernelGGL(long_find_kernel, grid, block, 0, st, sk, n, s.hdr, s.long_slot, s.long_head, max_slots);
    hipLaunchKernelGGL(long_plan_kernel, grid, block, 0, st, sk, n, s.hdr, s.long_head, s.long_len, s.long_piece,
                       s.long_count, s.long_base, s.piece_slot, max_slots, max_pieces);
#define ECRM_CHAIN_LAUNCH(NC)                                                                               \
    hipLaunchKernelGGL((long_piece_kernel<NC, false>), grid, block, 0, st, si, grads, s.hdr, s.long_head,   \
                       s.long_len, s.long_piece, s.long_base, s.piece_slot, s.partial, max_pieces, g);      \
    hipLaunchKernelGGL((long_scan_kernel<NC>), grid, block, 0, st, sk, A, s.hdr, s.long_head, s.long_count, \
                       s.long_base, s.partial, s.long_res, max_slots, g);                                   \
    hipLaunchKernelGGL((long_piece_kernel<NC, true>), grid, block, 0, st, si, grads, s.hdr, s.long_head,    \
                       s.long_len, s.long_piece, s.long_base, s.piece_slot, s.partial, max_pieces, g);      \
    hipLaunchKernelGGL((long_reduce_kernel<NC>), grid, block, 0, st, s.hdr, s.long_count, s.long_base,      \
                       s.partial, s.long_res, max_slots, g);
    if (g.nc == 1) { ECRM_CHAIN_LAUNCH(1) } else { ECRM_CHAIN_LAUNCH(2) }
#undef ECRM_CHAIN_LAUNCH
}

void launch_apply(const Scratch &s, const Geometry &g, float *E, float *A, float *PE, float *PA,
                  unsigned long long *load_data, unsigned long long *load_parity, const float *grads,
                  const uint32_t *sk, const uint32_t *si, uint32_t n, int grid_blocks, hipStream_t st)
{
    ApplyArgs a;
    a.E = E; a.A = A; a.PE = PE; a.PA = PA;
    a.grads = grads; a.sk = sk; a.si = si;
    a.long_slot = s.long_slot; a.long_len = s.long_len; a.long_res = s.long_res;
    a.hdr = s.hdr; a.cnt = s.cnt;
    a.load_data = load_data; a.load_parity = load_parity;
    a.n = n; a.geo = g;
    const dim3 grid(grid_blocks), block(256);
    if (g.nc == 1) hipLaunchKernelGGL(apply_stripes_kernel<1>, grid, block, 0, st, a);
    else hipLaunchKernelGGL(apply_stripes_kernel<2>, grid, block, 0, st, a);
}

void launch_encode(const Geometry &g, const float *E, const float *A, float *PE, float *PA,
                   int grid_blocks, hipStream_t st)
{
    hipLaunchKernelGGL(encode_kernel, dim3(grid_blocks), dim3(256), 0, st, E, A, PE, PA, g.rows / g.k, g.D, g.k);
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
