// Shared by the kernels of the update path (update.hip, chains.hip): whole-row access through buffer
// resources, the update rules, a few wave-level helpers, and the dispatch over (row width, rule).
#pragma once

#include "ecrm_internal.h"

namespace ecrm {


// A row (or the part of it that starts at column block cb) as a bounds-checked buffer resource:
// the base is wave-uniform and lives in scalar registers, each lane adds only its 32-bit byte
// offset, loads past the end of the row return 0 and stores past it are dropped -- so rows shorter
// than the 128 floats a wave spans need no lane predicates.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr int kRsrcFlags = 0x00020000;     // raw 32-bit data format (gfx9 family)

__device__ __forceinline__ rsrc_t row_f32(const float *table, uint32_t row, uint32_t D, uint32_t col0)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(table + (size_t)row * D + col0), 0,
                                             (int)((D - col0) * 4u), kRsrcFlags);
}
__device__ __forceinline__ rsrc_t row_f64(const double *table, size_t row, uint32_t D, uint32_t col0)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<double *>(table + row * D + col0), 0,
                                             (int)((D - col0) * 8u), kRsrcFlags);
}
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
// Cache policy of the row accesses (buffer instruction aux bits; 2 = non-temporal).  Every row is
// read once and written at most once per call, so nothing is worth keeping in L2 or the MALL;
// streaming hints measured 4 % faster on the apply kernel and 10 % on the chain kernels.
#ifndef ECRM_AUX_GRAD
#define ECRM_AUX_GRAD 2
#endif
#ifndef ECRM_AUX_LOAD
#define ECRM_AUX_LOAD 2
#endif
#ifndef ECRM_AUX_STORE
#define ECRM_AUX_STORE 2
#endif
// lane's float2 of 128-float slice i of the row
template <int AUX = ECRM_AUX_LOAD>
__device__ __forceinline__ float2 ld2(rsrc_t r, int i)
{
    return __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)(lane_id() * 8u + i * 512u), 0, AUX));
}
__device__ __forceinline__ float2 ldg2(rsrc_t r, int i) { return ld2<ECRM_AUX_GRAD>(r, i); }   // gradients: read once
__device__ __forceinline__ void st2(rsrc_t r, int i, float2 v)
{
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), r, (int)(lane_id() * 8u + i * 512u), 0, ECRM_AUX_STORE);
}

struct D2 { double x, y; };
__device__ __forceinline__ D2 ldd2(rsrc_t r, int i)
{
    const double2 v = __builtin_bit_cast(double2, __builtin_amdgcn_raw_buffer_load_b128(r, (int)(lane_id() * 16u + i * 1024u), 0, 0));
    return D2{v.x, v.y};
}
__device__ __forceinline__ void std2(rsrc_t r, int i, D2 d)
{
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, double2{d.x, d.y}), r, (int)(lane_id() * 16u + i * 1024u), 0, 0);
}
__device__ __forceinline__ D2 widen2(float2 f) { return D2{(double)f.x, (double)f.y}; }
__device__ __forceinline__ float2 narrow2(D2 d) { return float2{(float)d.x, (float)d.y}; }

// ---- update rules --------------------------------------------------------------------------------
// MODE = optimizer + how several updates to one entry inside a call are treated:
//   sequential: applied one after the other in arrival order (asynchronous training, Sec. 2.1, 3.3.2);
//   combined:   their gradients are summed and applied as ONE update (the synchronous variant sketched
//               in Sec. 4.4 "Synchronous training").
// Adagrad is the rule printed in Sec. 3.3.1.  Momentum SGD (the optimizer of the paper's evaluation,
// Sec. 4.1, which gives no formula) is taken as v <- mu*v + g, e <- e - lr*v, one state float per
// parameter.  For every rule a chain keeps a running value s and the sum acc of the steps taken; the
// entry moves by -acc and its state becomes s.
enum { kAdagradSeq = 0, kMomentumSeq = 1, kAdagradCombine = 2, kMomentumCombine = 3 };
struct RuleParams { double lr, eps, mu; };

template <int MODE>
struct Rule {
    static constexpr bool combine = MODE == kAdagradCombine || MODE == kMomentumCombine;
    static __device__ __forceinline__ double start(double state0) { return combine ? 0.0 : state0; }
    // one update g of the chain
    static __device__ __forceinline__ void item(double &s, double &acc, float gf, const RuleParams &p)
    {
        if (MODE == kAdagradSeq) adagrad_step(s, acc, gf, p.lr, p.eps);
        else if (MODE == kMomentumSeq) { s = fma(p.mu, s, (double)gf); acc = fma(p.lr, s, acc); }
        else s += (double)gf;
    }
    // what a piece of a long chain contributes when started from zero (phase 1 of the split chain)
    static __device__ __forceinline__ void summary(double &s, float gf, const RuleParams &p)
    {
        if (MODE == kAdagradSeq) s = fma((double)gf, (double)gf, s);
        else if (MODE == kMomentumSeq) s = fma(p.mu, s, (double)gf);
        else s += (double)gf;
    }
    // end of the chain: the combined rules take their single step here
    static __device__ __forceinline__ void finish(double &s, double &acc, double state0, const RuleParams &p)
    {
        if (MODE == kAdagradCombine) {
            const double g = s;
            double G = state0, a = 0.0;
            // one Adagrad step with the summed gradient (g is not an fp32 value: inline the step)
            G = fma(g, g, G);
            const double x = G + p.eps;
            double y = (double)__builtin_amdgcn_rsqf((float)x);
            const double h = 0.5 * x * y;
            y = fma(y, fma(-h, y, 0.5), y);
            a = p.lr * g * y;
            s = G;
            acc = a;
        } else if (MODE == kMomentumCombine) {
            const double v = fma(p.mu, state0, s);
            s = v;
            acc = p.lr * v;
        }
    }
};

template <int MODE>
__device__ __forceinline__ void item2(D2 &s, D2 &acc, float2 g, const RuleParams &p)
{
    Rule<MODE>::item(s.x, acc.x, g.x, p);
    Rule<MODE>::item(s.y, acc.y, g.y, p);
}
template <int MODE>
__device__ __forceinline__ void summary2(D2 &s, float2 g, const RuleParams &p)
{
    Rule<MODE>::summary(s.x, g.x, p);
    Rule<MODE>::summary(s.y, g.y, p);
}
template <int MODE>
__device__ __forceinline__ D2 start2(D2 state0) { return D2{Rule<MODE>::start(state0.x), Rule<MODE>::start(state0.y)}; }
template <int MODE>
__device__ __forceinline__ void finish2(D2 &s, D2 &acc, D2 state0, const RuleParams &p)
{
    Rule<MODE>::finish(s.x, acc.x, state0.x, p);
    Rule<MODE>::finish(s.y, acc.y, state0.y, p);
}
__device__ __forceinline__ RuleParams rule_params(const Geometry &g)
{
    return RuleParams{(double)g.lr, (double)g.eps, (double)g.mu};
}

__device__ __forceinline__ uint32_t wave_id() { return (blockIdx.x * blockDim.x + threadIdx.x) / kWave; }
__device__ __forceinline__ uint32_t wave_count() { return (gridDim.x * blockDim.x) / kWave; }
// value of v in lane j, j wave-uniform: the result is wave-uniform (scalar)
__device__ __forceinline__ uint32_t from_lane(uint32_t v, uint32_t j)
{
    return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)j);
}
__device__ __forceinline__ uint32_t uniform(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }
__device__ __forceinline__ uint32_t lowest_bit(unsigned long long m) { return (uint32_t)__builtin_ctzll(m); }
__device__ __forceinline__ unsigned long long bits_below(uint32_t j)      // j in 0..64
{
    return j >= 64 ? ~0ull : ((1ull << j) - 1ull);
}

// Blocks of `threads` threads of `kernel` that are resident on the whole device at once: the grid-stride
// kernels are launched with exactly that many, so that every block starts at time zero.  0 = the
// occupancy query failed.
template <typename K>
static int resident_grid(K kernel, int cus, int threads = 256)
{
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1) return 0;
    return cus * per_cu;
}

#define ECRM_DISPATCH(FN, ...)                                                   \
    do {                                                                         \
        if (g.nc == 1) {                                                         \
            switch (g.mode) {                                                    \
                case kAdagradSeq: FN<1, kAdagradSeq>(__VA_ARGS__); break;        \
                case kMomentumSeq: FN<1, kMomentumSeq>(__VA_ARGS__); break;      \
                case kAdagradCombine: FN<1, kAdagradCombine>(__VA_ARGS__); break; \
                default: FN<1, kMomentumCombine>(__VA_ARGS__); break;            \
            }                                                                    \
        } else {                                                                 \
            switch (g.mode) {                                                    \
                case kAdagradSeq: FN<2, kAdagradSeq>(__VA_ARGS__); break;        \
                case kMomentumSeq: FN<2, kMomentumSeq>(__VA_ARGS__); break;      \
                case kAdagradCombine: FN<2, kAdagradCombine>(__VA_ARGS__); break; \
                default: FN<2, kMomentumCombine>(__VA_ARGS__); break;            \
            }                                                                    \
        }                                                                        \
    } while (0)

}  // namespace ecrm
