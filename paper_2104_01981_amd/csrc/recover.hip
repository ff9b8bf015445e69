// Recovery side of ECRM (Sec. 3.4) with the r = 1 sum code of Sec. 3.2: a lost entry is the parity
// minus the k-1 surviving entries of its stripe, a lost parity is the sum of its k entries.  All
// kernels stream whole rows: one wavefront per stripe (or per requested key), 64 lanes x float2 per
// 128-float slice through bounds-checked buffer resources with wave-uniform bases.
#include "ecrm_internal.h"

namespace ecrm {

typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
constexpr int kRsrcFlags = 0x00020000;

__device__ __forceinline__ rsrc_t row_of(const float *table, size_t row, uint32_t D)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(table + row * D), 0, (int)(D * 4u), kRsrcFlags);
}
__device__ __forceinline__ float2 ldr(rsrc_t r, uint32_t slice)
{
    return __builtin_bit_cast(float2, __builtin_amdgcn_raw_buffer_load_b64(r, (int)(lane_id() * 8u + slice * 512u), 0, 2));
}
__device__ __forceinline__ void str(rsrc_t r, uint32_t slice, float2 v)
{
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, v), r, (int)(lane_id() * 8u + slice * 512u), 0, 2);
}
__device__ __forceinline__ uint32_t uni(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

__global__ __launch_bounds__(256) void fail_server_kernel(float *E, float *A, float *PE, float *PA, uint32_t stripes,
                                                          uint32_t D, uint32_t k, uint32_t S, uint32_t server)
{
    const uint32_t nslices = (D + 127u) / 128u;
    const float nan = __builtin_nanf("");
    // 64-bit stripe counter: with close to 2^32 stripes (k = 1) g + nw would wrap a 32-bit one
    const uint64_t w0 = (blockIdx.x * blockDim.x + threadIdx.x) / kWave, nw = (gridDim.x * blockDim.x) / kWave;
    for (uint64_t g64 = w0; g64 < stripes; g64 += nw) {
        const uint32_t g = (uint32_t)g64;
        const int u = unit_on_server(g, k, S, server);
        if (u < 0) continue;
        const rsrc_t r0 = u == (int)k ? row_of(PE, g, D) : row_of(E, (size_t)g * k + u, D);
        const rsrc_t r1 = u == (int)k ? row_of(PA, g, D) : row_of(A, (size_t)g * k + u, D);
        for (uint32_t s = 0; s < nslices; ++s) {
            str(r0, s, float2{nan, nan});
            str(r1, s, float2{nan, nan});
        }
    }
}

// value of the lost unit of one table: parity lost -> sum of members; member lost -> p - others
__device__ __forceinline__ void rebuild_row(float *T, float *P, uint32_t g, int lost, uint32_t D, uint32_t k)
{
    const uint32_t nslices = (D + 127u) / 128u;
    for (uint32_t s = 0; s < nslices; ++s) {
        double x = 0.0, y = 0.0;
        if (lost != (int)k) {
            const float2 p = ldr(row_of(P, g, D), s);
            x = (double)p.x;
            y = (double)p.y;
        }
        // the surviving members only (the lost row is never read): m-th survivor is member m, or m+1 past the lost one
        const uint32_t nsrc = lost == (int)k ? k : k - 1u;
        for (uint32_t m0 = 0; m0 < nsrc; m0 += 4) {          // four member rows in flight
            float2 v[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t m = m0 + u;
                const uint32_t j = (int)m < lost ? m : m + 1u;
                v[u] = float2{0.f, 0.f};
                if (m < nsrc) v[u] = ldr(row_of(T, (size_t)g * k + j, D), s);
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                if (m0 + u < nsrc) {
                    if (lost == (int)k) { x += (double)v[u].x; y += (double)v[u].y; }
                    else { x -= (double)v[u].x; y -= (double)v[u].y; }
                }
            }
        }
        const rsrc_t out = lost == (int)k ? row_of(P, g, D) : row_of(T, (size_t)g * k + lost, D);
        str(out, s, float2{(float)x, (float)y});
    }
}

// stripes [g_lo, g_hi).  per_wave == 0: the waves of a resident grid stride over the range (a recovery
// that has the device to itself).  per_wave > 0: wave w takes stripes g_lo + w * per_wave ... of a grid
// sized to the range, so that workgroups retire all the time and the kernels of another stream -- the
// updates that go on during a recovery, Sec. 3.4 -- get their share of the device.
__global__ __launch_bounds__(256) void recover_server_kernel(float *E, float *A, float *PE, float *PA, uint32_t g_lo,
                                                             uint32_t g_hi, uint32_t D, uint32_t k, uint32_t S, uint32_t server,
                                                             uint32_t per_wave)
{
    const uint64_t w0 = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave, nw = ((uint64_t)gridDim.x * blockDim.x) / kWave;
    uint64_t first = (uint64_t)g_lo + w0, last = g_hi, step = nw;
    if (per_wave) {
        first = (uint64_t)g_lo + w0 * per_wave;
        last = first + per_wave < (uint64_t)g_hi ? first + per_wave : (uint64_t)g_hi;
        step = 1;
    }
    for (uint64_t g64 = first; g64 < last; g64 += step) {
        const uint32_t g = (uint32_t)g64;
        const int u = unit_on_server(g, k, S, server);
        if (u < 0) continue;
        rebuild_row(E, PE, g, u, D, k);
        rebuild_row(A, PA, g, u, D, k);
    }
}

// The encoder (Sec. 3.2 "Encoder and decoder"; run once before training, Sec. 3.1) is the same walk
// with every stripe's parity as the unit to build: PE[g] = sum_j E[k*g+j], PA likewise, summed in
// fp64 by increasing j and rounded once.
__global__ __launch_bounds__(256) void encode_kernel(const float *E, const float *A, float *PE, float *PA, uint32_t stripes,
                                                     uint32_t D, uint32_t k)
{
    const uint64_t w0 = (blockIdx.x * blockDim.x + threadIdx.x) / kWave, nw = (gridDim.x * blockDim.x) / kWave;
    for (uint64_t g64 = w0; g64 < stripes; g64 += nw) {
        const uint32_t g = (uint32_t)g64;
        rebuild_row(const_cast<float *>(E), PE, g, (int)k, D, k);
        rebuild_row(const_cast<float *>(A), PA, g, (int)k, D, k);
    }
}

__device__ __forceinline__ void read_row(const float *T, const float *P, uint32_t x, uint32_t g, uint32_t j, bool decode,
                                         float *out, size_t i, uint32_t D, uint32_t k)
{
    const uint32_t nslices = (D + 127u) / 128u;
    const rsrc_t dst = row_of(out, i, D);
    for (uint32_t s = 0; s < nslices; ++s) {
        if (!decode) {
            str(dst, s, ldr(row_of(T, x, D), s));
            continue;
        }
        const float2 p = ldr(row_of(P, g, D), s);
        double a = (double)p.x, b = (double)p.y;
        for (uint32_t m = 0; m < k; ++m) {
            if (m == j) continue;
            const float2 v = ldr(row_of(T, (size_t)g * k + m, D), s);
            a -= (double)v.x;
            b -= (double)v.y;
        }
        str(dst, s, float2{(float)a, (float)b});
    }
}

__global__ __launch_bounds__(256) void degraded_read_kernel(const float *E, const float *A, const float *PE, const float *PA,
                                                            const uint64_t *keys, uint64_t n, uint32_t rows, uint32_t D,
                                                            uint32_t k, uint32_t S, uint32_t lost, float *out_E, float *out_A,
                                                            Header *hdr)
{
    const uint64_t w0 = ((uint64_t)blockIdx.x * blockDim.x + threadIdx.x) / kWave, nw = ((uint64_t)gridDim.x * blockDim.x) / kWave;
    for (uint64_t i = w0; i < n; i += nw) {
        const uint64_t key = keys[i];
        const uint32_t hi = uni((uint32_t)(key >> 32)), x = uni((uint32_t)key);
        if (hi != 0 || x >= rows) {
            if (lane_id() == 0) atomicOr(&hdr->err_sticky, 1u);
            continue;
        }
        const uint32_t g = x / k, j = x - g * k;
        const bool decode = lost != ECRM_NO_SERVER && (g + 1u + j) % S == lost;
        read_row(E, PE, x, g, j, decode, out_E, i, D, k);
        if (out_A) read_row(A, PA, x, g, j, decode, out_A, i, D, k);
    }
}

void launch_encode(const Geometry &g, const float *E, const float *A, float *PE, float *PA,
                   int grid_blocks, hipStream_t st)
{
    hipLaunchKernelGGL(encode_kernel, dim3(grid_blocks), dim3(256), 0, st, E, A, PE, PA, g.rows / g.k, g.D, g.k);
}

void launch_fail_server(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                        int grid_blocks, hipStream_t st)
{
    hipLaunchKernelGGL(fail_server_kernel, dim3(grid_blocks), dim3(256), 0, st, E, A, PE, PA, g.rows / g.k, g.D, g.k, g.S, server);
}

void launch_recover_server(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                           int grid_blocks, hipStream_t st)
{
    launch_recover_range(g, E, A, PE, PA, server, 0, g.rows / g.k, grid_blocks, st);
}

// grid_blocks > 0: a resident grid of that many workgroups; 0: a grid sized to the range (see the kernel)
void launch_recover_range(const Geometry &g, float *E, float *A, float *PE, float *PA, uint32_t server,
                          uint32_t g_lo, uint32_t g_hi, int grid_blocks, hipStream_t st)
{
    if (g_lo >= g_hi) return;
    uint32_t per_wave = 0;
    if (grid_blocks <= 0) {
        constexpr uint32_t kWavesPerBlock = 256 / kWave;
        per_wave = 16;
        uint64_t blocks = ((uint64_t)(g_hi - g_lo) + per_wave * kWavesPerBlock - 1) / (per_wave * kWavesPerBlock);
        while (blocks > (1u << 24)) {                  // keep the grid moderate for the very largest tables
            per_wave *= 2;
            blocks = ((uint64_t)(g_hi - g_lo) + per_wave * kWavesPerBlock - 1) / (per_wave * kWavesPerBlock);
        }
        grid_blocks = (int)blocks;
    }
    hipLaunchKernelGGL(recover_server_kernel, dim3(grid_blocks), dim3(256), 0, st, E, A, PE, PA, g_lo, g_hi, g.D, g.k, g.S,
                       server, per_wave);
}

void launch_degraded_read(const Scratch &s, const Geometry &g, const float *E, const float *A, const float *PE,
                          const float *PA, const uint64_t *keys, uint64_t n, uint32_t lost, float *out_E,
                          float *out_A, int grid_blocks, hipStream_t st)
{
    hipLaunchKernelGGL(degraded_read_kernel, dim3(grid_blocks), dim3(256), 0, st, E, A, PE, PA, keys, n, g.rows, g.D, g.k, g.S,
                       lost, out_E, out_A, s.hdr);
}

}  // namespace ecrm
