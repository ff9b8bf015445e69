// Measurement aid, not part of the method: the access pattern of the update path's tables -- whole rows of 128
// floats at random row numbers, read and written back -- on two caller tables, so that a benchmark can see what the
// device's memory delivers for it depending on where the tables lie.
#include "ecrm_internal.h"

namespace ecrm {

typedef float probe_f2 __attribute__((ext_vector_type(2)));

// One wave per row, eight rows in flight per wave; rows alternate between the two tables.  WRITE: every row read
// is written back (plus one); otherwise the values are only summed.
template <bool WRITE>
__global__ __launch_bounds__(256) void row_traffic_kernel(float *ta, float *tb, const uint32_t *rows, uint32_t n,
                                                          float *sink)
{
    constexpr uint32_t U = 8;
    const uint32_t lane = lane_id(), wave = (blockIdx.x * blockDim.x + threadIdx.x) / kWave;
    const uint32_t nw = (gridDim.x * blockDim.x) / kWave;
    probe_f2 acc = {0.f, 0.f};
    for (uint32_t r = wave * U; r + U <= n; r += nw * U) {          // a tail of fewer than U rows is left out
        probe_f2 v[U];
        probe_f2 *p[U];
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            const uint32_t row = (uint32_t)__builtin_amdgcn_readfirstlane((int)rows[r + u]);
            p[u] = (probe_f2 *)(((u & 1u) ? tb : ta) + (size_t)row * 128u) + lane;
            v[u] = __builtin_nontemporal_load(p[u]);
        }
#pragma unroll
        for (uint32_t u = 0; u < U; ++u) {
            if (WRITE) {
                __builtin_nontemporal_store(v[u] + 1.0f, p[u]);
            } else {
                acc.x += v[u].x;
                acc.y += v[u].y;
            }
        }
    }
    if (!WRITE && acc.x == 12345.678f) sink[0] = acc.y;           // keeps the loads; practically never true
}

}  // namespace ecrm

extern "C" int ecrm_probe_row_traffic(float *table_a, float *table_b, uint64_t table_rows, const uint32_t *rows,
                                      uint64_t n, int write, float *sink, void *stream)
{
    using namespace ecrm;
    if (!table_a || !table_b || !rows || !sink || table_rows == 0 || n == 0 || n > 0xFFFFFFFFull) return ECRM_EINVAL;
    if (((uintptr_t)table_a | (uintptr_t)table_b) % 8 != 0) return ECRM_EINVAL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess) return ECRM_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return ECRM_EHIP;
    const dim3 grid(cus * 8), block(256);
    if (write)
        hipLaunchKernelGGL(row_traffic_kernel<true>, grid, block, 0, (hipStream_t)stream, table_a, table_b, rows, (uint32_t)n, sink);
    else
        hipLaunchKernelGGL(row_traffic_kernel<false>, grid, block, 0, (hipStream_t)stream, table_a, table_b, rows, (uint32_t)n, sink);
    return hipGetLastError() == hipSuccess ? ECRM_OK : ECRM_EHIP;
}
