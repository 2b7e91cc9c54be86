// libsegkv measurement helper: the rate the matrix cores sustain on operands held in
// registers.  It puts the prefill kernel's TFLOP/s next to what the part delivers under
// its power limit: a chain of v_mfma_f32_32x32x16_f16 on constant operands runs near the
// published peak clock, the same chain on random operands (as Q, K and V are) settles at a
// much lower one.  No attention arithmetic here; nothing in the attention paths calls it.
#include "segkv_common.h"
#include "segkv_launch.h"

namespace segkv {

// One work-group of 4 waves; every wave cycles through 8 A and 8 B operands (its own 16
// bytes per lane of each) into 4 accumulators: 16 MFMAs per iteration, no memory traffic
// inside the loop.  clocks[2 g] = shader cycles, clocks[2 g + 1] = 100 MHz ticks of group g.
__global__ __launch_bounds__(256) void mfma_rate_probe_kernel(const half8_t* __restrict__ operands,
                                                              float* __restrict__ out,
                                                              unsigned long long* __restrict__ clocks,
                                                              int iters)
{
    const long long w0 = wall_clock64();
    const long long c0 = clock64();
    half8_t a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = operands[i * 256 + threadIdx.x];
        b[i] = operands[(8 + i) * 256 + threadIdx.x];
    }
    float16_t acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[i], acc[i & 3], 0, 0, 0);
            acc[(i + 1) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[(i + 3) & 7], b[(i + 5) & 7],
                                                                      acc[(i + 1) & 3], 0, 0, 0);
        }
    }
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[j][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
    if (threadIdx.x == 0) {
        clocks[2 * (size_t)blockIdx.x] = (unsigned long long)(clock64() - c0);
        clocks[2 * (size_t)blockIdx.x + 1] = (unsigned long long)(wall_clock64() - w0);
    }
}

hipError_t launch_mfma_rate_probe(const void* operands, float* out, unsigned long long* clocks,
                                  int n_groups, int iters, hipStream_t st)
{
    return SEGKV_LAUNCH(mfma_rate_probe_kernel, dim3((unsigned)n_groups), dim3(256), st,
                        (const half8_t*)operands, out, clocks, iters);
}

}  // namespace segkv
