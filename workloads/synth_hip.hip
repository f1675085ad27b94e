// gfx950 build of the counter-based row generator (see synth_core.h): fills a
// staging block [count][2][d] on the GPU.  The exported function has the
// signature of the balancing library's generator callback.
#include <hip/hip_runtime.h>

#include "synth_core.h"

namespace {

__global__ __launch_bounds__(256) void synth_fill_kernel(synth_params p, uint64_t seed_mixed,
                                                         int64_t first_pair, float *__restrict__ staging)
{
    const int64_t r = blockIdx.y;  // row inside the block: 2*q + which
    const int64_t row = syn_row_of_pair(&p, first_pair + (r >> 1), (int)(r & 1));
    float *out = staging + r * p.d;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
    for (int64_t e = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; e < p.d; e += stride) {
        float v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = (e + q < p.d) ? syn_element(&p, seed_mixed, row, e + q) : 0.0f;
        if (e + 3 < p.d && (p.d & 3) == 0) {
            *reinterpret_cast<float4 *>(out + e) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) if (e + q < p.d) out[e + q] = v[q];
        }
    }
}

}  // namespace

extern "C" int synth_fill_pairs_device(void *ctx, int64_t first_pair, int64_t count, float *staging,
                                       void *stream)
{
    const synth_params *p = static_cast<const synth_params *>(ctx);
    if (!p || !staging || first_pair < 0 || count < 1 || count > 32767) return -1;
    if (first_pair + count > p->m * (p->n / 2)) return -2;
    int64_t per_row = (p->d + 1023) / 1024;
    unsigned gx = (unsigned)(per_row < 2048 ? per_row : 2048);
    hipLaunchKernelGGL(synth_fill_kernel, dim3(gx, (unsigned)(2 * count)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), *p, syn_seed_mixed(p->seed), first_pair, staging);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}
