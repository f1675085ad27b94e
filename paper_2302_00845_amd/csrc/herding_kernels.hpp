// Parallel herding objective (Sec. 3.2):
//     max_k || sum_{j<=k} sum_i ( z_{i, perm_i(j)} - zbar ) ||_inf ,  zbar = mean of all m*n vectors.
// The prefix over the n steps is cut into segments so that the evaluation is
// parallel over (segment, element): pass A sums every segment, pass B turns the
// segment sums into the mean and into each segment's centred starting prefix,
// pass C replays every segment from its starting prefix and keeps the largest
// magnitude.  All sums are double; the result is a maximum, so the order in which
// segments finish does not matter.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdgrab {

struct HerdingShape {
    int64_t m, n, d;
    int64_t segments;  // number of step segments
    int64_t seg_len;   // steps per segment (last one may be shorter)
};

__device__ __forceinline__ double herding_step_sum(const float *__restrict__ z, const int32_t *__restrict__ perm,
                                                   const HerdingShape &sh, int64_t j, int64_t e) {
    double v = 0.0;
    for (int64_t i = 0; i < sh.m; ++i) {
        int64_t id = perm ? (int64_t)perm[i * sh.n + j] : j;
        v += (double)z[(i * sh.n + id) * sh.d + e];
    }
    return v;
}

// Pass A: segsum[s][e] = sum over the segment's steps and all workers.
__global__ __launch_bounds__(256) void herding_segment_sums(const float *__restrict__ z,
                                                            const int32_t *__restrict__ perm, HerdingShape sh,
                                                            double *__restrict__ segsum)
{
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (g >= sh.segments * sh.d) return;
    const int64_t s = g / sh.d, e = g - s * sh.d;
    const int64_t j0 = s * sh.seg_len;
    const int64_t j1 = (j0 + sh.seg_len < sh.n) ? j0 + sh.seg_len : sh.n;
    double acc = 0.0;
    for (int64_t j = j0; j < j1; ++j) acc += herding_step_sum(z, perm, sh, j, e);
    segsum[g] = acc;
}

// Pass B (one thread per element): zbar[e] and start[s][e], the centred prefix
// before segment s.
__global__ __launch_bounds__(256) void herding_segment_offsets(const double *__restrict__ segsum, HerdingShape sh,
                                                               double *__restrict__ zbar,
                                                               double *__restrict__ start)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= sh.d) return;
    double total = 0.0;
    for (int64_t s = 0; s < sh.segments; ++s) total += segsum[s * sh.d + e];
    const double mean = total / (double)(sh.m * sh.n);
    zbar[e] = mean;
    double run = 0.0;
    for (int64_t s = 0; s < sh.segments; ++s) {
        start[s * sh.d + e] = run;
        const int64_t j0 = s * sh.seg_len;
        const int64_t len = ((j0 + sh.seg_len < sh.n) ? sh.seg_len : sh.n - j0);
        run += segsum[s * sh.d + e] - (double)(len * sh.m) * mean;
    }
}

// Pass C: replay each segment from its starting prefix; the largest |prefix| seen
// anywhere is folded into *bound with an integer max on the bit pattern (valid
// for non-negative doubles).
__global__ __launch_bounds__(256) void herding_prefix_max(const float *__restrict__ z,
                                                          const int32_t *__restrict__ perm, HerdingShape sh,
                                                          const double *__restrict__ zbar,
                                                          const double *__restrict__ start,
                                                          unsigned long long *__restrict__ bound_bits)
{
    __shared__ double wave_max[4];
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double mx = 0.0;
    if (g < sh.segments * sh.d) {
        const int64_t s = g / sh.d, e = g - s * sh.d;
        const int64_t j0 = s * sh.seg_len;
        const int64_t j1 = (j0 + sh.seg_len < sh.n) ? j0 + sh.seg_len : sh.n;
        const double centre = (double)sh.m * zbar[e];
        double acc = start[g];
        for (int64_t j = j0; j < j1; ++j) {
            acc += herding_step_sum(z, perm, sh, j, e) - centre;
            mx = fmax(mx, fabs(acc));
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmax(mx, __shfl_xor(mx, off, 64));
    if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = mx;
    __syncthreads();
    if (threadIdx.x == 0) {
        double b = fmax(fmax(wave_max[0], wave_max[1]), fmax(wave_max[2], wave_max[3]));
        atomicMax(bound_bits, (unsigned long long)__double_as_longlong(b));
    }
}

__global__ void herding_clear(unsigned long long *bound_bits) { *bound_bits = 0ull; }

}  // namespace cdgrab
