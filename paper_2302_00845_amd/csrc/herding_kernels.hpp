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

#include "balance_kernels.hpp"

namespace cdgrab {

struct HerdingShape {
    int64_t m, n, d;
    int64_t segments;  // number of step segments
    int64_t seg_len;   // steps per segment (last one may be shorter)
    int32_t spw;       // segments per workgroup: 1 for long rows (a workgroup spans 1024 elements of
                       // one segment); 256 / quads for short rows (thread = (segment, four elements)),
                       // so that a 64-byte row still keeps every lane busy
    int32_t quads;     // ceil(d / 4)
};

// Which (segment, group of four elements) a thread serves.  Returns false for an idle thread.
__device__ __forceinline__ bool herding_thread_role(const HerdingShape &sh, int64_t &s, int64_t &qd) {
    if (sh.spw == 1) {
        s = blockIdx.y;
        qd = (int64_t)blockIdx.x * 256 + threadIdx.x;
        return qd < sh.quads;
    }
    const int sl = (int)threadIdx.x / sh.quads;
    qd = (int)threadIdx.x - sl * sh.quads;
    s = (int64_t)blockIdx.y * sh.spw + sl;
    return sl < sh.spw && s < sh.segments;
}

// Sum over the workers of elements e .. e+3 of step j's vectors.  VW = widest
// aligned load every row start allows (as in the balancing kernels).  ids: the m
// example ids of the step (LDS), or null: read perm (or take j) per worker.
template <int VW>
__device__ __forceinline__ void herding_step_sum(const float *__restrict__ z, const int32_t *__restrict__ perm,
                                                 const int32_t *ids, const HerdingShape &sh, int64_t j, int64_t e,
                                                 double v[4]) {
    v[0] = v[1] = v[2] = v[3] = 0.0;
#pragma unroll 8
    for (int64_t i = 0; i < sh.m; ++i) {
        const int64_t id = ids ? (int64_t)ids[i] : (perm ? (int64_t)perm[i * sh.n + j] : j);
        const float4 x = load4_nb<VW>(z + (i * sh.n + id) * sh.d, true, e, sh.d);  // branch-free: loads overlap
        v[0] += (double)x.x;
        v[1] += (double)x.y;
        v[2] += (double)x.z;
        v[3] += (double)x.w;
    }
}

// A workgroup serves one segment (blockIdx.y).  With lds_ids it first copies the
// segment's example ids perm[i][j0 .. j1) into LDS as ids[j - j0][i], so that the row
// loads of a step do not wait for a lookup of their own.
__device__ __forceinline__ const int32_t *herding_stage_ids(const int32_t *__restrict__ perm, const HerdingShape &sh,
                                                            int64_t j0, int64_t j1, int lds_ids, int32_t *ids_lds) {
    if (!lds_ids) return nullptr;
    const int64_t count = (j1 - j0) * sh.m;
    for (int64_t t = threadIdx.x; t < count; t += blockDim.x) {
        const int64_t jj = t / sh.m, i = t - jj * sh.m;
        ids_lds[t] = perm[i * sh.n + j0 + jj];
    }
    __syncthreads();
    return ids_lds;
}

// Pass A: segsum[s][e] = sum over the segment's steps and all workers.  One thread
// per (segment = blockIdx.y, four consecutive elements).
template <int VW>
__global__ __launch_bounds__(256) void herding_segment_sums(const float *__restrict__ z,
                                                            const int32_t *__restrict__ perm, HerdingShape sh,
                                                            int lds_ids, double *__restrict__ segsum)
{
    extern __shared__ int32_t ids_lds[];
    int64_t s, qd;
    const bool active = herding_thread_role(sh, s, qd);
    const int64_t j0 = s * sh.seg_len;
    const int64_t j1 = (j0 + sh.seg_len < sh.n) ? j0 + sh.seg_len : sh.n;
    // (ids are staged per workgroup, i.e. only when a workgroup serves one segment)
    const int32_t *ids = herding_stage_ids(perm, sh, j0, j1, sh.spw == 1 ? lds_ids : 0, ids_lds);
    if (!active) return;
    const int64_t e = qd * 4;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int64_t j = j0; j < j1; ++j) {
        double v[4];
        herding_step_sum<VW>(z, perm, ids ? ids + (j - j0) * sh.m : nullptr, sh, j, e, v);
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[q] += v[q];
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
        if (e + q < sh.d) segsum[s * sh.d + e + q] = acc[q];
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
#pragma unroll 8
    for (int64_t s = 0; s < sh.segments; ++s) total += segsum[s * sh.d + e];
    const double mean = total / (double)(sh.m * sh.n);
    zbar[e] = mean;
    double run = 0.0;
#pragma unroll 8
    for (int64_t s = 0; s < sh.segments; ++s) {
        start[s * sh.d + e] = run;
        const int64_t j0 = s * sh.seg_len;
        const int64_t len = ((j0 + sh.seg_len < sh.n) ? sh.seg_len : sh.n - j0);
        run += segsum[s * sh.d + e] - (double)(len * sh.m) * mean;
    }
}

// Pass B for short rows, where there are many segments and few elements: one workgroup per
// element; thread t takes a run of consecutive segments, the workgroup adds the runs' sums
// (mean), scans the centred run sums in thread order, and every thread then walks its run.
__global__ __launch_bounds__(256) void herding_segment_offsets_scan(const double *__restrict__ segsum,
                                                                    HerdingShape sh, double *__restrict__ zbar,
                                                                    double *__restrict__ start)
{
    __shared__ double part[256];
    const int64_t e = blockIdx.x;
    const int64_t run_len = (sh.segments + 255) / 256;
    const int64_t s0 = (int64_t)threadIdx.x * run_len;
    const int64_t s1 = (s0 + run_len < sh.segments) ? s0 + run_len : sh.segments;
    double local = 0.0;
    for (int64_t s = s0; s < s1; ++s) local += segsum[s * sh.d + e];
    part[threadIdx.x] = local;
    __syncthreads();
    double total = 0.0;
    for (int q = 0; q < 256; ++q) total += part[q];
    const double mean = total / (double)(sh.m * sh.n);
    __syncthreads();
    // steps covered by this thread's run (the last segment may be shorter)
    int64_t steps = 0;
    if (s0 < s1) {
        const int64_t j_first = s0 * sh.seg_len;
        const int64_t j_end = (s1 * sh.seg_len < sh.n) ? s1 * sh.seg_len : sh.n;
        steps = j_end - j_first;
    }
    part[threadIdx.x] = local - (double)(steps * sh.m) * mean;
    __syncthreads();
    double run = 0.0;
    for (int q = 0; q < (int)threadIdx.x; ++q) run += part[q];
    for (int64_t s = s0; s < s1; ++s) {
        start[s * sh.d + e] = run;
        const int64_t j0 = s * sh.seg_len;
        const int64_t len = ((j0 + sh.seg_len < sh.n) ? sh.seg_len : sh.n - j0);
        run += segsum[s * sh.d + e] - (double)(len * sh.m) * mean;
    }
    if (threadIdx.x == 0) zbar[e] = mean;
}

// Pass C: replay each segment from its starting prefix; the largest |prefix| seen
// anywhere is folded into *bound with an integer max on the bit pattern (valid
// for non-negative doubles).
template <int VW>
__global__ __launch_bounds__(256) void herding_prefix_max(const float *__restrict__ z,
                                                          const int32_t *__restrict__ perm, HerdingShape sh,
                                                          int lds_ids, const double *__restrict__ zbar,
                                                          const double *__restrict__ start,
                                                          unsigned long long *__restrict__ bound_bits)
{
    __shared__ double wave_max[4];
    extern __shared__ int32_t ids_lds[];
    int64_t s, qd;
    const bool active = herding_thread_role(sh, s, qd);
    const int64_t j0 = s * sh.seg_len;
    const int64_t j1 = (j0 + sh.seg_len < sh.n) ? j0 + sh.seg_len : sh.n;
    const int32_t *ids = herding_stage_ids(perm, sh, j0, j1, sh.spw == 1 ? lds_ids : 0, ids_lds);
    double mx = 0.0;
    if (active) {
        const int64_t e = qd * 4;
        double centre[4], acc[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool in = e + q < sh.d;  // elements beyond d load as zero and stay zero
            centre[q] = in ? (double)sh.m * zbar[e + q] : 0.0;
            acc[q] = in ? start[s * sh.d + e + q] : 0.0;
        }
        for (int64_t j = j0; j < j1; ++j) {
            double v[4];
            herding_step_sum<VW>(z, perm, ids ? ids + (j - j0) * sh.m : nullptr, sh, j, e, v);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                acc[q] += v[q] - centre[q];
                mx = fmax(mx, fabs(acc[q]));
            }
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
