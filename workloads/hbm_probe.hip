// Measurement aids for bench.py -- not part of the method and not part of the
// balancing library: kernels of known HBM traffic against which the passes'
// achieved bandwidth and rocprofv3's traffic counters can be set.
//
//   hbm_probe_read : plain streaming read (non-temporal 16-byte loads, nothing else)
//   hbm_probe_copy : plain streaming copy (16-byte loads and stores)
//
// Both work on caller-provided device buffers and enqueue on the caller's stream;
// timing is done here with HIP events on that stream.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void probe_read_kernel(const f4v *__restrict__ p, int64_t count4,
                                                         float *__restrict__ sink)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    float acc = 0.f;
    for (; i < count4; i += stride) {
        f4v v = __builtin_nontemporal_load(p + i);
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 1234.5678f) sink[0] = acc;  // keeps the loads; never true for a zero-filled buffer
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const f4v *__restrict__ src, f4v *__restrict__ dst,
                                                         int64_t count4)
{
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * 256;
    for (; i < count4; i += stride) dst[i] = src[i];
}

int timed(hipStream_t stream, int reps, double *ms_out, void (*launch)(hipStream_t, void *), void *ctx) {
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return -3;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return -3; }
    int rc = 0;
    launch(stream, ctx);  // warm-up
    if (hipEventRecord(e0, stream) != hipSuccess) rc = -3;
    for (int q = 0; q < reps && rc == 0; ++q) launch(stream, ctx);
    if (rc == 0 && hipEventRecord(e1, stream) != hipSuccess) rc = -3;
    if (rc == 0 && hipEventSynchronize(e1) != hipSuccess) rc = -3;
    float ms = 0.f;
    if (rc == 0 && hipEventElapsedTime(&ms, e0, e1) != hipSuccess) rc = -3;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc == 0 && hipGetLastError() != hipSuccess) rc = -3;
    *ms_out = (double)ms / reps;
    return rc;
}

struct ReadCtx { const f4v *p; int64_t count4; float *sink; unsigned grid; };
struct CopyCtx { const f4v *src; f4v *dst; int64_t count4; unsigned grid; };

void launch_read(hipStream_t s, void *v) {
    ReadCtx *c = static_cast<ReadCtx *>(v);
    hipLaunchKernelGGL(probe_read_kernel, dim3(c->grid), dim3(256), 0, s, c->p, c->count4, c->sink);
}
void launch_copy(hipStream_t s, void *v) {
    CopyCtx *c = static_cast<CopyCtx *>(v);
    hipLaunchKernelGGL(probe_copy_kernel, dim3(c->grid), dim3(256), 0, s, c->src, c->dst, c->count4);
}

}  // namespace

// GB/s of a plain streaming read of buf[bytes] (dev, 16-byte aligned, zero-filled by the
// caller; the last 16 bytes serve as the sink).  Returns 0, -1 (bad argument) or -3 (HIP).
extern "C" int hbm_probe_read(const void *buf, int64_t bytes, int reps, void *stream, double *gb_per_s_out) {
    if (!buf || bytes < 4096 || reps < 1 || !gb_per_s_out || (reinterpret_cast<uintptr_t>(buf) & 15)) return -1;
    const int64_t count4 = bytes / 16 - 1;
    ReadCtx c{static_cast<const f4v *>(buf), count4,
              reinterpret_cast<float *>(const_cast<void *>(buf)) + count4 * 4, 2048u};
    double ms = 0.0;
    const int rc = timed(static_cast<hipStream_t>(stream), reps, &ms, launch_read, &c);
    if (rc == 0) *gb_per_s_out = (double)count4 * 16.0 / (ms * 1e-3) / 1e9;
    return rc;
}

// GB/s (read + written bytes) of a plain copy of `bytes` bytes from src to dst (dev, 16-byte
// aligned, not overlapping).  Returns 0, -1 or -3.
extern "C" int hbm_probe_copy(const void *src, void *dst, int64_t bytes, int reps, void *stream,
                              double *gb_per_s_out) {
    if (!src || !dst || bytes < 4096 || reps < 1 || !gb_per_s_out) return -1;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15) return -1;
    CopyCtx c{static_cast<const f4v *>(src), static_cast<f4v *>(dst), bytes / 16, 2048u};
    double ms = 0.0;
    const int rc = timed(static_cast<hipStream_t>(stream), reps, &ms, launch_copy, &c);
    if (rc == 0) *gb_per_s_out = 2.0 * (double)c.count4 * 16.0 / (ms * 1e-3) / 1e9;
    return rc;
}
