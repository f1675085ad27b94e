// gfx950 build of the counter-based row generator (see synth_core.h): fills a
// staging block [count][2][d] on the GPU.  The exported function has the
// signature of the balancing library's generator callback.
#include <hip/hip_runtime.h>

#include "synth_core.h"

namespace {

typedef float syn_f4v __attribute__((ext_vector_type(4)));

// STREAM: the rows are written with streaming (non-temporal) stores, as a producer of
// write-once data would; otherwise with ordinary stores.
template <bool STREAM>
__global__ __launch_bounds__(256) void synth_fill_kernel(synth_params p, uint64_t seed_mixed,
                                                         int64_t first_pair, float *__restrict__ staging)
{
    const int64_t r = blockIdx.y;  // row inside the block: 2*q + which
    const int64_t row = syn_row_of_pair(&p, first_pair + (r >> 1), (int)(r & 1));
    float *out = staging + r * p.d;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x * 4;
    for (int64_t e = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 4; e < p.d; e += stride) {
        float v[4];
        // one division per four elements: the scale block of e, stepped when an element crosses into the next
        int64_t block = 0, left = 0;
        if (p.n_block_scales > 0) {
            block = (p.d <= 0xffffffffll) ? (int64_t)((uint32_t)e / (uint32_t)p.block_len) : e / p.block_len;
            left = (block + 1) * p.block_len - e;  // elements of this block from e on
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            // (blocks shorter than four elements can be crossed twice: divide again)
            const int64_t b = (p.n_block_scales <= 0 || q < left) ? block
                              : (p.block_len >= 4)                 ? block + 1
                                                                   : (e + q) / p.block_len;
            v[q] = (e + q < p.d) ? syn_element_in_block(&p, seed_mixed, row, e + q, b) : 0.0f;
        }
        if (e + 3 < p.d && (p.d & 3) == 0) {
            if constexpr (STREAM) {
                const syn_f4v val = {v[0], v[1], v[2], v[3]};
                __builtin_nontemporal_store(val, reinterpret_cast<syn_f4v *>(out + e));
            } else {
                *reinterpret_cast<float4 *>(out + e) = make_float4(v[0], v[1], v[2], v[3]);
            }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) if (e + q < p.d) out[e + q] = v[q];
        }
    }
}

// Reads `count4` float4 of a scratch buffer: run after the fill, it displaces the
// fill's not-yet-written-back lines from the last-level cache, so that the rows are
// in HBM (not half-way there) when the consumer's timed region starts.
__global__ __launch_bounds__(256) void synth_drain_kernel(const float4 *__restrict__ scratch, int64_t count4,
                                                          float *__restrict__ sink)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    float acc = 0.f;
    for (; i < count4; i += stride) {
        float4 v = scratch[i];
        acc += v.x + v.y + v.z + v.w;
    }
    if (acc == 123456.789f) sink[0] = acc;  // never true for the zero-filled scratch; keeps the loads
}

}  // namespace

// Optional cache drain after each fill: scratch must hold `floats` zero-filled floats.
static float *g_drain_scratch = nullptr;
static int64_t g_drain_floats = 0;
extern "C" int synth_set_drain(float *scratch /*dev or NULL*/, int64_t floats) {
    g_drain_scratch = scratch;
    g_drain_floats = scratch ? floats : 0;
    return 0;
}

// Store flavour of the fill kernel: 0 ordinary stores, 1 streaming (non-temporal) stores,
// 2 (default) chosen per block as a producer on the same GPU would: a block that fits the
// last-level cache (256 MB Infinity Cache + L2) is left cacheable, because the consumer reads
// it right away; a larger one is streamed, because most of it would only pass through the
// cache as dirty lines whose write-back then competes with the consumer's reads.
static int g_streaming_stores = 2;
static const int64_t kStreamAboveBytes = (int64_t)384 << 20;
extern "C" int synth_set_streaming_stores(int mode) {
    if (mode < 0 || mode > 2) return -1;
    g_streaming_stores = mode;
    return 0;
}

extern "C" int synth_fill_pairs_device(void *ctx, int64_t first_pair, int64_t count, float *staging,
                                       void *stream)
{
    const synth_params *p = static_cast<const synth_params *>(ctx);
    if (!p || !staging || first_pair < 0 || count < 1 || count > 32767) return -1;
    if (first_pair + count > p->m * (p->n / 2)) return -2;
    int64_t per_row = (p->d + 1023) / 1024;
    unsigned gx = (unsigned)(per_row < 2048 ? per_row : 2048);
    const bool stream_stores = g_streaming_stores == 1 ||
                               (g_streaming_stores == 2 && count * 2 * p->d * 4 > kStreamAboveBytes);
    if (stream_stores)
        hipLaunchKernelGGL(synth_fill_kernel<true>, dim3(gx, (unsigned)(2 * count)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), *p, syn_seed_mixed(p->seed), first_pair, staging);
    else
        hipLaunchKernelGGL(synth_fill_kernel<false>, dim3(gx, (unsigned)(2 * count)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), *p, syn_seed_mixed(p->seed), first_pair, staging);
    if (g_drain_scratch && g_drain_floats >= 8)
        hipLaunchKernelGGL(synth_drain_kernel, dim3(2048), dim3(256), 0, static_cast<hipStream_t>(stream),
                           reinterpret_cast<const float4 *>(g_drain_scratch), (g_drain_floats - 4) / 4,
                           g_drain_scratch + g_drain_floats - 1);
    return hipGetLastError() == hipSuccess ? 0 : -3;
}
