// Permutation builders and the per-example gradient kernel for gfx950.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdgrab {

// ---------------------------------------------------------------------------
// Pair form of the reorder (one-step server algorithm, App. C.1): pair k of a
// worker contributes exactly one row to the front list and one to the back list,
// so the front pointer is k and the back pointer n-1-k -- no scan is needed.
//   eps = +1: the second row (2k+1) carries +1 and goes to the front.
__global__ void build_pair_permutations(const int8_t *__restrict__ signs, const int32_t *__restrict__ perm_in,
                                        int32_t *__restrict__ perm_out, int64_t m, int64_t n)
{
    const int64_t half = n / 2;
    int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= m * half) return;
    int64_t i = idx / half, k = idx - i * half;
    int eps = signs[idx];
    int64_t front = (eps == 1) ? 2 * k + 1 : 2 * k;
    int64_t back = (eps == 1) ? 2 * k : 2 * k + 1;
    const int32_t *pin = perm_in ? perm_in + i * n : nullptr;
    int32_t *pout = perm_out + i * n;
    pout[k] = pin ? pin[front] : (int32_t)front;
    pout[n - 1 - k] = pin ? pin[back] : (int32_t)back;
}

// ---------------------------------------------------------------------------
// General reorder from per-example signs (Sec. 2.1): a stable partition with the
// negative part reversed.  One workgroup per worker walks the n signs in chunks;
// an exclusive prefix count of +1 signs gives each positive its slot from the
// front and each negative its slot from the back.
constexpr int kScanThreads = 256;

__device__ __forceinline__ int wave_inclusive_scan(int v, int lane) {
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        int up = __shfl_up(v, off, 64);
        if (lane >= off) v += up;
    }
    return v;
}

__global__ __launch_bounds__(kScanThreads) void reorder_from_signs(const int8_t *__restrict__ signs,
                                                                   const int32_t *__restrict__ perm_in,
                                                                   int32_t *__restrict__ perm_out, int64_t n,
                                                                   int32_t *__restrict__ bad_flag)
{
    __shared__ int wave_tot[kScanThreads / 64];
    const int64_t i = blockIdx.x;
    const int8_t *sg = signs + i * n;
    const int32_t *pin = perm_in ? perm_in + i * n : nullptr;
    int32_t *pout = perm_out + i * n;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t pos_before = 0;  // +1 signs in earlier chunks
    for (int64_t base = 0; base < n; base += kScanThreads) {
        int64_t jpos = base + threadIdx.x;
        int s = (jpos < n) ? (int)sg[jpos] : 0;
        if (jpos < n && s != 1 && s != -1) atomicExch(bad_flag, 1);
        int is_pos = (s == 1) ? 1 : 0;
        int incl = wave_inclusive_scan(is_pos, lane);
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int wave_off = 0, chunk_tot = 0;
#pragma unroll
        for (int w = 0; w < kScanThreads / 64; ++w) {
            int tw = wave_tot[w];
            if (w < wave) wave_off += tw;
            chunk_tot += tw;
        }
        if (jpos < n) {
            int64_t pos_rank = pos_before + wave_off + incl - is_pos;  // exclusive count of +1
            int32_t id = pin ? pin[jpos] : (int32_t)jpos;
            if (is_pos) pout[pos_rank] = id;
            else pout[n - 1 - (jpos - pos_rank)] = id;                 // negatives fill from the back
        }
        pos_before += chunk_tot;
        __syncthreads();
    }
}

// s <- -s for n signs (the pair walk exports the sign of a pair's second row).
__global__ void negate_signs(int8_t *__restrict__ signs, int64_t n) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) signs[i] = (int8_t)(-signs[i]);
}

// mean_out[e] = (1/n) sum_j rows[j][e], accumulated in double, one thread per element.
__global__ void column_mean(const float *__restrict__ rows, int64_t n, int64_t d, float *__restrict__ mean_out) {
    int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d) return;
    double acc = 0.0;
    for (int64_t j = 0; j < n; ++j) acc += (double)rows[j * d + e];
    mean_out[e] = (float)(acc / (double)n);
}

// ---------------------------------------------------------------------------
// Per-example gradient of softmax cross-entropy for a linear model ("CD-GraB
// Workers", line 4).  One wavefront per example, each wavefront looping over
// examples: the example's features are staged in LDS, the logits are
// wave-reduced one class at a time, and the (in_dim+1) x classes outer product
// is written with coalesced 16-byte stores -- the kernel is bound by that write
// (about ten times the bytes it reads).  WLDS: the workgroup first copies the
// weights into LDS (rows padded to the odd length `wstride`, so that lanes on
// consecutive rows hit distinct banks); without it the weights are read from
// global memory with row length wstride = classes.
constexpr int kGradWaves = 8;  // wavefronts per workgroup (fewer when the features are long)
constexpr int kGradPrefetch = 16;  // feature registers per lane of the prefetch variant

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Orders one wavefront's LDS writes before its later LDS reads from other lanes.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <bool WLDS, bool PREFETCH>
__global__ __launch_bounds__(kGradWaves * 64) void softmax_pergrad(const float *__restrict__ X,
                                                                   const int32_t *__restrict__ y,
                                                                   const float *__restrict__ W,
                                                                   float *__restrict__ G, int64_t N,
                                                                   int in_dim, int classes, int wstride)
{
    // [WLDS: (in_dim + 1) x wstride weights] then per wave: in_dim + 1 features, `classes` deltas
    extern __shared__ float dyn[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nthreads = blockDim.x, nwaves = blockDim.x >> 6;  // 1 .. kGradWaves wavefronts
    const int per_wave = in_dim + 1 + classes;
    const int dd = (in_dim + 1) * classes;
    const float *Wv = W;
    float *xs = dyn + wave * per_wave;
    if (WLDS) {
        float *Wl = dyn;
        xs += (in_dim + 1) * wstride;
        const int qs = nthreads / classes, rs = nthreads % classes;
        int r = (int)threadIdx.x / classes;
        int c = (int)threadIdx.x - r * classes;
        for (int f = threadIdx.x; f < dd; f += nthreads) {
            Wl[r * wstride + c] = W[f];
            r += qs;
            c += rs;
            if (c >= classes) { c -= classes; ++r; }
        }
        __syncthreads();
        Wv = Wl;
    }
    float *delta = xs + in_dim + 1;

    // PREFETCH (in_dim <= 64 * kGradPrefetch): the next example's features are loaded
    // into registers while this example is worked on.
    const int64_t e_step = (int64_t)gridDim.x * nwaves;
    int64_t e = (int64_t)blockIdx.x * nwaves + wave;
    float xn[kGradPrefetch];
    if (PREFETCH && e < N) {
#pragma unroll
        for (int k = 0; k < kGradPrefetch; ++k) {
            const int r = lane + 64 * k;
            xn[k] = X[e * in_dim + (r < in_dim ? r : in_dim - 1)];  // clamped, not branched: the loads overlap
        }
    }
    for (; e < N; e += e_step) {
        if (PREFETCH) {
#pragma unroll
            for (int k = 0; k < kGradPrefetch; ++k) {
                const int r = lane + 64 * k;
                if (r < in_dim) xs[r] = xn[k];
            }
            if (e + e_step < N) {
#pragma unroll
                for (int k = 0; k < kGradPrefetch; ++k) {
                    const int r = lane + 64 * k;
                    xn[k] = X[(e + e_step) * in_dim + (r < in_dim ? r : in_dim - 1)];
                }
            }
        } else {
            const float *x = X + e * in_dim;
#pragma unroll 8
            for (int r = lane; r < in_dim; r += 64) xs[r] = x[r];
        }
        if (lane == 0) xs[in_dim] = 1.0f;  // bias input
        wave_lds_sync();

        float mx = -INFINITY;
        for (int c = 0; c < classes; ++c) {
            float part = 0.f;
#pragma unroll 4
            for (int r = lane; r <= in_dim; r += 64) part = fmaf(xs[r], Wv[r * wstride + c], part);
            const float z = wave_sum(part);
            if (lane == 0) delta[c] = z;
            mx = fmaxf(mx, z);
        }
        wave_lds_sync();
        float Z = 0.f;
        for (int c = lane; c < classes; c += 64) Z += expf(delta[c] - mx);
        Z = wave_sum(Z);
        const int label = y[e];
        for (int c = lane; c < classes; c += 64) {  // each lane rewrites only what it read
            const float p = expf(delta[c] - mx) / Z;
            delta[c] = p - (c == label ? 1.0f : 0.0f);
        }
        wave_lds_sync();

        // row e of G, element idx = r * classes + c.  A scalar head brings the row to a
        // 16-byte boundary, the body goes out as four-element stores, a scalar tail ends
        // it; (r, c) advances by increments, with no division inside the loop.
        float *g = G + e * (int64_t)dd;
        int head = (int)(((16u - (uint32_t)(reinterpret_cast<uintptr_t>(g) & 15u)) & 15u) >> 2);
        if (head > dd) head = dd;
        const int nvec = (dd - head) >> 2;
        const int tail0 = head + 4 * nvec;
        if (lane < head) g[lane] = xs[lane / classes] * delta[lane % classes];
        if (lane < dd - tail0) {
            const int idx = tail0 + lane;
            g[idx] = xs[idx / classes] * delta[idx % classes];
        }
        const int qs = 256 / classes, rs = 256 % classes;
        int r = (head + 4 * lane) / classes;
        int c = (head + 4 * lane) - r * classes;
#pragma unroll 2
        for (int v = lane; v < nvec; v += 64) {
            int rr = r, cc = c;
            float o[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                o[q] = xs[rr] * delta[cc];
                if (++cc == classes) { cc = 0; ++rr; }
            }
            *reinterpret_cast<float4 *>(g + head + 4 * v) = make_float4(o[0], o[1], o[2], o[3]);
            r += qs;
            c += rs;
            if (c >= classes) { c -= classes; ++r; }
        }
        wave_lds_sync();  // the next example overwrites xs and delta
    }
}

// ---------------------------------------------------------------------------
// One optimisation step of the m simulated workers ("CD-GraB Workers" lines 4-7
// with the server's average, "CD-GraB Parameter Server" lines 5-7), for the
// softmax-regression model.  Step j: worker i takes example perm[i][j].
//
// train_step_delta: one workgroup per worker computes delta_i = softmax(W^T [x;1]) - onehot(y)
// at the current weights, and the example's loss.  Each of the sixteen wavefronts
// takes classes w, w + 16, ..: its lanes split the rows of the dot product, with
// all loads of one class in flight together (the step is a chain of dependent
// launches, so latency is what counts), and a wave reduction gives the logit.
// One wavefront then takes the softmax.
constexpr int kDeltaWaves = 16;

__global__ __launch_bounds__(kDeltaWaves * 64) void train_step_delta(const float *__restrict__ X,
                                                                     const int32_t *__restrict__ y,
                                                                     const int32_t *__restrict__ perm,
                                                                     const float *__restrict__ W,
                                                                     float *__restrict__ delta_out,
                                                                     float *__restrict__ loss_out, int64_t m,
                                                                     int64_t n, int64_t j, int in_dim,
                                                                     int classes)
{
    extern __shared__ float logit[];  // `classes` floats
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t i = blockIdx.x;  // worker
    const int64_t id = perm ? (int64_t)perm[i * n + j] : j;
    const float *x = X + (i * n + id) * in_dim;
    for (int c = wave; c < classes; c += kDeltaWaves) {
        // sixteen rows per lane at a time, every load issued before the first use
        // (clamped indices instead of a ragged last batch: no branch between the loads)
        float part = 0.f;
        for (int r0 = lane; r0 <= in_dim; r0 += 64 * 16) {
            float xv[16], wv[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int r = r0 + 64 * u;
                const int rw = r <= in_dim ? r : in_dim;
                xv[u] = x[rw < in_dim ? rw : in_dim - 1];
                wv[u] = W[rw * classes + c];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int r = r0 + 64 * u;
                if (r <= in_dim) part = fmaf(r < in_dim ? xv[u] : 1.0f, wv[u], part);  // bias input 1
            }
        }
        const float z = wave_sum(part);
        if (lane == 0) logit[c] = z;
    }
    __syncthreads();
    if (wave != 0) return;
    float mx = -INFINITY;
    for (int c = lane; c < classes; c += 64) mx = fmaxf(mx, logit[c]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off, 64));
    float Z = 0.f;
    for (int c = lane; c < classes; c += 64) Z += expf(logit[c] - mx);
    Z = wave_sum(Z);
    const int label = y[i * n + id];
    for (int c = lane; c < classes; c += 64) {
        const float p = expf(logit[c] - mx) / Z;
        delta_out[i * classes + c] = p - (c == label ? 1.0f : 0.0f);
        if (c == label && loss_out) loss_out[i * n + j] = -(logit[c] - mx - logf(Z));
    }
}

// train_step_update: one thread per parameter p = (r, c).  Writes every worker's
// gradient row of this step into the staging chunk (pair-major: pair (k, i) of the
// chunk holds rows [2q], [2q+1] with q = (k - k_first) m + i) and optionally into
// grads_out[m][n][d], forms the average gradient and applies SGD with momentum
// (v <- momentum v + gbar; w <- w - lr v).
template <bool PERM>
__global__ __launch_bounds__(256) void train_step_update(const float *__restrict__ X,
                                                         const int32_t *__restrict__ perm,
                                                         const float *__restrict__ delta,
                                                         float *__restrict__ W, float *__restrict__ velocity,
                                                         float *__restrict__ staging,
                                                         float *__restrict__ grads_out, int64_t m, int64_t n,
                                                         int64_t j, int64_t k_first, int in_dim, int classes,
                                                         float lr, float momentum)
{
    const int64_t d = (int64_t)(in_dim + 1) * classes;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= d) return;
    const int r = (int)(p / classes);
    const int c = (int)(p - (int64_t)r * classes);
    const int rx = r < in_dim ? r : in_dim - 1;  // the bias row reads a valid feature and drops it
    const int64_t k = j >> 1;
    const int which = (int)(j & 1);
    constexpr int U = 8;  // workers per batch: all of a batch's loads are issued before its stores
    float sum = 0.f;
    for (int64_t i0 = 0; i0 < m; i0 += U) {
        float g[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = (i0 + u < m) ? i0 + u : m - 1;
            const int64_t id = PERM ? (int64_t)perm[i * n + j] : j;
            const float xv = X[(i * n + id) * in_dim + rx];
            g[u] = (r < in_dim ? xv : 1.0f) * delta[i * classes + c];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t i = i0 + u;
            if (i < m) {
                const int64_t q = (k - k_first) * m + i;
                staging[(2 * q + which) * d + p] = g[u];
                if (grads_out) grads_out[(i * n + j) * d + p] = g[u];
                sum += g[u];
            }
        }
    }
    const float gbar = sum / (float)m;
    float step = gbar;
    if (velocity) {
        step = momentum * velocity[p] + gbar;
        velocity[p] = step;
    }
    W[p] = W[p] - lr * step;
}

}  // namespace cdgrab
