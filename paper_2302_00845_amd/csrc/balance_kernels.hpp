// Blocked pair-balancing kernels for gfx950 (CDNA4).
//
// The greedy walk of CD-GraB (App. B.2 "Balancing without normalization" applied
// pair by pair in the server algorithm's order, Sec. 3.3) decides each sign from
// <r, d_k>, where r already contains the earlier differences.  For a block of Bb
// consecutive differences
//     <r + sum_{j<k} eps_j d_j, d_k> = <r, d_k> + sum_{j<k} eps_j <d_j, d_k>,
// so one pass over the rows yields everything the Bb decisions need: the Bb dots
// with the block-start running sum and the Bb x Bb Gram matrix.  A single
// wavefront then resolves the signs in order, and a second pass applies
// r += sum_k eps_k d_k.  Each gradient row is read from HBM twice per epoch.
//
// Arithmetic: rows are fp32; differences are formed in double (exact), dots with
// r are double FMAs, the Gram matrix is accumulated by the double-precision MFMA
// (products of two exact fp32 differences are exact in double), and all
// cross-lane / cross-workgroup sums are taken in a fixed order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace cdgrab {

constexpr int kThreads = 256;       // workgroup size of the streaming kernels
constexpr int kWaves = kThreads / 64;
constexpr int kPadE = 128;          // the running sum is padded to a multiple of this many elements

typedef double double4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef float float2_t __attribute__((ext_vector_type(2)));

// Where the rows of the current block live: element offsets from `base` of the
// first and second row of each pair, filled in by the host (dense input [m][n][d]:
// flattened pair p belongs to worker p % m and is its pair p / m; a staging block
// is [Bb][2][d]).  Passed by value: uniform indices become scalar loads.
constexpr int kMaxBlockPairs = 64;

struct RowMap {
    const float *base;
    int64_t d;
    int64_t n;
    int64_t k0;     // pair index (per worker) of the block's first flattened pair
    int32_t i0;     // worker of the block's first flattened pair
    int32_t m;
    int32_t nb;     // valid pairs in this block (<= Bb)
    int32_t dense;  // 1: the rows are those of a dense input [m][n][d] in its own order
    int64_t off[2 * kMaxBlockPairs];  // off[2 j + which]

    __device__ __forceinline__ const float *row(int j, int which) const { return base + off[2 * j + which]; }
    // Same address without the table, for dense input: pair j of the block is pair
    // k0 + (i0 + j) / m of worker (i0 + j) % m.  A per-thread j costs a memory round trip
    // through the table and a few integer instructions this way.
    __device__ __forceinline__ const float *dense_row(int j, int which) const {
        const uint32_t q = (uint32_t)(i0 + j);
        const uint32_t dk = q / (uint32_t)m;
        const int64_t i = (int64_t)(q - dk * (uint32_t)m), k = k0 + (int64_t)dk;
        return base + (i * n + 2 * k + which) * d;
    }
};

// Four consecutive fp32 elements starting at element e of a row, zero beyond d or
// for a missing row.  VW is the widest load the row alignment allows (4, 2 or 1
// floats).  Rows are read exactly once per pass, so the loads carry the
// non-temporal hint: the streamed rows then do not evict the running sum, which
// is re-read and rewritten every block, from the last-level cache.
template <int VW>
__device__ __forceinline__ float4 load4(const float *row, int64_t e, int64_t d) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (row == nullptr) return v;
    if constexpr (VW == 4) {
        if (e < d) {
            float4_t t = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(row + e));
            v = make_float4(t.x, t.y, t.z, t.w);
        }
    } else if constexpr (VW == 2) {
        if (e < d) { float2_t t = __builtin_nontemporal_load(reinterpret_cast<const float2_t *>(row + e)); v.x = t.x; v.y = t.y; }
        if (e + 2 < d) { float2_t t = __builtin_nontemporal_load(reinterpret_cast<const float2_t *>(row + e + 2)); v.z = t.x; v.w = t.y; }
    } else {
        if (e < d) v.x = __builtin_nontemporal_load(row + e);
        if (e + 1 < d) v.y = __builtin_nontemporal_load(row + e + 1);
        if (e + 2 < d) v.z = __builtin_nontemporal_load(row + e + 2);
        if (e + 3 < d) v.w = __builtin_nontemporal_load(row + e + 3);
    }
    return v;
}

// The same without a branch, for launches that are bound by latency rather than by
// bytes: `row` must be readable at its first elements whether or not `have` is set,
// out-of-range parts read the row's start instead and are replaced by zero afterwards.
// (A load inside an `if` ends in a wait for it before the next one is issued; with
// straight-line code all loads of a thread are in flight together.)
template <int VW>
__device__ __forceinline__ float4 load4_nb(const float *row, bool have, int64_t e, int64_t d) {
    float4 v;
    if constexpr (VW == 4) {
        const bool in = have && e < d;
        const float4_t t = __builtin_nontemporal_load(reinterpret_cast<const float4_t *>(row + (in ? e : 0)));
        v = make_float4(in ? t.x : 0.f, in ? t.y : 0.f, in ? t.z : 0.f, in ? t.w : 0.f);
    } else if constexpr (VW == 2) {
        const bool in0 = have && e < d, in1 = have && e + 2 < d;
        const float2_t t0 = __builtin_nontemporal_load(reinterpret_cast<const float2_t *>(row + (in0 ? e : 0)));
        const float2_t t1 = __builtin_nontemporal_load(reinterpret_cast<const float2_t *>(row + (in1 ? e + 2 : 0)));
        v = make_float4(in0 ? t0.x : 0.f, in0 ? t0.y : 0.f, in1 ? t1.x : 0.f, in1 ? t1.y : 0.f);
    } else {
        float o[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool in = have && e + q < d;
            const float t = __builtin_nontemporal_load(row + (in ? e + q : 0));
            o[q] = in ? t : 0.f;
        }
        v = make_float4(o[0], o[1], o[2], o[3]);
    }
    return v;
}

// Number of doubles one workgroup of the dot/Gram pass emits: the Gram tiles in
// the MFMA accumulator layout (tile * 256 + v * 64 + lane) followed by Bb dots.
template <int BB> struct PartLayout {
    static constexpr int RG = BB / 16;               // 16-row groups
    static constexpr int NT = RG * (RG + 1) / 2;     // upper-triangular 16x16 tiles
    static constexpr int GRAM = NT * 256;
    static constexpr int PART = GRAM + BB;
};

// Row / column of accumulator element v of lane `lane` in the 16x16 result of
// v_mfma_f64_16x16x4_f64: column = lane % 16, row = 4 * v + lane / 16
// (measured on gfx950 with a rank-one probe).
__device__ __forceinline__ void mfma_f64_16x16_coord(int lane, int v, int &i, int &j) {
    j = lane & 15;
    i = 4 * v + (lane >> 4);
}

// ---------------------------------------------------------------------------
// Pass 1: partial dots <r, d_k> and partial Gram <d_j, d_k> over a strided set
// of TE-element tiles of d.  One workgroup = 4 waves; each tile is staged
// through LDS (coalesced 16 B global loads -> row-per-lane MFMA operands), with
// the next tile's loads in flight while the current one is consumed.
// Lane (row = lane % 16, kslot = lane / 16) of wave w owns elements
// (TE/4) w + 16 s + 4 kslot .. +3 (s = 0 .. TE/64-1) of the tile for pair `row`
// of each 16-pair group.  TE = 128 halves the barriers per byte and is the
// streaming configuration; TE = 64 gives short rows more workgroups.
//
// With APPLY the same launch first applies the PREVIOUS block to the tile's slice
// of the running sum (r += sum_k eps_k d_k over prev's rows, the work of pass 2):
// every thread adds up the signed rows it loads, the RPI partial sums per element
// are added in row order through LDS, the new slice is written back and is the one
// the current block's dots are taken against.  The running sum is then read once
// and written once per block, and a block costs one streaming launch instead of two.
struct PrevBlock {
    RowMap rm;           // rows of the previous block
    const int8_t *eps;   // its resolved signs
};

// Several independent walks of the same shape in one launch (the uncoordinated baseline:
// every worker balances its own rows on its own running sum).  The walk is a grid
// coordinate; everything a walk owns lies at a fixed element stride from the first walk's.
// All strides are zero for a single walk.
struct WalkStrides {
    int64_t rows;   // floats from walk w's rows to walk w+1's
    int64_t r;      // doubles between running sums
    int64_t gram;   // doubles between the walks' reduced Gram tiles
    int64_t dots;   // doubles between the walks' per-workgroup dots
    int64_t out;    // entries between the walks' slices of signs_out / dots_out
    int64_t maps;   // row maps per walk
};

// `group` of `ngroups` workgroups share the tiles; the workgroup's result goes to `out`.
template <int BB, int VW, int TE, bool APPLY, bool NB>
__device__ __forceinline__ void pass1_body(const RowMap &rm, const PrevBlock &prev, double *__restrict__ r_sum,
                                           double *__restrict__ out, int64_t ntiles, int group, int ngroups)
{
    using L = PartLayout<BB>;
    constexpr int RG = L::RG;
    constexpr int TPR = TE / 4;               // threads covering one row of the tile
    constexpr int RPI = kThreads / TPR;       // rows covered by one load instruction
    constexpr int LOADS = 2 * BB / RPI;       // 16 B loads per thread per tile
    constexpr int STRIDE = TE + 4;            // floats per LDS row (16 B aligned, bank-skewed)
    constexpr int TILE_FLOATS = BB * STRIDE;
    constexpr int EPW = TE / kWaves;          // elements per wave per tile
    // LDS: two stages of (first rows, second rows, running-sum chunk), with APPLY one
    // buffer of RPI partial sums per element; the final cross-wave reduction reuses
    // the same bytes.
    constexpr int STAGE_BYTES = 2 * TILE_FLOATS * 4 + TE * 8;
    constexpr int APPLY_BYTES = APPLY ? RPI * TE * 8 : 0;
    constexpr int RED_BYTES = kWaves * (L::GRAM + RG * 64) * 8;
    constexpr int SMEM = (2 * STAGE_BYTES + APPLY_BYTES > RED_BYTES) ? 2 * STAGE_BYTES + APPLY_BYTES : RED_BYTES;
    __shared__ __attribute__((aligned(16))) unsigned char smem[SMEM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int64_t d = rm.d;

    const int lrow = tid / TPR;
    const int chunk = tid % TPR;
    const float *src[LOADS];
    const float *psrc[APPLY ? LOADS : 1];
    float psign[APPLY ? LOADS : 1];
    int lds_off[LOADS];
    uint32_t have_mask = 0;  // bit u: load u's pair exists in this block
#pragma unroll
    for (int u = 0; u < LOADS; ++u) {
        int rr = u * RPI + lrow;       // 0 .. 2*BB-1
        int j = rr >> 1, which = rr & 1;
        // the table is read without a branch (entries of missing pairs are readable rows:
        // zero, or those of an earlier block), so that the lookups overlap
        src[u] = rm.row(j, which);
        if (j < rm.nb) have_mask |= 1u << u;
        lds_off[u] = (which * TILE_FLOATS + j * STRIDE + chunk * 4) * 4;
        if constexpr (APPLY) {
            const bool have = j < prev.rm.nb;
            psrc[u] = prev.rm.row(j, which);
            const float ej = (float)prev.eps[j];  // 64 entries, always readable
            // d_k = second - first, so the second row enters with eps and the first with -eps
            // (a missing pair enters with sign 0)
            psign[u] = have ? ej * (which ? 1.0f : -1.0f) : 0.0f;
        }
    }

    // NB (one block of short rows: one or two tiles per workgroup, the launch is bound by
    // latency): loads without branches; the streaming uses keep the plain loads.  Rows of
    // the previous block that do not exist enter with sign 0, so they need no zeroing.
    auto tile_load = [&](const float *row, bool have, int64_t e) {
        if constexpr (NB) return load4_nb<VW>(row, have, e, d);
        else return load4<VW>(have ? row : nullptr, e, d);
    };

    double4_t acc[L::NT];
#pragma unroll
    for (int q = 0; q < L::NT; ++q) acc[q] = (double4_t){0.0, 0.0, 0.0, 0.0};
    double pdot[RG];
#pragma unroll
    for (int g = 0; g < RG; ++g) pdot[g] = 0.0;

    const int mrow = lane & 15;
    const int kslot = lane >> 4;

    float4 stage_regs[LOADS];
    float4 prev_regs[APPLY ? LOADS : 1];
    double2 stage_s = make_double2(0.0, 0.0);

    int64_t tile = group;
    if (tile < ntiles) {
#pragma unroll
        for (int u = 0; u < LOADS; ++u) stage_regs[u] = tile_load(src[u], (have_mask >> u) & 1u, tile * TE + chunk * 4);
        if constexpr (APPLY) {
#pragma unroll
            for (int u = 0; u < LOADS; ++u) prev_regs[u] = tile_load(psrc[u], true, tile * TE + chunk * 4);
        }
        if (tid < TE / 2) stage_s = *reinterpret_cast<const double2 *>(r_sum + tile * TE + tid * 2);
    }
    int buf = 0;
    for (; tile < ntiles; tile += ngroups) {
        unsigned char *stage = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int u = 0; u < LOADS; ++u)
            *reinterpret_cast<float4 *>(stage + lds_off[u]) = stage_regs[u];
        if constexpr (APPLY) {
            // this thread's signed sum of the previous block's rows it holds
            double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
#pragma unroll
            for (int u = 0; u < LOADS; ++u) {
                const double sg = (double)psign[u];
                a0 = __builtin_fma(sg, (double)prev_regs[u].x, a0);
                a1 = __builtin_fma(sg, (double)prev_regs[u].y, a1);
                a2 = __builtin_fma(sg, (double)prev_regs[u].z, a2);
                a3 = __builtin_fma(sg, (double)prev_regs[u].w, a3);
            }
            double *ap = reinterpret_cast<double *>(smem + 2 * STAGE_BYTES) + lrow * TE + chunk * 4;
            *reinterpret_cast<double2 *>(ap) = make_double2(a0, a1);
            *reinterpret_cast<double2 *>(ap + 2) = make_double2(a2, a3);
            __syncthreads();
            if (tid < TE / 2) {
                const double *col = reinterpret_cast<const double *>(smem + 2 * STAGE_BYTES) + tid * 2;
                double s0 = 0.0, s1 = 0.0;
#pragma unroll
                for (int q = 0; q < RPI; ++q) { s0 += col[q * TE]; s1 += col[q * TE + 1]; }
                stage_s.x += s0;
                stage_s.y += s1;
                *reinterpret_cast<double2 *>(r_sum + tile * TE + tid * 2) = stage_s;
            }
        }
        if (tid < TE / 2)
            *reinterpret_cast<double2 *>(stage + 2 * TILE_FLOATS * 4 + tid * 16) = stage_s;
        __syncthreads();

        // prefetch the next tile while this one is consumed
        int64_t nxt = tile + ngroups;
        if (nxt < ntiles) {
#pragma unroll
            for (int u = 0; u < LOADS; ++u) stage_regs[u] = tile_load(src[u], (have_mask >> u) & 1u, nxt * TE + chunk * 4);
            if constexpr (APPLY) {
#pragma unroll
                for (int u = 0; u < LOADS; ++u) prev_regs[u] = tile_load(psrc[u], true, nxt * TE + chunk * 4);
            }
            if (tid < TE / 2) stage_s = *reinterpret_cast<const double2 *>(r_sum + nxt * TE + tid * 2);
        }

        const float *first = reinterpret_cast<const float *>(stage);
        const float *second = first + TILE_FLOATS;
        const double *sv = reinterpret_cast<const double *>(stage + 2 * TILE_FLOATS * 4);
#pragma unroll
        for (int ks = 0; ks < EPW / 16; ++ks) {
            const int eo = EPW * wave + 16 * ks + 4 * kslot;  // element offset inside the tile
            float4 a[RG], b[RG];
#pragma unroll
            for (int g = 0; g < RG; ++g) {
                a[g] = *reinterpret_cast<const float4 *>(first + (16 * g + mrow) * STRIDE + eo);
                b[g] = *reinterpret_cast<const float4 *>(second + (16 * g + mrow) * STRIDE + eo);
            }
            double2 s01 = *reinterpret_cast<const double2 *>(sv + eo);
            double2 s23 = *reinterpret_cast<const double2 *>(sv + eo + 2);
            const double se[4] = {s01.x, s01.y, s23.x, s23.y};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                double dd[RG];
#pragma unroll
                for (int g = 0; g < RG; ++g) {
                    float fa = (t == 0) ? a[g].x : (t == 1) ? a[g].y : (t == 2) ? a[g].z : a[g].w;
                    float fb = (t == 0) ? b[g].x : (t == 1) ? b[g].y : (t == 2) ? b[g].z : b[g].w;
                    dd[g] = (double)fb - (double)fa;
                    pdot[g] = __builtin_fma(se[t], dd[g], pdot[g]);
                }
                // upper-triangular tiles, row group g (A operand) x row group h >= g (B operand)
                int q = 0;
#pragma unroll
                for (int g = 0; g < RG; ++g)
#pragma unroll
                    for (int h = g; h < RG; ++h) {
                        acc[q] = __builtin_amdgcn_mfma_f64_16x16x4f64(dd[g], dd[h], acc[q], 0, 0, 0);
                        ++q;
                    }
            }
        }
        buf ^= 1;
    }

    // cross-wave reduction in a fixed order
    __syncthreads();
    double *red = reinterpret_cast<double *>(smem);
    constexpr int PER_WAVE = L::GRAM + RG * 64;
#pragma unroll
    for (int q = 0; q < L::NT; ++q)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave * PER_WAVE + q * 256 + v * 64 + lane] = acc[q][v];
#pragma unroll
    for (int g = 0; g < RG; ++g) red[wave * PER_WAVE + L::GRAM + g * 64 + lane] = pdot[g];
    __syncthreads();
    for (int idx = tid; idx < L::GRAM; idx += kThreads) {
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) sum += red[w * PER_WAVE + idx];
        out[idx] = sum;
    }
    if (tid < BB) {
        int g = tid >> 4, rw = tid & 15;
        double sum = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sum += red[w * PER_WAVE + L::GRAM + g * 64 + ks * 16 + rw];
        out[L::GRAM + tid] = sum;
    }
}

template <int BB, int VW, int TE, bool APPLY>
__global__ __launch_bounds__(kThreads) void pass1_dots_gram(RowMap rm, PrevBlock prev, double *__restrict__ r_sum,
                                                            double *__restrict__ partials,
                                                            int64_t ntiles)
{
    pass1_body<BB, VW, TE, APPLY, TE == 64>(rm, prev, r_sum, partials + (int64_t)blockIdx.x * PartLayout<BB>::PART,
                                            ntiles, (int)blockIdx.x, (int)gridDim.x);
}

// The Gram matrices of many blocks in one launch (they depend on the rows only, not on
// the running sum or on earlier signs): blockIdx.y picks the block, whose row map is
// read from device memory, and gridDim.x workgroups share its tiles.  The dots this
// form also emits are taken against whatever the running sum holds and are not used.
template <int BB, int VW, int TE>
__global__ __launch_bounds__(kThreads) void gram_batched(const RowMap *__restrict__ maps,
                                                         double *__restrict__ r_sum,
                                                         double *__restrict__ partials, int64_t ntiles,
                                                         int64_t maps_per_walk)
{
    // blockIdx.z: the walk (its maps follow the previous walk's)
    const RowMap &rm = maps[(int64_t)blockIdx.z * maps_per_walk + blockIdx.y];
    PrevBlock none;
    none.rm.nb = 0;
    none.eps = nullptr;
    const int64_t slot = ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x;
    pass1_body<BB, VW, TE, false, false>(rm, none, r_sum, partials + slot * PartLayout<BB>::PART, ntiles,
                                         (int)blockIdx.x, (int)gridDim.x);
}

// Sum over the `groups` workgroups of each block of the batched form, in group order:
// gram_all[b][idx] = sum_g partials[(b * groups + g)][idx].
__global__ __launch_bounds__(kThreads) void reduce_batched(const double *__restrict__ partials,
                                                           double *__restrict__ gram_all, int part, int groups,
                                                           int64_t walk_gram_stride)
{
    const int idx = blockIdx.x * kThreads + threadIdx.x;
    if (idx >= part) return;
    // blockIdx.y: block of the batch, blockIdx.z: walk
    const double *src = partials + ((int64_t)blockIdx.z * gridDim.y + blockIdx.y) * groups * part + idx;
    double sum = 0.0;
#pragma unroll 8
    for (int g = 0; g < groups; ++g) sum += src[(int64_t)g * part];
    gram_all[(int64_t)blockIdx.z * walk_gram_stride + (int64_t)blockIdx.y * part + idx] = sum;
}

// ---------------------------------------------------------------------------
// Fixed-order reduction of the per-workgroup partials, first level: the list of
// workgroups is cut into kReduceSlices slices (blockIdx.y); each workgroup sums
// its slice for 32 consecutive entries, 8 sub-ranges per entry combined in order.
// The resolver adds the kReduceSlices slice sums, again in order.
constexpr int kReduceEntries = 32;
constexpr int kReduceSubs = kThreads / kReduceEntries;
constexpr int kReduceSlices = 8;

__global__ __launch_bounds__(kThreads) void reduce_partials(const double *__restrict__ partials,
                                                            double *__restrict__ sliced, int part,
                                                            int groups)
{
    __shared__ double subsum[kReduceSubs][kReduceEntries];
    const int ent = threadIdx.x % kReduceEntries;
    const int sub = threadIdx.x / kReduceEntries;
    const int entry = blockIdx.x * kReduceEntries + ent;
    const int slice = blockIdx.y;
    const int s0 = (int)((int64_t)slice * groups / kReduceSlices);
    const int s1 = (int)((int64_t)(slice + 1) * groups / kReduceSlices);
    const int g0 = s0 + (int)((int64_t)sub * (s1 - s0) / kReduceSubs);
    const int g1 = s0 + (int)((int64_t)(sub + 1) * (s1 - s0) / kReduceSubs);
    double sum = 0.0;
    if (entry < part) {
        // the loads are independent: keep eight in flight (the adds stay in order)
#pragma unroll 8
        for (int g = g0; g < g1; ++g) sum += partials[(int64_t)g * part + entry];
    }
    subsum[sub][ent] = sum;
    __syncthreads();
    if (sub == 0 && entry < part) {
        double tot = 0.0;
#pragma unroll
        for (int q = 0; q < kReduceSubs; ++q) tot += subsum[q][ent];
        sliced[(int64_t)slice * part + entry] = tot;
    }
}

// ---------------------------------------------------------------------------
// Sequential sign resolution.  All threads of the workgroup finish the reduction and unpack
// the Gram tiles into LDS; then one wavefront walks the block: lane k carries
// t_k = <r, d_k> + sum_{j<k, decided} eps_j G[j][k]; step j broadcasts t_j,
// fixes eps_j = +1 if t_j <= 0 else -1 (or, given uniform draws, the randomized
// rule) and updates the later lanes.
// Threads of the resolver's load phase: 1024, but 512 for 64-pair blocks, whose walk
// keeps 64 doubles of the Gram matrix per lane in registers.
template <int BB> constexpr int kResolveThreads = BB > 32 ? 512 : 1024;

// The resolver's body, run by all NT threads of a workgroup (the walk by its first
// wavefront).  write_out: store the signs (and resolved dots) to global memory; eps_lds
// (LDS, BB entries, or null): the block's signs for the rest of the workgroup, valid after
// the barrier this function ends with.
template <int BB, bool RANDOM, int SLICES, int NT>
__device__ __forceinline__ void resolve_body(const double *__restrict__ gram_src, int64_t gram_stride,
                                             const double *__restrict__ dot_src, int dot_groups,
                                             int64_t dot_stride, int nb, int64_t k0, int32_t i0, int32_t m,
                                             int64_t half_n, bool write_out, int8_t *__restrict__ eps_blk,
                                             int8_t *__restrict__ signs_out, double *__restrict__ dots_out,
                                             const float *__restrict__ uniforms, int8_t *eps_lds)
{
    // Gram tiles: sum of SLICES arrays gram_src[s * gram_stride + idx];
    // dots: sum of dot_groups arrays dot_src[g * dot_stride + k]; both in index order.
    using L = PartLayout<BB>;
    constexpr int SUBS = (NT / BB < 16) ? NT / BB : 16;  // threads sharing one dot
    __shared__ double G[BB][BB + 1];
    __shared__ double P[BB];
    __shared__ double psub[BB][SUBS + 1];
    // The dots' first DV groups per thread are requested before anything else and
    // consumed after the Gram tiles: indices beyond the last group re-read it and count
    // as zero, so that no branch separates the loads.
    constexpr int DV = (256 / SUBS < 32) ? 256 / SUBS : 32;  // loads per thread in the first batch
    const int dk = (threadIdx.x / SUBS) % BB, dsub = threadIdx.x % SUBS;
    double dv[DV];
#pragma unroll
    for (int u = 0; u < DV; ++u) {
        const int g = dsub + u * SUBS;
        dv[u] = dot_src[(int64_t)(g < dot_groups ? g : dot_groups - 1) * dot_stride + dk];
    }
    // Two consecutive entries per thread and step (16 B loads; GRAM is even).  All loads
    // of a thread are issued before the first is used: entries beyond the end re-read
    // entry 0 and are dropped.
    constexpr int ITER = (L::GRAM + 2 * NT - 1) / (2 * NT);
    double2 raw[ITER][SLICES];
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = 2 * (int)threadIdx.x + it * 2 * NT;
        const int idc = idx < L::GRAM ? idx : 0;
#pragma unroll
        for (int sl = 0; sl < SLICES; ++sl)
            raw[it][sl] = *reinterpret_cast<const double2 *>(gram_src + (int64_t)sl * gram_stride + idc);
    }
#pragma unroll
    for (int it = 0; it < ITER; ++it) {
        const int idx = 2 * (int)threadIdx.x + it * 2 * NT;
        if (idx >= L::GRAM) continue;
        double2 val = make_double2(0.0, 0.0);
#pragma unroll
        for (int sl = 0; sl < SLICES; ++sl) {
            val.x += raw[it][sl].x;
            val.y += raw[it][sl].y;
        }
        const int tile = idx >> 8, v = (idx >> 6) & 3, ln = idx & 63;
        // tiles are stored row group by row group, upper triangle only: (0,0), (0,1), .., (1,1), ..
        int tg = 0, th = tile;
        while (th >= L::RG - tg) { th -= L::RG - tg; ++tg; }
        th += tg;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            int i, j;
            mfma_f64_16x16_coord(ln + q, v, i, j);
            const double x = q ? val.y : val.x;
            G[16 * tg + i][16 * th + j] = x;
            if (th != tg) G[16 * th + j][16 * tg + i] = x;
        }
    }
    if (threadIdx.x < BB * SUBS) {
        double sum = 0.0;
#pragma unroll
        for (int u = 0; u < DV; ++u) sum += (dsub + u * SUBS < dot_groups) ? dv[u] : 0.0;
        // (more than DV * SUBS groups: the rest in further batches of sixteen loads)
        for (int g0 = dsub + DV * SUBS; g0 < dot_groups; g0 += 16 * SUBS) {
            double v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int g = g0 + u * SUBS;
                v[u] = dot_src[(int64_t)(g < dot_groups ? g : dot_groups - 1) * dot_stride + dk];
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) sum += (g0 + u * SUBS < dot_groups) ? v[u] : 0.0;
        }
        psub[dk][dsub] = sum;
    }
    __syncthreads();
    if (threadIdx.x < BB) {
        double sum = 0.0;
#pragma unroll
        for (int q = 0; q < SUBS; ++q) sum += psub[threadIdx.x][q];
        P[threadIdx.x] = sum;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const int lane = threadIdx.x;
        // lane k keeps column k of the Gram matrix (= row k, it is symmetric) in registers
        // (entries j >= lane are zeroed: lane k is updated at steps j < k only, and the walk
        // then needs no lane test of its own)
        double col[BB];
#pragma unroll
        for (int j = 0; j < BB; ++j) col[j] = (lane < BB && lane > j) ? G[lane][j] : 0.0;
        double t = (lane < nb) ? P[lane] : 0.0;
        // flattened pair of this lane -> (worker, pair) slot of the [m][n/2] arrays
        int64_t slot = 0;
        if (lane < nb) {
            uint32_t q = (uint32_t)(i0 + lane);
            uint32_t dq = q / (uint32_t)m;
            slot = (int64_t)(q - dq * (uint32_t)m) * half_n + (k0 + dq);
        }
        // randomized rule (PairBalance's RandomizedBalance subroutine, Sec. 3.2): with
        // c = z1 - z2 = -d, the first row gets +1 with probability p = (1 - <r,c>)/2 =
        // (1 + t)/2, so the exported sign (of the second row) is -1 when u < p.
        const float my_u = (RANDOM && lane < nb) ? uniforms[slot] : 0.f;
        auto rule = [&](double tv) { return RANDOM ? !((double)my_u < 0.5 * (1.0 + tv)) : (tv <= 0.0); };
        // Every lane applies the rule to its own t at every step; a wave-wide vote turns
        // lane j's answer into a scalar.  Lane k is updated at steps j < k only, so after
        // the loop its t is the resolved dot of pair k and the rule on it is pair k's sign.
        // (Steps j >= nb of a short last block run too: they only touch lanes above j, which
        // hold no pair.  Straight-line code, five instructions per step.)
#pragma unroll
        for (int j = 0; j < BB; ++j) {
            // +col[j] or -col[j]: the vote's bit j picks the sign bit to flip (a scalar)
            const uint32_t flip = ((__ballot(rule(t)) >> j) & 1ull) ? 0u : 0x80000000u;
            t += __hiloint2double(__double2hiint(col[j]) ^ (int)flip, __double2loint(col[j]));
        }
        const double my_t = t;
        const int my_eps = rule(t) ? 1 : -1;
        if (eps_lds && lane < BB) eps_lds[lane] = (lane < nb) ? (int8_t)my_eps : (int8_t)0;
        if (write_out && lane < nb) {
            eps_blk[lane] = (int8_t)my_eps;
            signs_out[slot] = (int8_t)my_eps;
            if (dots_out) dots_out[slot] = my_t;
        }
    }
    __syncthreads();
}

template <int BB, bool RANDOM, int SLICES>
__global__ __launch_bounds__(kResolveThreads<BB>) void resolve_signs(const double *__restrict__ gram_src,
                                                                     int64_t gram_stride,
                                                                     const double *__restrict__ dot_src,
                                                                     int dot_groups, int64_t dot_stride, int nb,
                                                                     int64_t k0, int32_t i0, int32_t m, int64_t half_n,
                                                                     int8_t *__restrict__ eps_blk,
                                                                     int8_t *__restrict__ signs_out,
                                                                     double *__restrict__ dots_out,
                                                                     const float *__restrict__ uniforms,
                                                                     WalkStrides ws)
{
    const int64_t w = blockIdx.y;  // the walk
    resolve_body<BB, RANDOM, SLICES, kResolveThreads<BB>>(gram_src + w * ws.gram, gram_stride, dot_src + w * ws.dots,
                                                          dot_groups, dot_stride, nb, k0, i0, m, half_n, true,
                                                          eps_blk + w * kMaxBlockPairs, signs_out + w * ws.out,
                                                          dots_out ? dots_out + w * ws.out : nullptr, uniforms,
                                                          nullptr);
}

// ---------------------------------------------------------------------------
// Pass 2: r += sum_k eps_k d_k.  Each thread owns four consecutive elements and
// streams the block's rows through registers.  FULL = the block holds all BB
// pairs (no per-pair test inside the unrolled loop).
template <int BB, int VW, bool FULL>
__global__ __launch_bounds__(kThreads) void pass2_apply(RowMap rm, const int8_t *__restrict__ eps_blk,
                                                        double *__restrict__ r_sum)
{
    const int64_t d = rm.d;
    const int64_t e = ((int64_t)blockIdx.x * kThreads + threadIdx.x) * 4;
    if (e >= d) return;
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll 8
    for (int j = 0; j < BB; ++j) {
        if (FULL || j < rm.nb) {
            float4 a = load4<VW>(rm.row(j, 0), e, d);
            float4 b = load4<VW>(rm.row(j, 1), e, d);
            double sg = (double)eps_blk[j];
            acc[0] = __builtin_fma(sg, (double)b.x - (double)a.x, acc[0]);
            acc[1] = __builtin_fma(sg, (double)b.y - (double)a.y, acc[1]);
            acc[2] = __builtin_fma(sg, (double)b.z - (double)a.z, acc[2]);
            acc[3] = __builtin_fma(sg, (double)b.w - (double)a.w, acc[3]);
        }
    }
    // the running sum is padded to a multiple of the tile; the padding stays zero
    // because elements beyond d load as zero
    double2 lo = *reinterpret_cast<double2 *>(r_sum + e);
    double2 hi = *reinterpret_cast<double2 *>(r_sum + e + 2);
    lo.x += acc[0]; lo.y += acc[1]; hi.x += acc[2]; hi.y += acc[3];
    *reinterpret_cast<double2 *>(r_sum + e) = lo;
    *reinterpret_cast<double2 *>(r_sum + e + 2) = hi;
}

// ---------------------------------------------------------------------------
// Pass 2 for long rows, with the running-sum traffic gathered into bursts.  The grid is
// wholly resident (two workgroups per CU); a thread owns up to kResidentGroups groups of
// four elements (group g of slab s at element ((s * kuse + g) * T + t) * 4, T threads in
// all), streams all rows of the block for one group after the other and keeps the sums in
// registers; only when all its groups are done does it read, update and write the running
// sum.  All workgroups run in step, so the launch is a long stretch of pure row reads
// followed by one short burst of running-sum reads and writes.  A row longer than the
// registers of the chip hold (kuse * T * 4 elements) is cut into slabs, ONE LAUNCH PER SLAB:
// the launch boundary brings the workgroups back into step -- inside one launch they drift
// apart from slab to slab, the bursts smear out into the row reads, and the gain is lost
// (d = 124M, eleven slabs: 6.06 ms in one launch, the same as the flat form).
// Writes scattered through a read stream cost this chip about 1 us per MB (the flat form
// above: 0.52 ms per 32-pair block at d = 11.2M, of which 0.09 ms for 180 MB of running-sum
// traffic); gathered at the end they cost a third of that (0.46 ms).  Same sums in the
// same order as the flat form: bit-identical results.
constexpr int kResidentGroups = 22;

template <int BB, int VW, bool FULL>
__global__ __launch_bounds__(kThreads, 2) void pass2_apply_resident(RowMap rm, const int8_t *__restrict__ eps_blk,
                                                                    double *__restrict__ r_sum, int kuse,
                                                                    int64_t g0)
{
    // this launch: groups g0 .. g0 + kuse - 1 of every thread (one slab)
    constexpr int K = kResidentGroups;
    const int64_t d = rm.d;
    const int64_t T = (int64_t)gridDim.x * kThreads;
    const int64_t t = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    double acc[K][4];
#pragma unroll
    for (int g = 0; g < K; ++g) {
        acc[g][0] = acc[g][1] = acc[g][2] = acc[g][3] = 0.0;
        const int64_t e = ((g0 + g) * T + t) * 4;
        if (g < kuse && e < d) {
#pragma unroll 2
            for (int j = 0; j < BB; ++j) {
                if (FULL || j < rm.nb) {
                    float4 a = load4<VW>(rm.row(j, 0), e, d);
                    float4 b = load4<VW>(rm.row(j, 1), e, d);
                    double sg = (double)eps_blk[j];
                    acc[g][0] = __builtin_fma(sg, (double)b.x - (double)a.x, acc[g][0]);
                    acc[g][1] = __builtin_fma(sg, (double)b.y - (double)a.y, acc[g][1]);
                    acc[g][2] = __builtin_fma(sg, (double)b.z - (double)a.z, acc[g][2]);
                    acc[g][3] = __builtin_fma(sg, (double)b.w - (double)a.w, acc[g][3]);
                }
            }
        }
    }
    // the running sum is padded to a multiple of the tile; the padding stays zero
    // because elements beyond d load as zero
#pragma unroll
    for (int g = 0; g < K; ++g) {
        const int64_t e = ((g0 + g) * T + t) * 4;
        if (g < kuse && e < d) {
            double2 lo = *reinterpret_cast<double2 *>(r_sum + e);
            double2 hi = *reinterpret_cast<double2 *>(r_sum + e + 2);
            lo.x += acc[g][0]; lo.y += acc[g][1]; hi.x += acc[g][2]; hi.y += acc[g][3];
            *reinterpret_cast<double2 *>(r_sum + e) = lo;
            *reinterpret_cast<double2 *>(r_sum + e + 2) = hi;
        }
    }
}

// ---------------------------------------------------------------------------
// Pass 2 for short rows: a workgroup owns 64 consecutive elements; its 256 threads
// are 16 element-quads x 16 pair groups, each thread sums BB/16 pairs for its quad,
// the 16 partial sums are added in group order through LDS, and 64 threads update
// one element each.  Sixteen times the workgroups and a sixteenth of the loads per
// thread of the flat form, which is what a latency-bound launch needs.
constexpr int kSplitGroups = 16;
constexpr int kSplitElems = (kThreads / kSplitGroups) * 4;  // 64 elements per workgroup

template <int BB, int VW, bool FULL>
__global__ __launch_bounds__(kThreads) void pass2_apply_split(RowMap rm, const int8_t *__restrict__ eps_blk,
                                                              double *__restrict__ r_sum, WalkStrides ws)
{
    __shared__ double part[kSplitGroups][kSplitElems];
    const int64_t d = rm.d;
    const int64_t woff = (int64_t)blockIdx.y * ws.rows;  // blockIdx.y: the walk
    eps_blk += (int64_t)blockIdx.y * kMaxBlockPairs;
    r_sum += (int64_t)blockIdx.y * ws.r;
    const int quad = threadIdx.x % (kThreads / kSplitGroups), grp = threadIdx.x / (kThreads / kSplitGroups);
    const int64_t e = (int64_t)blockIdx.x * kSplitElems + quad * 4;
    const int64_t mine = (int64_t)blockIdx.x * kSplitElems + threadIdx.x;
    // the running-sum element is requested first so that its latency overlaps the row loads
    const double r_old = (threadIdx.x < kSplitElems && mine < d) ? r_sum[mine] : 0.0;
    constexpr int PER = BB / kSplitGroups;
    float4 a[PER], b[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int j = grp * PER + q;
        // (offsets of missing pairs are readable rows: zero, or those of an earlier block)
        const bool have = FULL || j < rm.nb;
        a[q] = load4_nb<VW>(rm.row(j, 0) + woff, have, e, d);
        b[q] = load4_nb<VW>(rm.row(j, 1) + woff, have, e, d);
    }
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int j = grp * PER + q;
        const double sg = (FULL || j < rm.nb) ? (double)eps_blk[j] : 0.0;
        acc[0] = __builtin_fma(sg, (double)b[q].x - (double)a[q].x, acc[0]);
        acc[1] = __builtin_fma(sg, (double)b[q].y - (double)a[q].y, acc[1]);
        acc[2] = __builtin_fma(sg, (double)b[q].z - (double)a[q].z, acc[2]);
        acc[3] = __builtin_fma(sg, (double)b[q].w - (double)a[q].w, acc[3]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) part[grp][quad * 4 + q] = acc[q];
    __syncthreads();
    if (threadIdx.x < kSplitElems && mine < d) {
        double sum = 0.0;
#pragma unroll
        for (int g = 0; g < kSplitGroups; ++g) sum += part[g][threadIdx.x];
        r_sum[mine] = r_old + sum;
    }
}

// ---------------------------------------------------------------------------
// Short rows with the Gram matrices computed ahead (gram_batched): the chain of a block
// in ONE launch.  What is left on the chain is the resolver of the PREVIOUS block,
// r += sum_k eps_k d_k over it, and the dots <r, d_k> of this block against the result.
// Every workgroup resolves the previous block for itself (its reduced Gram tiles and the
// per-workgroup dots the previous launch wrote: the resolver's body on 256 threads,
// redundantly in each of the d/64 workgroups -- a few tens of KB from the L2 and a walk of
// Bb steps, cheaper than a launch boundary).  Then, with the thread layout of
// pass2_apply_split (a workgroup owns 64 elements, group g of 16 threads takes the pairs
// g*PER .. g*PER+PER-1 of either block), it applies the previous block and writes its share
// of this block's Bb dots to dots_out_part[blockIdx.x][BB], which must not be the array
// being read.  Workgroup 0 also stores the previous block's signs.  DENSE: row addresses by
// arithmetic (RowMap::dense_row) instead of through the offset table.
template <int BB, int VW, bool DENSE, bool RANDOM>
__global__ __launch_bounds__(kThreads) void resolve_dots_apply_split(
    RowMap rm, PrevBlock prev, const double *__restrict__ prev_gram, const double *__restrict__ dots_in_part,
    double *__restrict__ dots_out_part, int dot_groups, double *__restrict__ r_sum, int8_t *__restrict__ eps_blk,
    int8_t *__restrict__ signs_out, double *__restrict__ dots_out, const float *__restrict__ uniforms,
    WalkStrides ws)
{
    __shared__ double part[kSplitGroups][kSplitElems];
    __shared__ double rnew[kSplitElems];
    __shared__ int8_t eps_s[kMaxBlockPairs];
    const int64_t d = rm.d;
    // blockIdx.y: the walk; what it owns lies at a fixed stride from the first walk's
    const int64_t w = blockIdx.y;
    const int64_t woff = w * ws.rows;
    prev_gram += w * ws.gram;
    dots_in_part += w * ws.dots;
    dots_out_part += w * ws.dots;
    r_sum += w * ws.r;
    eps_blk += w * kMaxBlockPairs;
    signs_out += w * ws.out;
    if (dots_out) dots_out += w * ws.out;
    constexpr int QUADS = kThreads / kSplitGroups;  // 16 threads, four elements each
    const int quad = threadIdx.x % QUADS, grp = threadIdx.x / QUADS;
    const int64_t e = (int64_t)blockIdx.x * kSplitElems + quad * 4;
    const int64_t mine = (int64_t)blockIdx.x * kSplitElems + threadIdx.x;
    // the rows of both blocks are requested before the resolver's inputs
    const double r_old = (threadIdx.x < kSplitElems) ? r_sum[mine] : 0.0;  // padded to a multiple of 128
    constexpr int PER = BB / kSplitGroups;
    float4 pa[PER], pb[PER], ca[PER], cb[PER];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const int j = grp * PER + q;
        const int jp = j < prev.rm.nb ? j : 0, jc = j < rm.nb ? j : 0;
        pa[q] = load4_nb<VW>((DENSE ? prev.rm.dense_row(jp, 0) : prev.rm.row(j, 0)) + woff, true, e, d);
        pb[q] = load4_nb<VW>((DENSE ? prev.rm.dense_row(jp, 1) : prev.rm.row(j, 1)) + woff, true, e, d);
        ca[q] = load4_nb<VW>((DENSE ? rm.dense_row(jc, 0) : rm.row(j, 0)) + woff, true, e, d);
        cb[q] = load4_nb<VW>((DENSE ? rm.dense_row(jc, 1) : rm.row(j, 1)) + woff, true, e, d);
    }
    if (prev.rm.nb > 0) {  // uniform
        resolve_body<BB, RANDOM, 1, kThreads>(prev_gram, 0, dots_in_part, dot_groups, BB, prev.rm.nb, prev.rm.k0,
                                              prev.rm.i0, prev.rm.m, prev.rm.n / 2, blockIdx.x == 0, eps_blk,
                                              signs_out, dots_out, uniforms, eps_s);
    } else {
        if (threadIdx.x < BB) eps_s[threadIdx.x] = 0;
        __syncthreads();
    }
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        const double sg = (double)eps_s[grp * PER + q];  // 0 for a pair the previous block does not have
        acc[0] = __builtin_fma(sg, (double)pb[q].x - (double)pa[q].x, acc[0]);
        acc[1] = __builtin_fma(sg, (double)pb[q].y - (double)pa[q].y, acc[1]);
        acc[2] = __builtin_fma(sg, (double)pb[q].z - (double)pa[q].z, acc[2]);
        acc[3] = __builtin_fma(sg, (double)pb[q].w - (double)pa[q].w, acc[3]);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) part[grp][quad * 4 + q] = acc[q];
    __syncthreads();
    if (threadIdx.x < kSplitElems) {
        double sum = 0.0;
#pragma unroll
        for (int g = 0; g < kSplitGroups; ++g) sum += part[g][threadIdx.x];
        const double r = r_old + sum;  // elements beyond d load as zero, so the padding stays zero
        r_sum[mine] = r;
        rnew[threadIdx.x] = r;
    }
    __syncthreads();
    const double r0 = rnew[quad * 4], r1 = rnew[quad * 4 + 1], r2 = rnew[quad * 4 + 2], r3 = rnew[quad * 4 + 3];
#pragma unroll
    for (int q = 0; q < PER; ++q) {
        double p = r0 * ((double)cb[q].x - (double)ca[q].x);
        p = __builtin_fma(r1, (double)cb[q].y - (double)ca[q].y, p);
        p = __builtin_fma(r2, (double)cb[q].z - (double)ca[q].z, p);
        p = __builtin_fma(r3, (double)cb[q].w - (double)ca[q].w, p);
#pragma unroll
        for (int off = 1; off < QUADS; off <<= 1) p += __shfl_xor(p, off, 64);
        if (quad == 0) dots_out_part[(int64_t)blockIdx.x * BB + grp * PER + q] = p;
    }
}

// ---------------------------------------------------------------------------
// Clears `count` 32-bit words.  The library clears its flags and scratch with fill
// kernels rather than memset nodes, so that a caller may capture its stream in a graph.
__global__ void fill_zero_b32(uint32_t *p, int64_t count) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0u;
}

__global__ void fill_zero_f64(double *p, int64_t count) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < count; i += stride) p[i] = 0.0;
}

// Row maps of `count` consecutive blocks starting at flattened pair first_pair: block b
// holds the pairs first_pair + b*bb .. (up to total_pairs).  One thread per (block, pair).
__global__ __launch_bounds__(kMaxBlockPairs) void fill_row_maps(RowMap *__restrict__ maps, const float *base,
                                                                int64_t m, int64_t n, int64_t d, int bb,
                                                                int64_t first_pair, int64_t total_pairs,
                                                                int64_t center_off, int layout,
                                                                int64_t walk_rows_stride)
{
    // layout 0: dense [m][n][d];  1: single rows paired with the row at center_off;
    // 2: a staging chunk [q][2][d] that starts at first_pair (base = the chunk)
    // blockIdx.y: the walk (its rows start walk_rows_stride floats after the previous walk's)
    const int use_center = layout == 1;
    base += (int64_t)blockIdx.y * walk_rows_stride;
    RowMap &rm = maps[(int64_t)blockIdx.y * gridDim.x + blockIdx.x];
    const int j = threadIdx.x;
    const int64_t p0 = first_pair + (int64_t)blockIdx.x * bb;
    const int64_t left = total_pairs - p0;
    const int nb = (int)(left < bb ? left : bb);
    if (j == 0) {
        rm.base = base;
        rm.d = d;
        rm.n = n;
        rm.k0 = p0 / m;
        rm.i0 = (int32_t)(p0 - (p0 / m) * m);
        rm.m = (int32_t)m;
        rm.nb = nb;
        rm.dense = layout == 0 ? 1 : 0;
    }
    int64_t o0 = 0, o1 = 0;
    if (j < nb) {
        const int64_t p = p0 + j;
        if (use_center) {
            o0 = p * d;
            o1 = center_off;
        } else if (layout == 2) {
            o0 = (p - first_pair) * 2 * d;
            o1 = o0 + d;
        } else {
            const int64_t k = p / m, i = p - k * m;
            o0 = (i * n + 2 * k) * d;
            o1 = o0 + d;
        }
    }
    rm.off[2 * j] = o0;
    rm.off[2 * j + 1] = o1;
}

__global__ void export_running_sum(const double *__restrict__ r_sum, int64_t d, float *__restrict__ r32,
                                   double *__restrict__ r64)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (; i < d; i += stride) {
        double v = r_sum[i];
        if (r32) r32[i] = (float)v;
        if (r64) r64[i] = v;
    }
}

}  // namespace cdgrab
