// C ABI of the CD-GraB pair-balancing library (see include/cdgrab.h for the
// contract of every entry point).  Host orchestration only: every arithmetic
// step of the path runs in the kernels of balance_kernels.hpp / order_kernels.hpp.
#include "../../include/cdgrab.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "balance_kernels.hpp"
#include "order_kernels.hpp"
#include "herding_kernels.hpp"

using namespace cdgrab;

namespace {

thread_local std::string g_create_error;

enum Interval { kGen = 0, kBalance, kPass1, kReduce, kResolve, kPass2, kFinish, kIntervalKinds };

struct Mark {
    hipEvent_t ev;
    int kind_after;  // what runs between this mark and the next one (-1: nothing timed)
};

}  // namespace

struct cdgrab_handle {
    int device = 0;
    hipStream_t stream = nullptr;
    int block_pairs_opt = 0;
    int timing = 0;
    int pass1_groups_opt = 0;
    int apply_mode = 0;  // 0 choose by row length, 1 separate apply launch, 2 apply fused into the next block's launch,
                         // 3 / 4 separate launch, always in the resident / the flat form
    int apply_groups_opt = 0;  // cap on the resident apply grid (0: two workgroups per CU)
    int gram_mode = 0;   // 0 choose, 1 each block's Gram in its own launch, 2 Grams of many blocks ahead in one launch
    int num_cu = 256;
    std::string err;

    double *r_sum = nullptr;   int64_t r_cap = 0;         // doubles
    double *partials = nullptr; int64_t partials_cap = 0; // doubles
    double *reduced = nullptr;                            // kReduceSlices x PartLayout<64>::PART doubles
    int8_t *eps_blk = nullptr; int64_t eps_cap = 0;       // 64 signs of the current block per walk
    int32_t *flag = nullptr;                              // reorder's bad-sign flag
    const float *uniforms = nullptr;                      // caller's draws while a randomized epoch runs
    int64_t walks = 1;                                    // independent walks per launch while such an epoch runs
    WalkStrides ws{};                                     // their strides (all zero for one walk)
    float *zero_row = nullptr; int64_t zero_row_cap = 0;  // a zero vector standing in for a missing stale mean
    float *train_delta = nullptr; int64_t train_delta_cap = 0;  // [m][classes] softmax deltas of one step
    int32_t *train_perm = nullptr; int64_t train_perm_cap = 0;  // spare [m][n] order of the multi-epoch driver
    int8_t *train_signs = nullptr; int64_t train_signs_cap = 0; // its [m][n/2] signs when the caller wants none
    double *herd_ws = nullptr; int64_t herd_cap = 0;      // herding evaluator: segment sums, starts, mean
    double *gram_all = nullptr; int64_t gram_all_cap = 0; // Grams-ahead form: reduced tiles of up to kGramBatch blocks
    double *dot_partials = nullptr; int64_t dot_partials_cap = 0;  // its per-workgroup dots of one block
    RowMap *maps = nullptr; int64_t maps_cap = 0;         // its row maps (device)
    float *staging = nullptr;  int64_t staging_cap = 0;   // floats: two staging chunks (the fused pass reads the previous block too)
    bool fixed_workspace = false;                         // the workspace pointers are borrowed: never grow or free them

    std::vector<hipEvent_t> event_pool;
    std::vector<Mark> marks;
    size_t events_used = 0;
    bool have_timing = false;
    cdgrab_timing last{};
};

namespace {

int fail(cdgrab_handle *h, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (h) h->err = buf; else g_create_error = buf;
    return code;
}

#define HIP_TRY(h, expr)                                                                  \
    do {                                                                                  \
        hipError_t e_ = (expr);                                                           \
        if (e_ != hipSuccess)                                                             \
            return fail(h, CDGRAB_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_));   \
    } while (0)

int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }

// Do the byte ranges [a, a + na) and [b, b + nb) share a byte?  (Null ranges never do.)
bool ranges_overlap(const void *a, int64_t na, const void *b, int64_t nb) {
    if (!a || !b || na <= 0 || nb <= 0) return false;
    const uintptr_t a0 = reinterpret_cast<uintptr_t>(a), b0 = reinterpret_cast<uintptr_t>(b);
    return a0 < b0 + (uintptr_t)nb && b0 < a0 + (uintptr_t)na;
}

int pick_vector_width(int64_t d, int64_t base_align) {
    if (d % 4 == 0 && base_align % 16 == 0) return 4;
    if (d % 2 == 0 && base_align % 8 == 0) return 2;
    return 1;
}

// 32 pairs per block keep the double-precision Gram tiles under the HBM time for
// long rows; short rows are bound by launches, not bytes, and take 64.
int pick_block_pairs(int64_t pairs, int64_t d, int32_t requested) {
    if (requested == 16 || requested == 32 || requested == 64) return requested;
    if (pairs <= 16) return 16;
    if (pairs > 32 && d <= 65536) return 64;
    return 32;
}

// Measured on MI355X: applying a block inside the next block's dot/Gram launch wins up
// to about 1.2M elements per row (one launch and one read of the running sum less: 3 % at
// 1M, 4 % at 512K, 15 % at 8K); beyond that the heavier fused kernel streams 8-12 % slower
// than the dot/Gram launch and the resident apply launch together (1.5M: 158 against 141 us
// per 32-pair block, 2M: 213 against 198, 4M: 423 against 388).
bool fuse_apply_by_default(int64_t d) { return d <= (int64_t)5 << 18; }

// Dense input with short rows: a block is bound by its chain of launches, so the Gram
// matrices (which depend on the rows only) are taken off the chain: one launch computes
// them for up to kGramBatch blocks, and a block then costs one launch (resolver of the
// previous block, its apply, this block's dots).  Measured on MI355X (m = 16, 64-pair blocks), time per block of the per-block
// form -> this form: d = 256: 22.0 -> 8.9 us; 4096: 23.3 -> 11.2; 7850: 26.1 -> 15.8;
// 16 384: 26.3 -> 19.3; 32 768: 35.9 -> 44.0; 65 536: 48.6 -> 132 (the rows are read three
// times instead of twice, and every workgroup repeats the previous block's resolver).
constexpr int64_t kGramBatch = 512;
constexpr int64_t kGramAheadMaxD = 16384;     // chosen by default up to here
constexpr int64_t kGramAheadLimitD = 131072;  // refused beyond (gram_mode 2)
bool gram_ahead_by_default(int64_t d, int64_t blocks, bool streamed) {
    return !streamed && blocks >= 2 && d <= kGramAheadMaxD;
}

int part_size(int bb) {
    return bb == 64 ? PartLayout<64>::PART : bb == 32 ? PartLayout<32>::PART : PartLayout<16>::PART;
}

// The launch plan of one epoch.  `chunk_pairs` is the number of flattened pairs staged per
// generator call (streamed input; 0 = one block).  Every decision an epoch takes is taken
// here, so that cdgrab_plan_epoch reports exactly what a handle with the same options runs.
int plan_epoch(int64_t m, int64_t n, int64_t d, int32_t block_pairs, int32_t streamed,
               int64_t base_align, int num_cu, int32_t pass1_groups_opt, int apply_mode, int gram_mode,
               int64_t chunk_pairs, cdgrab_plan *plan) {
    if (m < 1 || n < 2 || (n & 1) || d < 1 || !plan) return CDGRAB_EINVAL;
    if (block_pairs != 0 && block_pairs != 16 && block_pairs != 32 && block_pairs != 64) return CDGRAB_EINVAL;
    if (base_align < 4 || (base_align & (base_align - 1))) return CDGRAB_EINVAL;
    if (m > (INT64_MAX / n) / d || m > (1 << 30)) return CDGRAB_EINVAL;
    plan->pairs = m * (n / 2);
    plan->block_pairs = pick_block_pairs(plan->pairs, d, block_pairs);
    const int64_t bb = plan->block_pairs;
    plan->blocks = (plan->pairs + bb - 1) / bb;
    plan->vector_width = pick_vector_width(d, streamed ? 256 : base_align);
    // long rows stream through 128-element tiles with two resident workgroups per CU;
    // short rows use 64-element tiles so that more workgroups share the work
    plan->tile_elems = (d >= (int64_t)128 * 2 * num_cu) ? 128 : 64;
    int64_t ntiles = (d + plan->tile_elems - 1) / plan->tile_elems;
    int64_t want = pass1_groups_opt > 0 ? pass1_groups_opt
                                        : (int64_t)num_cu * (plan->tile_elems == 128 ? 2 : 4);
    plan->pass1_groups = (int32_t)std::max<int64_t>(1, std::min<int64_t>(want, ntiles));
    plan->pass2_groups = (int32_t)((d + kThreads * 4 - 1) / (kThreads * 4));
    if (chunk_pairs <= 0) chunk_pairs = bb;

    // Grams ahead: asked for, or chosen for short rows when the caller left both choices
    // open; for streamed rows when a staging chunk holds several whole blocks.
    const bool ahead_dense = !streamed && plan->blocks >= 2 &&
                             (gram_mode == 2 || (gram_mode == 0 && apply_mode == 0 &&
                                                 gram_ahead_by_default(d, plan->blocks, false)));
    const bool ahead_streamed = streamed && gram_mode != 1 && apply_mode == 0 && d <= kGramAheadMaxD &&
                                plan->pairs > bb && chunk_pairs >= 2 * bb && chunk_pairs % bb == 0 &&
                                chunk_pairs / bb <= kGramBatch;
    const bool ahead = ahead_dense || ahead_streamed;
    // the ahead form applies a block inside the next block's launch by construction
    const bool fused = !ahead && (apply_mode == 2 || (apply_mode == 0 && fuse_apply_by_default(d)));
    plan->gram_ahead = ahead ? 1 : 0;
    plan->fused_apply = fused ? 1 : 0;
    plan->reserved = 0;

    // two staging chunks when a launch reads the previous block's rows as well
    plan->staging_bytes = streamed ? ((fused || ahead) ? 2 : 1) * chunk_pairs * 2 * d * 4 : 0;
    const int64_t part = part_size(plan->block_pairs);
    int64_t partial_doubles = (int64_t)plan->pass1_groups * part;
    int64_t ahead_bytes = 0;
    if (ahead) {
        const int64_t batch = streamed ? chunk_pairs / bb : std::min<int64_t>(plan->blocks, kGramBatch);
        const int64_t gg = std::max<int64_t>(1, std::min<int64_t>(ntiles, (4 * (int64_t)num_cu + batch - 1) / batch));
        partial_doubles = std::max(partial_doubles, batch * gg * part);
        ahead_bytes = (batch + 1) * part * 8                               // reduced Gram tiles
                      + 2 * ((d + kSplitElems - 1) / kSplitElems * bb) * 8  // per-workgroup dots, two blocks
                      + batch * (int64_t)sizeof(RowMap);                    // row maps
    }
    plan->workspace_bytes = round_up(d, kPadE) * 8 + partial_doubles * 8 +
                            (int64_t)kReduceSlices * PartLayout<64>::PART * 8 + 64 + ahead_bytes +
                            plan->staging_bytes;
    // each row twice; the double running sum read twice and written once per block, or read
    // once and written once when the apply rides in the next block's launch; with the Gram
    // matrices ahead the rows are read three times
    plan->bytes_per_example = ahead ? 12.0 * (double)d + 8.0 * (double)d / (double)bb
                                    : 8.0 * (double)d + (fused ? 8.0 : 12.0) * (double)d / (double)bb;
    return CDGRAB_OK;
}

// ---- timing marks ----------------------------------------------------------
int mark(cdgrab_handle *h, int kind_after) {
    if (h->events_used == h->event_pool.size()) {
        hipEvent_t ev;
        HIP_TRY(h, hipEventCreate(&ev));
        h->event_pool.push_back(ev);
    }
    hipEvent_t ev = h->event_pool[h->events_used++];
    HIP_TRY(h, hipEventRecord(ev, h->stream));
    h->marks.push_back({ev, kind_after});
    return CDGRAB_OK;
}

#define MARK(h, level, kind)                                   \
    do {                                                       \
        if ((h)->timing >= (level)) {                          \
            int rc_ = mark((h), (kind));                       \
            if (rc_ != CDGRAB_OK) return rc_;                  \
        }                                                      \
    } while (0)

template <typename T>
int ensure(cdgrab_handle *h, T *&ptr, int64_t &cap, int64_t want) {
    if (cap >= want) return CDGRAB_OK;
    if (h->fixed_workspace)
        return fail(h, CDGRAB_ENOMEM, "the fixed workspace is too small (%lld elements needed, %lld there)",
                    (long long)want, (long long)cap);
    if (ptr) { HIP_TRY(h, hipStreamSynchronize(h->stream)); HIP_TRY(h, hipFree(ptr)); ptr = nullptr; cap = 0; }
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&ptr), (size_t)want * sizeof(T));
    if (e != hipSuccess) {
        ptr = nullptr;
        (void)hipGetLastError();
        return fail(h, CDGRAB_ENOMEM, "workspace allocation of %lld bytes failed: %s",
                    (long long)(want * (int64_t)sizeof(T)), hipGetErrorString(e));
    }
    cap = want;
    return CDGRAB_OK;
}

template <int BB, int VW>
void launch_pass1(cdgrab_handle *h, const RowMap &rm, const PrevBlock *prev, const cdgrab_plan &plan) {
    PrevBlock none;
    none.rm = rm;
    none.rm.nb = 0;
    none.eps = h->eps_blk;
    const dim3 grid(plan.pass1_groups), block(kThreads);
    const int64_t ntiles = (rm.d + plan.tile_elems - 1) / plan.tile_elems;
    auto launch = [&](auto kernel, const PrevBlock &pb) {
        hipLaunchKernelGGL(kernel, grid, block, 0, h->stream, rm, pb, h->r_sum, h->partials, ntiles);
    };
    if (plan.tile_elems == 128) {
        if (prev) launch(pass1_dots_gram<BB, VW, 128, true>, *prev);
        else launch(pass1_dots_gram<BB, VW, 128, false>, none);
    } else {
        if (prev) launch(pass1_dots_gram<BB, VW, 64, true>, *prev);
        else launch(pass1_dots_gram<BB, VW, 64, false>, none);
    }
}
// Rows from this length on take the resident form of the apply pass (the running-sum
// traffic in one burst); shorter ones the flat form, whose launch ramps up faster
// (block of 32 pairs, dot/Gram launch included: 1M elements 106 against 115 us, 768K 84
// against 80 us).
constexpr int64_t kResidentMinD = (int64_t)1 << 20;

template <int BB, int VW>
void launch_pass2(cdgrab_handle *h, const RowMap &rm, int groups) {
    // short rows: too few flat workgroups to hide latency -> split the pairs over thread groups
    // (several independent walks per launch exist for short rows only, in this form)
    if ((groups < 2 * h->num_cu && h->apply_mode < 3) || h->walks > 1) {
        const dim3 grid((unsigned)((rm.d + kSplitElems - 1) / kSplitElems), (unsigned)h->walks);
        if (rm.nb == BB)
            hipLaunchKernelGGL((pass2_apply_split<BB, VW, true>), grid, dim3(kThreads), 0, h->stream, rm,
                               h->eps_blk, h->r_sum, h->ws);
        else
            hipLaunchKernelGGL((pass2_apply_split<BB, VW, false>), grid, dim3(kThreads), 0, h->stream, rm,
                               h->eps_blk, h->r_sum, h->ws);
        return;
    }
    if (h->apply_mode == 3 || (h->apply_mode != 4 && rm.d >= kResidentMinD)) {
        // a wholly resident grid: two workgroups per CU, each thread up to kResidentGroups groups of four
        const int64_t quads = (rm.d + 3) / 4;
        int64_t grid = std::min<int64_t>(2 * (int64_t)h->num_cu, (quads + kThreads - 1) / kThreads);
        if (h->apply_groups_opt > 0) grid = std::min<int64_t>(grid, h->apply_groups_opt);
        const int64_t T = grid * kThreads;
        const int64_t per_thread = (quads + T - 1) / T;
        const int64_t slabs = (per_thread + kResidentGroups - 1) / kResidentGroups;
        const int kuse = (int)((per_thread + slabs - 1) / slabs);
        // one launch per slab: the boundary keeps the workgroups in step, so that each slab ends in
        // one burst of running-sum traffic
        for (int64_t sl = 0; sl < slabs; ++sl) {
            if (rm.nb == BB)
                hipLaunchKernelGGL((pass2_apply_resident<BB, VW, true>), dim3((unsigned)grid), dim3(kThreads), 0,
                                   h->stream, rm, h->eps_blk, h->r_sum, kuse, sl * kuse);
            else
                hipLaunchKernelGGL((pass2_apply_resident<BB, VW, false>), dim3((unsigned)grid), dim3(kThreads), 0,
                                   h->stream, rm, h->eps_blk, h->r_sum, kuse, sl * kuse);
        }
        return;
    }
    if (rm.nb == BB)
        hipLaunchKernelGGL((pass2_apply<BB, VW, true>), dim3(groups), dim3(kThreads), 0, h->stream, rm,
                           h->eps_blk, h->r_sum);
    else
        hipLaunchKernelGGL((pass2_apply<BB, VW, false>), dim3(groups), dim3(kThreads), 0, h->stream, rm,
                           h->eps_blk, h->r_sum);
}
template <int BB>
void launch_resolve(cdgrab_handle *h, const RowMap &rm, int8_t *signs_out, double *dots_out) {
    // Gram tiles and dots both come from the kReduceSlices slice sums
    constexpr int part = PartLayout<BB>::PART;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(1), dim3(kResolveThreads<BB>), 0, h->stream, h->reduced,
                           (int64_t)part, h->reduced + PartLayout<BB>::GRAM, kReduceSlices, (int64_t)part, rm.nb,
                           rm.k0, rm.i0, rm.m, rm.n / 2, h->eps_blk, signs_out, dots_out, h->uniforms, WalkStrides{});
    };
    if (h->uniforms) launch(resolve_signs<BB, true, kReduceSlices>);
    else launch(resolve_signs<BB, false, kReduceSlices>);
}

// Grams-ahead form of one block, one launch: every workgroup resolves the previous block
// (its Gram tiles at prev_gram, its per-workgroup dots in dots_in), applies it and takes
// this block's dots (into dots_out).  The first block of an epoch has prev.rm.nb == 0.
template <int BB>
int run_block_ahead(cdgrab_handle *h, const RowMap &rm, const PrevBlock &prev, const cdgrab_plan &plan,
                    const double *prev_gram, const double *dots_in, double *dots_out, int8_t *signs_out,
                    double *dots_export) {
    const unsigned groups = (unsigned)((rm.d + kSplitElems - 1) / kSplitElems);
    MARK(h, 2, kPass1);
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(groups, (unsigned)h->walks), dim3(kThreads), 0, h->stream, rm, prev,
                           prev_gram, dots_in, dots_out, (int)groups, h->r_sum, h->eps_blk, signs_out, dots_export,
                           h->uniforms, h->ws);
    };
    auto by_width = [&](auto dense_tag, auto random_tag) {
        constexpr bool DENSE = decltype(dense_tag)::value, RANDOM = decltype(random_tag)::value;
        switch (plan.vector_width) {
            case 4: launch(resolve_dots_apply_split<BB, 4, DENSE, RANDOM>); break;
            case 2: launch(resolve_dots_apply_split<BB, 2, DENSE, RANDOM>); break;
            default: launch(resolve_dots_apply_split<BB, 1, DENSE, RANDOM>); break;
        }
    };
    if (rm.dense) {
        if (h->uniforms) by_width(std::true_type{}, std::true_type{});
        else by_width(std::true_type{}, std::false_type{});
    } else {
        if (h->uniforms) by_width(std::false_type{}, std::true_type{});
        else by_width(std::false_type{}, std::false_type{});
    }
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

// The resolver alone, for the epoch's last block in the Grams-ahead form.
template <int BB>
int run_resolve_ahead(cdgrab_handle *h, const RowMap &rm, const double *gram, const double *dots_in,
                      int8_t *signs_out, double *dots_export) {
    const int groups = (int)((rm.d + kSplitElems - 1) / kSplitElems);
    MARK(h, 2, kResolve);
    auto resolve = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, dim3(1, (unsigned)h->walks), dim3(kResolveThreads<BB>), 0, h->stream, gram,
                           (int64_t)0, dots_in, groups, (int64_t)BB, rm.nb, rm.k0, rm.i0, rm.m, rm.n / 2,
                           h->eps_blk, signs_out, dots_export, h->uniforms, h->ws);
    };
    if (h->uniforms) resolve(resolve_signs<BB, true, 1>);
    else resolve(resolve_signs<BB, false, 1>);
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

// Gram tiles of `count` blocks (row maps already in h->maps) into gram_out[count][PART].
template <int BB>
int run_grams_ahead(cdgrab_handle *h, int64_t d, const cdgrab_plan &plan, int64_t count, int groups,
                    double *gram_out) {
    constexpr int part = PartLayout<BB>::PART;
    const dim3 grid((unsigned)groups, (unsigned)count, (unsigned)h->walks), block(kThreads);
    MARK(h, 2, kPass1);
    const int64_t ntiles = (d + plan.tile_elems - 1) / plan.tile_elems;
    auto launch = [&](auto kernel) {
        hipLaunchKernelGGL(kernel, grid, block, 0, h->stream, h->maps, h->r_sum, h->partials, ntiles, count);
    };
    if (plan.tile_elems == 128) {
        switch (plan.vector_width) {
            case 4: launch(gram_batched<BB, 4, 128>); break;
            case 2: launch(gram_batched<BB, 2, 128>); break;
            default: launch(gram_batched<BB, 1, 128>); break;
        }
    } else {
        switch (plan.vector_width) {
            case 4: launch(gram_batched<BB, 4, 64>); break;
            case 2: launch(gram_batched<BB, 2, 64>); break;
            default: launch(gram_batched<BB, 1, 64>); break;
        }
    }
    MARK(h, 2, kReduce);
    hipLaunchKernelGGL(reduce_batched, dim3((part + kThreads - 1) / kThreads, (unsigned)count, (unsigned)h->walks),
                       block, 0, h->stream, h->partials, gram_out, part, groups, h->ws.gram);
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

// One block: dots + Gram (with the previous block applied in the same launch when
// `prev` is given), reduction, sign resolution, and -- unless the apply is left to the
// next block's launch -- the apply pass.
template <int BB>
int run_block_vw(cdgrab_handle *h, const RowMap &rm, const PrevBlock *prev, bool apply_now,
                 const cdgrab_plan &plan, int8_t *signs_out, double *dots_out) {
    const int part = PartLayout<BB>::PART;
    MARK(h, 2, kPass1);
    switch (plan.vector_width) {
        case 4: launch_pass1<BB, 4>(h, rm, prev, plan); break;
        case 2: launch_pass1<BB, 2>(h, rm, prev, plan); break;
        default: launch_pass1<BB, 1>(h, rm, prev, plan); break;
    }
    MARK(h, 2, kReduce);
    hipLaunchKernelGGL(reduce_partials,
                       dim3((part + kReduceEntries - 1) / kReduceEntries, kReduceSlices),
                       dim3(kThreads), 0, h->stream, h->partials, h->reduced, part, plan.pass1_groups);
    MARK(h, 2, kResolve);
    launch_resolve<BB>(h, rm, signs_out, dots_out);
    if (apply_now) {
        MARK(h, 2, kPass2);
        switch (plan.vector_width) {
            case 4: launch_pass2<BB, 4>(h, rm, plan.pass2_groups); break;
            case 2: launch_pass2<BB, 2>(h, rm, plan.pass2_groups); break;
            default: launch_pass2<BB, 1>(h, rm, plan.pass2_groups); break;
        }
    }
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

template <int BB>
int apply_block_vw(cdgrab_handle *h, const RowMap &rm, const cdgrab_plan &plan) {
    MARK(h, 2, kPass2);
    switch (plan.vector_width) {
        case 4: launch_pass2<BB, 4>(h, rm, plan.pass2_groups); break;
        case 2: launch_pass2<BB, 2>(h, rm, plan.pass2_groups); break;
        default: launch_pass2<BB, 1>(h, rm, plan.pass2_groups); break;
    }
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

}  // namespace

extern "C" {

int cdgrab_create(cdgrab_handle **out, const cdgrab_options *opt) {
    if (!out) return fail(nullptr, CDGRAB_EINVAL, "cdgrab_create: out is NULL");
    *out = nullptr;
    cdgrab_options o{};
    if (opt) o = *opt;
    if (o.block_pairs != 0 && o.block_pairs != 16 && o.block_pairs != 32 && o.block_pairs != 64)
        return fail(nullptr, CDGRAB_EINVAL, "block_pairs must be 0, 16, 32 or 64 (got %d)", o.block_pairs);
    if (o.timing < 0 || o.timing > 2) return fail(nullptr, CDGRAB_EINVAL, "timing must be 0, 1 or 2");
    if (o.pass1_groups < 0 || o.pass1_groups > 65536)
        return fail(nullptr, CDGRAB_EINVAL, "pass1_groups out of range");
    if (o.apply_mode < 0 || o.apply_mode > 4) return fail(nullptr, CDGRAB_EINVAL, "apply_mode must be 0 .. 4");
    if (o.apply_groups < 0 || o.apply_groups > 65536)
        return fail(nullptr, CDGRAB_EINVAL, "apply_groups out of range");
    if (o.gram_mode < 0 || o.gram_mode > 2) return fail(nullptr, CDGRAB_EINVAL, "gram_mode must be 0, 1 or 2");
    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess || o.device < 0 || o.device >= count)
        return fail(nullptr, CDGRAB_EHIP, "no HIP device %d (%d visible): %s", o.device, count,
                    hipGetErrorString(e));
    cdgrab_handle *h = new (std::nothrow) cdgrab_handle();
    if (!h) return fail(nullptr, CDGRAB_ENOMEM, "out of host memory");
    h->device = o.device;
    h->stream = reinterpret_cast<hipStream_t>(o.stream);
    h->block_pairs_opt = o.block_pairs;
    h->timing = o.timing;
    h->pass1_groups_opt = o.pass1_groups;
    h->apply_mode = o.apply_mode;
    h->gram_mode = o.gram_mode;
    h->apply_groups_opt = o.apply_groups;
    hipDeviceProp_t prop;
    if (hipSetDevice(h->device) == hipSuccess && hipGetDeviceProperties(&prop, h->device) == hipSuccess)
        h->num_cu = prop.multiProcessorCount;
    *out = h;
    return CDGRAB_OK;
}

int cdgrab_destroy(cdgrab_handle *h) {
    if (!h) return CDGRAB_OK;
    (void)hipSetDevice(h->device);
    (void)hipStreamSynchronize(h->stream);
    for (hipEvent_t ev : h->event_pool) (void)hipEventDestroy(ev);
    if (h->r_sum) (void)hipFree(h->r_sum);
    if (h->partials) (void)hipFree(h->partials);
    if (h->reduced) (void)hipFree(h->reduced);
    if (h->eps_blk) (void)hipFree(h->eps_blk);
    if (h->flag) (void)hipFree(h->flag);
    if (h->herd_ws) (void)hipFree(h->herd_ws);
    if (h->train_delta) (void)hipFree(h->train_delta);
    if (h->train_perm) (void)hipFree(h->train_perm);
    if (h->train_signs) (void)hipFree(h->train_signs);
    if (h->zero_row) (void)hipFree(h->zero_row);
    if (h->staging) (void)hipFree(h->staging);
    if (h->gram_all) (void)hipFree(h->gram_all);
    if (h->dot_partials) (void)hipFree(h->dot_partials);
    if (h->maps) (void)hipFree(h->maps);
    delete h;
    return CDGRAB_OK;
}

const char *cdgrab_last_error(const cdgrab_handle *h) {
    return h ? h->err.c_str() : g_create_error.c_str();
}

int cdgrab_plan_epoch(int64_t m, int64_t n, int64_t d, int32_t block_pairs, int32_t streamed,
                      int64_t base_align, cdgrab_plan *plan) {
    return plan_epoch(m, n, d, block_pairs, streamed, base_align, 256, 0, 0, 0, 0, plan);
}

int cdgrab_pergrad(cdgrab_handle *h, int64_t N, int64_t in_dim, int64_t classes, const float *X,
                   const int32_t *y, const float *W, float *G_out) {
    if (!h) return CDGRAB_EINVAL;
    if (N < 0 || in_dim < 1 || classes < 1 || classes > 1024 || in_dim > (1 << 20))
        return fail(h, CDGRAB_EINVAL, "cdgrab_pergrad: bad sizes N=%lld in_dim=%lld classes=%lld",
                    (long long)N, (long long)in_dim, (long long)classes);
    if (N == 0) return CDGRAB_OK;
    if (!X || !y || !W || !G_out) return fail(h, CDGRAB_EINVAL, "cdgrab_pergrad: null pointer");
    // per-wave staging of one example; fewer wavefronts per workgroup when it is long
    const size_t per_wave = (size_t)(in_dim + 1 + classes) * sizeof(float);
    if (per_wave > 64 * 1024)
        return fail(h, CDGRAB_EINVAL, "cdgrab_pergrad: in_dim + classes too large for LDS staging");
    int waves = kGradWaves;
    while (waves > 1 && waves * per_wave > 64 * 1024) waves >>= 1;
    const size_t lds_waves = waves * per_wave;
    HIP_TRY(h, hipSetDevice(h->device));
    // weights in LDS when they fit beside the per-wave staging (64 KB per workgroup)
    const int wstride = (int)classes | 1;
    const size_t lds_w = (size_t)(in_dim + 1) * (size_t)wstride * sizeof(float);
    const bool wlds = lds_waves + lds_w <= 64 * 1024;
    const size_t lds = lds_waves + (wlds ? lds_w : 0);
    // each wavefront loops over examples: as many workgroups as stay resident
    int64_t per_cu = (int64_t)((160 * 1024) / lds);
    per_cu = std::max<int64_t>(1, std::min<int64_t>(per_cu, 32 / waves));
    int64_t groups = std::min<int64_t>((N + waves - 1) / waves, per_cu * h->num_cu);
    const bool prefetch = in_dim <= 64 * kGradPrefetch;
    auto launch = [&](auto kernel, int stride) {
        hipLaunchKernelGGL(kernel, dim3((unsigned)groups), dim3(waves * 64), lds, h->stream, X, y, W,
                           G_out, N, (int)in_dim, (int)classes, stride);
    };
    if (wlds && prefetch) launch(softmax_pergrad<true, true>, wstride);
    else if (wlds) launch(softmax_pergrad<true, false>, wstride);
    else if (prefetch) launch(softmax_pergrad<false, true>, (int)classes);
    else launch(softmax_pergrad<false, false>, (int)classes);
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

// Dispatch on the block size, which is a template parameter of the launch helpers.
#define BY_BLOCK_PAIRS(bb, call64, call32, call16) ((bb) == 64 ? (call64) : (bb) == 32 ? (call32) : (call16))

namespace {

// One epoch's state: what the caller gave, the plan, the launch form chosen, and the
// row map of the current and of the previous block.
struct Epoch {
    cdgrab_handle *h;
    int64_t m, n, d;
    const float *grads;        // dense input, or null: rows come from gen
    cdgrab_gen_fn gen;
    void *gen_ctx;
    int64_t chunk_pairs;       // flattened pairs staged per generator call
    const float *center_row;   // dense, m == 1: every row is paired with this one
    int8_t *signs_out;
    double *dots_out;

    bool streamed = false;
    cdgrab_plan plan{};
    int bb = 0;
    bool fused = false;        // apply inside the next block's dot/Gram launch
    bool ahead = false;        // Gram matrices of a batch of blocks ahead, one launch per block
    int64_t batch = 0;         // blocks per ahead-launch (a staging chunk's blocks when streaming)
    int gram_groups = 1;       // workgroups per block of the ahead-launch
    int64_t staging_chunk = 0; // floats per staging chunk
    int64_t center_off = 0;    // element offset of center_row from grads
    int64_t walks = 1;         // independent walks of this shape run side by side (m == 1, dense, Grams ahead)

    RowMap rm;
    PrevBlock prev;
    bool have_prev = false;

    int prepare();
    void set_block(int64_t p0, int64_t nb, const float *stage_base);
    int generate(int64_t first, int64_t count, float *stage_buf);
    int chain_ahead();
    int chain_blocks();
    int apply_last();
};

// Validation, plan, choice of the launch form, workspace.
int Epoch::prepare() {
    if (m < 1 || n < 2 || (n & 1) || d < 1)
        return fail(h, CDGRAB_EINVAL,
                    "cdgrab_balance_epoch: need m>=1, even n>=2, d>=1 (got m=%lld n=%lld d=%lld)",
                    (long long)m, (long long)n, (long long)d);
    if ((grads == nullptr) == (gen == nullptr))
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: give exactly one of grads and gen");
    if (n > INT32_MAX) return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: n exceeds int32 range");
    HIP_TRY(h, hipSetDevice(h->device));

    streamed = grads == nullptr;
    int64_t align = 16;
    if (!streamed) {
        uintptr_t a = reinterpret_cast<uintptr_t>(grads);
        if (center_row) a |= reinterpret_cast<uintptr_t>(center_row);
        align = (a % 16 == 0) ? 16 : (a % 8 == 0) ? 8 : 4;
        if (a % 4) return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: grads is not 4-byte aligned");
    }
    // (Every one of the d/64 workgroups of a block's launch in the Grams-ahead form reads all
    // d/64 x Bb partial dots of the previous block: quadratic in d, hence refused for long rows.)
    if (h->gram_mode == 2 && !streamed && d > kGramAheadLimitD)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: gram_mode 2 is for rows up to %lld elements (d=%lld)",
                    (long long)kGramAheadLimitD, (long long)d);
    int rc = plan_epoch(m, n, d, h->block_pairs_opt, streamed, align, h->num_cu, h->pass1_groups_opt,
                        h->apply_mode, h->gram_mode, chunk_pairs, &plan);
    if (rc != CDGRAB_OK) return fail(h, rc, "cdgrab_balance_epoch: sizes overflow or are invalid");
    bb = plan.block_pairs;
    if (chunk_pairs <= 0) chunk_pairs = bb;
    staging_chunk = chunk_pairs * 2 * d;
    fused = plan.fused_apply != 0;
    ahead = plan.gram_ahead != 0;
    batch = streamed ? chunk_pairs / bb : std::min<int64_t>(plan.blocks, kGramBatch);

    // workspace (per walk when several independent walks run side by side)
    const int64_t r_pad = round_up(d, kPadE);
    if (walks > 1 && !(ahead && !streamed && !center_row && m == 1))
        return fail(h, CDGRAB_EINVAL, "several walks per launch need dense short rows (the Grams-ahead form)");
    int64_t fixed_cap = 0;
    rc = ensure(h, h->r_sum, h->r_cap, walks * r_pad);
    if (rc) return rc;
    rc = ensure(h, h->partials, h->partials_cap, (int64_t)plan.pass1_groups * part_size(bb));
    if (rc) return rc;
    if (!h->reduced) { fixed_cap = 0; rc = ensure(h, h->reduced, fixed_cap, (int64_t)kReduceSlices * PartLayout<64>::PART); if (rc) return rc; }
    rc = ensure(h, h->eps_blk, h->eps_cap, walks * kMaxBlockPairs);
    if (rc) return rc;
    if (streamed) {
        // two chunks when a launch reads the previous block's rows as well: they must outlive the next fill
        rc = ensure(h, h->staging, h->staging_cap, ((fused || ahead) ? 2 : 1) * staging_chunk);
        if (rc) return rc;
    }
    h->ws = WalkStrides{};
    if (ahead) {
        // enough workgroups to fill the chip, at least one tile each
        const int64_t ntiles = (d + plan.tile_elems - 1) / plan.tile_elems;
        const int64_t launches = batch * walks;
        gram_groups = (int)std::max<int64_t>(1, std::min<int64_t>(ntiles, (4 * h->num_cu + launches - 1) / launches));
        const int64_t dot_len = (d + kSplitElems - 1) / kSplitElems * bb;
        rc = ensure(h, h->partials, h->partials_cap, walks * batch * gram_groups * part_size(bb));
        if (rc) return rc;
        rc = ensure(h, h->gram_all, h->gram_all_cap, walks * (batch + 1) * part_size(bb));
        if (rc) return rc;
        rc = ensure(h, h->dot_partials, h->dot_partials_cap, walks * 2 * dot_len);
        if (rc) return rc;
        rc = ensure(h, h->maps, h->maps_cap, walks * batch);
        if (rc) return rc;
        if (walks > 1) {
            h->ws.rows = n * d;
            h->ws.r = r_pad;
            h->ws.gram = (batch + 1) * part_size(bb);
            h->ws.dots = 2 * dot_len;
            h->ws.out = n / 2;
            h->ws.maps = batch;
        }
    }
    h->walks = walks;

    center_off = center_row ? (int64_t)((reinterpret_cast<intptr_t>(center_row) - reinterpret_cast<intptr_t>(grads)) /
                                        (intptr_t)sizeof(float))
                            : 0;
    rm.d = d; rm.m = (int32_t)m; rm.n = n; rm.dense = (!streamed && !center_row) ? 1 : 0;
    rm.k0 = 0; rm.i0 = 0; rm.nb = 0;
    // (a copy of this map stands in for "no previous block": its rows must be readable)
    rm.base = streamed ? h->staging : grads;
    for (int64_t &o : rm.off) o = 0;
    prev.eps = h->eps_blk;
    prev.rm = rm;
    have_prev = false;
    return CDGRAB_OK;
}

// Row offsets of the block of flattened pairs p0 .. p0+nb-1 (dense input), or of a
// staging chunk's rows [2 q], [2 q + 1] starting at stage_base.
void Epoch::set_block(int64_t p0, int64_t nb, const float *stage_base) {
    rm.k0 = p0 / m;
    rm.i0 = (int32_t)(p0 - rm.k0 * m);
    rm.nb = (int32_t)nb;
    if (stage_base) rm.base = stage_base;
    for (int j = 0; j < rm.nb; ++j) {
        if (stage_base) {
            rm.off[2 * j] = (int64_t)(2 * j) * d;
        } else if (center_row) {
            rm.off[2 * j] = (p0 + j) * d;
            rm.off[2 * j + 1] = center_off;
            continue;
        } else {
            const int64_t p = p0 + j, k = p / m, i = p - k * m;
            rm.off[2 * j] = (i * n + 2 * k) * d;
        }
        rm.off[2 * j + 1] = rm.off[2 * j] + d;
    }
    // The kernels read the table without a branch, also for pairs the block does not have:
    // those entries point at the block's first row, which is always readable (an entry left
    // over from an earlier, fuller block could point past the end of a staging chunk).
    for (int j = rm.nb; j < kMaxBlockPairs; ++j) rm.off[2 * j] = rm.off[2 * j + 1] = 0;
}

int Epoch::generate(int64_t first, int64_t count, float *stage_buf) {
    MARK(h, 1, kGen);
    const int grc = gen(gen_ctx, first, count, stage_buf, h->stream);
    if (grc != 0)
        return fail(h, CDGRAB_EGEN, "generator callback returned %d at pair %lld", grc, (long long)first);
    return CDGRAB_OK;
}

// Gram matrices of a batch of blocks in one launch, then one launch per block.  Slot 0 of
// gram_all carries the last block of the previous batch over; the per-workgroup dots
// alternate between two arrays (a launch reads the previous block's while it writes its own).
int Epoch::chain_ahead() {
    const int64_t part = part_size(bb);
    const int64_t dot_len = (d + kSplitElems - 1) / kSplitElems * bb;
    int64_t blk = 0, prev_slot = 0, batch_index = 0;
    int rc = CDGRAB_OK;
    for (int64_t b0 = 0; b0 < plan.blocks; b0 += batch, ++batch_index) {
        const int64_t count = std::min<int64_t>(batch, plan.blocks - b0);
        const int64_t first = b0 * bb, cnt_pairs = std::min<int64_t>(count * bb, plan.pairs - first);
        float *stage_buf = streamed ? h->staging + (batch_index & 1) * staging_chunk : nullptr;
        if (streamed && (rc = generate(first, cnt_pairs, stage_buf))) return rc;
        MARK(h, 1, kBalance);
        if (b0 > 0)
            for (int64_t w = 0; w < walks; ++w)
                HIP_TRY(h, hipMemcpyAsync(h->gram_all + w * h->ws.gram, h->gram_all + w * h->ws.gram + prev_slot * part,
                                          (size_t)part * sizeof(double), hipMemcpyDeviceToDevice, h->stream));
        hipLaunchKernelGGL(fill_row_maps, dim3((unsigned)count, (unsigned)walks), dim3(kMaxBlockPairs), 0, h->stream,
                           h->maps, streamed ? stage_buf : grads, m, n, d, bb, first, plan.pairs, center_off,
                           streamed ? 2 : (center_row ? 1 : 0), h->ws.rows);
        double *gram_out = h->gram_all + part;
        rc = BY_BLOCK_PAIRS(bb, run_grams_ahead<64>(h, d, plan, count, gram_groups, gram_out),
                            run_grams_ahead<32>(h, d, plan, count, gram_groups, gram_out),
                            run_grams_ahead<16>(h, d, plan, count, gram_groups, gram_out));
        if (rc) return rc;
        for (int64_t b = 0; b < count; ++b, ++blk) {
            const int64_t p0 = (b0 + b) * bb;
            set_block(p0, std::min<int64_t>(bb, plan.pairs - p0), streamed ? stage_buf + (p0 - first) * 2 * d : nullptr);
            // block b of this batch sits in slot b + 1, its predecessor in slot b
            const double *prev_gram = h->gram_all + b * part;
            const double *dots_in = h->dot_partials + ((blk + 1) & 1) * dot_len;
            double *dots_mine = h->dot_partials + (blk & 1) * dot_len;
            rc = BY_BLOCK_PAIRS(bb,
                                run_block_ahead<64>(h, rm, prev, plan, prev_gram, dots_in, dots_mine, signs_out, dots_out),
                                run_block_ahead<32>(h, rm, prev, plan, prev_gram, dots_in, dots_mine, signs_out, dots_out),
                                run_block_ahead<16>(h, rm, prev, plan, prev_gram, dots_in, dots_mine, signs_out, dots_out));
            if (rc) return rc;
            prev.rm = rm;
            have_prev = true;
        }
        prev_slot = count;
    }
    // the last block: the resolver alone (its apply follows)
    const double *gram = h->gram_all + prev_slot * part;
    const double *dots_in = h->dot_partials + ((blk + 1) & 1) * dot_len;
    MARK(h, 1, kBalance);
    return BY_BLOCK_PAIRS(bb, run_resolve_ahead<64>(h, prev.rm, gram, dots_in, signs_out, dots_out),
                          run_resolve_ahead<32>(h, prev.rm, gram, dots_in, signs_out, dots_out),
                          run_resolve_ahead<16>(h, prev.rm, gram, dots_in, signs_out, dots_out));
}

// Block by block: dot/Gram launch (with the previous block's apply inside it when
// fused), reduction, resolver, and the apply launch when it is not fused.
int Epoch::chain_blocks() {
    const int64_t chunk = streamed ? chunk_pairs : plan.pairs;
    int64_t chunk_index = 0;
    int rc = CDGRAB_OK;
    for (int64_t first = 0; first < plan.pairs; first += chunk, ++chunk_index) {
        const int64_t cnt = std::min<int64_t>(chunk, plan.pairs - first);
        // with the fused pass the previous block's rows must outlive this chunk's staging
        float *stage_buf = h->staging + ((fused && (chunk_index & 1)) ? staging_chunk : 0);
        if (streamed && (rc = generate(first, cnt, stage_buf))) return rc;
        for (int64_t p0 = first; p0 < first + cnt; p0 += bb) {
            set_block(p0, std::min<int64_t>(bb, first + cnt - p0), streamed ? stage_buf + (p0 - first) * 2 * d : nullptr);
            MARK(h, 1, kBalance);
            const PrevBlock *pp = (fused && have_prev) ? &prev : nullptr;
            rc = BY_BLOCK_PAIRS(bb, run_block_vw<64>(h, rm, pp, !fused, plan, signs_out, dots_out),
                                run_block_vw<32>(h, rm, pp, !fused, plan, signs_out, dots_out),
                                run_block_vw<16>(h, rm, pp, !fused, plan, signs_out, dots_out));
            if (rc) return rc;
            prev.rm = rm;
            have_prev = true;
        }
    }
    return CDGRAB_OK;
}

// The epoch's last block has no successor to apply it.
int Epoch::apply_last() {
    if (!(fused || ahead) || !have_prev) return CDGRAB_OK;
    MARK(h, 1, kBalance);
    return BY_BLOCK_PAIRS(bb, apply_block_vw<64>(h, prev.rm, plan), apply_block_vw<32>(h, prev.rm, plan),
                          apply_block_vw<16>(h, prev.rm, plan));
}

}  // namespace

// One epoch.  With a generator, `chunk_pairs` flattened pairs are staged per callback
// (0 = one block) and balanced block by block out of the staging buffer.
// With `center_row` (dense input, m == 1) every row j is paired with that one row
// instead of with its neighbour: "pair" j is (row j, center_row), n pairs in all, and
// the permutation is left to the caller (perm_out may be null).
static int balance_epoch_impl(cdgrab_handle *h, int64_t m, int64_t n, int64_t d, const float *grads,
                              cdgrab_gen_fn gen, void *gen_ctx, int64_t chunk_pairs,
                              const int32_t *perm_in, int8_t *signs_out, int32_t *perm_out,
                              float *r_out, double *r64_out, double *dots_out,
                              const float *center_row = nullptr, int64_t walks = 1) {
    if (!h) return CDGRAB_EINVAL;
    if (!signs_out || (!perm_out && !center_row))
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: signs_out and perm_out are required");
    Epoch ep{h, m, n, d, grads, gen, gen_ctx, chunk_pairs, center_row, signs_out, dots_out};
    ep.walks = walks;
    int rc = ep.prepare();
    if (rc) return rc;
    // the permutation kernel reads perm_in while other threads write perm_out
    if (ranges_overlap(perm_in, walks * m * n * 4, perm_out, walks * m * n * 4))
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch: perm_in and perm_out must not overlap");

    h->marks.clear();
    h->events_used = 0;
    h->have_timing = false;
    hipLaunchKernelGGL(fill_zero_f64, dim3(std::min<int64_t>(4096, (h->r_cap + 255) / 256)), dim3(256), 0,
                       h->stream, h->r_sum, h->r_cap);
    rc = ep.ahead ? ep.chain_ahead() : ep.chain_blocks();
    if (rc) return rc;
    rc = ep.apply_last();
    if (rc) return rc;

    MARK(h, 1, kFinish);
    if (!center_row)  // (side-by-side walks are one-worker walks: `walks` rows of signs and orders)
        hipLaunchKernelGGL(build_pair_permutations, dim3((unsigned)((walks * m * (n / 2) + 255) / 256)), dim3(256),
                           0, h->stream, signs_out, perm_in, perm_out, walks * m, n);
    if (r_out || r64_out)
        hipLaunchKernelGGL(export_running_sum, dim3((unsigned)std::min<int64_t>(8192, (d + 255) / 256)), dim3(256),
                           0, h->stream, h->r_sum, d, r_out, r64_out);
    MARK(h, 1, -1);
    HIP_TRY(h, hipGetLastError());
    const int64_t cp = ep.chunk_pairs, bb = ep.bb;
    h->last = cdgrab_timing{};
    h->last.blocks = ep.streamed ? ((ep.plan.pairs / cp) * ((cp + bb - 1) / bb) + ((ep.plan.pairs % cp) + bb - 1) / bb)
                                 : ep.plan.blocks;
    h->last.block_pairs = (int32_t)bb;
    h->last.pass1_groups = ep.plan.pass1_groups;
    h->have_timing = h->timing >= 1;
    h->walks = 1;
    h->ws = WalkStrides{};
    return CDGRAB_OK;
}

int cdgrab_balance_epoch(cdgrab_handle *h, int64_t m, int64_t n, int64_t d, const float *grads,
                         cdgrab_gen_fn gen, void *gen_ctx, const int32_t *perm_in,
                         int8_t *signs_out, int32_t *perm_out, float *r_out, double *r64_out,
                         double *dots_out) {
    return balance_epoch_impl(h, m, n, d, grads, gen, gen_ctx, 0, perm_in, signs_out, perm_out, r_out,
                              r64_out, dots_out);
}

// ---- the epoch on a static workspace (for callers that cannot allocate) -------------
namespace {

// Workspace of cdgrab_balance_epoch_static, in doubles: the running sum, the per-workgroup
// partials of the dot/Gram pass, the slice sums of the reduction, and the block's signs.
constexpr int64_t kStaticMaxD = CDGRAB_STATIC_MAX_D;
constexpr int kStaticGroups = 128;  // workgroups of the dot/Gram pass at most
constexpr int64_t kStaticRsum = kStaticMaxD;
constexpr int64_t kStaticPartials = (int64_t)kStaticGroups * PartLayout<64>::PART;
constexpr int64_t kStaticReduced = (int64_t)kReduceSlices * PartLayout<64>::PART;
constexpr int64_t kStaticEps = 64 / 8;
constexpr int64_t kStaticDoubles = kStaticRsum + kStaticPartials + kStaticReduced + kStaticEps;
static_assert(kStaticMaxD % kPadE == 0, "the running sum is padded to whole tiles");

constexpr int kMaxDevices = 64;
double *g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, once resolved
std::mutex g_scratch_mutex;

}  // namespace

// Every GPU the library runs on holds its own copy of this array (about 3.9 MB) until the
// process ends.  In host code the name is only a stand-in: its device address comes from
// hipGetSymbolAddress with that device current.
static __device__ __align__(256) double scratch[kStaticDoubles];

namespace {

int static_scratch(cdgrab_handle *h, double **out) {
    if (h->device < 0 || h->device >= kMaxDevices)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_static: device ordinal %d not supported", h->device);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[h->device]) {
        HIP_TRY(h, hipSetDevice(h->device));
        void *ptr = nullptr;
        HIP_TRY(h, hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return fail(h, CDGRAB_EHIP, "cdgrab_balance_epoch_static: no device address for the workspace");
        g_scratch_ptr[h->device] = static_cast<double *>(ptr);
    }
    *out = g_scratch_ptr[h->device];
    return CDGRAB_OK;
}

}  // namespace

int cdgrab_balance_epoch_static(cdgrab_handle *h, int64_t m, int64_t n, int64_t d, const float *grads,
                                const int32_t *perm_in, int8_t *signs_out, int32_t *perm_out,
                                float *r_out, double *r64_out, double *dots_out) {
    if (!h) return CDGRAB_EINVAL;
    if (!grads) return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_static: grads is NULL (dense input only)");
    if (d > kStaticMaxD)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_static: d=%lld exceeds the static workspace (at most %lld)",
                    (long long)d, (long long)kStaticMaxD);
    double *base = nullptr;
    int rc = static_scratch(h, &base);
    if (rc) return rc;

    // Borrow the static array as the handle's workspace for this call: the per-block launch
    // form, no timing events, at most kStaticGroups workgroups in the dot/Gram pass.
    struct Saved {
        double *r_sum, *partials, *reduced; int8_t *eps_blk;
        int64_t r_cap, partials_cap, eps_cap; int timing, gram_mode, pass1_groups_opt; bool fixed;
    } sv{h->r_sum, h->partials, h->reduced, h->eps_blk, h->r_cap, h->partials_cap, h->eps_cap,
         h->timing, h->gram_mode, h->pass1_groups_opt, h->fixed_workspace};
    h->r_sum = base;
    h->r_cap = d > 0 ? round_up(d, kPadE) : 0;  // only this much is cleared and used
    h->partials = base + kStaticRsum;
    h->partials_cap = kStaticPartials;
    h->reduced = h->partials + kStaticPartials;
    h->eps_blk = reinterpret_cast<int8_t *>(h->reduced + kStaticReduced);
    h->eps_cap = kMaxBlockPairs;
    h->fixed_workspace = true;
    h->timing = 0;
    h->gram_mode = 1;
    h->pass1_groups_opt = (sv.pass1_groups_opt > 0 && sv.pass1_groups_opt < kStaticGroups) ? sv.pass1_groups_opt
                                                                                            : kStaticGroups;
    rc = balance_epoch_impl(h, m, n, d, grads, nullptr, nullptr, 0, perm_in, signs_out, perm_out, r_out,
                            r64_out, dots_out);
    h->r_sum = sv.r_sum; h->partials = sv.partials; h->reduced = sv.reduced; h->eps_blk = sv.eps_blk;
    h->r_cap = sv.r_cap; h->partials_cap = sv.partials_cap; h->eps_cap = sv.eps_cap;
    h->timing = sv.timing; h->gram_mode = sv.gram_mode; h->pass1_groups_opt = sv.pass1_groups_opt;
    h->fixed_workspace = sv.fixed;
    h->have_timing = false;
    return rc;
}

int cdgrab_balance_epoch_randomized(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                                    const float *grads, const float *uniforms, const int32_t *perm_in,
                                    int8_t *signs_out, int32_t *perm_out, double *r64_out,
                                    double *dots_out) {
    if (!h) return CDGRAB_EINVAL;
    if (!uniforms) return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_randomized: uniforms is NULL");
    h->uniforms = uniforms;
    int rc = balance_epoch_impl(h, m, n, d, grads, nullptr, nullptr, 0, perm_in, signs_out, perm_out, nullptr,
                                r64_out, dots_out);
    h->uniforms = nullptr;
    return rc;
}

int cdgrab_balance_epoch_stale_mean(cdgrab_handle *h, int64_t n, int64_t d, const float *grads,
                                    const float *stale_mean, const int32_t *perm_in,
                                    int8_t *signs_out, int32_t *perm_out, float *mean_out,
                                    double *r64_out) {
    if (!h) return CDGRAB_EINVAL;
    if (n < 1 || d < 1 || n > INT32_MAX / 2)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_stale_mean: need n>=1, d>=1");
    if (!grads || !signs_out || !perm_out)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_stale_mean: null pointer");
    if (ranges_overlap(perm_in, n * 4, perm_out, n * 4))
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_stale_mean: perm_in and perm_out must not overlap");
    if (ranges_overlap(stale_mean, d * 4, mean_out, d * 4))
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_stale_mean: stale_mean and mean_out must not overlap");
    HIP_TRY(h, hipSetDevice(h->device));
    int rc = CDGRAB_OK;
    if (!stale_mean) {
        rc = ensure(h, h->zero_row, h->zero_row_cap, d);
        if (rc) return rc;
        hipLaunchKernelGGL(fill_zero_b32, dim3((unsigned)std::min<int64_t>(4096, (d + 255) / 256)), dim3(256), 0,
                           h->stream, reinterpret_cast<uint32_t *>(h->zero_row), d);
        stale_mean = h->zero_row;
    }
    if (!h->flag) { int64_t cap = 0; rc = ensure(h, h->flag, cap, (int64_t)1); if (rc) return rc; }
    // single vectors as pairs (g_j, stale mean): the pair walk then balances
    // mean - g_j = -z_j and its exported sign is minus the sign of z_j, ties included
    rc = balance_epoch_impl(h, 1, 2 * n, d, grads, nullptr, nullptr, 0, nullptr, signs_out, nullptr, nullptr,
                            r64_out, nullptr, stale_mean);
    if (rc) return rc;
    hipLaunchKernelGGL(negate_signs, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, h->stream, signs_out, n);
    hipLaunchKernelGGL(fill_zero_b32, dim3(1), dim3(64), 0, h->stream, reinterpret_cast<uint32_t *>(h->flag), (int64_t)1);
    hipLaunchKernelGGL(reorder_from_signs, dim3(1), dim3(kScanThreads), 0, h->stream, signs_out, perm_in,
                       perm_out, n, h->flag);
    if (mean_out)
        hipLaunchKernelGGL(column_mean, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, h->stream, grads, n, d,
                           mean_out);
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

int cdgrab_balance_epoch_independent(cdgrab_handle *h, int64_t m, int64_t n, int64_t d,
                                     const float *grads, const int32_t *perm_in, int8_t *signs_out,
                                     int32_t *perm_out) {
    if (!h) return CDGRAB_EINVAL;
    if (m < 1) return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_independent: need m>=1");
    if (!grads || !signs_out || !perm_out)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_independent: null pointer");
    if (n < 2 || (n & 1) || d < 1 || m > (INT64_MAX / n) / d)
        return fail(h, CDGRAB_EINVAL, "cdgrab_balance_epoch_independent: need even n >= 2, d >= 1");
    // Short rows (the Grams-ahead form): the m one-worker walks run side by side, the worker
    // as a grid coordinate, each on its own running sum -- every launch of the chain serves all
    // workers.  Same kernels, same sums in the same order as a one-worker epoch.  (A worker's
    // rows start n*d floats after the previous worker's: as aligned as the first worker's
    // whenever d suits the load width.)
    if (m > 1 && m <= 65535) {
        const uintptr_t a = reinterpret_cast<uintptr_t>(grads);
        cdgrab_plan one{};
        const int prc = plan_epoch(1, n, d, h->block_pairs_opt, 0, (a % 16 == 0) ? 16 : (a % 8 == 0) ? 8 : 4,
                                   h->num_cu, h->pass1_groups_opt, h->apply_mode, h->gram_mode, 0, &one);
        if (prc == CDGRAB_OK && one.gram_ahead)
            return balance_epoch_impl(h, 1, n, d, grads, nullptr, nullptr, 0, perm_in, signs_out, perm_out,
                                      nullptr, nullptr, nullptr, nullptr, m);
    }
    // long rows: m separate one-worker epochs, each bound by bytes, not by launches
    for (int64_t i = 0; i < m; ++i) {
        int rc = balance_epoch_impl(h, 1, n, d, grads + i * n * d, nullptr, nullptr, 0,
                                    perm_in ? perm_in + i * n : nullptr, signs_out + i * (n / 2),
                                    perm_out + i * n, nullptr, nullptr, nullptr);
        if (rc) return rc;
    }
    return CDGRAB_OK;
}

namespace {
// State of the internal generator of cdgrab_train_epoch_softmax: it produces the rows
// of a chunk of whole step pairs by running the workers' steps at the evolving weights.
struct TrainCtx {
    cdgrab_handle *h;
    int64_t m, n, in_dim, classes, d;
    const float *X; const int32_t *y; const int32_t *perm_in;
    float *W, *velocity, *grads_out, *loss_out;
    float lr, momentum;
};

int train_generate(void *vctx, int64_t first_pair, int64_t count, float *staging, void *stream) {
    TrainCtx *c = static_cast<TrainCtx *>(vctx);
    cdgrab_handle *h = c->h;
    if (first_pair % c->m != 0 || count % c->m != 0) return 1;  // chunks are whole step pairs
    const int64_t k_first = first_pair / c->m, k_count = count / c->m;
    const size_t lds = (size_t)c->classes * sizeof(float);
    for (int64_t j = 2 * k_first; j < 2 * (k_first + k_count); ++j) {
        hipLaunchKernelGGL(train_step_delta, dim3((unsigned)c->m), dim3(kDeltaWaves * 64), lds,
                           static_cast<hipStream_t>(stream), c->X, c->y,
                           c->perm_in, c->W, h->train_delta, c->loss_out, c->m, c->n, j, (int)c->in_dim,
                           (int)c->classes);
        if (c->perm_in)
            hipLaunchKernelGGL(train_step_update<true>, dim3((unsigned)((c->d + 255) / 256)), dim3(256), 0,
                               static_cast<hipStream_t>(stream), c->X, c->perm_in, h->train_delta, c->W,
                               c->velocity, staging, c->grads_out, c->m, c->n, j, k_first, (int)c->in_dim,
                               (int)c->classes, c->lr, c->momentum);
        else
            hipLaunchKernelGGL(train_step_update<false>, dim3((unsigned)((c->d + 255) / 256)), dim3(256), 0,
                               static_cast<hipStream_t>(stream), c->X, c->perm_in, h->train_delta, c->W,
                               c->velocity, staging, c->grads_out, c->m, c->n, j, k_first, (int)c->in_dim,
                               (int)c->classes, c->lr, c->momentum);
    }
    return hipGetLastError() == hipSuccess ? 0 : 2;
}
}  // namespace

int cdgrab_train_epoch_softmax(cdgrab_handle *h, int64_t m, int64_t n, int64_t in_dim, int64_t classes,
                               const float *X, const int32_t *y, const int32_t *perm_in, float *W,
                               float *velocity, float lr, float momentum, int8_t *signs_out,
                               int32_t *perm_out, float *grads_out, float *loss_out) {
    if (!h) return CDGRAB_EINVAL;
    if (m < 1 || n < 2 || (n & 1) || in_dim < 1 || classes < 1 || classes > 1024 || in_dim > (1 << 20))
        return fail(h, CDGRAB_EINVAL, "cdgrab_train_epoch_softmax: bad sizes");
    if (!X || !y || !W || !signs_out || !perm_out)
        return fail(h, CDGRAB_EINVAL, "cdgrab_train_epoch_softmax: null pointer");
    if (ranges_overlap(perm_in, m * n * 4, perm_out, m * n * 4))
        return fail(h, CDGRAB_EINVAL, "cdgrab_train_epoch_softmax: perm_in and perm_out must not overlap");
    if (momentum != 0.0f && !velocity)
        return fail(h, CDGRAB_EINVAL, "cdgrab_train_epoch_softmax: momentum needs a velocity buffer");
    HIP_TRY(h, hipSetDevice(h->device));
    int rc = ensure(h, h->train_delta, h->train_delta_cap, m * classes);
    if (rc) return rc;
    TrainCtx ctx{h, m, n, in_dim, classes, (in_dim + 1) * classes, X, y, perm_in, W, velocity,
                 grads_out, loss_out, lr, momentum};
    // a chunk is a whole number of step pairs: about one block's worth of pairs, at least one step pair;
    // for short rows eight blocks' worth (or as many as make it whole blocks), so that the Gram
    // matrices of a chunk are computed in one launch and a block costs a single one
    const int64_t step_pairs = std::max<int64_t>(1, 64 / m);
    int64_t chunk = step_pairs * m;
    if (ctx.d <= kGramAheadMaxD && h->gram_mode != 1 && h->apply_mode == 0) {
        const int64_t bb = pick_block_pairs(m * (n / 2), ctx.d, h->block_pairs_opt);
        int64_t k = 8;
        if ((chunk * k) % bb != 0) k = bb;  // chunk * bb is a multiple of bb
        if (chunk * k / bb <= kGramBatch && chunk * k * 2 * ctx.d * 4 * 2 <= ((int64_t)1 << 30)) chunk *= k;
    }
    return balance_epoch_impl(h, m, n, ctx.d, nullptr, train_generate, &ctx, chunk, perm_in,
                              signs_out, perm_out, nullptr, nullptr, nullptr);
}

int cdgrab_train_softmax(cdgrab_handle *h, int64_t m, int64_t n, int64_t in_dim, int64_t classes,
                         const float *X, const int32_t *y, int32_t *perm, float *W, float *velocity,
                         float lr, float momentum, int64_t epochs, int8_t *signs_out, float *loss_out) {
    if (!h) return CDGRAB_EINVAL;
    if (epochs < 1 || !perm) return fail(h, CDGRAB_EINVAL, "cdgrab_train_softmax: need epochs>=1 and perm");
    if (m < 1 || n < 2 || (n & 1) || m > INT32_MAX || n > INT32_MAX)
        return fail(h, CDGRAB_EINVAL, "cdgrab_train_softmax: bad sizes");
    HIP_TRY(h, hipSetDevice(h->device));
    int rc = ensure(h, h->train_perm, h->train_perm_cap, m * n);
    if (rc) return rc;
    if (!signs_out) {
        rc = ensure(h, h->train_signs, h->train_signs_cap, m * (n / 2));
        if (rc) return rc;
        signs_out = h->train_signs;
    }
    // the order ping-pongs between the caller's buffer and the spare one
    int32_t *cur = perm, *nxt = h->train_perm;
    for (int64_t t = 0; t < epochs; ++t) {
        rc = cdgrab_train_epoch_softmax(h, m, n, in_dim, classes, X, y, cur, W, velocity, lr, momentum,
                                        signs_out, nxt, nullptr, loss_out ? loss_out + t * m * n : nullptr);
        if (rc) return rc;
        std::swap(cur, nxt);
    }
    if (cur != perm)
        HIP_TRY(h, hipMemcpyAsync(perm, cur, (size_t)(m * n) * sizeof(int32_t), hipMemcpyDeviceToDevice,
                                  h->stream));
    return CDGRAB_OK;
}

int cdgrab_reorder(cdgrab_handle *h, int64_t m, int64_t n, const int8_t *signs,
                   const int32_t *perm_in, int32_t *perm_out) {
    if (!h) return CDGRAB_EINVAL;
    if (m < 1 || n < 1 || n > INT32_MAX || m > INT32_MAX)
        return fail(h, CDGRAB_EINVAL, "cdgrab_reorder: need m>=1, n>=1");
    if (!signs || !perm_out) return fail(h, CDGRAB_EINVAL, "cdgrab_reorder: null pointer");
    if (ranges_overlap(perm_in, m * n * 4, perm_out, m * n * 4))
        return fail(h, CDGRAB_EINVAL, "cdgrab_reorder: perm_in and perm_out must not overlap");
    HIP_TRY(h, hipSetDevice(h->device));
    if (!h->flag) { int64_t cap = 0; int rc = ensure(h, h->flag, cap, (int64_t)1); if (rc) return rc; }
    hipLaunchKernelGGL(fill_zero_b32, dim3(1), dim3(64), 0, h->stream, reinterpret_cast<uint32_t *>(h->flag), (int64_t)1);
    hipLaunchKernelGGL(reorder_from_signs, dim3((unsigned)m), dim3(kScanThreads), 0, h->stream, signs,
                       perm_in, perm_out, n, h->flag);
    HIP_TRY(h, hipGetLastError());
    int32_t bad = 0;
    HIP_TRY(h, hipMemcpyAsync(&bad, h->flag, sizeof bad, hipMemcpyDeviceToHost, h->stream));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    if (bad) return fail(h, CDGRAB_EINVAL, "cdgrab_reorder: a sign is neither +1 nor -1");
    return CDGRAB_OK;
}

int cdgrab_herding_bound(cdgrab_handle *h, int64_t m, int64_t n, int64_t d, const float *z,
                         const int32_t *perm, double *bound_out) {
    if (!h) return CDGRAB_EINVAL;
    if (m < 1 || n < 1 || d < 1 || m > (INT64_MAX / n) / d)
        return fail(h, CDGRAB_EINVAL, "cdgrab_herding_bound: need m>=1, n>=1, d>=1");
    if (!z || !bound_out) return fail(h, CDGRAB_EINVAL, "cdgrab_herding_bound: null pointer");
    HIP_TRY(h, hipSetDevice(h->device));
    HerdingShape sh;
    sh.m = m; sh.n = n; sh.d = d;
    // enough (segment, four elements) threads to fill the chip, at least one step per segment
    const int64_t quads = (d + 3) / 4;
    sh.quads = (int32_t)std::min<int64_t>(quads, INT32_MAX);
    // short rows: a workgroup serves several segments (thread = (segment, four elements))
    sh.spw = quads <= 128 ? (int32_t)(256 / quads) : 1;
    int64_t want_threads = (int64_t)h->num_cu * 2048;
    // blockIdx.y counts workgroups of spw segments (at most 65 535 of them)
    int64_t segs = std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(n, (int64_t)65535 * sh.spw),
                                                          (want_threads + quads - 1) / quads));
    sh.seg_len = (n + segs - 1) / segs;
    sh.segments = (n + sh.seg_len - 1) / sh.seg_len;
    int rc = ensure(h, h->herd_ws, h->herd_cap, 2 * sh.segments * d + d);
    if (rc) return rc;
    double *segsum = h->herd_ws, *start = segsum + sh.segments * d, *zbar = start + sh.segments * d;
    const dim3 grid(sh.spw == 1 ? (unsigned)((quads + 255) / 256) : 1u,
                    (unsigned)((sh.segments + sh.spw - 1) / sh.spw));
    unsigned long long *bits = reinterpret_cast<unsigned long long *>(bound_out);
    // the segment's example ids go through LDS when they fit (48 KB)
    const size_t ids_bytes = (size_t)(sh.seg_len * m) * sizeof(int32_t);
    const int lds_ids = (perm && sh.spw == 1 && ids_bytes <= 48 * 1024) ? 1 : 0;
    const size_t lds = lds_ids ? ids_bytes : 0;
    // widest load every row start allows
    const uintptr_t zb = reinterpret_cast<uintptr_t>(z);
    const int vw = (d % 4 == 0 && zb % 16 == 0) ? 4 : (d % 2 == 0 && zb % 8 == 0) ? 2 : 1;
    hipLaunchKernelGGL(herding_clear, dim3(1), dim3(1), 0, h->stream, bits);
    auto launch = [&](auto vw_tag) {
        constexpr int VW = decltype(vw_tag)::value;
        hipLaunchKernelGGL((herding_segment_sums<VW>), grid, dim3(256), lds, h->stream, z, perm, sh, lds_ids, segsum);
        // the prefix over segments: one thread per element for long rows, a workgroup scan per
        // element for short ones (many segments, few elements)
        if (sh.spw == 1)
            hipLaunchKernelGGL(herding_segment_offsets, dim3((unsigned)((d + 255) / 256)), dim3(256), 0, h->stream,
                               segsum, sh, zbar, start);
        else
            hipLaunchKernelGGL(herding_segment_offsets_scan, dim3((unsigned)d), dim3(256), 0, h->stream,
                               segsum, sh, zbar, start);
        hipLaunchKernelGGL((herding_prefix_max<VW>), grid, dim3(256), lds, h->stream, z, perm, sh, lds_ids, zbar,
                           start, bits);
    };
    if (vw == 4) launch(std::integral_constant<int, 4>{});
    else if (vw == 2) launch(std::integral_constant<int, 2>{});
    else launch(std::integral_constant<int, 1>{});
    HIP_TRY(h, hipGetLastError());
    return CDGRAB_OK;
}

int cdgrab_get_timing(cdgrab_handle *h, cdgrab_timing *out) {
    if (!h || !out) return CDGRAB_EINVAL;
    if (!h->have_timing) return fail(h, CDGRAB_EINVAL, "cdgrab_get_timing: no timed epoch on this handle");
    HIP_TRY(h, hipSetDevice(h->device));
    HIP_TRY(h, hipStreamSynchronize(h->stream));
    double sum[kIntervalKinds] = {0};
    for (size_t q = 0; q + 1 < h->marks.size(); ++q) {
        int kind = h->marks[q].kind_after;
        if (kind < 0) continue;
        float ms = 0.f;
        HIP_TRY(h, hipEventElapsedTime(&ms, h->marks[q].ev, h->marks[q + 1].ev));
        sum[kind] += ms;
    }
    cdgrab_timing t = h->last;
    t.generator_ms = sum[kGen];
    t.pass1_ms = sum[kPass1];
    t.reduce_ms = sum[kReduce];
    t.resolve_ms = sum[kResolve];
    t.pass2_ms = sum[kPass2];
    t.finish_ms = sum[kFinish];
    // with per-kernel marks the balancer interval is split into its four kernels
    t.balance_ms = sum[kBalance] + sum[kPass1] + sum[kReduce] + sum[kResolve] + sum[kPass2];
    h->last = t;
    *out = t;
    return CDGRAB_OK;
}

}  // extern "C"
