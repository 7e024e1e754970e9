// One group of instances of the fused scan kernel and its launcher.  Compiled once per
// (TRIM_INST_MODE: 0 kNN / 1 range, TRIM_INST_E: result entries per lane of the merging wave,
// TRIM_INST_BITS: 8- or 4-bit codes, TRIM_INST_LEAN: an 80-register small-k kNN instance), each
// time into an object of its own.
#include <atomic>

#include "trim_launch.h"

#if !defined(TRIM_INST_MODE) || !defined(TRIM_INST_E) || !defined(TRIM_INST_BITS)
#error "define TRIM_INST_MODE, TRIM_INST_E and TRIM_INST_BITS"
#endif
#ifndef TRIM_INST_LEAN
#define TRIM_INST_LEAN 0   // 1, 2: the 80-register instances of small-k kNN (see LeanKind)
#endif

#define TRIM_CAT_(a, b, c, d, e, f) a##b##c##d##e##f
#define TRIM_CAT(a, b, c, d, e, f) TRIM_CAT_(a, b, c, d, e, f)
#if TRIM_INST_MODE == 0 && TRIM_INST_LEAN == 2
#define TRIM_INST_NAME TRIM_CAT(launch_search_, knnleanlong, _e, TRIM_INST_E, _c, TRIM_INST_BITS)
#elif TRIM_INST_MODE == 0 && TRIM_INST_LEAN
#define TRIM_INST_NAME TRIM_CAT(launch_search_, knnlean, _e, TRIM_INST_E, _c, TRIM_INST_BITS)
#elif TRIM_INST_MODE == 0
#define TRIM_INST_NAME TRIM_CAT(launch_search_, knn, _e, TRIM_INST_E, _c, TRIM_INST_BITS)
#else
#define TRIM_INST_NAME TRIM_CAT(launch_search_, range, _e, TRIM_INST_E, _c, TRIM_INST_BITS)
#endif

namespace trim {

namespace {

constexpr int kMode = TRIM_INST_MODE;
constexpr int kE = TRIM_INST_E;
constexpr bool kFs = TRIM_INST_BITS == 4;
constexpr int kLean = TRIM_INST_LEAN;   // a LeanKind

template <bool ACCT>
int launch_instance(const SearchArgs &a, const Plan &pl, dim3 grid, hipStream_t st) {
    void (*fn)(const SearchArgs) = nullptr;
    switch (pl.vec) {
        case 4: fn = search_kernel<kMode, 4, kE, ACCT, kFs, kLean>; break;
        case 2: fn = search_kernel<kMode, 2, kE, ACCT, kFs, kLean>; break;
        default:
            // 4-bit codes come in rows of a multiple of 8 bytes: no 4-byte code loads there
            if constexpr (kFs) return TRIM_UNSUPPORTED_SHAPE;
            else fn = search_kernel<kMode, 1, kE, ACCT, kFs, kLean>;
            break;
    }
    // The kernel addresses its distance table with immediate offsets from LDS address 0, so it
    // must own the workgroup's LDS from the first byte: an instance that was built with static
    // LDS in front of the dynamic area is refused here instead of being launched.
    static std::atomic<int> lds_checked[3];   // per instance (ACCT) and code-load width
    std::atomic<int> &seen = lds_checked[pl.vec == 4 ? 2 : pl.vec == 2 ? 1 : 0];
    if (seen.load(std::memory_order_acquire) == 0) {
        hipFuncAttributes fa;
        HIP_TRY(hipFuncGetAttributes(&fa, reinterpret_cast<const void *>(fn)));
        seen.store(fa.sharedSizeBytes == 0 ? 1 : -1, std::memory_order_release);
    }
    if (seen.load(std::memory_order_acquire) < 0) return TRIM_INTERNAL;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)pl.lds));
    hipLaunchKernelGGL(fn, grid, dim3(pl.threads), pl.lds, st, a);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

}  // namespace

int TRIM_INST_NAME(const SearchArgs &a, const Plan &pl, dim3 grid, hipStream_t st) {
    return a.work ? launch_instance<true>(a, pl, grid, st) : launch_instance<false>(a, pl, grid, st);
}

}  // namespace trim
