// What the translation units of libtrim share on the host side: the launch plan of a search,
// the error bookkeeping, and the launchers of the search kernel's instances.  The instances are
// compiled in translation units of their own (trim_search_inst.hip, once per search mode,
// result-set width and code width), so that they build in parallel.
#pragma once

#include <hip/hip_runtime.h>

#include "../../include/trim.h"
#include "trim_search.h"

namespace trim {

// Table phases, block size and LDS layout of a search launch (made by make_plan).
struct Plan {
    int threads;
    int P, Mp, vec;
    size_t lds;
    uint32_t off_q, off_segp, off_segd, off_rest, off_seglb, off_spos, off_sd2, off_sidx, off_rd2, off_rid, off_ctl;
    uint32_t off_plb, off_cnt, off_wq;
    int span, wqcap, cruise, poss_cap, scap, rcap, bucket;
    int lean;    // a LeanKind; small-k kNN: launch an 80-register instance (six waves per SIMD, or short codes)
};

// Records a failed HIP call for trim_last_hip_error and returns TRIM_HIP_ERROR.
int hip_fail(hipError_t e);

#define HIP_TRY(expr)                                         \
    do {                                                      \
        hipError_t _e = (expr);                               \
        if (_e != hipSuccess) return ::trim::hip_fail(_e);    \
    } while (0)

// launch_search_<mode>_e<result entries per lane>_c<bits per code>: enqueue the matching
// instance of search_kernel (with or without the work counters, by SearchArgs::work).
#define TRIM_DECLARE_LAUNCH(name) \
    int name(const SearchArgs &a, const Plan &pl, dim3 grid, hipStream_t st)
TRIM_DECLARE_LAUNCH(launch_search_knnlean_e1_c8);
TRIM_DECLARE_LAUNCH(launch_search_knnlean_e1_c4);
TRIM_DECLARE_LAUNCH(launch_search_knnleanlong_e1_c8);
TRIM_DECLARE_LAUNCH(launch_search_knnleanlong_e1_c4);
TRIM_DECLARE_LAUNCH(launch_search_knn_e1_c8);
TRIM_DECLARE_LAUNCH(launch_search_knn_e2_c8);
TRIM_DECLARE_LAUNCH(launch_search_knn_e4_c8);
TRIM_DECLARE_LAUNCH(launch_search_knn_e16_c8);
TRIM_DECLARE_LAUNCH(launch_search_range_e1_c8);
TRIM_DECLARE_LAUNCH(launch_search_knn_e1_c4);
TRIM_DECLARE_LAUNCH(launch_search_knn_e2_c4);
TRIM_DECLARE_LAUNCH(launch_search_knn_e4_c4);
TRIM_DECLARE_LAUNCH(launch_search_knn_e16_c4);
TRIM_DECLARE_LAUNCH(launch_search_range_e1_c4);

}  // namespace trim
