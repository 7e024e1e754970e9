// C ABI of libtrim (see include/trim.h): argument checks, LDS carve-up, launches.
// No device allocation, no synchronisation, no state between calls.
#include "../../include/trim.h"

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdio>
#include <mutex>

#include "trim_aux.h"
#include "trim_launch.h"

// Scratch area of trim_search_range_static (see below): device memory inside the library's code
// object; every GPU the library runs on holds its own copy at its own address.
static __device__ __align__(256) unsigned char scratch[TRIM_STATIC_SCRATCH_BYTES];

namespace trim {
thread_local int g_last_hip_error = 0;
int hip_fail(hipError_t e) {
    g_last_hip_error = (int)e;
    return TRIM_HIP_ERROR;
}
}  // namespace trim

namespace {

using namespace trim;

static_assert(kWorkCounters == TRIM_WORK_COUNTERS && kWorkFirstPass == TRIM_WORK_FIRST_PASS &&
              kWorkSkipped == TRIM_WORK_SKIPPED && kWorkCodeBytes == TRIM_WORK_CODE_BYTES &&
              kWorkLookups == TRIM_WORK_LOOKUPS && kWorkRows == TRIM_WORK_ROWS &&
              kWorkFullCode == TRIM_WORK_FULL_CODE, "header and kernel disagree on the work counters");

constexpr size_t kLdsBytes = 160 * 1024;  // LDS per workgroup on gfx950


inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t up16(size_t x) { return (x + 15u) & ~size_t(15); }


// Decide table phases, block size and LDS layout for a search launch.
// cap = survivor-list capacity (max(batch,k) for kNN, round size for range).
// batch = candidates per threshold update (range: = cap).  The span of candidates bounded
// between two barriers on the span-by-span path is the largest multiple of batch up to the
// span target (at least one batch, at most kMaxBatchesPerSpan batches).  In kNN mode that
// path only serves the first stretch after the seed and the rare overflow of a cruise
// stretch, so its span is kept short and the LDS goes to residency instead: the layout is
// fitted to the smallest footprint tier (most workgroups per CU) that holds it.
constexpr int kSpanKnn = 1024;
constexpr int kSpanRange = 4096;
constexpr int kSpanLong = 4096;   // kNN span target when the table leaves one workgroup per CU anyway
constexpr int kMaxBatchesPerSpan = 1024;
constexpr int kPossMin = 512;    // smallest possibles list worth cruising with
constexpr int kPossMax = 2048;

// Block size and LDS bytes per workgroup for 4, 3, 2 and 1 workgroups per CU (LDS is handed
// out in 1280-byte granules).  Three 512-thread workgroups, or two of 768 threads, are 6 waves
// per SIMD: only the kernel instances built for that register budget (result_slots == 1) can use
// those tiers.  The second is for tables too long for three workgroups (M = 40..60): with 24
// instead of 16 waves per CU more rows and code blocks are in flight (5M x 384, M = 48: the
// scan went 5.06 -> 4.70 ms); it is kept to codes under 64 bytes, which the 80-register
// instance is the better one for anyway.
struct Tier { int threads; size_t lds; bool needs_6_waves; bool short_codes_only; };
constexpr Tier kTiers[] = {{256, 40960, false, false}, {512, 53760, true, false}, {768, 81920, true, true},
                           {512, 81920, false, false}, {1024, kLdsBytes, false, false}};

// One attempt: table phases P, a footprint tier, a span; need_poss: only layouts with a possibles
// list (a cruise) count.
bool fit_plan(int d, int M, int row_bytes, int nsegs, int cap, int batch, int k, bool range, int P,
              const Tier &tier, int span, bool need_poss, Plan *pl) {
    const int Mp = M / P;
    const int nbatch = span / batch;
    // cruise stretches (kNN): up to 61440 candidates (16-bit queue entries).  Their possibles
    // are counted per bucket of `bucket` candidates (a whole number of batches, at most 1024
    // buckets).
    int cruise = 61440 / batch * batch;
    if (range || cruise < 2 * span) cruise = 0;
    int bucket = batch;
    if (cruise / batch > 1024) bucket = batch * (((cruise + 1023) / 1024 + batch - 1) / batch);
    const int nbucket = cruise > 0 ? (cruise + bucket - 1) / bucket : 0;
    const int ncnt = nbucket > nbatch ? nbucket : nbatch;
    // (4-bit codes: 8 KB in front of the table for the pair table of the first filter pass)
    const size_t tab = (size_t)Mp * row_bytes + (row_bytes == (int)kByteRow<true> ? 8 * kC * 4 : 0);
    const bool can_cruise = cruise > 0 && P == 1;  // table phases need block-wide barriers
    if (need_poss && !can_cruise) return false;
    const int nwaves = tier.threads / 64;
    // a wave's share of a span is rounded up to 64; two queue arrays of 16-bit entries
    const int wqcap = ((span + nwaves - 1) / nwaves + 63) / 64 * 64;
    size_t wq_min = (size_t)2 * nwaves * wqcap * 2;
    if (can_cruise && wq_min < (size_t)nwaves * kRing * 4) wq_min = (size_t)nwaves * kRing * 4;
    const size_t rest = tab + up16((size_t)d * 4) + up16((size_t)(nsegs + 1) * 4) +
                        up16((size_t)nsegs * 4) + up16((size_t)(Mp / 4 + 1) * 4) +
                        up16((size_t)nsegs * 8) +
                        (range ? up16((size_t)cap * 4) : 0) +
                        up16((size_t)kWave * result_slots(k) * 4) * 2 + up16(sizeof(Ctl)) +
                        up16((size_t)ncnt * 4);
    // The possibles list of a cruise stretch takes what is left, largest first.  Its
    // capacity p also sizes the arrays of the stretch's replay: spos[] holds p entries,
    // and the queue area holds p exact distances and p bounds (queues are only live
    // while bounds are computed, distances and bounds only afterwards).
    static const int kPossTry[] = {kPossMax, 1536, 1024, 768, kPossMin, 0};
    for (int p : kPossTry) {
        if (p > 0 && !can_cruise) continue;
        if (p == 0 && need_poss) continue;
        const int scap = cap > p ? cap : p;
        size_t wq_bytes = wq_min;
        if (wq_bytes < (size_t)(scap + p) * 4) wq_bytes = (size_t)(scap + p) * 4;
        // a span that ends in a replay keeps up to min(scap, span) bounds behind the
        // scap exact distances
        const int span_poss = scap < span ? scap : span;
        if (!range && wq_bytes < (size_t)(scap + span_poss) * 4) wq_bytes = (size_t)(scap + span_poss) * 4;
        wq_bytes = up16(wq_bytes);
        size_t plb = up16((size_t)span * 4);             // bounds of a span / the possibles list
        if (plb < (size_t)p * 8) plb = (size_t)p * 8;
        const size_t total = rest + up16((size_t)scap * 4) + plb + wq_bytes;
        if (total > tier.lds) continue;
        pl->P = P;
        pl->Mp = Mp;
        pl->vec = (M % 16 == 0 && Mp % 16 == 0) ? 4 : (M % 8 == 0 && Mp % 8 == 0) ? 2 : 1;
        size_t off = tab;
        pl->off_q = (uint32_t)off;    off += up16((size_t)d * 4);
        pl->off_segp = (uint32_t)off; off += up16((size_t)(nsegs + 1) * 4);
        pl->off_segd = (uint32_t)off; off += up16((size_t)nsegs * 4);
        pl->off_rest = (uint32_t)off; off += up16((size_t)(Mp / 4 + 1) * 4);
        pl->off_seglb = (uint32_t)off; off += up16((size_t)nsegs * 8);
        pl->off_spos = (uint32_t)off; off += up16((size_t)scap * 4);
        pl->off_sidx = (uint32_t)off; if (range) off += up16((size_t)cap * 4);
        pl->off_rd2 = (uint32_t)off;  off += up16((size_t)kWave * result_slots(k) * 4);
        pl->off_rid = (uint32_t)off;  off += up16((size_t)kWave * result_slots(k) * 4);
        pl->off_ctl = (uint32_t)off;  off += up16(sizeof(Ctl));
        pl->off_plb = (uint32_t)off;  off += plb;
        pl->off_cnt = (uint32_t)off;  off += up16((size_t)ncnt * 4);
        pl->off_wq = (uint32_t)off;   off += wq_bytes;
        pl->off_sd2 = pl->off_wq;
        pl->span = span;
        pl->lds = off;
        pl->threads = tier.threads;
        // the 80-register instance: needed for three workgroups per CU, and the better one for short
        // codes in any case (the other's bulk rounds and deeper refine pipelines pay from 64 code bytes on)
        pl->lean = !(P == 1 && M <= 256 && (tier.needs_6_waves || M < 64)) ? kFullInstance
                   : d <= 128 ? kLeanShortRows : kLeanLongRows;
        pl->wqcap = wqcap;
        pl->cruise = p > 0 ? cruise : 0;
        pl->poss_cap = p;
        pl->scap = scap;
        pl->rcap = (int)(wq_bytes / 4) - scap;
        pl->bucket = bucket;
        return true;
    }
    return false;
}

// M counts code bytes; fs: 4-bit codes (two subspaces of 16 centroids per byte), else 8-bit.
bool make_plan(int d, int M, bool fs, int nseg, int cap, int batch, int k, bool range, Plan *pl) {
    if (d <= 0 || M <= 0 || d % 4 || M % 4) return false;
    if (fs ? (d % (2 * M) || M % 8 || d / (2 * M) > 64) : (d % M || d / M > 64)) return false;
    const int row_bytes = fs ? (int)kByteRow<true> : (int)kByteRow<false>;
    const int nsegs = nseg > 0 ? nseg : 1;
    int nbatch = (range ? kSpanRange : kSpanKnn) / batch;
    if (nbatch < 1) nbatch = 1;
    if (nbatch > kMaxBatchesPerSpan) nbatch = kMaxBatchesPerSpan;
    const int span = nbatch * batch;
    if (span > 65535) return false;
    constexpr int nt = (int)(sizeof(kTiers) / sizeof(kTiers[0]));
    for (int P = 1; P <= M / 4; ++P) {
        if (M % P || (M / P) % 4) continue;
        for (int t = 0; t < nt; ++t) {
            const Tier &tier = kTiers[t];
            if (tier.needs_6_waves && (range || result_slots(k) != 1)) continue;
            if (tier.short_codes_only && M >= 64) continue;
            // a short table would fit four small workgroups per CU (16 waves); the instance built
            // for six waves per SIMD does better as three 512-thread ones (24 waves)
            if (t == 0 && !range && result_slots(k) == 1 && fs) continue;
            if (t + 1 < nt) {
                // below the last tier a layout must leave room for a cruise when one is possible
                // at all (else the next tier is tried first)
                const bool cruise_possible = !range && P == 1 && 61440 / batch * batch >= 2 * span;
                if (fit_plan(d, M, row_bytes, nsegs, cap, batch, k, range, P, tier, span, cruise_possible, pl)) return true;
                continue;
            }
            // One workgroup per CU whatever the span: kNN takes the longest span that fits (fewer
            // barriers and more survivors per refine step on the span-by-span path), first among the
            // layouts that keep a possibles list, then among those without.
            if (!range) {
                for (int pass = 0; pass < 2; ++pass)
                    for (int target = kSpanLong; target > span; target -= 1024) {
                        const int longer = target / batch * batch;
                        if (longer <= span || longer / batch > kMaxBatchesPerSpan) continue;
                        if (fit_plan(d, M, row_bytes, nsegs, cap, batch, k, range, P, tier, longer, pass == 0, pl)) return true;
                    }
            }
            if (fit_plan(d, M, row_bytes, nsegs, cap, batch, k, range, P, tier, span, false, pl)) return true;
        }
    }
    return false;
}

// The search kernel's instances are compiled in translation units of their own
// (trim_search_inst.hip); this picks the one for a launch.
int launch_search(bool range, bool fs, const SearchArgs &a, const Plan &pl, dim3 grid, hipStream_t st) {
    if (range) return fs ? launch_search_range_e1_c4(a, pl, grid, st) : launch_search_range_e1_c8(a, pl, grid, st);
    // k decides how many result entries a lane of the merging wave holds (result_slots)
    switch (result_slots(a.k)) {
        case 1:
            if (pl.lean == kLeanLongRows) return fs ? launch_search_knnleanlong_e1_c4(a, pl, grid, st) : launch_search_knnleanlong_e1_c8(a, pl, grid, st);
            if (pl.lean) return fs ? launch_search_knnlean_e1_c4(a, pl, grid, st) : launch_search_knnlean_e1_c8(a, pl, grid, st);
            return fs ? launch_search_knn_e1_c4(a, pl, grid, st) : launch_search_knn_e1_c8(a, pl, grid, st);
        case 2: return fs ? launch_search_knn_e2_c4(a, pl, grid, st) : launch_search_knn_e2_c8(a, pl, grid, st);
        case 4: return fs ? launch_search_knn_e4_c4(a, pl, grid, st) : launch_search_knn_e4_c8(a, pl, grid, st);
        default: return fs ? launch_search_knn_e16_c4(a, pl, grid, st) : launch_search_knn_e16_c8(a, pl, grid, st);
    }
}

// 4-bit codes (two per byte, 16 centroids per subspace)?  Bytes of one stored code.
inline bool is_fs(const trim_index_view *ix) { return ix->code_bits == 4; }
inline int code_bytes(const trim_index_view *ix) { return is_fs(ix) ? ix->M / 2 : ix->M; }

int check_index(const trim_index_view *ix) {
    if (!ix) return TRIM_INVALID_ARG;
    if (ix->n < 0 || ix->n >= (int64_t(1) << 31)) return TRIM_INVALID_ARG;
    if (ix->d <= 0 || ix->M <= 0) return TRIM_INVALID_ARG;
    if (ix->code_bits != 0 && ix->code_bits != 8 && ix->code_bits != 4) return TRIM_INVALID_ARG;
    if (!(is_fs(ix) ? trim_fs_shape_supported(ix->d, ix->M) : trim_shape_supported(ix->d, ix->M)))
        return TRIM_UNSUPPORTED_SHAPE;
    if (ix->n > 0 && (!ix->base || !ix->codes || !ix->dlx)) return TRIM_INVALID_ARG;
    if (!aligned16(ix->base) || !aligned16(ix->codes) || !aligned16(ix->codebooks))
        return TRIM_INVALID_ARG;
    if (ix->scan_head && ((reinterpret_cast<uintptr_t>(ix->scan_head) & 3u) || code_bytes(ix) % 8))
        return TRIM_INVALID_ARG;
    if (ix->codes_tiled && (!aligned16(ix->codes_tiled) || code_bytes(ix) % 16)) return TRIM_INVALID_ARG;
    return TRIM_OK;
}

int check_cand(const trim_candidates *c) {
    if (!c) return TRIM_OK;
    if (c->nlist <= 0 || c->nprobe <= 0 || c->nprobe > TRIM_MAX_NPROBE) return TRIM_INVALID_ARG;
    if (!c->list_offsets || !c->probes) return TRIM_INVALID_ARG;
    if (c->list_bounds && !aligned16(c->list_bounds)) return TRIM_INVALID_ARG;
    return TRIM_OK;
}

void fill_common(SearchArgs &a, const trim_index_view *ix, const float *queries, const float *lut,
                 const trim_candidates *cand, float gamma, const trim_stats *stats,
                 uint32_t *mask, int64_t mask_words, const Plan &pl) {
    a.base = ix->base; a.codes = ix->codes; a.dlx = ix->dlx; a.ids = ix->ids;
    a.codebooks = ix->codebooks; a.head = static_cast<const uint32_t *>(ix->scan_head);
    a.codes_tiled = static_cast<const uint8_t *>(ix->codes_tiled); a.n = ix->n; a.d = ix->d;
    a.M = code_bytes(ix);       // the kernel counts code bytes
    a.dsub = ix->d / ix->M;     // length of one subspace's sub-vectors (8- or 4-bit codes alike)
    a.queries = queries; a.lut = lut; a.order = nullptr;
    a.list_offsets = cand ? cand->list_offsets : nullptr;
    a.probes = cand ? cand->probes : nullptr;
    a.nlist = cand ? cand->nlist : 0;
    a.nseg = cand ? cand->nprobe : 0;
    const int64_t hard = (int64_t(1) << 31) - 1 - TRIM_MAX_BATCH - 2048;
    int64_t mc = cand ? cand->max_candidates : ix->n;
    if (mc <= 0 || mc > hard) mc = hard;
    a.max_cand = (int32_t)mc;
    a.P = pl.P; a.Mp = pl.Mp;
    a.two_gamma = 2.0f * gamma;
    a.n_scanned = stats ? stats->n_scanned : nullptr;
    a.n_exact = stats ? stats->n_exact : nullptr;
    a.work = stats ? stats->work : nullptr;
    a.mask = mask; a.mask_words = mask_words;
    a.off_q = pl.off_q; a.off_segp = pl.off_segp; a.off_segd = pl.off_segd; a.off_rest = pl.off_rest;
    a.off_seglb = pl.off_seglb;
    a.list_bounds = cand ? static_cast<const uint8_t *>(cand->list_bounds) : nullptr;
    a.off_spos = pl.off_spos; a.off_sd2 = pl.off_sd2; a.off_sidx = pl.off_sidx;
    a.off_rd2 = pl.off_rd2; a.off_rid = pl.off_rid; a.off_ctl = pl.off_ctl;
    a.off_plb = pl.off_plb; a.off_cnt = pl.off_cnt; a.span = pl.span;
    a.off_wq = pl.off_wq; a.wqcap = pl.wqcap; a.cruise = pl.cruise; a.poss_cap = pl.poss_cap; a.scap = pl.scap; a.rcap = pl.rcap; a.bucket = pl.bucket;
    a.small_addr = ix->n < (int64_t(1) << 24) && ix->n * (int64_t)ix->M < (int64_t(1) << 32) &&
                   ix->M < (1 << 24);
    // Thresholds that count on the remaining table minima (and list summaries) rest on an error
    // bound of 2 * (table additions) * 2^-24 <= 3.1e-5 (see abandon_threshold): at most 256
    // additions per table sum, and the whole table resident.
    a.use_rest = pl.P == 1 && ix->M <= 256;
}

int fill_u32(uint32_t *p, size_t count, uint32_t v, hipStream_t st) {
    if (count == 0) return TRIM_OK;
    size_t blocks = (count + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, count, v);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

constexpr int kRangeRound = 2048;   // survivor-list capacity per round in range mode
constexpr int kRangeSplitTarget = 2048;  // aim for at least this many workgroups

int range_nsplit(int64_t nq, int64_t max_cand) {
    int64_t want = (kRangeSplitTarget + nq - 1) / (nq > 0 ? nq : 1);
    if (want < 1) want = 1;
    // at least 4096 candidates per chunk so that the table fill is amortised
    int64_t most = (max_cand + 4095) / 4096;
    if (most < 1) most = 1;
    if (want > most) want = most;
    if (want > 65535) want = 65535;
    return (int)want;
}

struct RangeLayout {
    int nsplit;
    int chunk;
    int64_t rmask_words;
    size_t off_counts, off_cbase, off_d2, total;
};

RangeLayout range_layout(int64_t nq, int64_t max_cand) {
    RangeLayout L;
    L.nsplit = range_nsplit(nq, max_cand);
    int64_t chunk = (max_cand + L.nsplit - 1) / L.nsplit;
    chunk = (chunk + 63) / 64 * 64;
    if (chunk < 64) chunk = 64;
    L.chunk = (int)chunk;
    L.rmask_words = (int64_t)L.nsplit * (chunk / 32);
    size_t off = (size_t)nq * L.rmask_words * 4;
    off = (off + 255) & ~size_t(255);
    L.off_counts = off; off += (size_t)nq * L.nsplit * 4;
    off = (off + 255) & ~size_t(255);
    L.off_cbase = off; off += (size_t)nq * L.nsplit * 8;
    off = (off + 255) & ~size_t(255);
    // the exact distance of every result waits here, at its scan-order number, for the pass that
    // writes the CSR arrays (one binary32 per candidate slot; only result slots are touched)
    L.off_d2 = off; off += (size_t)nq * L.rmask_words * 32 * 4;
    L.total = (off + 255) & ~size_t(255);
    return L;
}

// The scratch area lives from the first use of the library on a GPU until the process ends.
// In host code the array's name is only a handle: its device address is asked for once per
// device (hipGetSymbolAddress with that device current) and kept here; host code passes that
// address, never the name, to kernels.
constexpr size_t kScratchBytes = TRIM_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int scratch_for_current_device(void **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return TRIM_INVALID_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || (reinterpret_cast<uintptr_t>(p) & 255u)) return TRIM_HIP_ERROR;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return TRIM_OK;
}

// The range search behind both entry points: `workspace` is the caller's buffer or this
// device's copy of the static scratch area.
int range_search(const trim_index_view *index, const float *queries, int64_t nq,
                 const float *lut, const trim_candidates *cand, float radius, float gamma,
                 const int32_t *query_order, int64_t *out_offsets, int32_t *out_ids,
                 float *out_d2, int64_t capacity,
                 int64_t *required, const trim_stats *stats, uint32_t *survivor_mask,
                 int64_t mask_words, void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_index(index);
    if (rc) return rc;
    if ((rc = check_cand(cand))) return rc;
    if (nq < 0 || nq > TRIM_MAX_QUERIES || capacity < 0) return TRIM_INVALID_ARG;
    if (!(gamma >= 0.0f) || std::isinf(gamma) || !(radius >= 0.0f)) return TRIM_INVALID_ARG;
    if (!out_offsets) return TRIM_INVALID_ARG;
    if (capacity > 0 && (!out_ids || !out_d2)) return TRIM_INVALID_ARG;
    if (lut && !aligned16(lut)) return TRIM_INVALID_ARG;
    if (!lut && !index->codebooks) return TRIM_INVALID_ARG;
    if (survivor_mask && mask_words <= 0) return TRIM_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (nq == 0) {
        if ((rc = fill_u32(reinterpret_cast<uint32_t *>(out_offsets), 2, 0u, st))) return rc;
        if (required && (rc = fill_u32(reinterpret_cast<uint32_t *>(required), 2, 0u, st))) return rc;
        return TRIM_OK;
    }
    if (!queries) return TRIM_INVALID_ARG;
    int64_t max_cand = cand ? cand->max_candidates : index->n;
    if (cand && max_cand <= 0) return TRIM_INVALID_ARG;  // needed to size the masks
    const RangeLayout L = range_layout(nq, max_cand);
    if (!workspace || workspace_bytes < L.total || (reinterpret_cast<uintptr_t>(workspace) & 255u))
        return TRIM_WORKSPACE;
    Plan pl;
    if (!make_plan(index->d, code_bytes(index), is_fs(index), cand ? cand->nprobe : 0, kRangeRound, kRangeRound, 1, true, &pl))
        return TRIM_UNSUPPORTED_SHAPE;

    unsigned char *ws = static_cast<unsigned char *>(workspace);
    uint32_t *rmask = reinterpret_cast<uint32_t *>(ws);
    int32_t *counts = reinterpret_cast<int32_t *>(ws + L.off_counts);
    int64_t *cbase = reinterpret_cast<int64_t *>(ws + L.off_cbase);
    float *rd2 = reinterpret_cast<float *>(ws + L.off_d2);

    if ((rc = fill_u32(rmask, (size_t)nq * L.rmask_words, 0u, st))) return rc;
    if (survivor_mask && (rc = fill_u32(survivor_mask, (size_t)nq * mask_words, 0u, st))) return rc;
    if (stats && stats->n_exact && (rc = fill_u32(reinterpret_cast<uint32_t *>(stats->n_exact), (size_t)nq, 0u, st)))
        return rc;
    if (stats && stats->work && (rc = fill_u32(stats->work, (size_t)nq * kWorkCounters, 0u, st))) return rc;

    SearchArgs a{};
    fill_common(a, index, queries, lut, cand, gamma, stats, survivor_mask, mask_words, pl);
    a.k = 1; a.batch = kRangeRound;
    a.radius2 = radius * radius;
    a.chunk = L.chunk; a.nsplit = L.nsplit;
    a.result_mask = rmask; a.rmask_words = L.rmask_words; a.chunk_counts = counts;
    a.result_d2 = rd2;
    a.order = query_order;
    // a query that the order does not name is not searched: its counts must read zero
    if (query_order && (rc = fill_u32(reinterpret_cast<uint32_t *>(counts), (size_t)nq * L.nsplit, 0u, st))) return rc;
    if (a.max_cand > max_cand) a.max_cand = (int32_t)max_cand;

    RangeFillArgs f{};
    f.base = index->base; f.ids = index->ids; f.queries = queries;
    f.list_offsets = a.list_offsets; f.probes = a.probes; f.n = index->n; f.d = index->d;
    f.nlist = a.nlist; f.nseg = a.nseg; f.max_cand = a.max_cand; f.chunk = L.chunk;
    f.nsplit = L.nsplit; f.result_mask = rmask; f.rmask_words = L.rmask_words; f.result_d2 = rd2;
    f.chunk_base = cbase; f.out_ids = out_ids; f.out_d2 = out_d2; f.capacity = capacity;
    const int nsegs = a.nseg > 0 ? a.nseg : 1;
    size_t off = 0;
    f.off_q = (uint32_t)off;    off += up16((size_t)index->d * 4);
    f.off_segp = (uint32_t)off; off += up16((size_t)(nsegs + 1) * 4);
    f.off_segd = (uint32_t)off; off += up16((size_t)nsegs * 4);
    f.off_list = (uint32_t)off; off += 2048 * 4;
    const size_t fill_lds = off;

    a.nq = nq;
    const int64_t slots = (nq + kXcds - 1) / kXcds * kXcds;
    if (slots * pl.threads >= (int64_t(1) << 32)) return TRIM_INVALID_ARG;  // threads per launch
    if ((rc = launch_search(true, is_fs(index), a, pl, dim3((unsigned)slots, (unsigned)L.nsplit), st))) return rc;
    hipLaunchKernelGGL(range_offsets_kernel, dim3(1), dim3(1024), 0, st, counts, nq, L.nsplit, cbase,
                       out_offsets, required);
    HIP_TRY(hipGetLastError());
    if (capacity > 0) {
        HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(range_fill_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)fill_lds));
        hipLaunchKernelGGL(range_fill_kernel, dim3((unsigned)nq, (unsigned)L.nsplit), dim3(256), fill_lds,
                           st, f);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

}  // namespace

extern "C" {

int trim_shape_supported(int32_t d, int32_t M) {
    Plan pl;
    if (d <= 0 || M <= 0 || d % M) return 0;
    return make_plan(d, M, false, 64, 2048, 2048, 10, true, &pl) ? 1 : 0;
}

int trim_fs_shape_supported(int32_t d, int32_t M) {
    Plan pl;
    if (d <= 0 || M <= 0 || M % 2 || d % M) return 0;
    return make_plan(d, M / 2, true, 64, 2048, 2048, 10, true, &pl) ? 1 : 0;
}

int trim_encode(const float *base, int64_t n, int32_t d, const float *codebooks, int32_t M,
                uint8_t *codes_out, float *dlx_out, void *stream) {
    if (n < 0 || d <= 0 || M <= 0) return TRIM_INVALID_ARG;
    if (d % M || M % 4) return TRIM_UNSUPPORTED_SHAPE;
    const int dsub = d / M;
    if ((size_t)kC * dsub * 4 > 64 * 1024) return TRIM_UNSUPPORTED_SHAPE;
    if (n == 0) return TRIM_OK;
    if (!base || !codebooks || !codes_out || !dlx_out) return TRIM_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(codes_out) & 3u) return TRIM_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)((n + 255) / 256)), block(256);
    const size_t lds = (size_t)kC * dsub * 4;
    if (dsub == 4)
        hipLaunchKernelGGL(encode_kernel<4>, grid, block, lds, st, base, n, d, codebooks, M, dsub, codes_out, dlx_out);
    else if (dsub == 8)
        hipLaunchKernelGGL(encode_kernel<8>, grid, block, lds, st, base, n, d, codebooks, M, dsub, codes_out, dlx_out);
    else
        hipLaunchKernelGGL(encode_kernel<0>, grid, block, lds, st, base, n, d, codebooks, M, dsub, codes_out, dlx_out);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

size_t trim_list_bounds_bytes(int32_t nlist, int32_t M) {
    if (nlist <= 0 || M <= 0) return 0;
    return (size_t)nlist * list_record_bytes(M);
}

int trim_pack_list_bounds(const trim_index_view *index, const int64_t *list_offsets, int32_t nlist,
                          void *out, void *stream) {
    const int rc = check_index(index);
    if (rc != TRIM_OK) return rc;
    if (nlist <= 0 || !list_offsets || !out || !aligned16(out)) return TRIM_INVALID_ARG;
    const int Mb = code_bytes(index);   // summaries are kept per code byte
    hipLaunchKernelGGL(list_bounds_kernel, dim3((unsigned)nlist), dim3(256), (size_t)Mb * 32,
                       static_cast<hipStream_t>(stream), index->codes, index->dlx, index->n, Mb,
                       list_offsets, static_cast<uint8_t *>(out));
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_ceiling_stream_read(const void *buf, size_t bytes, int32_t blocks, uint32_t *sink,
                             void *stream) {
    if (!buf || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(buf) & 15u)) return TRIM_INVALID_ARG;
    if (blocks < 1 || blocks > TRIM_CEILING_MAX_BLOCKS) return TRIM_INVALID_ARG;
    hipLaunchKernelGGL(stream_read_kernel, dim3(blocks), dim3(512), 0,
                       static_cast<hipStream_t>(stream), static_cast<const uint4 *>(buf), bytes / 16,
                       sink);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_ceiling_lds_gather(int32_t blocks, int32_t iters, int32_t entry_floats, uint32_t seed,
                            float *sink, void *stream) {
    if (!sink || iters < 1 || iters > (1 << 20)) return TRIM_INVALID_ARG;
    if (blocks < 1 || blocks > TRIM_CEILING_MAX_BLOCKS) return TRIM_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (entry_floats) {
        case 1:
            hipLaunchKernelGGL(lds_gather_kernel, dim3(blocks), dim3(512), 32 * kC * 4, st, iters, seed, sink);
            break;
        case 2:
            hipLaunchKernelGGL(lds_gather_wide_kernel<2>, dim3(blocks), dim3(512), 8 * kC * 8, st, iters, seed, sink);
            break;
        case 4:
            hipLaunchKernelGGL(lds_gather_wide_kernel<4>, dim3(blocks), dim3(512), 8 * kC * 16, st, iters, seed, sink);
            break;
        case 16:
            hipLaunchKernelGGL(lds_gather_fs_kernel, dim3(blocks), dim3(512), 64 * kC4 * 4, st, iters, seed, sink);
            break;
        default:
            return TRIM_INVALID_ARG;
    }
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_pack_scan_head(const uint8_t *codes, const float *dlx, int64_t n, int32_t M,
                        void *head_out, void *stream) {
    if (n < 0 || n >= (int64_t(1) << 31) || M <= 0) return TRIM_INVALID_ARG;
    if (M % 8) return TRIM_UNSUPPORTED_SHAPE;
    if (n == 0) return TRIM_OK;
    if (!codes || !dlx || !head_out) return TRIM_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(codes) & 7u) || (reinterpret_cast<uintptr_t>(head_out) & 3u))
        return TRIM_INVALID_ARG;
    size_t blocks = ((size_t)n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(pack_scan_head_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), codes, dlx, n, M,
                       static_cast<uint32_t *>(head_out));
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_train_pq(const float *train, int64_t ns, int32_t d, int32_t M, int32_t iters,
                  const int32_t *init_rows, float *codebooks_out, uint8_t *codes_ws, float *dlx_ws,
                  void *stream) {
    if (ns <= 0 || d <= 0 || M <= 0 || iters < 0) return TRIM_INVALID_ARG;
    if (d % M || M % 4 || M > 65535) return TRIM_UNSUPPORTED_SHAPE;
    if (!train || !init_rows || !codebooks_out || !codes_ws || !dlx_ws) return TRIM_INVALID_ARG;
    const int dsub = d / M;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int per = kC * dsub;  // centroid coordinates per subspace
    for (int j = 0; j < M; ++j) {
        hipLaunchKernelGGL(kmeans_init_kernel, dim3((per + 255) / 256), dim3(256), 0, st, train, ns,
                           (int64_t)d, j * dsub, dsub, init_rows, kC, codebooks_out + (size_t)j * per);
    }
    HIP_TRY(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        const int rc = trim_encode(train, ns, d, codebooks_out, M, codes_ws, dlx_ws, stream);
        if (rc) return rc;
        hipLaunchKernelGGL(kmeans_update_kernel<1>, dim3((per + 255) / 256, M), dim3(256), 0, st, train,
                           ns, (int64_t)d, 0, dsub, static_cast<const void *>(codes_ws), (int64_t)M, kC,
                           codebooks_out);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_train_ivf(const float *train, int64_t ns, int32_t d, int32_t nlist, int32_t iters,
                   const int32_t *init_rows, float *centroids_out, int32_t *assign_ws, void *stream) {
    if (ns <= 0 || d <= 0 || nlist <= 0 || iters < 0) return TRIM_INVALID_ARG;
    if (d % 4) return TRIM_UNSUPPORTED_SHAPE;
    if (!train || !init_rows || !centroids_out || !assign_ws) return TRIM_INVALID_ARG;
    if ((int64_t)nlist * d > 0x7fffffff) return TRIM_UNSUPPORTED_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int per = nlist * d;
    hipLaunchKernelGGL(kmeans_init_kernel, dim3((per + 255) / 256), dim3(256), 0, st, train, ns,
                       (int64_t)d, 0, d, init_rows, nlist, centroids_out);
    HIP_TRY(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        const int rc = trim_ivf_probe(train, ns, d, centroids_out, nlist, 1, assign_ws, stream);
        if (rc) return rc;
        hipLaunchKernelGGL(kmeans_update_kernel<4>, dim3((per + 255) / 256), dim3(256), 0, st, train, ns,
                           (int64_t)d, 0, d, static_cast<const void *>(assign_ws), (int64_t)1, nlist,
                           centroids_out);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_estimate_gamma(const trim_index_view *index, const int32_t *sample_rows, int32_t S,
                        const float *sample_queries, int32_t Q, float p, float *gamma_x_out,
                        float *gamma_out, void *stream) {
    if (!index || index->n <= 0 || index->d <= 0 || index->M <= 0) return TRIM_INVALID_ARG;
    if (index->code_bits == 4) return TRIM_UNSUPPORTED_SHAPE;   // 8-bit landmark codes only
    if (index->d % 4 || index->d % index->M) return TRIM_UNSUPPORTED_SHAPE;
    if (S <= 0 || Q <= 0 || !(p >= 0.0f && p <= 1.0f)) return TRIM_INVALID_ARG;
    if (Q > 16384) return TRIM_UNSUPPORTED_SHAPE;
    if (!index->base || !index->codes || !index->codebooks || !sample_rows || !sample_queries || !gamma_out)
        return TRIM_INVALID_ARG;
    if (!aligned16(sample_queries)) return TRIM_INVALID_ARG;
    int npow2 = 1;
    while (npow2 < Q) npow2 <<= 1;
    const size_t lds = ((size_t)2 * index->d + npow2) * 4;
    if (lds + 1024 > kLdsBytes) return TRIM_UNSUPPORTED_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = fill_u32(reinterpret_cast<uint32_t *>(gamma_out), 1, 0x7f800000u, st);  // +inf
    if (rc) return rc;
    GammaArgs a{};
    a.base = index->base; a.codes = index->codes; a.codebooks = index->codebooks;
    a.rows = sample_rows; a.queries = sample_queries; a.n = index->n; a.d = index->d; a.M = index->M;
    a.Q = Q; a.npow2 = npow2;
    long m = (long)std::ceil((double)p * (double)Q);
    if (m < 1) m = 1;
    if (m > Q) m = Q;
    a.rank = (int32_t)(Q - m);
    a.gamma_x = gamma_x_out; a.gamma_bits = reinterpret_cast<uint32_t *>(gamma_out);
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(gamma_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(gamma_kernel, dim3((unsigned)S), dim3(256), lds, st, a);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_estimate_gamma_normal(const trim_index_view *index, const int32_t *sample_rows, int32_t S,
                               const float *normals, int32_t Q, float p, int32_t grid, double *work,
                               float *gamma_x_out, float *gamma_out, void *stream) {
    if (!index || index->n <= 0 || index->d <= 0 || index->M <= 0) return TRIM_INVALID_ARG;
    if (index->code_bits == 4) return TRIM_UNSUPPORTED_SHAPE;   // 8-bit landmark codes only
    if (index->d % index->M || index->d < 3) return TRIM_UNSUPPORTED_SHAPE;
    if (S <= 0 || Q <= 0 || grid < 2 || !(p >= 0.0f && p <= 1.0f)) return TRIM_INVALID_ARG;
    if (Q > 16384 || grid > (1 << 24)) return TRIM_UNSUPPORTED_SHAPE;
    if (!index->base || !index->codes || !index->codebooks || !sample_rows || !normals || !work || !gamma_out)
        return TRIM_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(work) & 7u) return TRIM_INVALID_ARG;
    int npow2 = 1;
    while (npow2 < Q) npow2 <<= 1;
    const size_t lds = (size_t)npow2 * 8;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int rc = fill_u32(reinterpret_cast<uint32_t *>(gamma_out), 1, 0x7f800000u, st);  // +inf
    if (rc) return rc;
    hipLaunchKernelGGL(normal_triples_kernel, dim3((unsigned)((Q + 255) / 256)), dim3(256), 0, st, normals,
                       (int64_t)Q, index->d, work);
    HIP_TRY(hipGetLastError());
    GammaNormalArgs a{};
    a.base = index->base; a.codes = index->codes; a.codebooks = index->codebooks; a.rows = sample_rows;
    a.triples = work; a.n = index->n; a.d = index->d; a.M = index->M; a.Q = Q; a.npow2 = npow2;
    a.grid = grid; a.one_minus_p = 1.0 - (double)p;
    a.gamma_x = gamma_x_out; a.gamma_bits = reinterpret_cast<uint32_t *>(gamma_out);
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(gamma_normal_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(gamma_normal_kernel, dim3((unsigned)S), dim3(256), lds, st, a);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

size_t trim_codes_tiled_bytes(int64_t n, int32_t M) {
    if (n <= 0 || M <= 0) return 0;
    return (size_t)((n + 63) / 64) * 64 * (size_t)M;
}

int trim_pack_codes_tiled(const uint8_t *codes, int64_t n, int32_t M, void *tiled_out, void *stream) {
    if (n < 0 || n >= (int64_t(1) << 31) || M <= 0) return TRIM_INVALID_ARG;
    if (M % 16) return TRIM_UNSUPPORTED_SHAPE;
    if (n == 0) return TRIM_OK;
    if (!codes || !tiled_out || !aligned16(codes) || !aligned16(tiled_out)) return TRIM_INVALID_ARG;
    const size_t total = trim_codes_tiled_bytes(n, M) / 16;
    size_t blocks = (total + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(pack_codes_tiled_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), codes, n, M, static_cast<uint4 *>(tiled_out));
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_fs_encode(const float *base, int64_t n, int32_t d, const float *codebooks, int32_t M,
                   uint8_t *codes_out, float *dlx_out, void *stream) {
    if (n < 0 || d <= 0 || M <= 0) return TRIM_INVALID_ARG;
    if (d % M || M % 2) return TRIM_UNSUPPORTED_SHAPE;
    const int dsub = d / M;
    if ((size_t)2 * kC4 * dsub * 4 > 64 * 1024) return TRIM_UNSUPPORTED_SHAPE;
    if (n == 0) return TRIM_OK;
    if (!base || !codebooks || !codes_out || !dlx_out) return TRIM_INVALID_ARG;
    hipLaunchKernelGGL(encode_fs_kernel<true>, dim3((unsigned)((n + 255) / 256)), dim3(256),
                       (size_t)2 * kC4 * dsub * 4, static_cast<hipStream_t>(stream), base, n, d, codebooks,
                       M, dsub, codes_out, dlx_out);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

int trim_fs_train_pq(const float *train, int64_t ns, int32_t d, int32_t M, int32_t iters,
                     const int32_t *init_rows, float *codebooks_out, uint8_t *assign_ws, void *stream) {
    if (ns <= 0 || d <= 0 || M <= 0 || iters < 0) return TRIM_INVALID_ARG;
    if (d % M || M % 2 || M > 65535) return TRIM_UNSUPPORTED_SHAPE;
    if (!train || !init_rows || !codebooks_out || !assign_ws) return TRIM_INVALID_ARG;
    const int dsub = d / M;
    if ((size_t)2 * kC4 * dsub * 4 > 64 * 1024) return TRIM_UNSUPPORTED_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int per = kC4 * dsub;  // centroid coordinates per subspace
    for (int j = 0; j < M; ++j) {
        hipLaunchKernelGGL(kmeans_init_kernel, dim3((per + 255) / 256), dim3(256), 0, st, train, ns,
                           (int64_t)d, j * dsub, dsub, init_rows, kC4, codebooks_out + (size_t)j * per);
    }
    HIP_TRY(hipGetLastError());
    for (int it = 0; it < iters; ++it) {
        hipLaunchKernelGGL(encode_fs_kernel<false>, dim3((unsigned)((ns + 255) / 256)), dim3(256),
                           (size_t)2 * kC4 * dsub * 4, st, train, ns, d, codebooks_out, M, dsub, assign_ws,
                           static_cast<float *>(nullptr));
        HIP_TRY(hipGetLastError());
        hipLaunchKernelGGL(kmeans_update_kernel<1>, dim3((per + 255) / 256, M), dim3(256), 0, st, train,
                           ns, (int64_t)d, 0, dsub, static_cast<const void *>(assign_ws), (int64_t)M, kC4,
                           codebooks_out);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_fs_build_lut(const float *queries, int64_t nq, int32_t d, const float *codebooks, int32_t M,
                      float *lut_out, void *stream) {
    if (nq < 0 || d <= 0 || M <= 0) return TRIM_INVALID_ARG;
    if (d % M || M % 2) return TRIM_UNSUPPORTED_SHAPE;
    if (nq == 0) return TRIM_OK;
    if (!queries || !codebooks || !lut_out) return TRIM_INVALID_ARG;
    const int bper = 64;   // code bytes per block: 2048 entries
    for (int64_t q0 = 0; q0 < nq; q0 += 65535) {
        const int64_t cnt = nq - q0 < 65535 ? nq - q0 : 65535;
        hipLaunchKernelGGL(lut_fs_kernel, dim3((M / 2 + bper - 1) / bper, (unsigned)cnt), dim3(256),
                           (size_t)d * 4, static_cast<hipStream_t>(stream), queries + (size_t)q0 * d, d,
                           codebooks, M, d / M, bper, lut_out + (size_t)q0 * M * kC4);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_build_lut(const float *queries, int64_t nq, int32_t d, const float *codebooks, int32_t M,
                   float *lut_out, int32_t mfma, void *stream) {
    if (nq < 0 || d <= 0 || M <= 0) return TRIM_INVALID_ARG;
    if (d % M) return TRIM_UNSUPPORTED_SHAPE;
    const int dsub = d / M;
    if (mfma && dsub != 4 && dsub != 8) return TRIM_UNSUPPORTED_SHAPE;
    if (nq == 0) return TRIM_OK;
    if (!queries || !codebooks || !lut_out) return TRIM_INVALID_ARG;
    if (!aligned16(codebooks) || nq > 0x7fffffff) return TRIM_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (mfma) {
        const dim3 grid((unsigned)((nq + 15) / 16), (unsigned)((M + 3) / 4));
        if (grid.y > 65535) return TRIM_UNSUPPORTED_SHAPE;
        if (dsub == 4)
            hipLaunchKernelGGL(lut_mfma_kernel<4>, grid, dim3(256), 0, st, queries, nq, d, codebooks, M, lut_out);
        else
            hipLaunchKernelGGL(lut_mfma_kernel<8>, grid, dim3(256), 0, st, queries, nq, d, codebooks, M, lut_out);
        HIP_TRY(hipGetLastError());
        return TRIM_OK;
    }
    const int jper = 8;
    // grid.y is limited to 65535: walk the queries in slabs
    for (int64_t q0 = 0; q0 < nq; q0 += 65535) {
        const int64_t cnt = nq - q0 < 65535 ? nq - q0 : 65535;
        hipLaunchKernelGGL(lut_kernel, dim3((M + jper - 1) / jper, (unsigned)cnt), dim3(256),
                           (size_t)d * 4, st, queries + (size_t)q0 * d, d, codebooks, M, dsub, jper,
                           lut_out + (size_t)q0 * M * kC);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_search_knn(const trim_index_view *index, const float *queries, int64_t nq,
                    const float *lut, const trim_candidates *cand, int32_t k, float gamma,
                    int32_t batch, const int32_t *query_order,
                    int32_t *out_ids, float *out_d2,
                    const trim_stats *stats, uint32_t *survivor_mask, int64_t mask_words,
                    void *stream) {
    int rc = check_index(index);
    if (rc) return rc;
    if ((rc = check_cand(cand))) return rc;
    if (nq < 0 || nq > TRIM_MAX_QUERIES || k < 1 || k > TRIM_MAX_K || batch < 1 || batch > TRIM_MAX_BATCH)
        return TRIM_INVALID_ARG;
    if (!(gamma >= 0.0f) || std::isinf(gamma)) return TRIM_INVALID_ARG;
    if (nq == 0) return TRIM_OK;
    if (!queries || !out_ids || !out_d2) return TRIM_INVALID_ARG;
    if (!lut && !index->codebooks) return TRIM_INVALID_ARG;
    if (lut && !aligned16(lut)) return TRIM_INVALID_ARG;
    if (survivor_mask && mask_words <= 0) return TRIM_INVALID_ARG;
    Plan pl;
    const int cap = batch > k ? batch : k;
    if (!make_plan(index->d, code_bytes(index), is_fs(index), cand ? cand->nprobe : 0, cap, batch, k, false, &pl))
        return TRIM_UNSUPPORTED_SHAPE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (survivor_mask && (rc = fill_u32(survivor_mask, (size_t)nq * mask_words, 0u, st))) return rc;
    SearchArgs a{};
    fill_common(a, index, queries, lut, cand, gamma, stats, survivor_mask, mask_words, pl);
    a.k = k; a.batch = batch; a.radius2 = 0.0f;
    a.out_ids = out_ids; a.out_d2 = out_d2;
    a.chunk = 0; a.nsplit = 1;
    a.nq = nq; a.order = query_order;
    const int64_t slots = (nq + kXcds - 1) / kXcds * kXcds;
    if (slots * pl.threads >= (int64_t(1) << 32)) return TRIM_INVALID_ARG;  // threads per launch
    if ((rc = launch_search(false, is_fs(index), a, pl, dim3((unsigned)slots, 1), st))) return rc;
    return TRIM_OK;
}

size_t trim_range_workspace_bytes(int64_t nq, int64_t max_candidates) {
    if (nq <= 0 || max_candidates < 0) return 256;
    return range_layout(nq, max_candidates).total;
}

int trim_search_range(const trim_index_view *index, const float *queries, int64_t nq,
                      const float *lut, const trim_candidates *cand, float radius, float gamma,
                      const int32_t *query_order, int64_t *out_offsets, int32_t *out_ids,
                      float *out_d2, int64_t capacity,
                      int64_t *required, const trim_stats *stats, uint32_t *survivor_mask,
                      int64_t mask_words, void *workspace, size_t workspace_bytes, void *stream) {
    return range_search(index, queries, nq, lut, cand, radius, gamma, query_order, out_offsets, out_ids, out_d2,
                        capacity, required, stats, survivor_mask, mask_words, workspace,
                        workspace_bytes, stream);
}

int trim_search_range_static(const trim_index_view *index, const float *queries, int64_t nq,
                             const float *lut, const trim_candidates *cand, float radius, float gamma,
                             const int32_t *query_order, int64_t *out_offsets, int32_t *out_ids,
                             float *out_d2, int64_t capacity,
                             int64_t *required, const trim_stats *stats, uint32_t *survivor_mask,
                             int64_t mask_words, void *stream) {
    // refuse what does not fit before anything else: no device call has been made yet
    if (nq > 0 && index) {
        const int64_t max_cand = cand ? cand->max_candidates : index->n;
        if (max_cand >= 0 && nq <= TRIM_MAX_QUERIES && range_layout(nq, max_cand).total > kScratchBytes)
            return TRIM_WORKSPACE;
    }
    void *ws = nullptr;
    const int rc = scratch_for_current_device(&ws);
    if (rc) return rc;
    return range_search(index, queries, nq, lut, cand, radius, gamma, query_order, out_offsets, out_ids, out_d2,
                        capacity, required, stats, survivor_mask, mask_words, ws, kScratchBytes, stream);
}

size_t trim_static_scratch_bytes(void) { return kScratchBytes; }

int trim_ivf_probe(const float *queries, int64_t nq, int32_t d, const float *centroids,
                   int32_t nlist, int32_t nprobe, int32_t *probes_out, void *stream) {
    if (nq < 0 || d <= 0 || nlist <= 0 || nprobe <= 0) return TRIM_INVALID_ARG;
    if (nprobe > nlist || nprobe > TRIM_MAX_NPROBE) return TRIM_INVALID_ARG;
    if (d % 4) return TRIM_UNSUPPORTED_SHAPE;
    int npow2 = 1;
    while (npow2 < nlist) npow2 <<= 1;
    // queries per workgroup: 8 (one per wave for the selection), fewer if their key arrays do not
    // fit half of the LDS (so that two workgroups share a CU)
    int qt = 8;
    while (qt > 1 && (size_t)qt * ((size_t)npow2 * 8 + (size_t)d * 4) > kLdsBytes / 2) qt >>= 1;
    const size_t lds = (size_t)qt * ((size_t)npow2 * 8 + (size_t)d * 4);
    if (lds > kLdsBytes) return TRIM_UNSUPPORTED_SHAPE;
    if (nq == 0) return TRIM_OK;
    if (!queries || !centroids || !probes_out || !aligned16(centroids)) return TRIM_INVALID_ARG;
    if (nq > 0x7fffffff) return TRIM_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    void (*fn)(const float *, int64_t, int, const float *, int, int, int, int32_t *) =
        qt == 8 ? ivf_probe_kernel<8> : qt == 4 ? ivf_probe_kernel<4> : qt == 2 ? ivf_probe_kernel<2> : ivf_probe_kernel<1>;
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(fn),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    // a launch holds fewer than 2^32 threads: walk the queries in slabs
    const int64_t slab = (int64_t)qt * (1 << 22);
    for (int64_t q0 = 0; q0 < nq; q0 += slab) {
        const int64_t cnt = nq - q0 < slab ? nq - q0 : slab;
        hipLaunchKernelGGL(fn, dim3((unsigned)((cnt + qt - 1) / qt)), dim3(512), lds, st,
                           queries + (size_t)q0 * d, cnt, d, centroids, nlist, npow2, nprobe,
                           probes_out + (size_t)q0 * nprobe);
        HIP_TRY(hipGetLastError());
    }
    return TRIM_OK;
}

int trim_query_order(const int32_t *probes, int64_t nq, int32_t nprobe, int32_t nlist,
                     int32_t *order_out, void *stream) {
    if (nq < 0 || nq > 0x7fffffff - 8 || nprobe <= 0 || nlist <= 0) return TRIM_INVALID_ARG;
    if (nq == 0) return TRIM_OK;
    if (!probes || !order_out) return TRIM_INVALID_ARG;
    const int nbucket = nlist < 32768 ? nlist : 32768;
    const size_t lds = (size_t)nbucket * 4;
    hipStream_t st = static_cast<hipStream_t>(stream);
    HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(query_order_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    hipLaunchKernelGGL(query_order_kernel, dim3(1), dim3(1024), lds, st, probes, nq, nprobe, nbucket,
                       order_out);
    HIP_TRY(hipGetLastError());
    return TRIM_OK;
}

const char *trim_strerror(int status) {
    switch (status) {
        case TRIM_OK: return "ok";
        case TRIM_INVALID_ARG: return "invalid argument";
        case TRIM_UNSUPPORTED_SHAPE: return "unsupported shape (d, M) for this build";
        case TRIM_WORKSPACE: return "workspace missing, misaligned or too small (trim_search_range_static: the search needs more than TRIM_STATIC_SCRATCH_BYTES)";
        case TRIM_HIP_ERROR: return "HIP call failed (see trim_last_hip_error)";
        case TRIM_INTERNAL: return "the library was built wrongly (a search kernel carries static LDS)";
        default: return "unknown status";
    }
}

int trim_last_hip_error(void) { return trim::g_last_hip_error; }

const char *trim_version(void) { return "0.1"; }

}  // extern "C"
