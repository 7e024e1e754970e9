// The fused filter-then-refine scan (Section 4.2) as one workgroup per query, resident for the whole scan of it
// (kNN) or per (query, candidate chunk) (range).  Everything a query needs between
// batches (distance table, query, result set R, threshold tau, survivor list) stays in
// LDS; the only HBM traffic is the streamed codes + landmark distances, the raw rows of
// survivors, and the results.
#pragma once

#include "trim_device.h"

namespace trim {

enum Mode { kKnn = 0, kRange = 1 };
// The distance table sits at the very start of the workgroup's LDS (the search kernel has no
// static LDS), which lets table gathers use an immediate row offset.  The launch wrapper checks
// the kernel's static LDS size (it must be 0) before the first launch of an instance, and the
// build refuses a library in which it is not.
constexpr uint32_t kTabLds = 0;
// With 4-bit codes the first 8 KB of LDS hold a second, derived table for the first filter pass
// of the barrier-free stretches: P[i][c] = T[2i][c & 15] + T[2i+1][c >> 4] for the first 8 code
// bytes i and all 256 values c of a byte, so that the pass costs one lookup and one shift per
// code byte, as with 8-bit codes (a row of 16 entries never makes lanes collide, but costs two
// lookups and 2.5 times the address arithmetic per byte, which is what limits this kernel).
// The pass only decides who is looked at again: its sums may round differently from the
// table sum proper (a pair is added first), which the abandon margin covers like the other
// roundings of a partial sum (see abandon_threshold), and every candidate that passes has its
// sum redone from the 16-entry rows in subspace order.  The table proper follows at kTabAt.
template <bool FS> constexpr uint32_t kTabAt = FS ? 8 * kC * 4 : kTabLds;
constexpr int kXcds = 8;  // accelerator dies of an MI355X, each with its own L2

struct SearchArgs {
    // index (Section 3.3 preprocessing output)
    const float *base;
    const uint8_t *codes;
    const float *dlx;
    const int32_t *ids;
    const float *codebooks;
    const uint32_t *head;  // optional [n][3]: code bytes 0..7 and dlx of each vector
    const uint8_t *codes_tiled;  // optional: codes in blocks of 64 vectors x 16-byte pieces
    int64_t n;
    int32_t d, M, dsub;
    // queries, optional processing order, optional prebuilt tables
    const float *queries;
    int64_t nq;
    const int32_t *order;
    const float *lut;
    // candidate structure (nseg == 0: all n positions)
    const int64_t *list_offsets;
    const int32_t *probes;
    const uint8_t *list_bounds;  // per-list summaries (list_record_bytes(M) each) or null
    int32_t nlist, nseg;
    int32_t max_cand;  // per-query cut
    // table phases: the M subspaces are handled Mp at a time (P = M / Mp passes per batch)
    int32_t P, Mp;
    // search parameters
    int32_t k, batch;  // range: batch = span = survivor-list capacity per round
    int32_t span;      // candidates bounded between two barriers (a multiple of batch)
    float two_gamma;
    float radius2;
    // outputs
    int32_t *out_ids;
    float *out_d2;
    int32_t *n_scanned, *n_exact;
    uint32_t *work;   // optional [nq][kWorkCounters]: what the launch touched (see WorkCounter)
    uint32_t *mask;
    int64_t mask_words;
    // range only
    int32_t chunk;           // candidates per workgroup, multiple of 64
    int32_t nsplit;
    uint32_t *result_mask;   // [nq][rmask_words]
    float *result_d2;        // [nq][rmask_words * 32]: exact distance of each result, by scan-order number
    int64_t rmask_words;
    int32_t *chunk_counts;   // [nq][nsplit]
    // LDS carve-up (byte offsets)
    uint32_t off_q, off_segp, off_segd, off_rest, off_seglb, off_spos, off_sd2, off_sidx, off_rd2, off_rid, off_ctl;
    uint32_t off_plb, off_cnt, off_wq;
    int32_t wqcap;     // entries per wave in each of the two work-queue arrays
    int32_t cruise;    // candidates per cruise stretch (multiple of batch; 0 = disabled)
    int32_t small_addr;  // n < 2^24 and n*M < 2^32: 24-bit multiply and 32-bit offsets suffice
    int32_t use_rest;    // kNN: thresholds take the remaining table minima (and list summaries) into account
    int32_t poss_cap;  // capacity of the possibles list
    int32_t scap;      // entries of spos[] and of sd2[] (>= survivor capacity and >= poss_cap)
    int32_t rcap;      // entries behind sd2[scap] (bounds of a replay; >= poss_cap)
    int32_t bucket;    // cruise: possibles are counted per bucket of this many candidates (a multiple of batch)
};

// One record of the optional scan head.
struct __attribute__((packed, aligned(4))) HeadRecord {
    uint32_t w0, w1;  // code bytes 0..3, 4..7
    float b;          // landmark distance
};

struct Ctl {
    int32_t total;       // candidates of this query (after clamping)
    int32_t nsurv;       // survivors appended in the current batch
    float tau;
    int32_t nresult;     // range: results in this chunk
    int32_t nexact;
    int32_t nposs;       // cruise: number of possibles found in the stretch
    int32_t npassed;     // cruise: candidates of the stretch that passed the first subspaces
    int32_t hold;        // candidates still to be taken span by span before the next stretch is tried
    int32_t nfail;       // stretches that failed in a row (the next one is a short trial while > 0)
    uint32_t work[8];    // WorkCounter totals of this workgroup (only kept when asked for)
};

// Optional accounting of what a search touched, per query (trim_stats.work).
enum WorkCounter {
    kWorkFirstPass = 0,  // candidates whose first code bytes and landmark distance were read
    kWorkSkipped = 1,    // candidates passed over with their whole list, never read
    kWorkCodeBytes = 2,  // bytes of codes, scan-head records and landmark distances requested
    kWorkLookups = 3,    // table lookups issued
    kWorkRows = 4,       // raw rows read for an exact distance
    kWorkFullCode = 5,   // candidates whose code was read beyond the first pass
    kWorkCounters = 8
};
// Where the code bytes of one stored vector are.  Row-major: consecutive.  Tiled: the vectors
// are grouped in blocks of 64, and piece p (code bytes 16p..16p+15) of the 64 vectors of a
// block is contiguous (1 KB), so that 64 lanes reading the same piece of 64 consecutive
// vectors read one contiguous KB.  at(j) is valid for a load of 4, 8 or 16 bytes at a
// multiple of its size.
struct CodeRow {
    const uint8_t *p;
    uint32_t step;  // bytes from one 16-byte piece to the next
    __device__ __forceinline__ const uint8_t *at(int j) const {
        return p + (size_t)(uint32_t)(j >> 4) * step + (j & 15);
    }
};
template <bool TILED_OK>
__device__ __forceinline__ CodeRow code_row(const SearchArgs &a, int pos) {
    if (TILED_OK && a.codes_tiled)
        return CodeRow{a.codes_tiled + (((size_t)(pos >> 6) * (uint32_t)(a.M >> 4)) << 10) + ((pos & 63) << 4), 1024u};
    return CodeRow{a.codes + (size_t)pos * a.M, 16u};
}

constexpr int kSmallBatch = 512;  // below this: short first spans and the bulk form of the replay
constexpr int kRing = 256;  // entries of a wave's ring queue in cruise mode

// Load or build the table rows [j0, j0+nj) of query q into LDS.
template <bool FS>
__device__ __forceinline__ void fill_table(float *tab, const SearchArgs &a, const float *q_lds,
                                           int64_t q, int j0, int nj) {
    if (a.lut) {
        const float4 *src =
            reinterpret_cast<const float4 *>(a.lut + ((size_t)q * a.M + j0) * kByteEntries<FS>);
        float4 *dst = reinterpret_cast<float4 *>(tab);
        for (int e = threadIdx.x; e < nj * (kByteEntries<FS> / 4); e += blockDim.x) dst[e] = src[e];
    } else {
        build_table_rows<FS>(tab, q_lds, a.codebooks, a.dsub, j0, nj);
    }
}

// Per-thread cursor into the segment table: maps a scan-order number c to a storage
// position.  c must not decrease between calls.
struct SegCursor {
    int seg;
    int end;    // first scan-order number beyond the current segment
    int delta;  // position = c + delta inside the current segment
    __device__ __forceinline__ void init(const int *segp, const int *segd) {
        seg = 0; end = segp[1]; delta = segd[0];
    }
    __device__ __forceinline__ int pos(int c, const int *segp, const int *segd) {
        while (c >= end) {  // c < total guarantees termination
            ++seg;
            end = segp[seg + 1];
            delta = segd[seg];
        }
        return c + delta;
    }
};

constexpr int32_t kEmptyId = 0x7fffffff;  // id of an unused slot of R (its d2 is +inf)

// Entries per lane that hold a result set of size k in one wave's registers.
__host__ __device__ inline int result_slots(int k) { return k <= 64 ? 1 : k <= 128 ? 2 : k <= 256 ? 4 : 16; }

// Merge the refined survivors of a batch into R and publish tau (the "result queue update"
// of Section 4.2).  Executed by ONE whole wave.  R lives in LDS between calls (64*E
// entries, ascending by (d2,id), unused slots = (+inf, kEmptyId)); during the call lane l
// keeps entries l*E .. l*E+E-1 in registers, so an insertion is a ballot (rank), one
// cross-lane shift and a few selects, with no LDS round trip.
// The result set R in one wave's registers: 64*E entries ascending by (d2,id), lane l holding
// entries l*E .. l*E+E-1, unused slots = (+inf, kEmptyId).  R lives in LDS between uses.
template <int E>
struct ResultRegs {
    float r_d2[E];
    int32_t r_id[E];
    float t_d2;      // the k-th entry (tau): +inf while R holds fewer than k entries
    int32_t t_id;
    int k, lane, kl, ks;

    __device__ __forceinline__ void load(const float *rd2, const int32_t *rid, int k_, int lane_) {
        k = k_; lane = lane_;
        kl = (k - 1) / E; ks = (k - 1) % E;  // lane and slot of the k-th entry
#pragma unroll
        for (int s = 0; s < E; ++s) { r_d2[s] = rd2[lane * E + s]; r_id[s] = rid[lane * E + s]; }
        load_kth();
    }
    __device__ __forceinline__ void store(float *rd2, int32_t *rid) const {
#pragma unroll
        for (int s = 0; s < E; ++s) { rd2[lane * E + s] = r_d2[s]; rid[lane * E + s] = r_id[s]; }
    }
    __device__ __forceinline__ void load_kth() {
        float vd = r_d2[0];
        int32_t vi = r_id[0];
#pragma unroll
        for (int s = 1; s < E; ++s) if (s == ks) { vd = r_d2[s]; vi = r_id[s]; }
        t_d2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(vd), kl));  // kl is uniform
        t_id = __builtin_amdgcn_readlane(vi, kl);
    }
    // Insert the lanes' items (one per lane with `pending` set) that beat the k-th entry, one at
    // a time: an insertion is a ballot (rank), one cross-lane shift and a few selects.
    __device__ __forceinline__ void insert_pending(bool pending, float d2, int32_t id) {
        for (;;) {
            const unsigned long long m = __ballot(pending && hit_less(d2, id, t_d2, t_id));
            if (m == 0) break;
            const int src = __ffsll((long long)m) - 1;
            const float xd2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(d2), src));
            const int32_t xid = __builtin_amdgcn_readlane(id, src);  // src is the same in all lanes
            if (lane == src) pending = false;
            // rank = number of entries that are not greater than the item (a prefix of R)
            int rank = 0;
#pragma unroll
            for (int s = 0; s < E; ++s)
                rank += __popcll(__ballot(!hit_less(xd2, xid, r_d2[s], r_id[s])));
            // last slot of the lane below (whole-wave shift right by one lane; lane 0 unused)
            const float c_d2 = __int_as_float(
                __builtin_amdgcn_update_dpp(0, __float_as_int(r_d2[E - 1]), 0x138, 0xf, 0xf, false));
            const int32_t c_id = __builtin_amdgcn_update_dpp(0, r_id[E - 1], 0x138, 0xf, 0xf, false);
#pragma unroll
            for (int s = E - 1; s >= 0; --s) {
                const int g = lane * E + s;
                const float p_d2 = s > 0 ? r_d2[s > 0 ? s - 1 : 0] : c_d2;
                const int32_t p_id = s > 0 ? r_id[s > 0 ? s - 1 : 0] : c_id;
                if (g == rank) { r_d2[s] = xd2; r_id[s] = xid; }
                else if (g > rank) { r_d2[s] = p_d2; r_id[s] = p_id; }
                if (g >= k) { r_d2[s] = __builtin_inff(); r_id[s] = kEmptyId; }
            }
            load_kth();
        }
    }
};

// Merge the refined survivors of a batch into R and publish tau (the "result queue update"
// of Section 4.2).  Executed by ONE whole wave.
template <int E>
__device__ __forceinline__ void merge_batch(const float *sd2, const int32_t *sid, int ns,
                                            float *rd2, int32_t *rid, Ctl *ctl, int k, int lane) {
    ResultRegs<E> R;
    R.load(rd2, rid, k, lane);
    // A long list (the first batch after the seed) is pre-filtered: lane l takes the minimum of
    // entries l, l+64, ...; the k-th smallest of these 64 minima (distinct entries) is an upper
    // bound on the k-th distance after the merge, so entries above it never enter R and skip
    // the one-at-a-time insertion below.  (One entry per lane: result sets up to 64.)
    float cut = __builtin_inff();
    if constexpr (E == 1) {
        if (ns > 2 * kWave) {
            float cmin = __builtin_inff();
            for (int i = lane; i < ns; i += kWave) cmin = __builtin_fminf(cmin, sd2[i]);
#pragma unroll
            for (int size = 2; size <= kWave; size <<= 1) {
#pragma unroll
                for (int j = size >> 1; j > 0; j >>= 1) {   // bitonic network across the lanes
                    const float other = __shfl_xor(cmin, j);
                    const bool keep_min = ((lane & j) == 0) == ((lane & size) == 0);
                    cmin = keep_min ? __builtin_fminf(cmin, other) : __builtin_fmaxf(cmin, other);
                }
            }
            cut = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(cmin), k - 1));
        }
    }
    for (int i0 = 0; i0 < ns; i0 += kWave) {
        const int i = i0 + lane;
        bool pending = i < ns;
        float d2 = 0.0f;
        int32_t id = 0;
        if (pending) { d2 = sd2[i]; id = sid[i]; pending = d2 <= cut; }
        R.insert_pending(pending, d2, id);
    }
    R.store(rd2, rid);
    if (lane == 0) ctl->tau = R.t_d2;  // +inf while R holds fewer than k entries
}

// Replay of the batch rule over the possibles of a stretch (Section 4.2's threshold update,
// taken batch by batch), by ONE wave, with no barrier.  The entries 0..np-1 are grouped by
// batch in ascending batch order (any order inside a batch) and carry their candidate number
// (relative to the stretch), bound, exact distance and id.  For each batch in turn the threshold
// is frozen at the current k-th distance; the batch's entries whose bound passes it are its
// survivors: they are counted, marked, and merged into R.  Returns the number of survivors.
// BULK (for small batches): survivors that do not beat the k-th distance are handled all at once.
template <int E, bool BULK>
__device__ __forceinline__ int replay_batches(const int32_t *s_cl, const float *s_g, const float *s_d2,
                                              const int32_t *s_id, int np, int batch, int c0,
                                              uint32_t *mask_row, int64_t mask_words, float *rd2,
                                              int32_t *rid, Ctl *ctl, int k, int lane) {
    ResultRegs<E> R;
    R.load(rd2, rid, k, lane);
    int frozen_b = -1;
    float tau_f = R.t_d2;
    int total = 0;
    for (int i0 = 0; i0 < np; i0 += kWave) {
        const int i = i0 + lane;
        bool pending = i < np;
        int cl = 0, b = 0;
        int32_t id = 0;
        float g = __builtin_inff(), d2 = 0.0f;
        if (pending) { cl = s_cl[i]; g = s_g[i]; d2 = s_d2[i]; id = s_id[i]; b = cl / batch; }
        for (; !BULK;) {
            // thresholds only fall: an entry of a batch not yet begun whose bound exceeds the
            // current k-th distance can no longer survive
            pending = pending && (b == frozen_b || g <= R.t_d2);
            const unsigned long long m = __ballot(pending);
            if (m == 0) break;
            const int first = __ffsll((long long)m) - 1;   // lowest pending batch (entries are grouped)
            const int fb = __builtin_amdgcn_readlane(b, first);
            if (fb != frozen_b) { frozen_b = fb; tau_f = R.t_d2; }
            const bool grp = pending && b == fb;
            const bool sel = grp && g <= tau_f;
            total += __popcll(__ballot(sel));
            if (sel && mask_row) {
                const int c = c0 + cl;
                const int64_t wi = c >> 5;
                if (wi < mask_words) atomicOr(&mask_row[wi], 1u << (c & 31));
            }
            R.insert_pending(sel, d2, id);
            pending = pending && !grp;
        }
        for (; BULK;) {
            // An entry can still survive only if its bound passes the threshold of its batch: the
            // frozen one if its batch has begun, else the current k-th distance (thresholds only
            // fall, so failing it now is final).
            pending = pending && g <= (b == frozen_b ? tau_f : R.t_d2);
            // Only an entry that also beats the k-th distance changes anything.  Up to the first
            // such entry (in batch order) every pending entry is a survivor of a batch whose
            // threshold is the current k-th distance: counted and marked in one go.
            const unsigned long long mi = __ballot(pending && hit_less(d2, id, R.t_d2, R.t_id));
            int fb = 0x7fffffff;
            if (mi != 0) fb = __builtin_amdgcn_readlane(b, __ffsll((long long)mi) - 1);
            const bool plain = pending && b < fb;
            total += __popcll(__ballot(plain));
            if (plain && mask_row) {
                const int c = c0 + cl;
                const int64_t wi = c >> 5;
                if (wi < mask_words) atomicOr(&mask_row[wi], 1u << (c & 31));
            }
            pending = pending && !plain;
            // (a batch that goes on in the next chunk keeps its threshold: the frozen one if it
            // was frozen here, else the k-th distance, unchanged since that batch began)
            if (mi == 0) break;
            // the batch of the first improving entry: frozen threshold, all its passing entries
            // survive, those that beat the k-th distance are merged
            if (fb != frozen_b) { frozen_b = fb; tau_f = R.t_d2; }
            const bool sel = pending && b == fb;
            total += __popcll(__ballot(sel));
            if (sel && mask_row) {
                const int c = c0 + cl;
                const int64_t wi = c >> 5;
                if (wi < mask_words) atomicOr(&mask_row[wi], 1u << (c & 31));
            }
            R.insert_pending(sel, d2, id);
            pending = pending && !sel;
        }
    }
    R.store(rd2, rid);
    if (lane == 0) ctl->tau = R.t_d2;
    return total;
}

// E = result_slots(k) is a template parameter of the kernel, so that the common small-k case
// does not carry the registers of the wide result sets.
// LEAN_KIND (kNN, E = 1 only; see LeanKind): the instances held to 80 registers (6 waves per SIMD), so that three
// 512-thread workgroups share a CU when the table is short enough for that; it goes without
// the bulk rounds over long codes, the tiled code copy and the deeper refine pipelines, which
// the other instances (128 registers, at most 4 waves per SIMD) use.
constexpr int kLeanWavesPerSimd = 6;
// The lean instance comes in two kinds, one per shape of the refine step, so that neither carries
// the other's code: rows of at most 128 values (four rows per half wave, one 16-byte group per
// lane and row) and longer rows (two rows per half wave with three groups of each in flight).
enum LeanKind { kFullInstance = 0, kLeanShortRows = 1, kLeanLongRows = 2 };
// ACCT: the instance that keeps the work counters (SearchArgs::work); the plain one carries none
// of that code.
// FS: 4-bit codes, two per code byte, with rows of 16 table entries (see kByteRow); SearchArgs::M
// counts code bytes in either case.
template <int MODE, int VEC, int E, bool ACCT, bool FS, int LEAN_KIND>
__global__ __launch_bounds__(1024)
__attribute__((amdgpu_waves_per_eu(LEAN_KIND != kFullInstance ? kLeanWavesPerSimd : 4)))
void search_kernel(const SearchArgs a) {
    constexpr bool LEAN = LEAN_KIND != kFullInstance;
    static_assert(!LEAN || (MODE == kKnn && E == 1), "the lean instances are the small-k kNN ones");
    // The tiled copy of the codes is read by the instances with 16-byte code loads, except the
    // lean ones, whose codes are short (they read the row-major array).
    constexpr bool kTiledOk = VEC == 4 && !LEAN;
    extern __shared__ __align__(16) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem + kTabAt<FS>);
    float *pair_tab = reinterpret_cast<float *>(smem);   // 4-bit codes only: see kTabAt
    float *q_lds = reinterpret_cast<float *>(smem + a.off_q);
    int *segp = reinterpret_cast<int *>(smem + a.off_segp);   // [nseg+1] prefix of lengths
    int *segd = reinterpret_cast<int *>(smem + a.off_segd);   // [nseg] start - prefix
    float *restv = reinterpret_cast<float *>(smem + a.off_rest);  // [M/4+1] remaining minima (cruise)
    float *rowmin = reinterpret_cast<float *>(smem + a.off_plb);     // [M] smallest entry of each table row (prologue only)
    float2 *seglist = reinterpret_cast<float2 *>(smem + a.off_seglb); // [nseg] list-level pruning {slack, rest}: see the prologue
    int32_t *spos = reinterpret_cast<int32_t *>(smem + a.off_spos);  // survivor position -> id
    float *sd2 = reinterpret_cast<float *>(smem + a.off_sd2);        // exact d2 (shares the queue area)
    int32_t *sidx = reinterpret_cast<int32_t *>(smem + a.off_sidx);  // range: scan-order number
    float *plbs = reinterpret_cast<float *>(smem + a.off_plb);       // [span] partial s, then bound
    int *cnt0 = reinterpret_cast<int *>(smem + a.off_cnt);           // per-batch counts
    int *poss_cl = reinterpret_cast<int *>(smem + a.off_plb);        // cruise: possibles, aliasing
    float *poss_g = plbs + a.poss_cap;                               //   plbs ([poss_cap] each)
    float *rd2 = reinterpret_cast<float *>(smem + a.off_rd2);
    int32_t *rid = reinterpret_cast<int32_t *>(smem + a.off_rid);
    Ctl *ctl = reinterpret_cast<Ctl *>(smem + a.off_ctl);
    uint16_t *wq = reinterpret_cast<uint16_t *>(smem + a.off_wq);   // per-wave work queues

    const int tid = threadIdx.x;
    const int T = blockDim.x;
    const int lane = tid & (kWave - 1);
    // optional accounting of the work done (same for every thread); totals gather in LDS
    constexpr bool acct = ACCT;
    auto tally = [&](int which, uint32_t v) { atomicAdd(&ctl->work[which], v); };
    // The lean instances only run with the whole table in LDS and the tighter thresholds on (the
    // host sees to it), so the table phases and the switch are compiled out of them.
    const int nphase = LEAN ? 1 : a.P;
    const int Mp = LEAN ? a.M : a.Mp;
    const bool use_rest = LEAN ? true : a.use_rest != 0;
    // Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous run of the
    // (optionally sorted) query order so that concurrent workgroups of an XCD scan the same
    // lists and share its L2.
    const int64_t per_xcd = (a.nq + kXcds - 1) / kXcds;
    const int64_t slot = (int64_t)(blockIdx.x % kXcds) * per_xcd + blockIdx.x / kXcds;
    if (slot >= a.nq) return;  // the whole workgroup leaves together
    const int64_t q = a.order ? a.order[slot] : slot;
    if (q < 0 || q >= a.nq) return;  // not a permutation entry: nothing is done for it
    const int split = blockIdx.y;
    const int nseg = a.nseg > 0 ? a.nseg : 1;

    // ---- prologue: query, segment table, table ----
    for (int t = tid; t < a.d; t += T) q_lds[t] = a.queries[(size_t)q * a.d + t];
    if (MODE == kKnn)
        for (int g = tid; g < kWave * E; g += T) { rd2[g] = __builtin_inff(); rid[g] = kEmptyId; }
    // (list ids wait in the queue area, idle until the seed's barrier, for the list-level bounds)
    int *segl = reinterpret_cast<int *>(smem + a.off_wq);
    const bool segl_fits = nseg <= a.scap + a.rcap;
    for (int p = tid; p < nseg; p += T) {
        int64_t s = 0, e = a.n;
        int32_t lp = -1;
        if (a.nseg > 0) {
            const int32_t l = a.probes[(size_t)q * a.nseg + p];
            lp = l;
            if (l >= 0 && l < a.nlist) {
                s = a.list_offsets[l];
                e = a.list_offsets[l + 1];
                s = s < 0 ? 0 : (s > a.n ? a.n : s);
                e = e < s ? s : (e > a.n ? a.n : e);
            } else {
                s = e = 0;
            }
        }
        segd[p] = (int)s;            // start for now
        segp[p + 1] = (int)(e - s);  // length for now
        if (segl_fits) segl[p] = e > s ? lp : -1;
    }
    __syncthreads();
    if (tid == 0) {
        int64_t run = 0;
        segp[0] = 0;
        for (int p = 0; p < nseg; ++p) {
            int64_t len = segp[p + 1];
            if (run + len > a.max_cand) len = a.max_cand - run;
            segd[p] = segd[p] - (int)run;
            run += len;
            segp[p + 1] = (int)run;
        }
        ctl->total = (int)run;
        ctl->nsurv = 0;
        ctl->tau = MODE == kRange ? a.radius2 : __builtin_inff();
        ctl->nresult = 0;
        ctl->nexact = 0;
        ctl->hold = 0;
        // The first stretch of a query is a trial (a short one) where a long one is likely to
        // fail: with long codes (8 of 64 or more subspaces may abandon too few candidates for
        // stretches to pay at all), or when much of the first probed list is still to come after
        // the first batch (the rest of the query's nearest list passes every filter and would
        // fill the list of possibles).
        ctl->nfail = (a.M >= 64 || segp[1] - (a.k + a.batch) > a.poss_cap / 2) ? 1 : 0;
        for (int i = 0; i < kWorkCounters; ++i) ctl->work[i] = 0;
    }
    if (nphase == 1) fill_table<FS>(tab, a, q_lds, q, 0, a.M);
    __syncthreads();
    if constexpr (FS) {   // the pair table of the first 8 code bytes (read after later barriers)
        for (int e = tid; e < 8 * kC; e += T) {
            const float *row = tab + (size_t)(e >> 8) * kByteEntries<true>;
            pair_tab[e] = row[e & 15] + row[kC4 + ((e >> 4) & 15)];
        }
    }
    // restv[i] = sum over the subspaces j >= 4i of the smallest entry of table row j: what the
    // subspaces still to come add to a running sum at the very least (see abandon_threshold).
    // Here: the sums of four rows' minima, one wave per group; turned into suffix sums below.
    if (MODE == kKnn && use_rest) {
        for (int i = tid >> 6; i < a.M / 4; i += T >> 6) {
            float gsum = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float m;
                if constexpr (FS) {
                    // the byte's two rows of 16: lanes 0..15 and 16..31 take a minimum each, and
                    // the least a byte can add is their sum
                    m = tab[(size_t)(4 * i + r) * kByteEntries<true> + (lane & 31)];
#pragma unroll
                    for (int off = 8; off > 0; off >>= 1) m = __builtin_fminf(m, __shfl_xor(m, off));
                    m = m + __shfl_xor(m, 16);
                } else {
                    const float4 v = *reinterpret_cast<const float4 *>(tab + (size_t)(4 * i + r) * kC + 4 * lane);
                    m = __builtin_fminf(__builtin_fminf(v.x, v.y), __builtin_fminf(v.z, v.w));
#pragma unroll
                    for (int off = 32; off > 0; off >>= 1) m = __builtin_fminf(m, __shfl_xor(m, off));
                }
                gsum = gsum + m;
                if (lane == 0) rowmin[4 * i + r] = m;
            }
            if (lane == 0) restv[i] = gsum;
        }
    }
    __syncthreads();
    if (tid == 0) {
        float acc = 0.0f;
        restv[Mp / 4] = 0.0f;
        for (int i = Mp / 4 - 1; i >= 0; --i) {
            acc = (MODE == kKnn && use_rest) ? acc + restv[i] : 0.0f;
            restv[i] = acc;
        }
    }   // (read after the next barrier: the seed's, or the one at the top of the main loop)
    // List-level bounds (kNN over inverted lists whose summaries the caller supplies): for the
    // list of segment p, lb = sum over all subspaces j of the smallest T[j][c] over the codes c
    // that occur in the list, a lower bound of every table sum of the list; rest = the same
    // over the subspaces from H0 on; bm = the list's largest landmark distance.  Every abandon
    // threshold of the list is at most (c bm + st)^2 (abandon_threshold grows with the
    // landmark distance), so while lb exceeds that, nothing in the list can survive.
    // Two segments per wave and round; a lane takes 16 recorded codes of one subspace (4 lanes
    // per subspace, 32 subspaces of either list per step, all loads of a step issued together).
    if (MODE == kKnn && use_rest && a.nseg > 0 && a.list_bounds != nullptr) {
        constexpr int kH0 = VEC >= 2 ? 8 : 4;
        const size_t rec_bytes = list_record_bytes(a.M);
        if (acct && tid == 0) tally(kWorkCodeBytes, (uint32_t)(nseg * rec_bytes));
        // two segments per round and wave, 32 subspaces per step: all the loads of a step are
        // issued before the first is used
        for (int p0 = 2 * (tid >> 6); p0 < nseg; p0 += 2 * (T >> 6)) {
            const uint8_t *rec[2];
            float bm[2], lb[2] = {0.0f, 0.0f}, rest[2] = {0.0f, 0.0f};
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const int l = p0 + t >= nseg ? -1                     // same for the wave
                              : segl_fits ? segl[p0 + t] : a.probes[(size_t)q * a.nseg + p0 + t];
                rec[t] = (l >= 0 && l < a.nlist) ? a.list_bounds + (size_t)l * rec_bytes : nullptr;
                bm[t] = rec[t] ? *reinterpret_cast<const float *>(rec[t] + list_record_bmax_offset(a.M))
                               : __builtin_inff();
            }
            for (int j0 = 0; j0 < a.M; j0 += 32) {
                uint4 cw[2][2];
                int cnt[2][2];
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int j = j0 + 16 * g + (lane >> 2);
                        cw[t][g] = make_uint4(0, 0, 0, 0);
                        cnt[t][g] = 0;
                        if (rec[t] && j < a.M) {
                            cw[t][g] = *reinterpret_cast<const uint4 *>(rec[t] + (size_t)j * kSetCap + (lane & 3) * 16);
                            cnt[t][g] = rec[t][(size_t)a.M * kSetCap + j];
                        }
                    }
#pragma unroll
                for (int t = 0; t < 2; ++t)
#pragma unroll
                    for (int g = 0; g < 2; ++g) {
                        const int j = j0 + 16 * g + (lane >> 2);
                        const bool on = rec[t] && j < a.M;
                        const float *row = tab + (size_t)(on ? j : 0) * kByteEntries<FS>;
                        const uint32_t w4[4] = {cw[t][g].x, cw[t][g].y, cw[t][g].z, cw[t][g].w};
                        float m = __builtin_inff();
                        // (words past the recorded count repeat the first code: skipped)
                        const int nrec = cnt[t][g] == kSetAny ? 0 : cnt[t][g];
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (16 * (lane & 3) + 4 * v < nrec) {
#pragma unroll
                                for (int b = 0; b < 4; ++b) {
                                    const uint32_t c = (w4[v] >> (8 * b)) & 255u;
                                    // what a vector with this code byte adds (4-bit codes: both halves)
                                    m = __builtin_fminf(m, FS ? row[c & 15u] + row[kC4 + (c >> 4)] : row[c]);
                                }
                            }
                        m = __builtin_fminf(m, __shfl_xor(m, 1));
                        m = __builtin_fminf(m, __shfl_xor(m, 2));
                        if (on && (cnt[t][g] == 0 || cnt[t][g] == kSetAny)) m = rowmin[j];
                        if (on && (lane & 3) == 0) {
                            lb[t] = lb[t] + m;
                            if (j >= kH0) rest[t] = rest[t] + m;
                        }
                    }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
#pragma unroll
                for (int off = 32; off >= 4; off >>= 1) {
                    lb[t] = lb[t] + __shfl_xor(lb[t], off);
                    rest[t] = rest[t] + __shfl_xor(rest[t], off);
                }
                // the list is passed over while lb > (c bm + st)^2, i.e. while
                // sqrt(lb) - c bm > st: the left side is kept, rounded against passing over
                float slack = sqrt_rn(lb[t]) * (1.0f - 1e-6f) - kAbandonC * bm[t] * (1.0f + 1e-6f);
                if (!(slack == slack)) slack = -__builtin_inff();
                if (lane == 0 && p0 + t < nseg) seglist[p0 + t] = make_float2(slack, rest[t]);
            }
        }
    }

    const int total = ctl->total;
    int c_begin = 0, c_end = total;
    if (MODE == kRange) {
        c_begin = split * a.chunk;
        c_end = c_begin + a.chunk < total ? c_begin + a.chunk : total;
        if (c_begin > total) c_begin = total;
    }
    SegCursor cur;
    cur.init(segp, segd);
    (void)split;

    const int nhalf = T >> 5;
    const int half = tid >> 5;
    const int lane32 = tid & 31;
    const int kseed = MODE == kKnn ? (a.k < total ? a.k : total) : 0;

    // Storage position of the candidate with scan-order number c (binary search over the
    // segment prefix; used only for the few candidates that survive).
    auto locate = [&](int c) {
        int lo = 0, hi = nseg - 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (c >= segp[mid + 1]) lo = mid + 1; else hi = mid;
        }
        return c + segd[lo];
    };

    // Append the calling lane's candidate (if live) to the survivor list: wave ballot,
    // prefix count, one LDS atomic per wave.  Must be called by whole waves.
    auto append = [&](bool live, int c) {
        const unsigned long long m = __ballot(live);
        if (m == 0) return;
        int basei = 0;
        if (lane == 0) basei = atomicAdd(&ctl->nsurv, __popcll(m));
        basei = __shfl(basei, 0);
        if (live) {
            const int slot = basei + __popcll(m & ((1ull << lane) - 1ull));
            spos[slot] = locate(c);
            if (MODE == kRange) sidx[slot] = c;
            if (a.mask) {
                const int64_t wi = c >> 5;
                if (wi < a.mask_words)
                    atomicOr(&a.mask[(size_t)q * a.mask_words + wi], 1u << (c & 31));
            }
        }
    };

    // Exact distances of `ns` listed candidates: one half wave per raw row, four rows in flight
    // per half wave.  pos_of(i) gives the storage position of entry i; put(i, d2, id or
    // position) stores the result (called by the lane that holds the row's distance).
    auto refine_rows = [&](int ns, auto pos_of, auto put) {
        // Two rows per half wave with several 16-byte groups of each in flight, instead of four
        // rows step by step: the lean instance for long rows always (three groups: its register
        // budget), the full instance for the few long rows that survive a short span (eight).
        if (LEAN_KIND == kLeanLongRows || (!LEAN && a.d >= 512 && ns <= 8 * nhalf)) {
            for (int i = half; i < ns; i += 2 * nhalf) {
                const int i1 = i + nhalf;
                const bool ok1 = i1 < ns;               // uniform within the half wave
                const int p0 = pos_of(i), p1 = pos_of(ok1 ? i1 : i);
                const int32_t id0 = (MODE == kKnn && a.ids) ? a.ids[p0] : p0;
                const int32_t id1 = (MODE == kKnn && a.ids) ? a.ids[p1] : p1;
                float d2[2];
                exact_d2_half_x2_deep<LEAN ? 3 : 8>(a.base + (size_t)p0 * a.d, a.base + (size_t)p1 * a.d, q_lds,
                                                    a.d, lane32, d2);
                if (lane32 == 0) {
                    put(i, d2[0], id0);
                    if (ok1) put(i1, d2[1], id1);
                }
            }
            return;
        }
        if constexpr (LEAN_KIND != kLeanLongRows)   // (that instance goes without this loop)
        for (int i = half; i < ns; i += 4 * nhalf) {
            int idx[4], pos[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                idx[u] = i + u * nhalf;
                ok[u] = idx[u] < ns;              // uniform within the half wave
                pos[u] = pos_of(ok[u] ? idx[u] : i);
            }
            int32_t rid4[4];  // ids are fetched together with the rows, not after them
#pragma unroll
            for (int u = 0; u < 4; ++u) rid4[u] = (MODE == kKnn && a.ids) ? a.ids[pos[u]] : pos[u];
            const float d2 = exact_d2_half_x4<!LEAN, LEAN_KIND == kLeanShortRows>(
                a.base + (size_t)pos[0] * a.d, a.base + (size_t)pos[1] * a.d, a.base + (size_t)pos[2] * a.d,
                a.base + (size_t)pos[3] * a.d, q_lds, a.d, lane32);
            // four lanes of the half wave hold one row's distance each and store it
            const int mine = half_reduce_x4_row(lane32);
            const bool hi2 = (mine & 2) != 0, lo1 = (mine & 1) != 0;
            const bool my_ok = hi2 ? (lo1 ? ok[3] : ok[2]) : (lo1 ? ok[1] : ok[0]);
            const int my_idx = hi2 ? (lo1 ? idx[3] : idx[2]) : (lo1 ? idx[1] : idx[0]);
            const int32_t my_id = hi2 ? (lo1 ? rid4[3] : rid4[2]) : (lo1 ? rid4[1] : rid4[0]);
            if (half_reduce_x4_writer(lane32) && my_ok) put(my_idx, d2, my_id);
        }
    };

    // Refine the listed survivors, then select: merge into R and publish the new tau.  Called
    // by the whole block after a barrier that made the survivor list visible; ends with a
    // barrier.
    auto refine_and_select = [&](int ns) {
        refine_rows(ns, [&](int i) { return spos[i]; },
                    [&](int i, float d2, int32_t id) {
                        if (MODE == kKnn) {
                            sd2[i] = d2;
                            spos[i] = id;
                        } else if (d2 <= a.radius2) {
                            const int c = sidx[i];
                            atomicOr(&a.result_mask[(size_t)q * a.rmask_words + (c >> 5)], 1u << (c & 31));
                            a.result_d2[(size_t)q * a.rmask_words * 32 + c] = d2;
                            atomicAdd(&ctl->nresult, 1);
                        }
                    });
        __syncthreads();
        if (MODE == kKnn && tid < kWave) merge_batch<E>(sd2, spos, ns, rd2, rid, ctl, a.k, lane);
        if (tid == 0) {
            ctl->nexact += ns;
            ctl->nsurv = 0;
            if (acct) tally(kWorkRows, (uint32_t)ns);
        }
        __syncthreads();
    };

    // ---- stage B by replay (k <= 64): the possibles of a stretch or span, already laid out in
    // batch order in spos[] (candidate number relative to c0) and s_g[] (bound), ALL get their
    // exact distance in one parallel pass, and one wave then replays the batch rule over them
    // without any barrier.  A possible that turns out not to survive its batch has had its
    // distance computed in vain; that is the price of dropping the barriers (and the refine
    // latency) of every single batch.  Called after a barrier; the caller's next barrier waits
    // for the replaying wave.
    auto counts_to_offsets = [&](int nb) {   // cnt0[0..nb): counts -> exclusive prefix; total -> nposs
        if (tid < kWave) {
            const int per = (nb + kWave - 1) / kWave;
            int sum = 0;
            for (int e = 0; e < per; ++e) {
                const int idx = lane * per + e;
                if (idx < nb) sum += cnt0[idx];
            }
            int incl = sum;
#pragma unroll
            for (int off = 1; off < kWave; off <<= 1) {
                const int t = __shfl_up(incl, off);
                if (lane >= off) incl += t;
            }
            int run = incl - sum;
            for (int e = 0; e < per; ++e) {
                const int idx = lane * per + e;
                if (idx < nb) { const int v = cnt0[idx]; cnt0[idx] = run; run += v; }
            }
            if (lane == kWave - 1) ctl->nposs = incl;
        }
    };
    auto refine_and_replay = [&](int np, int c0) {
        float *s_g = sd2 + a.scap;                                 // bounds, in batch order
        int32_t *s_id = reinterpret_cast<int32_t *>(smem + a.off_plb);  // ids (that area is dead by now)
        refine_rows(np, [&](int i) { return locate(c0 + spos[i]); },
                    [&](int i, float d2, int32_t id) { sd2[i] = d2; s_id[i] = id; });
        __syncthreads();
        if (tid < kWave) {
            uint32_t *mrow = a.mask ? a.mask + (size_t)q * a.mask_words : nullptr;
            int n;
            if constexpr (E > 1) {
                n = replay_batches<E, true>(spos, s_g, sd2, s_id, np, a.batch, c0, mrow, a.mask_words,
                                            rd2, rid, ctl, a.k, lane);
            } else {
                n = a.batch < kSmallBatch
                    ? replay_batches<E, true>(spos, s_g, sd2, s_id, np, a.batch, c0, mrow, a.mask_words,
                                              rd2, rid, ctl, a.k, lane)
                    : replay_batches<E, false>(spos, s_g, sd2, s_id, np, a.batch, c0, mrow, a.mask_words,
                                               rd2, rid, ctl, a.k, lane);
            }
            if (lane == 0) {
                ctl->nexact += n;
                if (acct) tally(kWorkRows, (uint32_t)np);
            }
        }
    };

    // ---- seed: the first k candidates populate R, all with exact distances ----
    if (kseed > 0) {
        for (int i0 = 0; i0 < kseed; i0 += T) append(i0 + tid < kseed, i0 + tid);
        __syncthreads();
        refine_and_select(kseed);
    }

    // ---- main loop over spans of candidates (a whole number of batches each) ----
    // Stage A bounds every candidate of the span with no barrier in between and
    // keeps the bounds in LDS; it counts, per batch, the candidates that pass the
    // threshold in force at the start of the span.  Thresholds only fall, so that
    // set contains every later survivor, and batches whose count is zero are skipped
    // outright.  Stage B walks the remaining batches in order with the up-to-date
    // threshold, which reproduces the batch-by-batch rule exactly.
    constexpr int H0 = VEC >= 2 ? 8 : 4;   // subspaces bounded in round 0
    constexpr int U = 4;                   // candidates per lane in flight in round 0
    // the wave number, in a scalar register: everything derived from it stays uniform
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), nwaves = T >> 6;
    // This wave's slice [lo, hi) of a span of the given length.
    auto wave_slice = [&](int span_len, int &lo, int &hi) {
        const int wchunk = ((span_len + nwaves - 1) / nwaves + kWave - 1) & ~(kWave - 1);
        lo = wave * wchunk;
        hi = lo + wchunk < span_len ? lo + wchunk : span_len;
    };
    // Issue the loads (first H0 code bytes, landmark distance) of U x 64 candidates.
    auto issue_loads = [&](int c0n, int base, int hi, uint32_t (&w)[U][H0 / 4], float (&bq)[U],
                           int (&sg)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int cl = base + u * kWave + lane;
            bq[u] = __builtin_nanf("");  // out of range: never passes a threshold test
            sg[u] = 0;
#pragma unroll
            for (int v = 0; v < H0 / 4; ++v) w[u][v] = 0;
            if (cl < hi) {
                const int pos = cur.pos(c0n + cl, segp, segd);
                sg[u] = cur.seg;
                load_codes<H0 / 4>(w[u], code_row<kTiledOk>(a, pos).at(0));
                bq[u] = a.dlx[pos];
            }
        }
    };
    // number of set bits of a ballot below the calling lane
    auto below = [](unsigned long long m) {
        return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
    };
    int cruise = MODE == kKnn ? a.cruise : 0;  // candidates per cruise stretch (0 = never)
    // next span length while the spans of a small-batch search still grow (a multiple of batch)
    int small_span = (MODE == kKnn && a.batch < kSmallBatch) ? (64 + a.batch - 1) / a.batch * a.batch : a.span;
    for (int c0 = c_begin + kseed; c0 < c_end;) {
        __syncthreads();  // every thread is done with the previous stretch
        const float tau0 = ctl->tau;
        const float sqrt_tau0 = abandon_scale(tau0);  // scaled: see abandon_threshold

        // ---- cruise: once tau is finite, bound a long stretch of candidates with no block-wide
        // barrier at all.  Every wave runs its own software pipeline over interleaved blocks of
        // U x 64 candidates: the next block's loads are in flight while the current block is
        // bounded over the first H0 subspaces; the few candidates not abandoned there go on
        // the wave's ring queue and are finished 64 at a time.  Only candidates whose bound
        // passes tau0 ("possibles": a superset of all later survivors, since thresholds only
        // fall) are kept, as (number, bound) pairs in a shared list; the batches are then
        // replayed in order over that list.  If the list overflows, nothing has been
        // committed: the stretch is redone span by span below.
        // (The first span after the seed is always taken span by span: it is what makes tau tight.)
        int replay_np = -1;  // >= 0: the candidates [c0, c0 + advance) end in a replay of that many possibles
        int advance = 0;
        if (cruise > 0 && ctl->hold <= 0 && small_span >= a.span && c0 > c_begin + kseed &&
            tau0 < __builtin_inff() && c_end - c0 > a.span) {
            // (the first stretch of a query, and the first after a failed one, is a short trial:
            // it shows whether the first pass abandons enough for stretches to pay, see below)
            int want = cruise;
            const int nfail = ctl->nfail;
            if (nfail > 0) {
                const int probe = 4096 / a.batch * a.batch;
                if (probe >= a.batch && probe < want) want = probe;
            }
            const int S = c0 + want < c_end ? want : c_end - c0;
            const int nb = (S + a.bucket - 1) / a.bucket;   // buckets (= batches unless they are very small)
            for (int b = tid; b < nb; b += T) cnt0[b] = 0;
            if (tid == 0) { ctl->nposs = 0; ctl->npassed = 0; }
            __syncthreads();
            {
                uint32_t *ring = reinterpret_cast<uint32_t *>(wq) + (size_t)wave * kRing;  // (segment << 16) | number
                int head = 0, count = 0;  // same in every lane of the wave

                const bool long_codes = a.M >= 64;
                // A drain takes up to 64 queued candidates, one per lane.  It is split in two so
                // that its loads are in flight while the next block is bounded: drain_issue pops
                // the entries and starts the loads of the landmark distance and the first code
                // chunk; drain_finish redoes the table sum from the start (now with a test every
                // 8 subspaces), evaluates Equation 3 and records the candidate if it passes tau0.
                constexpr int DV = VEC;            // dwords per code chunk
                const bool two_chunks = a.M >= 8 * DV;  // the first two chunks are loaded ahead
                int d_n = 0, d_cl = 0, d_pos = 0;
                float d_b = 0.0f;
                uint32_t d_w0[DV], d_w1[DV];
                auto drain_issue = [&]() {
                    d_n = count < kWave ? count : kWave;
                    // (long codes: every candidate that passed is drained once; counted for the test below)
                    if (long_codes && lane == 0) atomicAdd(&ctl->npassed, d_n);
                    if (lane < d_n) {
                        const uint32_t e = ring[(head + lane) & (kRing - 1)];
                        d_cl = (int)(e & 0xffffu);
                        d_pos = c0 + d_cl + segd[e >> 16];
                        const CodeRow cr = code_row<kTiledOk>(a, d_pos);
                        d_b = a.dlx[d_pos];
                        load_codes<DV>(d_w0, cr.at(0));
                        if (two_chunks) load_codes<DV>(d_w1, cr.at(4 * DV));
                    }
                    head = (head + d_n) & (kRing - 1);
                    count -= d_n;
                };
                auto drain_finish = [&]() {
                    if (lane < d_n) {
                        const float thr = abandon_threshold(d_b, sqrt_tau0);
                        const CodeRow cr = code_row<kTiledOk>(a, d_pos);
                        // every test of a running sum is against the threshold less what the
                        // subspaces still to come add at the least (restv; a half-way stop inside
                        // a 16-subspace piece comes back as +inf)
                        float sum = gather_add<DV, true, FS>(0.0f, kTabAt<FS>, d_w0, thr - restv[DV == 4 ? 2 : 0]);
                        int j = 4 * DV;
                        if (two_chunks && !(sum > thr - restv[j >> 2])) {
                            sum = gather_add<DV, true, FS>(sum, kTabAt<FS> + 4 * DV * kByteRow<FS>, d_w1,
                                                       thr - restv[DV == 4 ? 6 : 0]);
                            j = 8 * DV;
                        }
                        while (j < a.M && !(sum > thr - restv[j >> 2])) {  // widest aligned load that fits
                            if (VEC == 4 && (j & 15) == 0 && j + 16 <= a.M) {
                                uint32_t w[4];
                                load_codes<4>(w, cr.at(j));
                                sum = gather_add<4, true, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr - restv[(j >> 2) + 2]);
                                j += 16;
                            } else if (VEC >= 2 && (j & 7) == 0 && j + 8 <= a.M) {
                                uint32_t w[2];
                                load_codes<2>(w, cr.at(j));
                                sum = gather_add<2, false, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr);
                                j += 8;
                            } else {
                                uint32_t w[1];
                                load_codes<1>(w, cr.at(j));
                                sum = gather_add<1, false, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr);
                                j += 4;
                            }
                        }
                        if (acct) {
                            // the first two chunks were loaded ahead whether or not the sum got
                            // that far; a sum stopped inside a 16-byte piece comes back as +inf
                            // and has looked up only the piece's first 8 subspaces
                            const int loaded = two_chunks && j < 8 * DV ? 8 * DV : j;
                            tally(kWorkCodeBytes, (uint32_t)(loaded + 4));
                            tally(kWorkLookups, (uint32_t)(j - (DV == 4 && sum == __builtin_inff() ? 8 : 0)) * kByteLookups<FS>);
                            tally(kWorkFullCode, 1u);
                        }
                        if (!(sum > thr - restv[j >> 2])) {
                            const float g = plb_from_s(sum, d_b, a.two_gamma);
                            if (g <= tau0) {
                                const int at = atomicAdd(&ctl->nposs, 1);
                                if (at < a.poss_cap) { poss_cl[at] = d_cl; poss_g[at] = g; }

                                atomicAdd(&cnt0[d_cl / a.bucket], 1);
                            }
                        }
                    }
                    d_n = 0;
                    // the list of possibles has run full (a loose threshold, or near lists): the
                    // stretch will be redone span by span anyway, so this wave stops bounding

                };
                const int nblk = (S + U * kWave - 1) / (U * kWave);
                // the wave's own cursor into the segment table, in scalar registers
                int s_seg = 0;
                int s_end = __builtin_amdgcn_readfirstlane(segp[1]);
                int s_delta = __builtin_amdgcn_readfirstlane(segd[0]);
                // what subspaces H0.. add at the least, in a scalar register
                const float rest_h0 = __builtin_bit_cast(
                    float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, restv[H0 / 4])));
                // list-level pruning: a list is passed over while its slack > st (both compared as
                // integers: st > 0, and a negative slack is a negative integer)
                const bool have_lb = use_rest && a.nseg > 0 && a.list_bounds != nullptr;
                const int st_bits = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sqrt_tau0));
                for (int blk = wave; blk < nblk; blk += nwaves) {
                    // this block's loads fly while the previous drain is finished; the next
                    // drain's loads fly while this block is bounded
                    uint32_t w[U][H0 / 4];
                    float bq[U];
                    int sg[U];
                    const int cb = blk * U * kWave;
                    // same for the whole wave
                    const bool full = H0 == 8 && a.head && a.small_addr && cb + U * kWave <= S;
                    // A block that lies inside one list takes that list's remaining minimum, or is
                    // passed over with the list; any other block takes the global minimum.
                    float blk_rest = rest_h0;
                    if (full && have_lb) {
                        const int cf = c0 + cb;
                        while (cf >= s_end) {                    // cf < total: terminates
                            ++s_seg;
                            s_end = __builtin_amdgcn_readfirstlane(segp[s_seg + 1]);
                            s_delta = __builtin_amdgcn_readfirstlane(segd[s_seg]);
                        }
                        if (cf + U * kWave <= s_end) {
                            const float2 sr = seglist[s_seg];
                            const int sl = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sr.x));
                            const int rs = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, sr.y));
                            if (sl > st_bits) {                  // same for the whole wave
                                if (acct && lane == 0) tally(kWorkSkipped, U * kWave);
                                continue;
                            }
                            blk_rest = __builtin_bit_cast(float, rs);
                        } else if (s_seg + 1 < nseg) {
                            // the block ends in the next list: passed over if both lists are
                            const int e2 = __builtin_amdgcn_readfirstlane(segp[s_seg + 2]);
                            const int sl1 = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, seglist[s_seg].x));
                            const int sl2 = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, seglist[s_seg + 1].x));
                            if (cf + U * kWave <= e2 && sl1 > st_bits && sl2 > st_bits) {
                                if (acct && lane == 0) tally(kWorkSkipped, U * kWave);
                                continue;
                            }
                        }
                    }
                    if (full) {
                        // whole block in range, 32-bit byte offsets from uniform bases; the
                        // segment of 64 consecutive candidates is found with scalar arithmetic
                        // unless they straddle a segment boundary
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const int cf = c0 + cb + u * kWave;  // uniform
                            while (cf >= s_end) {                // cf < total: terminates
                                ++s_seg;
                                s_end = __builtin_amdgcn_readfirstlane(segp[s_seg + 1]);
                                s_delta = __builtin_amdgcn_readfirstlane(segd[s_seg]);
                            }
                            uint32_t pos;
                            if (cf + kWave <= s_end) {
                                pos = (uint32_t)(cf + s_delta) + (uint32_t)lane;
                                sg[u] = s_seg << 16;
                            } else {
                                int seg = s_seg, end = s_end, delta = s_delta;
                                const int c = cf + lane;
                                while (c >= end) {
                                    ++seg;
                                    end = segp[seg + 1];
                                    delta = segd[seg];
                                }
                                pos = (uint32_t)(c + delta);
                                sg[u] = seg << 16;
                            }
                            const HeadRecord r = *reinterpret_cast<const HeadRecord *>(
                                reinterpret_cast<const char *>(a.head) + (size_t)(uint32_t)__umul24(pos, 12u));
                            w[u][0] = r.w0;
                            w[u][H0 / 4 - 1] = r.w1;  // H0 == 8 here
                            bq[u] = r.b;
                        }
                    } else {
                        issue_loads(c0, cb, S, w, bq, sg);
#pragma unroll
                        for (int u = 0; u < U; ++u) sg[u] <<= 16;
                    }
                    if (acct && lane == 0) {
                        const uint32_t nv = cb + U * kWave <= S ? U * kWave : S - cb;  // candidates of the block
                        tally(kWorkFirstPass, nv);
                        tally(kWorkCodeBytes, nv * (full ? (uint32_t)sizeof(HeadRecord) : H0 + 4u));
                        tally(kWorkLookups, nv * H0);   // (4-bit codes: one lookup per byte in the pair table)
                    }
                    // finish the drain in flight; drain whole waves while two or more wait (keep
                    // room), and leave the last one in flight behind the gathers below.  (One call
                    // site each for issue and finish: the kernel's speed follows its code size.)
#pragma clang loop unroll(disable)
                    for (;;) {
                        if (d_n > 0) drain_finish();
                        if (count < kWave) break;
                        drain_issue();
                        if (count < kWave) break;
                    }
                    float sums[U];
                    if constexpr (H0 == 8 && U % 2 == 0) {
#pragma unroll
                        for (int u = 0; u < U; u += 2)
                            gather8_pair<false>(kTabLds, w[u], w[u + 1], sums[u], sums[u + 1]);   // (4-bit codes: the pair table)
                    } else {
#pragma unroll
                        for (int u = 0; u < U; ++u)
                            sums[u] = gather_add<H0 / 4, false, FS>(0.0f, kTabAt<FS>, w[u], __builtin_inff());
                    }
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        if (u == U / 2 && count >= 2 * kWave) {
                            // a ring holds 4 x 64 entries: make room half way through the block
                            // (finish what is in flight, drain one wave and finish it)
#pragma clang loop unroll(disable)
                            for (int r = 0; r < 2; ++r) {
                                if (d_n > 0) drain_finish();
                                if (r == 0) drain_issue();
                            }
                        }
                        const float sum = sums[u];
                        const int cl = cb + u * kWave + lane;
                        const float thr = abandon_threshold(bq[u], sqrt_tau0) - blk_rest;
                        // lanes beyond the stretch carry a NaN landmark distance (issue_loads):
                        // their threshold is NaN and the comparison is false
                        const bool alive = sum <= thr;
                        const unsigned long long m = __builtin_amdgcn_ballot_w64(alive);
                        if (alive) {
                            const uint32_t at = __builtin_amdgcn_mbcnt_hi(
                                (uint32_t)(m >> 32),
                                __builtin_amdgcn_mbcnt_lo((uint32_t)m, (uint32_t)(head + count)));
                            ring[at & (kRing - 1)] = (uint32_t)sg[u] | (uint32_t)cl;
                        }
                        count += __popcll(m);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                    __builtin_amdgcn_wave_barrier();
                }
#pragma clang loop unroll(disable)
                for (;;) {
                    if (d_n > 0) drain_finish();
                    if (count <= 0) break;
                    drain_issue();
                }
            }
            __syncthreads();
            // A first pass that abandons less than half of the candidates only adds work (its
            // lookups are redone when the survivor's whole code is summed, piece after piece): the
            // query then goes on span by span, where a round takes a long piece of every code at
            // once, for a while (twice as long after every failure in a row), and tries again
            // with a short stretch: near lists pass the first subspaces, far ones do not.
            bool failed = 2 * ctl->npassed > S;
            const int np = ctl->nposs;
            if (np <= a.poss_cap) {
                // Stage B of a stretch.  The possibles are put in batch order (counting sort on
                // the per-batch counts), ALL get their exact distance in one parallel pass, and
                // one wave then replays the batch rule over them without any barrier.  A possible
                // that turns out not to survive its batch has had its distance computed in vain;
                // thresholds fall slowly this deep into the scan, so these are few.
                replay_np = np;
                advance = S;
                if (np > 0) {
                    counts_to_offsets(nb);
                    __syncthreads();
                    float *s_g = sd2 + a.scap;
                    for (int i = tid; i < np; i += T) {
                        const int cl = poss_cl[i];
                        const int slot = atomicAdd(&cnt0[cl / a.bucket], 1);
                        spos[slot] = cl;
                        s_g[slot] = poss_g[i];
                    }
                    if (a.bucket > a.batch) {
                        // a bucket holds several batches: put its few entries in scan order
                        __syncthreads();
                        for (int t = tid; t < nb; t += T) {
                            const int lo = t > 0 ? cnt0[t - 1] : 0, hi = cnt0[t];  // ends after the scatter
                            for (int x = lo + 1; x < hi; ++x) {
                                const int cx = spos[x];
                                const float gx = s_g[x];
                                int y = x - 1;
                                while (y >= lo && spos[y] > cx) { spos[y + 1] = spos[y]; s_g[y + 1] = s_g[y]; --y; }
                                spos[y + 1] = cx;
                                s_g[y + 1] = gx;
                            }
                        }
                    }
                }
            } else {
                // overflow: redo from c0 span by span, then try again with a short stretch (waves
                // stop as soon as they see the list full, so np is no measure of the length that
                // would have fitted: the stretch just failed)
                failed = true;
                cur.init(segp, segd);
                __syncthreads();
            }
            if (tid == 0) {   // (read again only after the barrier at the top of the loop)
                // (long codes: a first pass that fails once rarely pays later; short codes: the
                // near lists are soon over)
                ctl->hold = failed ? (a.M >= 64 ? 8192 : 2048) << (nfail < 7 ? nfail : 7) : 0;
                ctl->nfail = failed ? nfail + 1 : 0;
            }
        }
        if (replay_np < 0) {

        // The first stretch after the seed is a single batch: its threshold (from the k seeds)
        // is loose, so nothing is abandoned early; one batch is enough to make tau tight.
        // Small batches: the first spans are short too (64 candidates or one batch, then doubling), so that
        // tau is tight before a full span's possibles have to fit the replay.
        int span_len = c0 == c_begin + kseed ? a.batch : a.span;
        if (small_span < a.span) {
            span_len = small_span;
            small_span *= 2;
        }
        const int span = c0 + span_len < c_end ? span_len : c_end - c0;
        const int nb = (span + a.batch - 1) / a.batch;
        for (int b = tid; b < nb; b += T) cnt0[b] = 0;
        __syncthreads();
        // Rounds, wave by wave.  Each wave owns a contiguous slice of the span.  Round 0
        // bounds ALL its candidates over the first H0 subspaces, branch-free, U x 64
        // candidates in flight.  Whoever is not abandoned yet goes on the wave's own work
        // queue; each later round takes that queue densely (one candidate per lane),
        // continues the table sum over the next subspaces and queues what is still alive.
        // Lanes stay full although most candidates stop after a few subspaces, and since a
        // queue is private to its wave no block-wide barrier separates the rounds.  The
        // partial sum of a queued candidate waits in plbs[].
        int wlo, whi;
        wave_slice(span, wlo, whi);
        uint16_t *qin = wq + (size_t)wave * a.wqcap;
        uint16_t *qout = wq + (size_t)(nwaves + wave) * a.wqcap;
        int qn = 0;  // length of this wave's queue (same in every lane)
        // A batch that runs against a loose threshold (the first ones after the seed) abandons
        // nobody, so the rounds would only add dependent memory latencies: its candidates are
        // bounded in one go instead, two per lane, with all their loads issued together.
        constexpr int kDirectChunks = 2;  // code chunks of 4*VEC bytes a lane keeps per candidate
        const bool direct = MODE == kKnn && VEC == 4 && nphase == 1 && a.M <= 4 * VEC * kDirectChunks &&
                            a.M % (4 * VEC) == 0 && c0 == c_begin + kseed;
        if (direct) {
            constexpr int UD = 2;
            for (int base = wlo; base < whi; base += UD * kWave) {
                uint32_t w[UD][kDirectChunks][VEC];
                float b[UD];
#pragma unroll
                for (int u = 0; u < UD; ++u) {
                    const int cl = base + u * kWave + lane;
                    b[u] = 0.0f;
#pragma unroll
                    for (int c = 0; c < kDirectChunks; ++c)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) w[u][c][v] = 0;
                    if (cl < whi) {
                        const int pos = cur.pos(c0 + cl, segp, segd);
                        const CodeRow cr = code_row<kTiledOk>(a, pos);
                        b[u] = a.dlx[pos];
#pragma unroll
                        for (int c = 0; c < kDirectChunks; ++c)
                            if (c * 4 * VEC < a.M) load_codes<VEC>(w[u][c], cr.at(c * 4 * VEC));
                    }
                }
#pragma unroll
                for (int u = 0; u < UD; ++u) {
                    const int cl = base + u * kWave + lane;
                    float sum = 0.0f;
#pragma unroll
                    for (int c = 0; c < kDirectChunks; ++c)
                        if (c * 4 * VEC < a.M)
                            sum = gather_add<VEC, false, FS>(sum, kTabAt<FS> + c * 4 * VEC * kByteRow<FS>, w[u][c],
                                                  __builtin_inff());
                    if (cl < whi) {
                        const float g = plb_from_s(sum, b[u], a.two_gamma);
                        plbs[cl] = g;
                        if (g <= tau0) atomicAdd(&cnt0[cl / a.batch], 1);
                    }
                }
            }
            if (acct && lane == 0 && whi > wlo) {
                const uint32_t nv = whi - wlo;
                tally(kWorkFirstPass, nv);
                tally(kWorkFullCode, nv);
                tally(kWorkCodeBytes, nv * (uint32_t)(a.M + 4));
                tally(kWorkLookups, nv * (uint32_t)a.M * kByteLookups<FS>);
            }
        }
        int rnd = 0;  // rounds taken so far (the second one reads the rest of a code for the first time)
        for (int ph = 0; ph < (direct ? 0 : nphase); ++ph) {
            if (nphase > 1) {
                __syncthreads();
                fill_table<FS>(tab, a, q_lds, q, ph * Mp, Mp);
                __syncthreads();
            }
            const bool last_ph = ph == nphase - 1;
            for (int h0 = 0; h0 < Mp;) {
                int h1;
                int qnext = 0;
                // Long codes: the first 8 subspaces are a small share of the sum and abandon
                // nobody, so the first round of phase 0 is a bulk round over the whole slice.
                const bool slice_round = ph == 0 && h0 == 0;
                constexpr int kPieces = LEAN ? 0 : 6;
                const bool bulk_first = kPieces > 0 && VEC == 4 && a.M >= 64;
                if (slice_round && !bulk_first) {
                    // ---- round 0 ----
                    h1 = H0 < Mp ? H0 : Mp;
                    const bool fin = last_ph && h1 == Mp;
                    for (int base = wlo; base < whi; base += U * kWave) {
                        float bq[U];
                        uint32_t w[U][H0 / 4];
                        int sg_unused[U];
                        issue_loads(c0, base, whi, w, bq, sg_unused);
#pragma unroll
                        for (int u = 0; u < U; ++u) {
                            const float sum = gather_add<H0 / 4, false, FS>(0.0f, kTabAt<FS>, w[u], __builtin_inff());
                            const int cl = base + u * kWave + lane;
                            const float thr = abandon_threshold(bq[u], sqrt_tau0);
                            const bool valid = cl < whi;
                            bool alive = valid && !(sum > thr);
                            float keep = alive ? sum : __builtin_inff();
                            if (fin && alive) {  // the whole bound fits in round 0
                                keep = plb_from_s(sum, bq[u], a.two_gamma);
                                if (keep <= tau0) atomicAdd(&cnt0[cl / a.batch], 1);
                                alive = false;
                            }
                            if (valid) plbs[cl] = keep;
                            const unsigned long long m = __ballot(alive);
                            if (alive) qout[qnext + below(m)] = (uint16_t)cl;
                            qnext += __popcll(m);
                        }
                    }
                    if (acct && lane == 0 && whi > wlo) {
                        const uint32_t nv = whi - wlo;
                        tally(kWorkFirstPass, nv);
                        tally(kWorkCodeBytes, nv * (H0 + 4u));
                        tally(kWorkLookups, nv * (uint32_t)h1 * kByteLookups<FS>);
                    }
                } else {
                    // ---- later rounds: dense over the wave's queue ----
                    // With 16-byte code loads a round takes up to 104 subspaces (an 8-byte piece
                    // up to the next 16-byte boundary, then up to kPieces 16-byte pieces) and issues
                    // all its loads together with the landmark distance: one memory latency per
                    // queue entry instead of one per piece.  Otherwise: 32 subspaces, piece by piece.
                    // (not in the lean instance, which meets later rounds only on fallback)
                    const bool lead8 = kPieces > 0 && VEC == 4 && (h0 & 15) == 8 && h0 + 8 <= Mp;
                    const int ja = h0 + (lead8 ? 8 : 0);
                    int n16 = kPieces > 0 && VEC == 4 && (ja & 15) == 0 ? (Mp - ja) / 16 : 0;
                    if (n16 > kPieces) n16 = kPieces;
                    const bool bulk = lead8 || n16 > 0;
                    h1 = bulk ? ja + 16 * n16 : (h0 + 32 < Mp ? h0 + 32 : Mp);
                    const bool fin = last_ph && h1 == Mp;
                    // entries: the wave's queue, or (first round of phase 0) its whole slice
                    const int nent = slice_round ? (whi > wlo ? whi - wlo : 0) : qn;
                    for (int i0 = 0; i0 < nent; i0 += kWave) {
                        const int i = i0 + lane;
                        bool alive = i < nent;
                        int cl = 0;
                        if (alive) {
                            cl = slice_round ? wlo + i : qin[i];
                            const int pos = slice_round ? cur.pos(c0 + cl, segp, segd) : locate(c0 + cl);
                            const CodeRow cr = code_row<kTiledOk>(a, pos);
                            const int jp = ph * Mp;  // first subspace of this phase
                            uint32_t w8[2] = {0, 0};
                            uint32_t w16[kPieces > 0 ? kPieces : 1][4];
                            if (bulk) {
                                if (lead8) load_codes<2>(w8, cr.at(jp + h0));
#pragma unroll
                                for (int c = 0; c < kPieces; ++c)
                                    if (c < n16) load_codes<4>(w16[c], cr.at(jp + ja + 16 * c));
                            }
                            const float b = a.dlx[pos];
                            const float thr = abandon_threshold(b, sqrt_tau0);
                            float sum = slice_round ? 0.0f : plbs[cl];
                            int j = h0;
                            int used16 = 0;  // 16-byte pieces of a bulk round whose sum was begun
                            // (a sum stopped inside a 16-byte piece comes back as +inf: still
                            // above every threshold, and the accounting can tell)
                            if (bulk) {
                                if (lead8) sum = gather_add<2, false, FS>(sum, kTabAt<FS> + h0 * kByteRow<FS>, w8, thr);
#pragma unroll
                                for (int c = 0; c < kPieces; ++c)
                                    if (c < n16 && !(sum > thr)) {
                                        sum = gather_add<4, true, FS>(sum, kTabAt<FS> + (ja + 16 * c) * kByteRow<FS>,
                                                                  w16[c], thr);
                                        ++used16;
                                    }
                                j = h1;
                            }
                            while (j < h1) {  // widest aligned load that fits, test after each
                                if (VEC == 4 && (j & 15) == 0 && j + 16 <= h1) {
                                    uint32_t w[4];
                                    load_codes<4>(w, cr.at(jp + j));
                                    sum = gather_add<4, true, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr);
                                    j += 16;
                                } else if (VEC >= 2 && (j & 7) == 0 && j + 8 <= h1) {
                                    uint32_t w[2];
                                    load_codes<2>(w, cr.at(jp + j));
                                    sum = gather_add<2, false, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr);
                                    j += 8;
                                } else {
                                    uint32_t w[1];
                                    load_codes<1>(w, cr.at(jp + j));
                                    sum = gather_add<1, false, FS>(sum, kTabAt<FS> + j * kByteRow<FS>, w, thr);
                                    j += 4;
                                }
                                if (sum > thr) break;
                            }
                            if (acct) {
                                const int bytes = bulk ? (lead8 ? 8 : 0) + 16 * n16 : j - h0;
                                const int looks = (bulk ? (lead8 ? 8 : 0) + 16 * used16 : j - h0) -
                                                  (VEC == 4 && sum == __builtin_inff() ? 8 : 0);
                                tally(kWorkCodeBytes, (uint32_t)(bytes + 4));
                                tally(kWorkLookups, (uint32_t)looks * kByteLookups<FS>);
                                if (slice_round) tally(kWorkFirstPass, 1u);
                                else if (rnd == 1) tally(kWorkFullCode, 1u);
                            }
                            if (sum > thr) {
                                plbs[cl] = __builtin_inff();
                                alive = false;
                            } else if (fin) {
                                const float g = plb_from_s(sum, b, a.two_gamma);
                                plbs[cl] = g;
                                if (g <= tau0) atomicAdd(&cnt0[cl / a.batch], 1);
                                alive = false;
                            } else {
                                plbs[cl] = sum;
                            }
                        }
                        const unsigned long long m = __ballot(alive);
                        if (alive) qout[qnext + below(m)] = (uint16_t)cl;
                        qnext += __popcll(m);
                    }
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                qn = qnext;
                uint16_t *t = qin; qin = qout; qout = t;
                h0 = h1;
                ++rnd;
                if (qn == 0) break;  // this wave has nobody left in this phase
            }
        }
        __syncthreads();
        // Several batches in the span and a result set of at most 64: replay (see above), unless
        // the possibles do not fit its arrays (a loose threshold: then batch by batch as below).
        int np_span = -1;
        if (MODE == kKnn && nb > 1) {
            counts_to_offsets(nb);
            __syncthreads();
            np_span = ctl->nposs;
            if (np_span <= a.scap && np_span <= a.rcap) {
                replay_np = np_span;
                advance = span;
                if (np_span > 0) {
                    float *s_g = sd2 + a.scap;
                    for (int i = tid; i < span; i += T) {
                        const float g = plbs[i];
                        if (g <= tau0) {
                            const int slot = atomicAdd(&cnt0[i / a.batch], 1);
                            spos[slot] = i;
                            s_g[slot] = g;
                        }
                    }
                }
            }
        }
        for (int b = 0; replay_np < 0 && b < nb; ++b) {
            // same value for every thread: no barrier needed (np_span >= 0: counts were turned
            // into start offsets above)
            const int cb = np_span < 0 ? cnt0[b] : (b + 1 < nb ? cnt0[b + 1] : np_span) - cnt0[b];
            if (cb == 0) continue;

            const float tau = ctl->tau;
            const int l0 = b * a.batch;
            const int blen = l0 + a.batch < span ? a.batch : span - l0;
            for (int i0 = 0; i0 < blen; i0 += T) {
                const int i = i0 + tid;
                const bool live = i < blen && plbs[l0 + i] <= tau;
                append(live, c0 + l0 + i);
            }
            __syncthreads();
            const int ns = ctl->nsurv;
            __syncthreads();  // nobody appends for the next batch before everyone has read ns
            if (ns > 0) refine_and_select(ns);
        }
        if (replay_np < 0) advance = span;
        if (tid == 0) ctl->hold -= advance;   // (several barriers after everybody read it)
        }  // span path
        if (replay_np > 0) {
            __syncthreads();   // the possibles are in place
            refine_and_replay(replay_np, c0);
        }
        c0 += advance;
    }

    // ---- epilogue ----
    // (the last stretch may have ended in a replay by the first wave alone: every thread that
    // writes results must see its R)
    __syncthreads();
    if (MODE == kKnn) {
        for (int i = tid; i < a.k; i += T) {
            const int32_t id = rid[i];
            a.out_ids[(size_t)q * a.k + i] = id == kEmptyId ? -1 : id;
            a.out_d2[(size_t)q * a.k + i] = rd2[i];
        }
        if (tid == 0) {
            if (a.n_scanned) a.n_scanned[q] = total;
            if (a.n_exact) a.n_exact[q] = ctl->nexact;
        }
        if (acct && tid < kWorkCounters) a.work[(size_t)q * kWorkCounters + tid] = ctl->work[tid];
    } else {
        if (tid == 0) {
            a.chunk_counts[(size_t)q * a.nsplit + split] = ctl->nresult;
            if (a.n_scanned && split == 0) a.n_scanned[q] = total;
            if (a.n_exact && ctl->nexact) atomicAdd(&a.n_exact[q], ctl->nexact);
        }
        // (the host zeroed the array: a query's chunks add up)
        if (acct && tid < kWorkCounters && ctl->work[tid])
            atomicAdd(&a.work[(size_t)q * kWorkCounters + tid], ctl->work[tid]);
    }
}

}  // namespace trim
