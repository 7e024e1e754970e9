// The fused filter-then-refine scan (Section 4.2) as one persistent workgroup per query
// (kNN) or per (query, candidate chunk) (range).  Everything a query needs between
// batches (distance table, query, result set R, threshold tau, survivor list) stays in
// LDS; the only HBM traffic is the streamed codes + landmark distances, the raw rows of
// survivors, and the results.
#pragma once

#include "trim_device.h"

namespace trim {

enum Mode { kKnn = 0, kRange = 1 };

struct SearchArgs {
    // index (Section 3.3 preprocessing output)
    const float *base;
    const uint8_t *codes;
    const float *dlx;
    const int32_t *ids;
    const float *codebooks;
    int64_t n;
    int32_t d, M, dsub;
    // queries and (optional) prebuilt tables
    const float *queries;
    const float *lut;
    // candidate structure (nseg == 0: all n positions)
    const int64_t *list_offsets;
    const int32_t *probes;
    int32_t nlist, nseg;
    int32_t max_cand;  // per-query cut
    // table phases: the M subspaces are handled Mp at a time (P = M / Mp passes per batch)
    int32_t P, Mp;
    // search parameters
    int32_t k, batch;  // range: batch = survivor-list capacity per round
    float two_gamma;
    float radius2;
    // outputs
    int32_t *out_ids;
    float *out_d2;
    int32_t *n_scanned, *n_exact;
    uint32_t *mask;
    int64_t mask_words;
    // range only
    int32_t chunk;           // candidates per workgroup, multiple of 64
    int32_t nsplit;
    uint32_t *result_mask;   // [nq][rmask_words]
    int64_t rmask_words;
    int32_t *chunk_counts;   // [nq][nsplit]
    // LDS carve-up (byte offsets)
    uint32_t off_q, off_segp, off_segd, off_spos, off_sd2, off_sidx, off_rd2, off_rid, off_ctl;
};

struct Ctl {
    int32_t total;       // candidates of this query (after clamping)
    int32_t nsurv;       // survivors appended in the current batch
    float tau;
    int32_t rsize;
    int32_t nresult;     // range: results in this chunk
    int32_t nexact;
};

// Load or build the table rows [j0, j0+nj) of query q into LDS.
__device__ __forceinline__ void fill_table(float *tab, const SearchArgs &a, const float *q_lds,
                                           int64_t q, int j0, int nj) {
    if (a.lut) {
        const float4 *src =
            reinterpret_cast<const float4 *>(a.lut + ((size_t)q * a.M + j0) * kC);
        float4 *dst = reinterpret_cast<float4 *>(tab);
        for (int e = threadIdx.x; e < nj * (kC / 4); e += blockDim.x) dst[e] = src[e];
    } else {
        build_table_rows(tab, q_lds, a.codebooks, a.dsub, j0, nj);
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

// Insert (d2,id) into the sorted result set held in LDS; executed by one whole wave.
// Returns the new size.
__device__ __forceinline__ int result_insert(volatile float *rd2, volatile int32_t *rid,
                                             int rsize, int k, float d2, int32_t id, int lane) {
    // rank = number of entries e with !(item < R[e])
    int rank = 0;
    for (int e0 = 0; e0 < rsize; e0 += kWave) {
        const int e = e0 + lane;
        bool keep = false;
        if (e < rsize) keep = !hit_less(d2, id, rd2[e], rid[e]);
        rank += __popcll(__ballot(keep));
    }
    const int nsize = rsize < k ? rsize + 1 : k;
    if (rank >= nsize) return rsize;  // not better than the current k-th
    // shift R[rank .. nsize-2] up by one, highest chunk first
    for (int e0 = ((nsize - 1) / kWave) * kWave; e0 >= 0 && e0 + kWave > rank; e0 -= kWave) {
        const int e = e0 + lane;
        const bool mv = e > rank && e < nsize;
        float td2 = 0.0f;
        int32_t tid = 0;
        if (mv) { td2 = rd2[e - 1]; tid = rid[e - 1]; }
        __builtin_amdgcn_wave_barrier();
        if (mv) { rd2[e] = td2; rid[e] = tid; }
        __builtin_amdgcn_wave_barrier();
    }
    if (lane == 0) { rd2[rank] = d2; rid[rank] = id; }
    __builtin_amdgcn_wave_barrier();
    return nsize;
}

// Merge the refined survivors of a batch into R (wave 0 only) and publish tau.
__device__ __forceinline__ void merge_batch(float *sd2, int32_t *sid, int ns, float *rd2_,
                                            int32_t *rid_, Ctl *ctl, int k, int lane) {
    volatile float *rd2 = rd2_;
    volatile int32_t *rid = rid_;
    int rsize = ctl->rsize;
    for (int i0 = 0; i0 < ns; i0 += kWave) {
        const int i = i0 + lane;
        bool pending = i < ns;
        float d2 = 0.0f;
        int32_t id = 0;
        if (pending) { d2 = sd2[i]; id = sid[i]; }
        for (;;) {
            bool cand = pending;
            if (cand && rsize >= k) cand = hit_less(d2, id, rd2[k - 1], rid[k - 1]);
            const unsigned long long m = __ballot(cand);
            if (m == 0) break;
            const int src = __ffsll((long long)m) - 1;
            const float xd2 = __shfl(d2, src);
            const int32_t xid = __shfl(id, src);
            if (lane == src) pending = false;
            rsize = result_insert(rd2, rid, rsize, k, xd2, xid, lane);
        }
    }
    if (lane == 0) {
        ctl->rsize = rsize;
        ctl->tau = rsize >= k ? rd2[k - 1] : __builtin_inff();
    }
}

template <int MODE, int VEC>
__global__ __launch_bounds__(1024) void search_kernel(const SearchArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem);
    float *q_lds = reinterpret_cast<float *>(smem + a.off_q);
    int *segp = reinterpret_cast<int *>(smem + a.off_segp);   // [nseg+1] prefix of lengths
    int *segd = reinterpret_cast<int *>(smem + a.off_segd);   // [nseg] start - prefix
    int32_t *spos = reinterpret_cast<int32_t *>(smem + a.off_spos);  // survivor position -> id
    float *sd2 = reinterpret_cast<float *>(smem + a.off_sd2);        // partial s, then d2
    int32_t *sidx = reinterpret_cast<int32_t *>(smem + a.off_sidx);  // range: scan-order number
    float *rd2 = reinterpret_cast<float *>(smem + a.off_rd2);
    int32_t *rid = reinterpret_cast<int32_t *>(smem + a.off_rid);
    Ctl *ctl = reinterpret_cast<Ctl *>(smem + a.off_ctl);

    const int tid = threadIdx.x;
    const int T = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int64_t q = blockIdx.y;
    const int split = blockIdx.x;
    const int nseg = a.nseg > 0 ? a.nseg : 1;

    // ---- prologue: query, segment table, table ----
    for (int t = tid; t < a.d; t += T) q_lds[t] = a.queries[(size_t)q * a.d + t];
    for (int p = tid; p < nseg; p += T) {
        int64_t s = 0, e = a.n;
        if (a.nseg > 0) {
            const int32_t l = a.probes[(size_t)q * a.nseg + p];
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
        ctl->rsize = 0;
        ctl->tau = MODE == kRange ? a.radius2 : __builtin_inff();
        ctl->nresult = 0;
        ctl->nexact = 0;
    }
    if (a.P == 1) fill_table(tab, a, q_lds, q, 0, a.M);
    __syncthreads();

    const int total = ctl->total;
    int c_begin = 0, c_end = total;
    if (MODE == kRange) {
        c_begin = split * a.chunk;
        c_end = c_begin + a.chunk < total ? c_begin + a.chunk : total;
        if (c_begin > total) c_begin = total;
    }
    SegCursor cur;
    cur.init(segp, segd);

    const int nhalf = T >> 5;
    const int half = tid >> 5;
    const int lane32 = tid & 31;
    const int kseed = MODE == kKnn ? (a.k < total ? a.k : total) : 0;

    int c0 = c_begin;
    bool seed = MODE == kKnn && kseed > 0;
    while (c0 < c_end) {
        const int c1 = seed ? kseed : (c0 + a.batch < c_end ? c0 + a.batch : c_end);
        const float tau = ctl->tau;
        const float sqrt_tau = trim::sqrt_rn(tau);
        const int iters = (c1 - c0 + T - 1) / T;
        // ---- filter: bound every candidate of the batch, compact the survivors ----
        const SegCursor cur0 = cur;
        for (int ph = 0; ph < a.P; ++ph) {
            if (a.P > 1) {
                __syncthreads();
                fill_table(tab, a, q_lds, q, ph * a.Mp, a.Mp);
                __syncthreads();
                cur = cur0;
            }
            const bool last = ph == a.P - 1;
            for (int it = 0; it < iters; ++it) {
                const int cl = it * T + tid;  // batch-local number
                const int c = c0 + cl;
                const bool valid = c < c1;
                bool live = false;
                int pos = 0;
                if (valid) {
                    pos = cur.pos(c, segp, segd);
                    if (seed) {
                        live = true;
                    } else {
                        const float b = a.dlx[pos];
                        const float thr = abandon_threshold(b, sqrt_tau);
                        float s = ph == 0 ? 0.0f : sd2[cl];
                        if (!(s > thr))
                            s = table_sum<VEC>(s, tab, a.codes + (size_t)pos * a.M + ph * a.Mp,
                                               a.Mp, thr);
                        if (last) {
                            // an abandoned sum is certainly pruned; otherwise s is complete
                            live = !(s > thr) && plb_from_s(s, b, a.two_gamma) <= tau;
                        } else {
                            sd2[cl] = s;
                        }
                    }
                }
                if (last) {
                    // wave-level compaction: ballot + prefix count, one LDS atomic per wave
                    const unsigned long long m = __ballot(live);
                    if (m != 0) {
                        int basei = 0;
                        if (lane == 0) basei = atomicAdd(&ctl->nsurv, __popcll(m));
                        basei = __shfl(basei, 0);
                        if (live) {
                            const int slot = basei + __popcll(m & ((1ull << lane) - 1ull));
                            spos[slot] = pos;
                            if (MODE == kRange) sidx[slot] = c;
                            if (a.mask) {
                                const int64_t wi = c >> 5;
                                if (wi < a.mask_words)
                                    atomicOr(&a.mask[(size_t)q * a.mask_words + wi], 1u << (c & 31));
                            }
                        }
                    }
                }
            }
        }
        __syncthreads();
        const int ns = ctl->nsurv;
        if (ns > 0) {
            // ---- refine: exact distances of the survivors, one half wave per row ----
            for (int i = half; i < ns; i += nhalf) {
                const int pos = spos[i];
                const float d2 = exact_d2_half(a.base + (size_t)pos * a.d, q_lds, a.d, lane32);
                if (lane32 == 0) {
                    if (MODE == kKnn) {
                        sd2[i] = d2;
                        spos[i] = a.ids ? a.ids[pos] : pos;
                    } else if (d2 <= a.radius2) {
                        const int c = sidx[i];
                        atomicOr(&a.result_mask[(size_t)q * a.rmask_words + (c >> 5)], 1u << (c & 31));
                        atomicAdd(&ctl->nresult, 1);
                    }
                }
            }
            __syncthreads();
            // ---- select: merge into R, publish the new tau ----
            if (MODE == kKnn && tid < kWave) merge_batch(sd2, spos, ns, rd2, rid, ctl, a.k, lane);
            if (tid == 0) {
                ctl->nexact += ns;
                ctl->nsurv = 0;
            }
            __syncthreads();
        }
        c0 = c1;
        seed = false;
    }

    // ---- epilogue ----
    if (MODE == kKnn) {
        const int rsize = ctl->rsize;
        for (int i = tid; i < a.k; i += T) {
            a.out_ids[(size_t)q * a.k + i] = i < rsize ? rid[i] : -1;
            a.out_d2[(size_t)q * a.k + i] = i < rsize ? rd2[i] : __builtin_inff();
        }
        if (tid == 0) {
            if (a.n_scanned) a.n_scanned[q] = total;
            if (a.n_exact) a.n_exact[q] = ctl->nexact;
        }
    } else if (tid == 0) {
        a.chunk_counts[(size_t)q * a.nsplit + split] = ctl->nresult;
        if (a.n_scanned && split == 0) a.n_scanned[q] = total;
        if (a.n_exact && ctl->nexact) atomicAdd(&a.n_exact[q], ctl->nexact);
    }
}

}  // namespace trim
