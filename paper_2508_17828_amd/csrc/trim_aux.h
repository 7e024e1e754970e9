// Kernels around the scan: PQ encode, stand-alone distance tables, range-search output
// assembly, coarse-probe selection, small fills.
#pragma once

#include "trim_device.h"

namespace trim {

// ---- fills (used instead of memset nodes so that callers may capture the stream) ----
__global__ void fill_u32_kernel(uint32_t *p, size_t count, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count;
         i += (size_t)gridDim.x * blockDim.x)
        p[i] = v;
}

// ---- ceilings of the machine for the two resources the scan leans on (measurement aids) ----
// Streaming read: every 16-byte piece of the buffer is read once, four loads in flight per
// thread; the xor of everything read goes to sink[block] so that the loads cannot be dropped.
__global__ __launch_bounds__(512) void stream_read_kernel(const uint4 *__restrict__ p, size_t n16,
                                                          uint32_t *__restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    uint32_t acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const uint4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], e = p[i + 3 * stride];
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ e.x ^ e.y ^ e.z ^ e.w;
    }
    for (; i < n16; i += stride) {
        const uint4 a = p[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    for (int off = 32; off > 0; off >>= 1) acc ^= __shfl_xor(acc, off);
    __shared__ uint32_t part[8];
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t r = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) r ^= part[w];
        sink[blockIdx.x] = r;
    }
}

// Table gathers: the inner step of the scan and nothing else.  Each lane owns 32 code bytes
// (8 words) and sums, per iteration, the 32 entries T[j][byte j] of a [32][256] binary32 table
// in LDS with the scan's own gather routine; the code words are stirred between iterations so
// that the reads stay random.  gathers = grid * 512 * iters * 32.
__global__ __launch_bounds__(512) void lds_gather_kernel(int iters, uint32_t seed,
                                                         float *__restrict__ sink) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem);  // [32][256]
    for (int i = threadIdx.x; i < 32 * kC; i += blockDim.x) tab[i] = (float)((i * 2654435761u) >> 20);
    __syncthreads();
    const uint32_t tab_base = lds_addr(tab);
    uint32_t w[8];
    uint32_t h = seed ^ ((blockIdx.x * 512u + threadIdx.x) * 0x9e3779b9u);
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        h ^= h << 13; h ^= h >> 17; h ^= h << 5;
        w[v] = h;
    }
    float s = 0.0f;
    for (int it = 0; it < iters; ++it) {
        const uint32_t lo[4] = {w[0], w[1], w[2], w[3]};
        const uint32_t hi[4] = {w[4], w[5], w[6], w[7]};
        s = gather_add<4>(s, tab_base, lo, __builtin_inff());
        s = gather_add<4>(s, tab_base + 16 * kC * 4, hi, __builtin_inff());
        const uint32_t t = w[0];
#pragma unroll
        for (int v = 0; v < 7; ++v) w[v] = w[v + 1];
        w[7] = (t << 7 | t >> 25) ^ (uint32_t)it;
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same for 4-bit codes: a [64][16] table (32 code bytes of two subspaces each); every lane
// sums, per iteration, the 64 entries its 32 code bytes select, with the scan's own routine.
// A row of 16 consecutive words spans 16 banks, so these lookups never collide: this is also the
// rate of conflict-free 4-byte LDS reads.  lookups = grid * 512 * iters * 64.
__global__ __launch_bounds__(512) void lds_gather_fs_kernel(int iters, uint32_t seed,
                                                            float *__restrict__ sink) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem);  // [64][16]
    for (int i = threadIdx.x; i < 64 * kC4; i += blockDim.x) tab[i] = (float)((i * 2654435761u) >> 20);
    __syncthreads();
    const uint32_t tab_base = lds_addr(tab);
    uint32_t w[8];
    uint32_t h = seed ^ ((blockIdx.x * 512u + threadIdx.x) * 0x9e3779b9u);
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        h ^= h << 13; h ^= h >> 17; h ^= h << 5;
        w[v] = h;
    }
    float s = 0.0f;
    for (int it = 0; it < iters; ++it) {
        const uint32_t lo[4] = {w[0], w[1], w[2], w[3]};
        const uint32_t hi[4] = {w[4], w[5], w[6], w[7]};
        s = gather_add<4, false, true>(s, tab_base, lo, __builtin_inff());
        s = gather_add<4, false, true>(s, tab_base + 16 * kByteRow<true>, hi, __builtin_inff());
        const uint32_t t = w[0];
#pragma unroll
        for (int v = 0; v < 7; ++v) w[v] = w[v + 1];
        w[7] = (t << 7 | t >> 25) ^ (uint32_t)it;
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// The same with entries of W binary32 values (W = 2, 4: what a table shared by W queries would
// hold): 8 rows of 256 entries, every thread performs iters * 8 lookups of one whole entry and
// adds its W values up.
template <int W>
__global__ __launch_bounds__(512) void lds_gather_wide_kernel(int iters, uint32_t seed,
                                                              float *__restrict__ sink) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *tab = reinterpret_cast<float *>(smem);  // [8][256][W]
    for (int i = threadIdx.x; i < 8 * kC * W; i += blockDim.x) tab[i] = (float)(i & 1023);
    __syncthreads();
    uint32_t h = seed ^ ((blockIdx.x * 512u + threadIdx.x) * 0x9e3779b9u);
    h ^= h << 13; h ^= h >> 17; h ^= h << 5;
    uint32_t w0 = h;
    h ^= h << 13; h ^= h >> 17; h ^= h << 5;
    uint32_t w1 = h;
    float s = 0.0f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const uint32_t c = ((j < 4 ? w0 : w1) >> (8 * (j & 3))) & 255u;
            const float *e = tab + (j * kC + c) * W;
            if (W == 2) {
                const float2 v = *reinterpret_cast<const float2 *>(e);
                s += v.x; s += v.y;
            } else {
                const float4 v = *reinterpret_cast<const float4 *>(e);
                s += v.x; s += v.y; s += v.z; s += v.w;
            }
        }
        const uint32_t t = w0;
        w0 = w1;
        w1 = (t << 7 | t >> 25) ^ (uint32_t)it;
    }
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- per-list summaries for list-level pruning (record layout: list_record_bytes) ----
// One workgroup per inverted list: a presence bitmap of 256 bits per subspace is filled from
// the list's codes, then one wave per subspace writes the set codes in ascending order.
__global__ __launch_bounds__(256) void list_bounds_kernel(const uint8_t *__restrict__ codes,
                                                          const float *__restrict__ dlx, int64_t n,
                                                          int M, const int64_t *__restrict__ list_offsets,
                                                          uint8_t *__restrict__ out) {
    extern __shared__ __align__(16) unsigned char smem[];
    uint32_t *bits = reinterpret_cast<uint32_t *>(smem);  // [M][8]
    __shared__ float red[256];
    const int l = blockIdx.x, tid = threadIdx.x, lane = tid & 63;
    uint8_t *rec = out + (size_t)l * list_record_bytes(M);
    for (int i = tid; i < M * 8; i += blockDim.x) bits[i] = 0;
    __syncthreads();
    int64_t lo = list_offsets[l], hi = list_offsets[l + 1];
    lo = lo < 0 ? 0 : (lo > n ? n : lo);
    hi = hi < lo ? lo : (hi > n ? n : hi);
    float bmax = 0.0f;
    for (int64_t x = lo + tid; x < hi; x += blockDim.x) {
        for (int j = 0; j < M; ++j) {
            const uint32_t c = codes[(size_t)x * M + j];
            atomicOr(&bits[j * 8 + (c >> 5)], 1u << (c & 31));
        }
        bmax = fmaxf(bmax, dlx[x]);
    }
    red[tid] = bmax;
    __syncthreads();
    for (int h = blockDim.x >> 1; h > 0; h >>= 1) {
        if (tid < h) red[tid] = fmaxf(red[tid], red[tid + h]);
        __syncthreads();
    }
    if (tid == 0) *reinterpret_cast<float *>(rec + list_record_bmax_offset(M)) = red[0];
    for (int j = tid >> 6; j < M; j += blockDim.x >> 6) {   // one wave per subspace
        const uint32_t nib = (bits[j * 8 + (lane >> 3)] >> ((lane & 7) * 4)) & 15u;  // codes 4*lane..4*lane+3
        const int cnt = __popc(nib);
        int incl = cnt;                                  // inclusive prefix over the lanes
        for (int off = 1; off < 64; off <<= 1) {
            const int v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        const int total = __shfl(incl, 63);
        uint8_t *row = rec + (size_t)j * kSetCap;
        if (total == 0 || total > kSetCap) {
            row[lane] = 0;
            if (lane == 0) rec[(size_t)M * kSetCap + j] = total == 0 ? 0 : (uint8_t)kSetAny;
            continue;
        }
        const unsigned long long have = __ballot(nib != 0);
        const int fl = __ffsll((long long)have) - 1;
        const uint32_t fn = (uint32_t)__shfl((int)nib, fl);
        const uint8_t first = (uint8_t)(4 * fl + (__ffs((int)fn) - 1));
        if (lane >= total) row[lane] = first;            // padding
        int at = incl - cnt;
        for (int b = 0; b < 4; ++b)
            if ((nib >> b) & 1u) row[at++] = (uint8_t)(4 * lane + b);
        if (lane == 0) rec[(size_t)M * kSetCap + j] = (uint8_t)total;
    }
}

// ---- scan head: {code bytes 0..7, landmark distance} of every vector as one 12-byte record ----
__global__ void pack_scan_head_kernel(const uint8_t *__restrict__ codes, const float *__restrict__ dlx,
                                      int64_t n, int M, uint32_t *__restrict__ head) {
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
         i += (int64_t)gridDim.x * blockDim.x) {
        const uint2 c = *reinterpret_cast<const uint2 *>(codes + (size_t)i * M);  // M % 8 == 0
        head[3 * i + 0] = c.x;
        head[3 * i + 1] = c.y;
        head[3 * i + 2] = __float_as_uint(dlx[i]);
    }
}

// ---- tiled codes: blocks of 64 vectors, 16-byte pieces of a block's vectors contiguous ----
// One thread per (vector slot, piece); slots beyond n are written as zeros.
__global__ void pack_codes_tiled_kernel(const uint8_t *__restrict__ codes, int64_t n, int M,
                                        uint4 *__restrict__ tiled) {
    const int npiece = M >> 4;
    const int64_t total = ((n + 63) / 64) * 64 * npiece;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < total;
         t += (int64_t)gridDim.x * blockDim.x) {
        // t enumerates the output in order: block, piece, lane
        const int lane = (int)(t & 63);
        const int64_t bp = t >> 6;
        const int piece = (int)(bp % npiece);
        const int64_t x = (bp / npiece) * 64 + lane;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (x < n) v = *reinterpret_cast<const uint4 *>(codes + (size_t)x * M + piece * 16);
        tiled[t] = v;
    }
}

// ---- centroid training (Lloyd's k-means; Sections 2.2, 3.1, 6.1) ----
// Initial centroids: cent[c][t] = x[init_rows[c]][col0 + t].
__global__ void kmeans_init_kernel(const float *__restrict__ x, int64_t ns, int64_t stride, int col0,
                                   int dim, const int32_t *__restrict__ init_rows, int K,
                                   float *__restrict__ cent) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= K * dim) return;
    int64_t r = init_rows[e / dim];
    r = r < 0 ? 0 : (r >= ns ? ns - 1 : r);
    cent[e] = x[(size_t)r * stride + col0 + e % dim];
}

// Update step with every rounding fixed: thread (c, t) walks the rows in ascending order and
// adds, in float64, coordinate col0 + t of every row assigned to c; the centroid becomes
// sum / count rounded once to binary32; a cluster without rows keeps its centroid.
// Assignments are read as bytes (ABYTES = 1) or 32-bit integers (ABYTES = 4) with a stride,
// staged through LDS a chunk at a time.  grid.x * blockDim.x >= K * dim; grid.y = number of
// independent clusterings y (PQ subspaces): columns col0 + y*dim.., assignment element y of
// every row, centroid block y.
template <int ABYTES>
__global__ __launch_bounds__(256) void kmeans_update_kernel(const float *__restrict__ x, int64_t ns,
                                                            int64_t stride, int col0, int dim,
                                                            const void *__restrict__ assign,
                                                            int64_t astride, int K,
                                                            float *__restrict__ cent) {
    constexpr int kChunk = 2048;
    __shared__ int32_t a_lds[kChunk];
    const int y = blockIdx.y;
    col0 += y * dim;
    cent += (size_t)y * K * dim;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    const bool live = e < K * dim;
    const int c = live ? e / dim : -1;
    const int t = live ? e % dim : 0;
    double sum = 0.0;
    int64_t count = 0;
    for (int64_t i0 = 0; i0 < ns; i0 += kChunk) {
        const int m = ns - i0 < kChunk ? (int)(ns - i0) : kChunk;
        __syncthreads();
        for (int i = threadIdx.x; i < m; i += blockDim.x) {
            const size_t at = (size_t)(i0 + i) * astride + y;
            a_lds[i] = ABYTES == 1 ? (int32_t) static_cast<const uint8_t *>(assign)[at]
                                   : static_cast<const int32_t *>(assign)[at];
        }
        __syncthreads();
        for (int i = 0; i < m; ++i) {
            if (a_lds[i] == c) {
                sum += (double)x[(size_t)(i0 + i) * stride + col0 + t];
                ++count;
            }
        }
    }
    if (live && count > 0) cent[e] = (float)(sum / (double)count);
}

// ---- gamma from a confidence level p (Section 3.2), empirical route ----
// One workgroup per sampled data vector x: landmark l = PQ reconstruction of x; for every
// sampled query the value 1 - cos(x - l, q - l) (half waves, 16 bytes per lane and step);
// the values are sorted in LDS (bitonic) and the one of the given rank is gamma_x; the
// global gamma is the minimum over x (values are >= 0, so their bit patterns order like
// the numbers and a 32-bit atomic minimum does it).
struct GammaArgs {
    const float *base;
    const uint8_t *codes;
    const float *codebooks;
    const int32_t *rows;
    const float *queries;
    int64_t n;
    int32_t d, M, Q, npow2, rank;
    float *gamma_x;
    uint32_t *gamma_bits;
};

__global__ __launch_bounds__(256) void gamma_kernel(const GammaArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *l = reinterpret_cast<float *>(smem);   // [d]
    float *u = l + a.d;                           // [d]
    float *vals = u + a.d;                        // [npow2]
    __shared__ float red[256];
    const int tid = threadIdx.x;
    int64_t r = a.rows[blockIdx.x];
    r = r < 0 ? 0 : (r >= a.n ? a.n - 1 : r);
    const int dsub = a.d / a.M;
    float part = 0.0f;
    for (int t = tid; t < a.d; t += blockDim.x) {
        const int j = t / dsub;
        const float lt = a.codebooks[((size_t)j * kC + a.codes[(size_t)r * a.M + j]) * dsub + t % dsub];
        const float ut = a.base[(size_t)r * a.d + t] - lt;
        l[t] = lt;
        u[t] = ut;
        part = __builtin_fmaf(ut, ut, part);
    }
    red[tid] = part;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (tid < h) red[tid] += red[tid + h];
        __syncthreads();
    }
    const float nu = trim::sqrt_rn(red[0]);
    const int half = tid >> 5, lane32 = tid & 31, nhalf = blockDim.x >> 5;
    const float4 *l4 = reinterpret_cast<const float4 *>(l);
    const float4 *u4 = reinterpret_cast<const float4 *>(u);
    const int ng = a.d >> 2;
    for (int qi = half; qi < a.Q; qi += nhalf) {
        const float4 *q4 = reinterpret_cast<const float4 *>(a.queries + (size_t)qi * a.d);
        float dot = 0.0f, nn = 0.0f;
        for (int g = lane32; g < ng; g += 32) {
            const float4 qv = q4[g], lv = l4[g], uv = u4[g];
            float w;
            w = qv.x - lv.x; dot = __builtin_fmaf(w, uv.x, dot); nn = __builtin_fmaf(w, w, nn);
            w = qv.y - lv.y; dot = __builtin_fmaf(w, uv.y, dot); nn = __builtin_fmaf(w, w, nn);
            w = qv.z - lv.z; dot = __builtin_fmaf(w, uv.z, dot); nn = __builtin_fmaf(w, w, nn);
            w = qv.w - lv.w; dot = __builtin_fmaf(w, uv.w, dot); nn = __builtin_fmaf(w, w, nn);
        }
        dot = half_reduce(dot);
        nn = half_reduce(nn);
        if (lane32 == 0) {
            const float den = trim::sqrt_rn(nn) * nu;
            vals[qi] = 1.0f - (den > 0.0f ? dot / den : 0.0f);
        }
    }
    for (int i = a.Q + tid; i < a.npow2; i += blockDim.x) vals[i] = __builtin_inff();
    __syncthreads();
    for (int k = 2; k <= a.npow2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < a.npow2; i += blockDim.x) {
                const int p = i ^ j;
                if (p > i) {
                    const float x = vals[i], y = vals[p];
                    const bool up = (i & k) == 0;
                    if ((x > y) == up) { vals[i] = y; vals[p] = x; }
                }
            }
            __syncthreads();
        }
    }
    if (tid == 0) {
        const float g = vals[a.rank];
        if (a.gamma_x) a.gamma_x[blockIdx.x] = g;
        atomicMin(a.gamma_bits, __float_as_uint(g < 0.0f ? 0.0f : g));
    }
}

// ---- gamma from a confidence level p for standard-normal queries (Section 3.2) ----
// The theorem of Section 3.2 gives, for a query Q ~ N(0, I) rotated so that x - l lies on the
// first axis and l in the plane of the first two: Z^2 = A / (A + B + C), A = (Q1 + h1)^2,
// B = (Q2 - h2)^2, C = the sum of the squares of the other d - 2 coordinates,
// h1 = (x - l).l / |x - l|, h2 = sqrt(|l|^2 - h1^2); the transform theorem turns the
// distribution of Z^2 into that of 1 - Z.  Only (Q1, Q2, C) of a variate row matter, and they
// do not depend on x: a first kernel reduces every row of normal variates to that triple.
__global__ void normal_triples_kernel(const float *__restrict__ normals, int64_t Q, int d,
                                      double *__restrict__ triples) {
    const int64_t r = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= Q) return;
    const float *row = normals + (size_t)r * d;
    double c = 0.0;
    for (int t = 2; t < d; ++t) c += (double)row[t] * (double)row[t];
    triples[3 * r + 0] = (double)row[0];
    triples[3 * r + 1] = (double)row[1];
    triples[3 * r + 2] = c;
}

// One workgroup per sampled data vector: h1 and h2 in binary64, Z^2 for every triple, a bitonic
// sort of the Z^2 in LDS, then the largest y on the grid y_i = 2 i / (grid - 1) whose
// F_{1-Z}(y_i) = 1/2 -+ F_{Z^2}((1 - y_i)^2) / 2 (minus for y <= 1) is at most 1 - p
// (F_{1-Z} rises with y: binary search over i).  gamma = min over the vectors (32-bit atomic
// minimum on the bit pattern of the non-negative binary32 result).
struct GammaNormalArgs {
    const float *base;
    const uint8_t *codes;
    const float *codebooks;
    const int32_t *rows;
    const double *triples;
    int64_t n;
    int32_t d, M, Q, npow2, grid;
    double one_minus_p;
    float *gamma_x;
    uint32_t *gamma_bits;
};

__global__ __launch_bounds__(256) void gamma_normal_kernel(const GammaNormalArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    double *z2 = reinterpret_cast<double *>(smem);   // [npow2]
    __shared__ double red[3][256];
    const int tid = threadIdx.x;
    int64_t r = a.rows[blockIdx.x];
    r = r < 0 ? 0 : (r >= a.n ? a.n - 1 : r);
    const int dsub = a.d / a.M;
    double ul = 0.0, uu = 0.0, ll = 0.0;
    for (int t = tid; t < a.d; t += blockDim.x) {
        const int j = t / dsub;
        const double lt = (double)a.codebooks[((size_t)j * kC + a.codes[(size_t)r * a.M + j]) * dsub + t % dsub];
        const double ut = (double)a.base[(size_t)r * a.d + t] - lt;
        ul += ut * lt; uu += ut * ut; ll += lt * lt;
    }
    red[0][tid] = ul; red[1][tid] = uu; red[2][tid] = ll;
    __syncthreads();
    for (int h = 128; h > 0; h >>= 1) {
        if (tid < h) { red[0][tid] += red[0][tid + h]; red[1][tid] += red[1][tid + h]; red[2][tid] += red[2][tid + h]; }
        __syncthreads();
    }
    // a vector equal to its landmark has no angle: 1 - Z counts as 1 for every query (cos = 0)
    const bool no_angle = !(red[1][0] > 0.0);
    const double h1 = no_angle ? 0.0 : red[0][0] / sqrt(red[1][0]);
    const double h2sq = red[2][0] - h1 * h1;
    const double h2 = h2sq > 0.0 ? sqrt(h2sq) : 0.0;
    for (int i = tid; i < a.npow2; i += blockDim.x) {
        double v = __builtin_inf();
        if (i < a.Q) {
            const double q1 = a.triples[3 * (size_t)i], q2 = a.triples[3 * (size_t)i + 1], c = a.triples[3 * (size_t)i + 2];
            const double A = (q1 + h1) * (q1 + h1), B = (q2 - h2) * (q2 - h2);
            v = no_angle ? 0.0 : A / (A + B + c);
        }
        z2[i] = v;
    }
    __syncthreads();
    for (int k = 2; k <= a.npow2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < a.npow2; i += blockDim.x) {
                const int p = i ^ j;
                if (p > i) {
                    const double x = z2[i], y = z2[p];
                    const bool up = (i & k) == 0;
                    if ((x > y) == up) { z2[i] = y; z2[p] = x; }
                }
            }
            __syncthreads();
        }
    }
    if (tid == 0) {
        // F_{1-Z}(y_i) for grid point i: the share of Z^2 values <= (1 - y_i)^2, halved either way
        auto cdf = [&](int i) {
            const double y = i == a.grid - 1 ? 2.0 : (double)i * (2.0 / (double)(a.grid - 1));
            const double v = (1.0 - y) * (1.0 - y);
            int lo = 0, hi = a.Q;                 // first index with z2 > v
            while (lo < hi) { const int mid = (lo + hi) >> 1; if (z2[mid] <= v) lo = mid + 1; else hi = mid; }
            const double f = (double)lo / (double)a.Q;
            return y <= 1.0 ? 0.5 - 0.5 * f : 0.5 + 0.5 * f;
        };
        const double limit = a.one_minus_p + 1e-12;
        int lo = -1, hi = a.grid - 1;             // largest i with cdf(i) <= limit (-1: none)
        if (cdf(hi) <= limit) lo = hi;
        else {
            if (cdf(0) <= limit) lo = 0;
            int l2 = lo < 0 ? -1 : 0;
            while (l2 >= 0 && hi - l2 > 1) {
                const int mid = (l2 + hi) >> 1;
                if (cdf(mid) <= limit) l2 = mid; else hi = mid;
            }
            lo = l2;
        }
        const double y = lo < 0 ? 0.0 : (lo == a.grid - 1 ? 2.0 : (double)lo * (2.0 / (double)(a.grid - 1)));
        const float g = (float)y;
        if (a.gamma_x) a.gamma_x[blockIdx.x] = g;
        atomicMin(a.gamma_bits, __float_as_uint(g));
    }
}

// ---- PQ encode (Section 3.3, preprocessing step 1) ----
// One thread per vector; the block stages one subspace's 256 centroids in LDS at a time.
// DSUB > 0: sub-vector length known at compile time (kept in registers); DSUB == 0: generic.
template <int DSUB>
__global__ __launch_bounds__(256) void encode_kernel(const float *__restrict__ base, int64_t n,
                                                     int d, const float *__restrict__ codebooks,
                                                     int M, int dsub_rt,
                                                     uint8_t *__restrict__ codes,
                                                     float *__restrict__ dlx) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *cb = reinterpret_cast<float *>(smem);  // [256][dsub]
    const int dsub = DSUB > 0 ? DSUB : dsub_rt;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    const float *x = base + (size_t)(valid ? i : 0) * d;
    float tot = 0.0f;
    uint32_t packed = 0;
    for (int j = 0; j < M; ++j) {
        __syncthreads();
        for (int e = threadIdx.x; e < kC * dsub; e += blockDim.x)
            cb[e] = codebooks[(size_t)j * kC * dsub + e];
        __syncthreads();
        float best = __builtin_inff();
        int arg = 0;
        if constexpr (DSUB > 0) {
            float xr[DSUB];
#pragma unroll
            for (int t = 0; t < DSUB; ++t) xr[t] = x[j * DSUB + t];
            for (int c = 0; c < kC; ++c) {
                float acc = 0.0f;
#pragma unroll
                for (int t = 0; t < DSUB; ++t) {
                    const float e = xr[t] - cb[c * DSUB + t];
                    acc = __builtin_fmaf(e, e, acc);
                }
                if (acc < best) { best = acc; arg = c; }
            }
        } else {
            for (int c = 0; c < kC; ++c) {
                float acc = 0.0f;
                for (int t = 0; t < dsub; ++t) {
                    const float e = x[j * dsub + t] - cb[c * dsub + t];
                    acc = __builtin_fmaf(e, e, acc);
                }
                if (acc < best) { best = acc; arg = c; }
            }
        }
        tot = tot + best;
        packed |= (uint32_t)arg << (8 * (j & 3));
        if ((j & 3) == 3) {
            if (valid) *reinterpret_cast<uint32_t *>(codes + (size_t)i * M + (j - 3)) = packed;
            packed = 0;
        }
    }
    if (valid) dlx[i] = trim::sqrt_rn(tot);
}

// ---- PQ encode with 16 centroids per subspace (4-bit codes; Section 6.1, FastScan variants) ----
// One thread per vector; a subspace's 16 centroids are read through the cache (every thread of
// the block reads the same ones).  PACKED: two codes per byte, the even subspace's in the low
// half (the stored index); else one byte per subspace (the assignments training works on).
template <bool PACKED>
__global__ __launch_bounds__(256) void encode_fs_kernel(const float *__restrict__ base, int64_t n, int d,
                                                        const float *__restrict__ codebooks, int m,
                                                        int dsub, uint8_t *__restrict__ codes,
                                                        float *__restrict__ dlx) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *cb = reinterpret_cast<float *>(smem);  // [2][16][dsub]: the two subspaces of one code byte
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const bool valid = i < n;
    const float *x = base + (size_t)(valid ? i : 0) * d;
    float tot = 0.0f;
    for (int jb = 0; jb < m / 2; ++jb) {
        __syncthreads();
        for (int e = threadIdx.x; e < 2 * kC4 * dsub; e += blockDim.x)
            cb[e] = codebooks[(size_t)jb * 2 * kC4 * dsub + e];
        __syncthreads();
        uint32_t byte = 0;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int j = 2 * jb + h;
            float best = __builtin_inff();
            int arg = 0;
            for (int c = 0; c < kC4; ++c) {
                float acc = 0.0f;
                for (int t = 0; t < dsub; ++t) {
                    const float e = x[j * dsub + t] - cb[(h * kC4 + c) * dsub + t];
                    acc = __builtin_fmaf(e, e, acc);
                }
                if (acc < best) { best = acc; arg = c; }
            }
            tot = tot + best;
            if (PACKED) byte |= (uint32_t)arg << (4 * h);
            else if (valid) codes[(size_t)i * m + j] = (uint8_t)arg;
        }
        if (PACKED && valid) codes[(size_t)i * (m / 2) + jb] = (uint8_t)byte;
    }
    if (valid && dlx) dlx[i] = trim::sqrt_rn(tot);
}

// ---- stand-alone distance table for 4-bit codes: lut[q][j][c], c < 16 ----
// grid (ceil(m/2 / bper), nq); each block writes the entries of bper code bytes of one query.
__global__ __launch_bounds__(256) void lut_fs_kernel(const float *__restrict__ queries, int d,
                                                     const float *__restrict__ codebooks, int m,
                                                     int dsub, int bper, float *__restrict__ lut) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *q_lds = reinterpret_cast<float *>(smem);
    const int64_t q = blockIdx.y;
    const int b0 = blockIdx.x * bper;
    const int nb = b0 + bper <= m / 2 ? bper : m / 2 - b0;
    for (int t = threadIdx.x; t < d; t += blockDim.x) q_lds[t] = queries[(size_t)q * d + t];
    __syncthreads();
    build_table_rows<true>(lut + ((size_t)q * m + 2 * b0) * kC4, q_lds, codebooks, dsub, b0, nb);
}

// ---- stand-alone distance table (Section 3.3, query-processing operation 1) ----
// grid (ceil(M / jper), nq); each block writes jper table rows of one query.
__global__ __launch_bounds__(256) void lut_kernel(const float *__restrict__ queries, int d,
                                                  const float *__restrict__ codebooks, int M,
                                                  int dsub, int jper, float *__restrict__ lut) {
    extern __shared__ __align__(16) unsigned char smem[];
    float *q_lds = reinterpret_cast<float *>(smem);
    const int64_t q = blockIdx.y;
    const int j0 = blockIdx.x * jper;
    const int nj = j0 + jper <= M ? jper : M - j0;
    for (int t = threadIdx.x; t < d; t += blockDim.x) q_lds[t] = queries[(size_t)q * d + t];
    __syncthreads();
    build_table_rows(lut + ((size_t)q * M + j0) * kC, q_lds, codebooks, dsub, j0, nj);
}

// ---- distance table on the matrix cores (expanded form) ----
// T[q][j][c] = max(0, (||q_j||^2 + ||c||^2) - 2 q_j.c).  One wave computes a tile of 16 queries
// x 256 centroids of one subspace: the cross terms are 16 MFMA tiles 16x16 with depth 4
// (v_mfma_f32_16x16x4_f32; two of them per tile for sub-vectors of length 8).
// Operand layout of that instruction for lane l: A[row l%16][k l/16], B[k l/16][col l%16],
// D[row 4*(l/16)+r][col l%16] in result register r.
// The contraction depth is only d/M, so each MFMA (256 FMAs ... per 1 KB stored) leaves the
// kernel bound by writing the table, not by the matrix cores.
template <int DSUB>
__global__ __launch_bounds__(256) void lut_mfma_kernel(const float *__restrict__ queries, int64_t nq,
                                                       int d, const float *__restrict__ codebooks,
                                                       int M, float *__restrict__ lut) {
    typedef float v4f __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.y * 4 + (threadIdx.x >> 6);
    if (j >= M) return;  // whole wave
    const int64_t q0 = (int64_t)blockIdx.x * 16;
    const int li = lane & 15, lg = lane >> 4;
    // A operand: query row q0+li, elements k = lg (and lg+4 for DSUB == 8)
    const int64_t qa = q0 + li < nq ? q0 + li : nq - 1;
    const float *qrow = queries + (size_t)qa * d + (size_t)j * DSUB;
    const float a0 = qrow[lg];
    const float a1 = DSUB == 8 ? qrow[lg + 4] : 0.0f;
    // squared norms of the 4 query rows this lane stores (rows 4*lg + r)
    float qn[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int64_t qr = q0 + 4 * lg + r < nq ? q0 + 4 * lg + r : nq - 1;
        const float *p = queries + (size_t)qr * d + (size_t)j * DSUB;
        float acc = 0.0f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) acc = __builtin_fmaf(p[t], p[t], acc);
        qn[r] = acc;
    }
    const float *cb = codebooks + (size_t)j * kC * DSUB;
    for (int c0 = 0; c0 < kC; c0 += 16) {
        const float *crow = cb + (size_t)(c0 + li) * DSUB;   // centroid column li of this tile
        float cn = 0.0f;
#pragma unroll
        for (int t = 0; t < DSUB; ++t) cn = __builtin_fmaf(crow[t], crow[t], cn);
        v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a0, crow[lg], acc, 0, 0, 0);
        if (DSUB == 8) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a1, crow[lg + 4], acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t q = q0 + 4 * lg + r;
            if (q < nq) {
                const float t = __builtin_fmaf(-2.0f, acc[r], qn[r] + cn);
                lut[((size_t)q * M + j) * kC + c0 + li] = t > 0.0f ? t : 0.0f;
            }
        }
    }
}

// ---- range search: offsets from per-chunk counts (single workgroup) ----
// counts [nq*nsplit] -> chunk_base [nq*nsplit] (exclusive prefix), out_offsets [nq+1],
// *required = total.
__global__ __launch_bounds__(1024) void range_offsets_kernel(const int32_t *__restrict__ counts,
                                                             int64_t nq, int nsplit,
                                                             int64_t *__restrict__ chunk_base,
                                                             int64_t *__restrict__ out_offsets,
                                                             int64_t *__restrict__ required) {
    __shared__ int64_t part[1024];
    const int64_t total_items = nq * nsplit;
    const int T = blockDim.x;
    const int64_t per = (total_items + T - 1) / T;
    const int64_t lo = (int64_t)threadIdx.x * per;
    const int64_t hi = lo + per < total_items ? lo + per : total_items;
    int64_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += counts[i];
    part[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t run = 0;
        for (int t = 0; t < T; ++t) { const int64_t v = part[t]; part[t] = run; run += v; }
        out_offsets[nq] = run;
        if (required) *required = run;
    }
    __syncthreads();
    int64_t run = part[threadIdx.x];
    for (int64_t i = lo; i < hi; ++i) {
        chunk_base[i] = run;
        if (i % nsplit == 0) out_offsets[i / nsplit] = run;
        run += counts[i];
    }
}

// ---- range search: write the results of one (query, chunk) in scan order ----
struct RangeFillArgs {
    const float *base;
    const int32_t *ids;
    const float *queries;
    const int64_t *list_offsets;
    const int32_t *probes;
    int64_t n;
    int32_t d, nlist, nseg, max_cand, chunk, nsplit;
    const uint32_t *result_mask;
    int64_t rmask_words;
    const float *result_d2;   // exact distance of each result, by scan-order number
    const int64_t *chunk_base;
    int32_t *out_ids;
    float *out_d2;
    int64_t capacity;
    uint32_t off_q, off_segp, off_segd, off_list;
};

__global__ __launch_bounds__(256) void range_fill_kernel(const RangeFillArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    int *segp = reinterpret_cast<int *>(smem + a.off_segp);
    int *segd = reinterpret_cast<int *>(smem + a.off_segd);
    int *list = reinterpret_cast<int *>(smem + a.off_list);  // [2048] scan-order numbers
    __shared__ int s_total;

    const int tid = threadIdx.x, T = blockDim.x;
    const int lane = tid & (kWave - 1);
    const int64_t q = blockIdx.x;
    const int split = blockIdx.y;
    const int nseg = a.nseg > 0 ? a.nseg : 1;

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
        segd[p] = (int)s;
        segp[p + 1] = (int)(e - s);
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
        s_total = (int)run;
    }
    __syncthreads();
    const int total = s_total;
    const int c_begin = split * a.chunk;
    if (c_begin >= total) return;
    const int c_end = c_begin + a.chunk < total ? c_begin + a.chunk : total;
    int64_t out = a.chunk_base[(size_t)q * a.nsplit + split];

    // rounds of 64 mask words (2048 candidates); wave 0 expands set bits in order
    for (int r0 = c_begin; r0 < c_end; r0 += 2048) {
        __shared__ int s_cnt;
        if (tid < kWave) {
            const int c_w = r0 + lane * 32;
            uint32_t w = 0;
            if (c_w < c_end) w = a.result_mask[(size_t)q * a.rmask_words + (c_w >> 5)];
            int cnt = __popc(w);
            int incl = cnt;  // inclusive prefix over the wave
#pragma unroll
            for (int o = 1; o < kWave; o <<= 1) {
                const int v = __shfl_up(incl, o);
                if (lane >= o) incl += v;
            }
            int at = incl - cnt;
            while (w) {
                const int b = __ffs((int)w) - 1;
                w &= w - 1;
                list[at++] = c_w + b;
            }
            if (lane == kWave - 1) s_cnt = incl;
        }
        __syncthreads();
        const int cnt = s_cnt;
        for (int i = tid; i < cnt; i += T) {
            if (out + i >= a.capacity) break;
            const int c = list[i];
            // segment of c by binary search over the prefix table
            int lo = 0, hi = nseg - 1;
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (c >= segp[mid + 1]) lo = mid + 1; else hi = mid;
            }
            const int pos = c + segd[lo];
            a.out_ids[out + i] = a.ids ? a.ids[pos] : pos;
            a.out_d2[out + i] = a.result_d2[(size_t)q * a.rmask_words * 32 + c];   // as the search computed it
        }
        out += cnt;
        __syncthreads();
    }
}

// Half-wave totals of N (32, 16 or 8) lane sums per lane at once: v[i] is the calling lane's share
// of sum i; lane l of the half wave returns the total of sum l >> (5 - log2 N).  The additions are
// those of half_reduce, pair by pair (lane ^ 16, ^ 8, ^ 4, ^ 2, ^ 1; binary32 addition commutes,
// so it does not matter which lane of a pair adds): while a lane still holds several sums, it
// hands half of them to its partner at each step and keeps the other half, so N sums take
// N - 1 exchanges (plus one per remaining step) instead of 5 N.
template <int BIT>
__device__ __forceinline__ float lane_xor(float x) {
    const int v = __float_as_int(x);
    if constexpr (BIT == 16) return __int_as_float(__builtin_amdgcn_ds_swizzle(v, 0x401F));
    else if constexpr (BIT == 8) return __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x128, 0xf, 0xf, false));  // row rotation by 8
    else if constexpr (BIT == 4) return __int_as_float(__builtin_amdgcn_ds_swizzle(v, 0x101F));
    else if constexpr (BIT == 2) return __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false));
    else return __int_as_float(__builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false));
}
template <int N, int BIT, int CAP>
__device__ __forceinline__ void reduce_step(float (&v)[CAP], int lane32) {
    if constexpr (N > 1) {
        const bool up = (lane32 & BIT) != 0;   // these lanes keep the upper half of the sums
#pragma unroll
        for (int i = 0; i < N / 2; ++i) {
            const float keep = up ? v[i + N / 2] : v[i];
            const float send = up ? v[i] : v[i + N / 2];
            v[i] = keep + lane_xor<BIT>(send);
        }
    } else {
        v[0] = v[0] + lane_xor<BIT>(v[0]);
    }
}
template <int N>
__device__ __forceinline__ float reduce_pairs(float (&v)[N], int lane32) {
    static_assert(N == 32 || N == 16 || N == 8, "sums per lane");
    reduce_step<N, 16>(v, lane32);
    reduce_step<(N / 2 > 1 ? N / 2 : 1), 8>(v, lane32);
    reduce_step<(N / 4 > 1 ? N / 4 : 1), 4>(v, lane32);
    reduce_step<(N / 8 > 1 ? N / 8 : 1), 2>(v, lane32);
    reduce_step<(N / 16 > 1 ? N / 16 : 1), 1>(v, lane32);
    return v[0];
}

// ---- coarse probe selection (Section 6.1: IVFPQ with C' lists, nprobe probed) ----
// One workgroup handles QT queries: every centroid row is read once and measured against
// all QT queries (exact distances by half waves, rounding order as in exact_d2_half; the lane
// sums of eight rows x QT queries are reduced together), then
// the nprobe smallest of each query's (distance bits, list id) keys are selected in LDS
// (bitonic runs and pairwise merges) and their ids are written in ascending key order.
template <int QT>
__global__ __launch_bounds__(512) void ivf_probe_kernel(const float *__restrict__ queries,
                                                        int64_t nq, int d,
                                                        const float *__restrict__ centroids,
                                                        int nlist, int npow2, int nprobe,
                                                        int32_t *__restrict__ probes) {
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long *keys = reinterpret_cast<unsigned long long *>(smem);  // [QT][npow2]
    float *q_lds = reinterpret_cast<float *>(smem + (size_t)QT * npow2 * 8);  // [QT][d]
    const int tid = threadIdx.x, T = blockDim.x;
    const int64_t q0 = (int64_t)blockIdx.x * QT;
    const int nqt = (int)(nq - q0 < QT ? nq - q0 : QT);
    for (int t = tid; t < QT * d; t += T) {
        const int qi = t / d;
        q_lds[t] = qi < nqt ? queries[(size_t)q0 * d + t] : 0.0f;
    }
    for (int i = tid; i < QT * npow2; i += T) keys[i] = ~0ull;
    __syncthreads();
    const int lane32 = tid & 31;
    const int ng = d >> 2;
    const int nh = T >> 5;
    // Short vectors (at most 128 values: one 16-byte group per lane of the half wave): the lane's
    // share of every query stays in registers, and the distance loop reads no LDS at all.
    const bool in_regs = ng <= 32;
    float qrx[QT], qry[QT], qrz[QT], qrw[QT];
#pragma unroll
    for (int qi = 0; qi < QT; ++qi) {
        float4 t = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (in_regs && lane32 < ng) t = *reinterpret_cast<const float4 *>(q_lds + qi * d + 4 * lane32);
        qrx[qi] = t.x; qry[qi] = t.y; qrz[qi] = t.z; qrw[qi] = t.w;
    }
    // A half wave takes kRows (8; 4 with 8 queries) consecutive centroid rows per pass (their loads in flight together)
    // against the QT queries: kRows x QT lane sums per lane, reduced together (reduce_pairs), after
    // which lane l of the half wave holds the distance of pair l >> kShift = row * QT + query and
    // the pairs' keys are stored side by side.
    constexpr int kRows = QT == 8 ? 4 : 8, NP = kRows * QT;
    constexpr int kShift = NP == 32 ? 0 : NP == 16 ? 1 : 2;
    for (int l0 = (tid >> 5) * kRows; l0 < nlist; l0 += nh * kRows) {
        // (rows past the end: the last row again, never stored)
        const float4 *row0 = reinterpret_cast<const float4 *>(centroids + (size_t)l0 * d);
        const int last = nlist - 1 - l0;     // >= 0
        float acc[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) acc[i] = 0.0f;
        for (int g = lane32; g < ng; g += 32) {
            float4 x[kRows];
#pragma unroll
            for (int r = 0; r < kRows; ++r) x[r] = row0[(r < last ? r : last) * ng + g];
#pragma unroll
            for (int qi = 0; qi < QT; ++qi) {
                float4 qv = make_float4(qrx[qi], qry[qi], qrz[qi], qrw[qi]);
                if (!in_regs) qv = *reinterpret_cast<const float4 *>(q_lds + qi * d + 4 * g);
#pragma unroll
                for (int r = 0; r < kRows; ++r) {
                    float e, a0 = acc[r * QT + qi];
                    e = qv.x - x[r].x; a0 = __builtin_fmaf(e, e, a0);
                    e = qv.y - x[r].y; a0 = __builtin_fmaf(e, e, a0);
                    e = qv.z - x[r].z; a0 = __builtin_fmaf(e, e, a0);
                    e = qv.w - x[r].w; a0 = __builtin_fmaf(e, e, a0);
                    acc[r * QT + qi] = a0;
                }
            }
        }
        const float dist = reduce_pairs<NP>(acc, lane32);
        const int pair = lane32 >> kShift;
        const int l = l0 + pair / QT, qi = pair % QT;
        // a distance is >= 0 (or NaN): its bit pattern orders like its value
        if ((lane32 & ((1 << kShift) - 1)) == 0 && l < nlist)
            keys[(size_t)qi * npow2 + l] = ((unsigned long long)__float_as_uint(dist) << 32) | (uint32_t)l;
    }
    __syncthreads();
    // Short probe lists (nprobe <= 64, at least 256 lists): one wave per query.  The keys are seen
    // as 64 S interleaved columns (S = 1 for nprobe <= 32, else 2; lane l, slot s holds column
    // 64 s + l); the nprobe-th smallest of the column minima (sorted across lanes and slots) is
    // an upper bound of the nprobe-th smallest key, so only the keys not above it can be
    // selected.  If at most 64 S keys qualify they are sorted the same way and the first nprobe
    // are the result; otherwise (rare) the whole workgroup takes the general path below.  Keys
    // are distinct, so either path gives the same list.
    __shared__ int general_path;
    if (nprobe <= 64 && npow2 >= 256) {
        if (tid == 0) general_path = 0;
        __syncthreads();
        const int wave = tid >> 6, lane = tid & 63;
        const int S = nprobe <= 32 ? 1 : 2;
        // ascending bitonic sort of the 64 S elements (element e = 64 slot + lane)
        auto sort_across = [&](unsigned long long (&key)[2]) {
            for (int size = 2; size <= 64 * S; size <<= 1) {
                for (int j = size >> 1; j > 0; j >>= 1) {
                    if (j >= 64) {            // partner in the other slot of the same lane (S == 2, size 128: ascending)
                        if (key[1] < key[0]) { const unsigned long long t = key[0]; key[0] = key[1]; key[1] = t; }
                        continue;
                    }
#pragma unroll
                    for (int sl = 0; sl < 2; ++sl) {
                        if (sl >= S) break;
                        const uint32_t olo = (uint32_t)__shfl_xor((int)(uint32_t)key[sl], j);
                        const uint32_t ohi = (uint32_t)__shfl_xor((int)(uint32_t)(key[sl] >> 32), j);
                        const unsigned long long other = ((unsigned long long)ohi << 32) | olo;
                        const int e = 64 * sl + lane;
                        const bool keep_min = ((lane & j) == 0) == ((e & size) == 0);
                        if (keep_min ? other < key[sl] : other > key[sl]) key[sl] = other;
                    }
                }
            }
        };
        unsigned long long *kq = keys + ((size_t)(wave < nqt ? wave : 0) * npow2);
        unsigned long long cut = 0;
        int c = 0;
        if (wave < nqt) {
            unsigned long long cmin[2] = {~0ull, ~0ull};
            for (int i = lane; i < npow2; i += 64 * S) {
                cmin[0] = kq[i] < cmin[0] ? kq[i] : cmin[0];
                if (S == 2) cmin[1] = kq[i + 64] < cmin[1] ? kq[i + 64] : cmin[1];
            }
            if (nprobe == 1) {   // the nearest list alone (assignment of a base set): a minimum, no sort
                unsigned long long m = cmin[0];
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) {
                    const uint32_t olo = (uint32_t)__shfl_xor((int)(uint32_t)m, off);
                    const uint32_t ohi = (uint32_t)__shfl_xor((int)(uint32_t)(m >> 32), off);
                    const unsigned long long other = ((unsigned long long)ohi << 32) | olo;
                    m = other < m ? other : m;
                }
                cmin[0] = m;       // every lane holds it: the bound below is the key itself
            } else {
                sort_across(cmin);
            }
            const unsigned long long at = (nprobe - 1) >= 64 ? cmin[1] : cmin[0];   // same choice in every lane
            const int src = (nprobe - 1) & 63;
            cut = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(at >> 32), src) << 32) |
                  (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)at, src);
            for (int i0 = 0; i0 < npow2; i0 += 64) c += __popcll(__ballot(kq[i0 + lane] <= cut));
            if (c > 64 * S) atomicOr(&general_path, 1);
        }
        __syncthreads();   // nothing has been moved yet: the general path finds every key in place
        if (!general_path) {
            if (wave < nqt) {
                // move the qualifying keys to the front (in place: none moves backwards)
                int at0 = 0;
                for (int i0 = 0; i0 < npow2; i0 += 64) {
                    const unsigned long long key = kq[i0 + lane];
                    const bool take = key <= cut;
                    const unsigned long long m = __ballot(take);
                    if (take) kq[at0 + __popcll(m & ((1ull << lane) - 1ull))] = key;
                    at0 += __popcll(m);
                }
                unsigned long long key[2];
                key[0] = lane < c ? kq[lane] : ~0ull;
                key[1] = (S == 2 && 64 + lane < c) ? kq[64 + lane] : ~0ull;
                if (nprobe > 1) sort_across(key);   // (one probe: c == 1, the key sits in lane 0)
                if (lane < nprobe) probes[(size_t)(q0 + wave) * nprobe + lane] = (int32_t)(key[0] & 0xffffffffu);
                if (64 + lane < nprobe) probes[(size_t)(q0 + wave) * nprobe + 64 + lane] = (int32_t)(key[1] & 0xffffffffu);
            }
            return;
        }
    }
    // Selection of the nprobe smallest keys of each query with bitonic networks; all sizes are
    // powers of two, so the index arithmetic is shifts and masks (lg_* are base-2 logarithms).
    // (1) runs of R >= nprobe keys are sorted, ascending and descending in turn;
    // (2) neighbouring runs are merged pairwise, keeping only the R smallest of the two: the
    //     element-wise minimum of an ascending and a descending run holds them as a bitonic
    //     sequence, which log2(R) exchange stages sort (again ascending / descending in turn);
    //     the surviving run stays where the pair's first run was, so after round r the live
    //     runs sit at multiples of R << r.  The last survivor, at 0, is ascending.
    const int lg_n = 31 - __builtin_clz(npow2);
    const int lg_half = lg_n - 1;
    int lg_r = 0;
    while ((1 << lg_r) < nprobe) ++lg_r;
    for (int lg_size = 1; lg_size <= lg_r; ++lg_size) {
        for (int lg_stride = lg_size - 1; lg_stride >= 0; --lg_stride) {
            const int stride = 1 << lg_stride;
            for (int w = tid; w < (QT << lg_half); w += T) {
                const int qi = w >> lg_half, i = w & ((1 << lg_half) - 1);
                const int lo = ((i >> lg_stride) << (lg_stride + 1)) | (i & (stride - 1));
                const int hi = lo + stride;
                const bool up = ((lo >> lg_size) & 1) == 0;
                unsigned long long *kq = keys + ((size_t)qi << lg_n);
                const unsigned long long x = kq[lo], y = kq[hi];
                if ((x > y) == up) { kq[lo] = y; kq[hi] = x; }
            }
            __syncthreads();
        }
    }
    const int R = 1 << lg_r;
    for (int lg_gap = lg_r; lg_gap < lg_n; ++lg_gap) {   // partner run = first run + (1 << lg_gap)
        const int lg_pairs = lg_n - lg_gap - 1;          // pairs per query in this round
        // element-wise minimum into the first run of each pair
        for (int w = tid; w < ((QT << lg_pairs) << lg_r); w += T) {
            const int i = w & (R - 1);
            const int pr = (w >> lg_r) & ((1 << lg_pairs) - 1);
            const int qi = w >> (lg_r + lg_pairs);
            unsigned long long *kq = keys + ((size_t)qi << lg_n) + ((size_t)pr << (lg_gap + 1));
            const unsigned long long x = kq[i], y = kq[(1 << lg_gap) + i];
            if (y < x) kq[i] = y;
        }
        __syncthreads();
        // sort the bitonic survivors: ascending for even pairs, descending for odd ones
        for (int lg_stride = lg_r - 1; lg_stride >= 0; --lg_stride) {
            const int stride = 1 << lg_stride;
            const int lg_ce = lg_r - 1;                  // exchanges per run and stage = R / 2
            for (int w = tid; w < ((QT << lg_pairs) << lg_ce); w += T) {
                const int i = w & ((1 << lg_ce) - 1);
                const int pr = (w >> lg_ce) & ((1 << lg_pairs) - 1);
                const int qi = w >> (lg_ce + lg_pairs);
                const int lo = ((i >> lg_stride) << (lg_stride + 1)) | (i & (stride - 1));
                const bool up = (pr & 1) == 0;
                unsigned long long *kq = keys + ((size_t)qi << lg_n) + ((size_t)pr << (lg_gap + 1));
                const unsigned long long x = kq[lo], y = kq[lo + stride];
                if ((x > y) == up) { kq[lo] = y; kq[lo + stride] = x; }
            }
            __syncthreads();
        }
    }
    for (int w = tid; w < nqt * nprobe; w += T) {
        const int qi = w / nprobe, p = w - qi * nprobe;
        probes[(size_t)(q0 + qi) * nprobe + p] = (int32_t)(keys[(size_t)qi * npow2 + p] & 0xffffffffu);
    }
}

// ---- processing order: queries grouped by their first probed list ----
// Single workgroup, counting sort with an LDS histogram (nbucket <= 32768 buckets; list ids
// are folded modulo nbucket, which still puts equal lists together).  Lists appear in
// ascending bucket order; the order of the queries inside a bucket is unspecified.
__global__ __launch_bounds__(1024) void query_order_kernel(const int32_t *__restrict__ probes,
                                                           int64_t nq, int nprobe, int nbucket,
                                                           int32_t *__restrict__ order) {
    extern __shared__ __align__(16) unsigned char smem[];
    int *hist = reinterpret_cast<int *>(smem);  // [nbucket], then running cursors
    __shared__ int part[16];
    const int tid = threadIdx.x, T = blockDim.x;
    for (int b = tid; b < nbucket; b += T) hist[b] = 0;
    // the first kKeep queries of a thread stay in registers for both passes, their loads in flight together
    constexpr int kKeep = 16;
    uint32_t mine[kKeep];
#pragma unroll
    for (int i = 0; i < kKeep; ++i) {
        const int64_t q = tid + (int64_t)i * T;
        mine[i] = q < nq ? (uint32_t)probes[(size_t)q * nprobe] % (uint32_t)nbucket : 0xffffffffu;
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
        if (mine[i] != 0xffffffffu) atomicAdd(&hist[mine[i]], 1);
    for (int64_t q = tid + (int64_t)kKeep * T; q < nq; q += T) {
        const uint32_t l = (uint32_t)probes[(size_t)q * nprobe];
        atomicAdd(&hist[l % (uint32_t)nbucket], 1);
    }
    __syncthreads();
    // exclusive prefix over the buckets: each thread owns a contiguous run; the runs' sums are
    // scanned inside each wave, then across the (at most 16) waves
    const int per = (nbucket + T - 1) / T;
    const int lo = tid * per < nbucket ? tid * per : nbucket;
    const int hi = lo + per < nbucket ? lo + per : nbucket;
    int sum = 0;
    for (int b = lo; b < hi; ++b) sum += hist[b];
    const int lane = tid & 63, wave = tid >> 6;
    int incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) part[wave] = incl;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < wave; ++w) before += part[w];
    int run = before + incl - sum;
    for (int b = lo; b < hi; ++b) { const int c = hist[b]; hist[b] = run; run += c; }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kKeep; ++i)
        if (mine[i] != 0xffffffffu) order[atomicAdd(&hist[mine[i]], 1)] = (int32_t)(tid + i * T);
    for (int64_t q = tid + (int64_t)kKeep * T; q < nq; q += T) {
        const uint32_t l = (uint32_t)probes[(size_t)q * nprobe];
        order[atomicAdd(&hist[l % (uint32_t)nbucket], 1)] = (int32_t)q;
    }
}

}  // namespace trim
