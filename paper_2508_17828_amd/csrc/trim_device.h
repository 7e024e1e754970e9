// Device-side building blocks of the TRIM scan for gfx950 (wave64).
//
// Rounding order (binary32, no contraction; this file is compiled with -ffp-contract=off
// and every fused multiply-add is written as __builtin_fmaf):
//   sub-vector distance : acc = fma(x_t - c_t, x_t - c_t, acc), t ascending
//   Gamma(l,q)^2        : table entries added left to right over the subspaces
//   bound (Equation 3)  : a = sqrt(s); e = a - b; g = fma((2*gamma)*a, b, e*e)
//   exact distance      : lane l of a 32-lane group owns coordinate groups l, l+32, ...
//                         (4 coordinates each, fma in order); then a 5-step butterfly
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace trim {

constexpr int kC = 256;          // centroids per subspace (the paper's C)
constexpr int kC4 = 16;          // centroids per subspace with 4-bit codes (Section 6.1: FastScan variants)
constexpr int kWave = 64;

// Layout of a query's distance table in LDS, per code BYTE.  8-bit codes: a byte selects one of
// the 256 entries of its subspace's row.  4-bit codes (FS): a byte holds the codes of two
// subspaces (even one in the low half) and selects one of 16 entries in each of two rows of 16;
// the 16 consecutive words of such a row lie in 16 different LDS banks, so lanes that read
// different entries never collide.  Everything outside the table (code loads, scan head, list
// summaries, thresholds every 8 bytes) works on code bytes and is the same for both.
template <bool FS> constexpr int kByteEntries = FS ? 2 * kC4 : kC;      // table entries per code byte
template <bool FS> constexpr uint32_t kByteRow = kByteEntries<FS> * 4;  // their bytes
template <bool FS> constexpr int kByteLookups = FS ? 2 : 1;             // lookups per code byte

struct Hit {
    float d2;
    int32_t id;
};

// Correctly rounded binary32 square root.  (The __fsqrt_rn intrinsic maps to the bare
// hardware approximation, which is within 1 ulp but not always the nearest value; sqrtf
// is expanded by the compiler into the approximation plus a correction step.)
__device__ __forceinline__ float sqrt_rn(float x) { return __builtin_sqrtf(x); }

__device__ __forceinline__ bool hit_less(float d2a, int32_t ida, float d2b, int32_t idb) {
    return d2a < d2b || (d2a == d2b && ida < idb);
}

// Squared distance between a query sub-vector held in LDS and a centroid in global memory.
__device__ __forceinline__ float subvec_sqdist(const float *__restrict__ x,
                                               const float *__restrict__ c, int dsub) {
    float acc = 0.0f;
    if ((dsub & 3) == 0) {
        for (int t = 0; t < dsub; t += 4) {
            const float4 cv = *reinterpret_cast<const float4 *>(c + t);
            const float4 xv = *reinterpret_cast<const float4 *>(x + t);
            float e;
            e = xv.x - cv.x; acc = __builtin_fmaf(e, e, acc);
            e = xv.y - cv.y; acc = __builtin_fmaf(e, e, acc);
            e = xv.z - cv.z; acc = __builtin_fmaf(e, e, acc);
            e = xv.w - cv.w; acc = __builtin_fmaf(e, e, acc);
        }
    } else {
        for (int t = 0; t < dsub; ++t) {
            const float e = x[t] - c[t];
            acc = __builtin_fmaf(e, e, acc);
        }
    }
    return acc;
}

// Distance-table rows [j0, j0+nj) of one query (Section 2.2 / Section 3.3 operation 1):
// out[(j-j0)*256 + c] = || q_j - centroid_{j,c} ||^2.  q points at the whole query (LDS or
// global), out at LDS or global.  All threads of the block take part.
// FS: j0 and nj count code bytes; byte j covers subspaces 2j and 2j+1 of 16 centroids each, dsub
// is the length of one of THOSE sub-vectors, and the entries of a byte are [2][16].
template <bool FS = false>
__device__ __forceinline__ void build_table_rows(float *__restrict__ out,
                                                 const float *__restrict__ q,
                                                 const float *__restrict__ codebooks, int dsub,
                                                 int j0, int nj) {
    const int T = blockDim.x;
    int e = threadIdx.x;
    if constexpr (FS) {
        // entry e of the slab: subspace 2*j0 + e/16, centroid e%16 -- exactly the [m][16] order
        for (; e < nj * kByteEntries<true>; e += T) {
            const int sj = 2 * j0 + (e >> 4);
            out[e] = subvec_sqdist(q + sj * dsub, codebooks + ((size_t)sj * kC4 + (e & 15)) * dsub, dsub);
        }
        return;
    }
    if (dsub == 4) {  // four entries per step so that four centroid loads are in flight
        for (; e + 3 * T < nj * kC; e += 4 * T) {
            float4 cv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                cv[u] = *reinterpret_cast<const float4 *>(codebooks + ((size_t)j0 * kC + e + u * T) * 4);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float4 xv = *reinterpret_cast<const float4 *>(q + (j0 + ((e + u * T) >> 8)) * 4);
                float acc = 0.0f, t;
                t = xv.x - cv[u].x; acc = __builtin_fmaf(t, t, acc);
                t = xv.y - cv[u].y; acc = __builtin_fmaf(t, t, acc);
                t = xv.z - cv[u].z; acc = __builtin_fmaf(t, t, acc);
                t = xv.w - cv[u].w; acc = __builtin_fmaf(t, t, acc);
                out[e + u * T] = acc;
            }
        }
    }
    for (; e < nj * kC; e += T) {
        const int j = j0 + (e >> 8);
        const int c = e & (kC - 1);
        out[e] = subvec_sqdist(q + j * dsub, codebooks + ((size_t)j * kC + c) * dsub, dsub);
    }
}

// Equation 3 from s = Gamma(l,q)^2 and b = Gamma(l,x).
__device__ __forceinline__ float plb_from_s(float s, float b, float two_gamma) {
    const float a = sqrt_rn(s);
    const float e = a - b;
    const float t = two_gamma * a;
    return __builtin_fmaf(t, b, e * e);
}

// Sum over the 32 lanes of a half wave in the tree order p[l] += p[l+h], h = 16, 8, 4, 2, 1
// (the result is exact in lane 0 of the half wave; the other lanes hold the same tree with
// operands swapped, which is the same value).  Step 16 crosses 16-lane rows (swizzle:
// lane ^ 16); steps 8..1 are rotations inside a row done by the data-parallel primitives
// of the vector ALU, so only one LDS-crossbar operation is needed per reduction.
__device__ __forceinline__ float half_reduce(float v) {
    v = v + __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(v), 0x401F));
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128, 0xf, 0xf, false));
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x124, 0xf, 0xf, false));
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x122, 0xf, 0xf, false));
    v = v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x121, 0xf, 0xf, false));
    return v;
}

// Exact squared distance, computed by the 32 lanes of a half wave (all 32 must call it
// together).  row: global, 16-byte aligned; q: LDS.  Lane 0 of the half wave returns the result.
__device__ __forceinline__ float exact_d2_half(const float *__restrict__ row,
                                               const float *__restrict__ q, int d, int lane32) {
    float acc = 0.0f;
    const float4 *r4 = reinterpret_cast<const float4 *>(row);
    const float4 *q4 = reinterpret_cast<const float4 *>(q);
    const int ng = d >> 2;
    for (int g = lane32; g < ng; g += 32) {
        const float4 xv = r4[g];
        const float4 qv = q4[g];
        float e;
        e = qv.x - xv.x; acc = __builtin_fmaf(e, e, acc);
        e = qv.y - xv.y; acc = __builtin_fmaf(e, e, acc);
        e = qv.z - xv.z; acc = __builtin_fmaf(e, e, acc);
        e = qv.w - xv.w; acc = __builtin_fmaf(e, e, acc);
    }
    return half_reduce(acc);
}

// The lane sums of four rows at once.  Every lane of the half wave brings four values (one per
// row); the value returned in lane l is the half-wave total of row 2*(l >> 4) + ((l >> 1) & 1),
// bit for bit what half_reduce gives for that row: the same pairs are added at every step
// (binary32 addition commutes, so which lane of a pair does the adding does not matter).  At
// the step of 16 and at the step of 2 every lane hands one of its two rows to its partner and
// keeps the other, so 16 exchanges become 7.
__device__ __forceinline__ float half_reduce_x4(const float (&v)[4], int lane32) {
    const bool hi = (lane32 & 16) != 0;
    // lanes 0..15 keep rows 0 and 1, lanes 16..31 rows 2 and 3
    const float s0 = hi ? v[0] : v[2], s1 = hi ? v[1] : v[3];
    float k0 = hi ? v[2] : v[0], k1 = hi ? v[3] : v[1];
    k0 = k0 + __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(s0), 0x401F));
    k1 = k1 + __int_as_float(__builtin_amdgcn_ds_swizzle(__float_as_int(s1), 0x401F));
    k0 = k0 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(k0), 0x128, 0xf, 0xf, false));
    k1 = k1 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(k1), 0x128, 0xf, 0xf, false));
    k0 = k0 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(k0), 0x124, 0xf, 0xf, false));
    k1 = k1 + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(k1), 0x124, 0xf, 0xf, false));
    // lanes with bit 1 clear keep the first of their two rows, the others the second
    const bool odd = (lane32 & 2) != 0;
    const float send = odd ? k0 : k1;
    float k = odd ? k1 : k0;
    k = k + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0x4E, 0xf, 0xf, false));  // lane ^ 2
    k = k + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(k), 0xB1, 0xf, 0xf, false));     // lane ^ 1
    return k;
}
// The row whose total half_reduce_x4 leaves in a lane, and the lanes that store the four totals.
__device__ __forceinline__ int half_reduce_x4_row(int lane32) { return ((lane32 >> 4) << 1) | ((lane32 >> 1) & 1); }
__device__ __forceinline__ bool half_reduce_x4_writer(int lane32) { return (lane32 & 13) == 0; }

// Four rows at once (same arithmetic per row as exact_d2_half; the four loads of each step
// are in flight together).  PIPE: the next step's four loads are issued before the current
// step is reduced (twice the registers; for long rows).  ONE_STEP: the caller guarantees rows of
// at most 128 values.  Returns the distance of row
// half_reduce_x4_row(lane32) (see half_reduce_x4).
template <bool PIPE, bool ONE_STEP = false>
__device__ __forceinline__ float exact_d2_half_x4(const float *__restrict__ r0,
                                                  const float *__restrict__ r1,
                                                  const float *__restrict__ r2,
                                                  const float *__restrict__ r3,
                                                  const float *__restrict__ q, int d, int lane32) {
    const float4 *rows[4] = {reinterpret_cast<const float4 *>(r0), reinterpret_cast<const float4 *>(r1),
                             reinterpret_cast<const float4 *>(r2), reinterpret_cast<const float4 *>(r3)};
    const float4 *q4 = reinterpret_cast<const float4 *>(q);
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    const int ng = d >> 2;
    float4 nxt[4];
    if (PIPE && lane32 < ng) {
#pragma unroll
        for (int u = 0; u < 4; ++u) nxt[u] = rows[u][lane32];
    }
    // (ONE_STEP: rows of at most 128 values, one 16-byte group per lane)
    for (int g = lane32; g < ng; g += 32) {
        float4 xv[4];
        if (PIPE) {
#pragma unroll
            for (int u = 0; u < 4; ++u) xv[u] = nxt[u];
            if (g + 32 < ng) {
#pragma unroll
                for (int u = 0; u < 4; ++u) nxt[u] = rows[u][g + 32];
            }
        } else {
#pragma unroll
            for (int u = 0; u < 4; ++u) xv[u] = rows[u][g];
        }
        const float4 qv = q4[g];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            float e;
            e = qv.x - xv[u].x; acc[u] = __builtin_fmaf(e, e, acc[u]);
            e = qv.y - xv[u].y; acc[u] = __builtin_fmaf(e, e, acc[u]);
            e = qv.z - xv[u].z; acc[u] = __builtin_fmaf(e, e, acc[u]);
            e = qv.w - xv[u].w; acc[u] = __builtin_fmaf(e, e, acc[u]);
        }
        if (ONE_STEP) break;
    }
    return half_reduce_x4(acc, lane32);
}

// Two long rows at once with ALL their loads in flight together (up to kDeep steps of 128 values
// per row and pass; longer rows take several passes).  For the few survivors of a short span,
// where the latency of a row's dependent steps, not bandwidth, is what the refine step waits
// for.  Same arithmetic per row as exact_d2_half.
template <int kDeep = 8>
__device__ __forceinline__ void exact_d2_half_x2_deep(const float *__restrict__ r0,
                                                      const float *__restrict__ r1,
                                                      const float *__restrict__ q, int d, int lane32,
                                                      float (&out)[2]) {
    const float4 *rows[2] = {reinterpret_cast<const float4 *>(r0), reinterpret_cast<const float4 *>(r1)};
    const float4 *q4 = reinterpret_cast<const float4 *>(q);
    float acc[2] = {0.0f, 0.0f};
    const int ng = d >> 2;
    for (int g0 = lane32; g0 < ng; g0 += 32 * kDeep) {
        float4 xv[2][kDeep];
#pragma unroll
        for (int t = 0; t < kDeep; ++t) {
            const int g = g0 + 32 * t;
            if (g < ng) {
                xv[0][t] = rows[0][g];
                xv[1][t] = rows[1][g];
            }
        }
#pragma unroll
        for (int t = 0; t < kDeep; ++t) {
            const int g = g0 + 32 * t;
            if (g < ng) {
                const float4 qv = q4[g];
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    float e;
                    e = qv.x - xv[u][t].x; acc[u] = __builtin_fmaf(e, e, acc[u]);
                    e = qv.y - xv[u][t].y; acc[u] = __builtin_fmaf(e, e, acc[u]);
                    e = qv.z - xv[u][t].z; acc[u] = __builtin_fmaf(e, e, acc[u]);
                    e = qv.w - xv[u][t].w; acc[u] = __builtin_fmaf(e, e, acc[u]);
                }
            }
        }
    }
    out[0] = half_reduce(acc[0]);
    out[1] = half_reduce(acc[1]);
}

// 4 * (byte B of w): the byte offset of a table entry inside its 1 KB row.
template <int B>
__device__ __forceinline__ uint32_t byte_times4(uint32_t w) {
    uint32_t r;
    const uint32_t two = 2;
    if constexpr (B == 0)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(two), "v"(w));
    else if constexpr (B == 1)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(two), "v"(w));
    else if constexpr (B == 2)
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(two), "v"(w));
    else
        asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(two), "v"(w));
    return r;
}

// Sum of table entries selected by 4*VEC consecutive code bytes (VEC dwords), added to s
// in subspace order.  tab points at the table row of the first of these subspaces.  Stops
// early once s > thr; a stopped sum is a lower estimate of the full sum that is still > thr.
// Read a float at a byte address of the workgroup's LDS.
__device__ __forceinline__ float lds_f32(uint32_t byte_addr) {
    typedef __attribute__((address_space(3))) const float lds_float;
    return *reinterpret_cast<lds_float *>(static_cast<uintptr_t>(byte_addr));
}

// LDS byte address of a pointer into the workgroup's LDS.
__device__ __forceinline__ uint32_t lds_addr(const void *p) {
    typedef __attribute__((address_space(3))) const char lds_char;
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_char *)p));
}

// tab_base is the LDS byte address of the table row of the first of these subspaces.
// The reads of 8 subspaces are issued together, ahead of their additions, so that their LDS
// latencies overlap; the additions stay in subspace order.
// MARK: a sum stopped half way is returned as +inf (for callers whose later tests use larger
// thresholds than the half-way one: see the remaining-minimum thresholds of the cruise).

// The same for 4-bit codes: every code byte adds two entries, the even subspace's (low half)
// first; reads of 8 bytes (16 subspaces) are issued together; tests after every 8 bytes.
template <int VEC, bool MARK>
__device__ __forceinline__ float gather_add_fs(float s, uint32_t tab_base, const uint32_t (&w)[VEC],
                                               float thr) {
    constexpr uint32_t kRow = kByteRow<true>;   // bytes of table per code byte
    constexpr uint32_t kHalf = kC4 * 4;         // from the even subspace's row to the odd one's
#pragma unroll
    for (int v0 = 0; v0 < VEC; v0 += 2) {
        float t[16];
#pragma unroll
        for (int dv = 0; dv < 2; ++dv) {
            if (v0 + dv < VEC) {
                const uint32_t cw = w[v0 + dv < VEC ? v0 + dv : 0];
                const uint32_t row = tab_base + ((v0 + dv) * 4) * kRow;
                // the low halves and the high halves of the word's four bytes, each in a byte of
                // its own: one sub-dword-addressed shift per lookup turns a byte into 4 * code
                const uint32_t lo = cw & 0x0f0f0f0fu;
                const uint32_t hi = (cw >> 4) & 0x0f0f0f0fu;
                t[8 * dv + 0] = lds_f32(row + byte_times4<0>(lo));
                t[8 * dv + 1] = lds_f32(row + kHalf + byte_times4<0>(hi));
                t[8 * dv + 2] = lds_f32(row + 1 * kRow + byte_times4<1>(lo));
                t[8 * dv + 3] = lds_f32(row + 1 * kRow + kHalf + byte_times4<1>(hi));
                t[8 * dv + 4] = lds_f32(row + 2 * kRow + byte_times4<2>(lo));
                t[8 * dv + 5] = lds_f32(row + 2 * kRow + kHalf + byte_times4<2>(hi));
                t[8 * dv + 6] = lds_f32(row + 3 * kRow + byte_times4<3>(lo));
                t[8 * dv + 7] = lds_f32(row + 3 * kRow + kHalf + byte_times4<3>(hi));
            }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
            if (v0 + i / 8 < VEC) s = s + t[i];
        if (v0 + 2 < VEC && s > thr) return MARK ? __builtin_inff() : s;
    }
    return s;
}

template <int VEC, bool MARK = false, bool FS = false>
__device__ __forceinline__ float gather_add(float s, uint32_t tab_base, const uint32_t (&w)[VEC],
                                            float thr) {
    if constexpr (FS) return gather_add_fs<VEC, MARK>(s, tab_base, w, thr);
    constexpr int kRow = kC * 4;  // bytes per table row
#pragma unroll
    for (int v0 = 0; v0 < VEC; v0 += 2) {
        float t[8];
#pragma unroll
        for (int dv = 0; dv < 2; ++dv) {
            if (v0 + dv < VEC) {
                // byte b of the code word, times 4 (the byte offset inside table row v*4+b): one
                // sub-dword-addressed shift each instead of extract + scale
                const uint32_t cw = w[v0 + dv < VEC ? v0 + dv : 0];
                const uint32_t row = tab_base + ((v0 + dv) * 4) * kRow;
                t[4 * dv + 0] = lds_f32(row + byte_times4<0>(cw));
                t[4 * dv + 1] = lds_f32(row + 1 * kRow + byte_times4<1>(cw));
                t[4 * dv + 2] = lds_f32(row + 2 * kRow + byte_times4<2>(cw));
                t[4 * dv + 3] = lds_f32(row + 3 * kRow + byte_times4<3>(cw));
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (v0 + i / 4 < VEC) s = s + t[i];
        // early abandon every 8 subspaces (see abandon_threshold)
        if (v0 + 2 < VEC && s > thr) return MARK ? __builtin_inff() : s;
    }
    return s;
}

// Table sums of two candidates over the same 8 subspaces (2 code dwords each), with the
// sixteen LDS reads issued before the first addition so that their latencies overlap.
template <bool FS = false>
__device__ __forceinline__ void gather8_pair(uint32_t tab_base, const uint32_t (&wa)[2],
                                             const uint32_t (&wb)[2], float &sa, float &sb) {
    if constexpr (FS) {   // 16 subspaces per candidate: one candidate's reads at a time
        sa = gather_add_fs<2, false>(0.0f, tab_base, wa, __builtin_inff());
        sb = gather_add_fs<2, false>(0.0f, tab_base, wb, __builtin_inff());
        return;
    }
    float ta[8], tb[8];
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        const uint32_t row = tab_base + (v * 4) * kC * 4;
        ta[4 * v + 0] = lds_f32(row + byte_times4<0>(wa[v]));
        ta[4 * v + 1] = lds_f32(row + 1 * kC * 4 + byte_times4<1>(wa[v]));
        ta[4 * v + 2] = lds_f32(row + 2 * kC * 4 + byte_times4<2>(wa[v]));
        ta[4 * v + 3] = lds_f32(row + 3 * kC * 4 + byte_times4<3>(wa[v]));
    }
#pragma unroll
    for (int v = 0; v < 2; ++v) {
        const uint32_t row = tab_base + (v * 4) * kC * 4;
        tb[4 * v + 0] = lds_f32(row + byte_times4<0>(wb[v]));
        tb[4 * v + 1] = lds_f32(row + 1 * kC * 4 + byte_times4<1>(wb[v]));
        tb[4 * v + 2] = lds_f32(row + 2 * kC * 4 + byte_times4<2>(wb[v]));
        tb[4 * v + 3] = lds_f32(row + 3 * kC * 4 + byte_times4<3>(wb[v]));
    }
    float a = 0.0f, b = 0.0f;
#pragma unroll
    for (int i = 0; i < 8; ++i) { a = a + ta[i]; b = b + tb[i]; }
    sa = a;
    sb = b;
}

template <int VEC> struct CodeVec;
template <> struct CodeVec<4> { using type = uint4; };
template <> struct CodeVec<2> { using type = uint2; };
template <> struct CodeVec<1> { using type = uint32_t; };

template <int VEC>
__device__ __forceinline__ void load_codes(uint32_t (&w)[VEC], const uint8_t *__restrict__ p) {
    if constexpr (VEC == 4) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
    } else if constexpr (VEC == 2) {
        const uint2 v = *reinterpret_cast<const uint2 *>(p);
        w[0] = v.x; w[1] = v.y;
    } else {
        w[0] = *reinterpret_cast<const uint32_t *>(p);
    }
}

// Per-list summary record (list-level pruning): for each subspace j a row of kSetCap code bytes
// (the distinct codes that occur in the list, ascending, padded with the first one), then one
// count byte per subspace (0: empty list, kSetAny: more than kSetCap distinct codes, "any
// code"), then, 4-byte aligned, the list's largest landmark distance; records are 16-byte
// multiples.
constexpr int kSetCap = 64;
constexpr int kSetAny = 255;
__host__ __device__ inline size_t list_record_bmax_offset(int M) { return ((size_t)M * (kSetCap + 1) + 3) & ~size_t(3); }
__host__ __device__ inline size_t list_record_bytes(int M) { return (list_record_bmax_offset(M) + 4 + 15) & ~size_t(15); }

// Early-abandon threshold on the running table sum (an exact shortcut, not part of the
// paper's method).  Table entries are >= 0, so the binary32 running sum never decreases, and
// for a = sqrt(s) >= b the computed bound of Equation 3 is >= (a - b)^2.  Hence, once
// s > (b + sqrt(tau))^2 by a margin that covers all rounding, the finished bound is
// certain to exceed tau and the remaining subspaces need not be read: the candidate is
// pruned exactly as the full evaluation would prune it.  Margin: the computed chain
// sqrt -> subtract -> square loses < 4 ulp (2.4e-7 relative); the threshold is inflated by
// 1e-5.  tau = +inf gives +inf (never abandons).
//
// Per threshold tau:   st = abandon_scale(tau) = c * max(sqrt(tau), 1e-15), c = 1.000025
// Per candidate:       thr = (c*b + st)^2 = c^2 (b + max(sqrt(tau),1e-15))^2 >= 1.00005 (b + sqrt(tau))^2
// (the floor keeps thr >= 1e-30, inside the normal range, so the margin argument holds for
// arbitrarily small tau as well).
//
// The cruise tests a running sum s_j (subspaces 0..j-1) against thr - rest_j, where rest_j is
// the binary32 sum over the remaining subspaces of their smallest table entry: the finished
// sum is at least s_j + (true rest) up to the rounding of at most M additions on either side,
//   s_full >= (s_j + rest_j) (1 - 2 M u),  u = 2^-24,  2 M u <= 3.1e-5 for M <= 256,
// and the subtraction thr - rest_j errs by at most u thr; the 5e-5 of the margin cover the
// 1e-5 of the first argument, these 3.1e-5 and that u.
constexpr float kAbandonC = 1.000025f;
__device__ __forceinline__ float abandon_scale(float tau) {
    return kAbandonC * fmaxf(sqrt_rn(tau), 1e-15f);
}
__device__ __forceinline__ float abandon_threshold(float b, float st) {
    const float r = __builtin_fmaf(b, kAbandonC, st);
    return r * r;
}

}  // namespace trim
