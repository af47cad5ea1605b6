// Distance providers shared by the beamSearch and robustPrune kernels:
// a query (or pivot) vector held in registers, T lanes per stored record,
// 16-byte gathers, partial sums reduced inside each T-lane group.
//   K_U8  : uint8 vectors, exact int32 squared L2 via packed dot products
//   K_F32 : float32 vectors, float32 squared L2
//   K_RQ4 : 4-bit RaBitQ codes, packed 4-bit dot products against the two
//           nibble planes of an 8-bit integer query
//   K_RQ1 : 1-bit RaBitQ codes, AND + popcount against the query's bit planes
//   K_F16 : binary16 vectors, ||a||^2 - 2<a,q> + ||q||^2 with packed half dot
//           products accumulated in float32 (clamped at 0)
#pragma once
#include "jx_device.h"
#include "jx_internal.h"

namespace jx {

enum { K_U8 = 0, K_F32 = 1, K_RQ4 = 2, K_RQ1 = 3, K_F16 = 4 };

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float hdot2(uint32_t a, uint32_t b, float c) {
    return __builtin_amdgcn_fdot2(__builtin_bit_cast(half2_t, a), __builtin_bit_cast(half2_t, b), c, false);
}

// RaBitQ records whose code chunks are covered exactly by T lanes x 3 chunks: the lanes hold code chunks only and
// every lane reads the record's meta chunk (data_add, data_rescale, code sum) with a load of its own.  For the
// 208-byte 1-bit records of d = 1536 (12 code chunks + meta) this is 4 lanes x 3 chunks, 16 records per pass, against
// 8 lanes x 2 chunk slots of which 3 in 16 are idle and the meta lane counts bits of zero planes.
template <int KIND, int CPL>
constexpr bool sep_meta() {
    return (KIND == 2 || KIND == 3) && CPL == 3;
}

// popcount(x) + acc in one instruction (the compiler prefers popcount-to-zero plus three-operand adds)
__device__ __forceinline__ uint32_t bcnt_acc(uint32_t x, uint32_t acc) {
    uint32_t r;
    asm("v_bcnt_u32_b32 %0, %1, %2" : "=v"(r) : "v"(x), "v"(acc));
    return r;
}

// 1-bit codes covered by 3 chunks per lane against four query bit planes: the planes (48 registers per lane) stay in
// LDS, one 16-byte read per chunk and plane in the inner loop, which lets a fifth wavefront fit each SIMD
#ifndef JX_RQ1_QLDS
#define JX_RQ1_QLDS 1
#endif
template <int KIND, int CPL, int QB>
constexpr bool query_in_lds() {
    return JX_RQ1_QLDS && KIND == 3 && CPL == 3 && QB == 4;
}
template <int KIND, int T, int CPL, int QB>
constexpr int query_lds_bytes() {
    return query_in_lds<KIND, CPL, QB>() ? QB * CPL * T * 16 : 0;
}

template <int KIND, int CPL, int QB>
struct QueryRegs {
    static constexpr int PLANES = (KIND == K_RQ4) ? 2 : (KIND == K_RQ1 ? QB : 1);
    static constexpr int N = query_in_lds<KIND, CPL, QB>() ? 1 : 4 * CPL * PLANES;
    uint32_t w[N];
    const uint4* lq;      // query_in_lds: planes in LDS, entry (plane * CPL + chunk slot) * T + lane in group
    uint32_t ps[CPL];     // RaBitQ: left shift of this chunk slot's integer dot product (high code plane)
    // per-query scalars
    int32_t qq;           // U8: sum q^2
    float qqf;            // F16: sum q^2
    float lo, delta, qadd, qsumq;
};

// TILED (exact kinds; the load ablation of Sec. 4.4): register m of a lane holds the 4-byte element lig + T * m of
// the vector -- consecutive lanes of a group read consecutive elements, one element per load ("tiled") -- instead of
// the four elements of 16-byte chunk lig + T * (m / 4) ("chunked").  Query and records use the same assignment, so
// the distance is the same sum.
template <int KIND, int T, int CPL, int QB, bool TILED = false>
__device__ __forceinline__ void load_query(QueryRegs<KIND, CPL, QB>& q, const DistSrc& a, int64_t qi, int lig,
                                           uint4* lds_planes = nullptr) {
    const uint8_t* base = a.qrecs + qi * a.qrec_stride;
    q.lq = lds_planes;
    if constexpr (KIND == K_U8 || KIND == K_F32 || KIND == K_F16) {
        if constexpr (TILED) {
#pragma unroll
            for (int m = 0; m < 4 * CPL; m++) {
                const int e = lig + T * m;
                q.w[m] = e < 4 * a.nch ? reinterpret_cast<const uint32_t*>(base)[e] : 0u;
            }
        } else {
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                int ch = lig + T * j;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (ch < a.nch) v = load16(base + (size_t)ch * 16);
                q.w[4 * j + 0] = v.x;
                q.w[4 * j + 1] = v.y;
                q.w[4 * j + 2] = v.z;
                q.w[4 * j + 3] = v.w;
            }
        }
        if constexpr (KIND == K_U8) {
            int32_t s = 0;
#pragma unroll
            for (int i = 0; i < 4 * CPL; i++) s = (int32_t)__builtin_amdgcn_udot4(q.w[i], q.w[i], (uint32_t)s, false);
            q.qq = group_sum<T>(s);
        }
        if constexpr (KIND == K_F16) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < 4 * CPL; i++) s = hdot2(q.w[i], q.w[i], s);
            q.qqf = group_sum<T>(s);
        }
    } else {
        constexpr int PL = QueryRegs<KIND, CPL, QB>::PLANES;
#pragma unroll
        for (int j = 0; j < CPL; j++) q.ps[j] = (lig + T * j) >= a.plane_chunks ? (uint32_t)a.plane_shift : 0u;
        const float* hdr = reinterpret_cast<const float*>(base);
        q.lo = hdr[0];
        q.delta = hdr[1];
        q.qadd = hdr[2];
        q.qsumq = hdr[3];
#pragma unroll
        for (int p = 0; p < PL; p++) {
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                int ch = lig + T * j;
                uint4 v = make_uint4(0, 0, 0, 0);
                // the high code plane meets the same query planes as the low one
                const int qch = ch >= a.plane_chunks ? ch - a.plane_chunks : ch;
                if (ch < a.meta_chunk) v = load16(base + 16 + (size_t)p * a.qplane_stride + (size_t)qch * 16);
                if constexpr (query_in_lds<KIND, CPL, QB>()) {
                    if (lane_id() < T) lds_planes[(p * CPL + j) * T + lig] = v;
                } else {
                    q.w[(p * CPL + j) * 4 + 0] = v.x;
                    q.w[(p * CPL + j) * 4 + 1] = v.y;
                    q.w[(p * CPL + j) * 4 + 2] = v.z;
                    q.w[(p * CPL + j) * 4 + 3] = v.w;
                }
            }
        }
        if constexpr (query_in_lds<KIND, CPL, QB>()) wave_sync();
    }
}

// Distance of the query to up to G*U records; result keys go to cand_key[].
// FULL: every one of the T*CPL chunk slots maps to a chunk of the record, so no
// lane has to be masked.  Lane groups beyond the last candidate of a batch read
// the last candidate's record again (same cache lines, no extra traffic) and
// drop the result; this keeps the gathers free of per-lane predication.
template <int KIND, int T, int CPL, int QB, int U, bool FULL = false, bool TILED = false>
__device__ __forceinline__ void eval_batch(const QueryRegs<KIND, CPL, QB>& q, const DistSrc& a, int s0, int n_new,
                                           const uint32_t* cand_id, uint64_t* cand_key, int g, int lig) {
    constexpr int G = 64 / T;
    constexpr bool SEP = sep_meta<KIND, CPL>();
    uint4 data[U][CPL];
    uint4 mdat[SEP ? U : 1];
    uint32_t ids[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
        int c = s0 + u * G + g;
        ids[u] = cand_id[c < n_new ? c : n_new - 1];
    }
    const int nload = SEP ? a.meta_chunk : a.nch;  // chunks that the lanes' chunk slots cover
#pragma unroll
    for (int u = 0; u < U; u++) {
        if (s0 + u * G < n_new) {  // wave-uniform
            // the stride fits 32 bits (records are at most a few KB): one 32 x 32 -> 64-bit multiply-add per address
            const uint8_t* rec = a.recs + (size_t)ids[u] * (uint32_t)a.rec_stride;
            if constexpr (TILED) {
                const uint32_t* el = reinterpret_cast<const uint32_t*>(rec);
#pragma unroll
                for (int j = 0; j < CPL; j++) {
                    uint32_t w[4];
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const int e = lig + T * (4 * j + c);
                        w[c] = (FULL || e < 4 * a.nch) ? el[e] : 0u;
                    }
                    data[u][j] = make_uint4(w[0], w[1], w[2], w[3]);
                }
                continue;
            }
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                int ch = lig + T * j;
                if constexpr (FULL) {
                    data[u][j] = load16(rec + (size_t)ch * 16);
                } else {
                    data[u][j] = make_uint4(0, 0, 0, 0);
                    if (ch < nload) data[u][j] = load16(rec + (size_t)ch * 16);
                }
            }
            if constexpr (SEP) mdat[u] = load16(rec + (size_t)a.meta_chunk * 16);
        }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
        int c = s0 + u * G + g;
        // wave-uniform skip of batches that hold no candidate at all
        if (s0 + u * G >= n_new) break;
        uint32_t dist_code = 0;
        bool writer = (lig == 0);
        if constexpr (KIND == K_U8) {
            uint32_t aa = 0, aq = 0;
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                const uint4 v = data[u][j];
                aa = __builtin_amdgcn_udot4(v.x, v.x, aa, false);
                aa = __builtin_amdgcn_udot4(v.y, v.y, aa, false);
                aa = __builtin_amdgcn_udot4(v.z, v.z, aa, false);
                aa = __builtin_amdgcn_udot4(v.w, v.w, aa, false);
                aq = __builtin_amdgcn_udot4(v.x, q.w[4 * j + 0], aq, false);
                aq = __builtin_amdgcn_udot4(v.y, q.w[4 * j + 1], aq, false);
                aq = __builtin_amdgcn_udot4(v.z, q.w[4 * j + 2], aq, false);
                aq = __builtin_amdgcn_udot4(v.w, q.w[4 * j + 3], aq, false);
            }
            int32_t part = (int32_t)aa - 2 * (int32_t)aq;
            part = group_sum<T>(part);
            dist_code = (uint32_t)(part + q.qq);
        } else if constexpr (KIND == K_F16) {
            float aa = 0.f, aq = 0.f;
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                const uint4 v = data[u][j];
                aa = hdot2(v.x, v.x, aa);
                aa = hdot2(v.y, v.y, aa);
                aa = hdot2(v.z, v.z, aa);
                aa = hdot2(v.w, v.w, aa);
                aq = hdot2(v.x, q.w[4 * j + 0], aq);
                aq = hdot2(v.y, q.w[4 * j + 1], aq);
                aq = hdot2(v.z, q.w[4 * j + 2], aq);
                aq = hdot2(v.w, q.w[4 * j + 3], aq);
            }
            float part = group_sum<T>(aa - 2.f * aq);
            dist_code = f32_to_ordered(fmaxf(part + q.qqf, 0.f));
        } else if constexpr (KIND == K_F32) {
            float acc = 0.f;
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                const uint4 v = data[u][j];
                float d0 = __uint_as_float(v.x) - __uint_as_float(q.w[4 * j + 0]);
                float d1 = __uint_as_float(v.y) - __uint_as_float(q.w[4 * j + 1]);
                float d2 = __uint_as_float(v.z) - __uint_as_float(q.w[4 * j + 2]);
                float d3 = __uint_as_float(v.w) - __uint_as_float(q.w[4 * j + 3]);
                acc = fmaf(d0, d0, acc);
                acc = fmaf(d1, d1, acc);
                acc = fmaf(d2, d2, acc);
                acc = fmaf(d3, d3, acc);
            }
            acc = group_sum<T>(acc);
            dist_code = f32_to_ordered(acc);
        } else {
            // RaBitQ estimator, integer-query form (Sec. 5.1): exact integer
            // <u,q_int>, sum(u) read from the record (stored at encode time), then
            // five float32 operations in a fixed order.  The query planes are zero
            // for the meta chunk and beyond, so no chunk has to be masked.
            uint32_t I = 0, S = 0;
            float m_add = 0.f, m_rescale = 0.f;
            const int mj = a.meta_chunk / T, ml = a.meta_chunk % T;
            if constexpr (SEP) {
                m_add = __uint_as_float(mdat[u].x);
                m_rescale = __uint_as_float(mdat[u].y);
                S = mdat[u].z;
            } else {
                writer = (lig == ml);
            }
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                const uint4 v = data[u][j];
                if (!SEP && j == mj) {
                    m_add = __uint_as_float(v.x);
                    m_rescale = __uint_as_float(v.y);
                    S = v.z;
                }
                if constexpr (KIND == K_RQ4) {
                    uint32_t ih = 0, il = 0;
                    const uint32_t* qh = &q.w[(0 * CPL + j) * 4];
                    const uint32_t* ql = &q.w[(1 * CPL + j) * 4];
                    il = __builtin_amdgcn_udot8(v.x, ql[0], il, false);
                    il = __builtin_amdgcn_udot8(v.y, ql[1], il, false);
                    il = __builtin_amdgcn_udot8(v.z, ql[2], il, false);
                    il = __builtin_amdgcn_udot8(v.w, ql[3], il, false);
                    if constexpr (QB == 8) {
                        ih = __builtin_amdgcn_udot8(v.x, qh[0], ih, false);
                        ih = __builtin_amdgcn_udot8(v.y, qh[1], ih, false);
                        ih = __builtin_amdgcn_udot8(v.z, qh[2], ih, false);
                        ih = __builtin_amdgcn_udot8(v.w, qh[3], ih, false);
                    }
                    I += ((QB == 8) ? (16u * ih + il) : il) << q.ps[j];
                } else {
                    // sum_b 2^b popcount(code & plane_b): one AND and one accumulating popcount per dword and plane
                    uint32_t Ij = 0;
#pragma unroll
                    for (int b = QB - 1; b >= 0; b--) {
                        uint4 qp;
                        if constexpr (query_in_lds<KIND, CPL, QB>())
                            qp = q.lq[(b * CPL + j) * T + lig];
                        else
                            qp = make_uint4(q.w[(b * CPL + j) * 4 + 0], q.w[(b * CPL + j) * 4 + 1], q.w[(b * CPL + j) * 4 + 2],
                                            q.w[(b * CPL + j) * 4 + 3]);
                        uint32_t cnt = bcnt_acc(v.x & qp.x, 0u);
                        cnt = bcnt_acc(v.y & qp.y, cnt);
                        cnt = bcnt_acc(v.z & qp.z, cnt);
                        cnt = bcnt_acc(v.w & qp.w, cnt);
                        Ij = (Ij << 1) + cnt;  // Horner over the planes
                    }
                    I += Ij << q.ps[j];
                }
            }
            I = group_sum<T>(I);
            float t = __fmul_rn((float)I, q.delta);
            float t2 = __fmul_rn(q.lo, (float)S);
            t = __fadd_rn(t, t2);
            t = __fsub_rn(t, q.qsumq);
            float e = __fadd_rn(m_add, q.qadd);
            float p = __fmul_rn(m_rescale, t);
            e = __fadd_rn(e, p);
            dist_code = f32_to_ordered(e);
        }
        if (writer && c < n_new) cand_key[c] = make_key(dist_code, ids[u]);
    }
}

}  // namespace jx
