// beamSearch kernel (Alg. 1 / Alg. 2 of the paper, fused as in Sec. 4.1 and
// App. B): one wavefront serves one query for its whole life.
//
// Per expansion ("hop") the wavefront
//   1. picks the closest unexpanded frontier entry u (ballot over registers),
//   2. reads adjacency row adj[u] with one coalesced 4R-byte load,
//   3. drops ids it has seen before with a direct-mapped table of full ids in
//      LDS (a table that only ever forgets: no false positives, so the frontier
//      sequence equals that of an exact visited set -- the filter changes the
//      number of distance evaluations, never the result),
//   4. gathers the surviving neighbours' records (vector or RaBitQ code) with
//      16-byte loads, T lanes per record, several records in flight per lane,
//   5. reduces the partial distances inside each T-lane group,
//   6. merges the new (distance,id) keys into the sorted frontier, which lives
//      in registers (one key per lane per 64 entries): every candidate that
//      beats the current worst entry is broadcast once, every lane counts how
//      many candidates precede its entries, and one LDS scatter/gather applies
//      the permutation.  Keys are 64-bit (ordered distance, id, expanded flag),
//      so the order is the strict total order (distance, id).
#include "jx_device.h"
#include "jx_internal.h"

namespace jx {

enum { K_U8 = 0, K_F32 = 1, K_RQ4 = 2, K_RQ1 = 3 };

template <int KIND, int CPL, int QB>
struct QueryRegs {
    static constexpr int PLANES = (KIND == K_RQ4) ? 2 : (KIND == K_RQ1 ? QB : 1);
    static constexpr int N = 4 * CPL * PLANES;
    uint32_t w[N];
    uint32_t cmask[CPL];  // RaBitQ: all-ones for code chunks, 0 for the meta chunk and beyond
    // per-query scalars
    int32_t qq;           // U8: sum q^2
    float lo, delta, qadd, qsumq;
};

template <int KIND, int T, int CPL, int QB>
__device__ __forceinline__ void load_query(QueryRegs<KIND, CPL, QB>& q, const BeamArgs& a, int64_t qi, int lig) {
    const uint8_t* base = a.qrecs + qi * a.qrec_stride;
    if constexpr (KIND == K_U8 || KIND == K_F32) {
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
        if constexpr (KIND == K_U8) {
            int32_t s = 0;
#pragma unroll
            for (int i = 0; i < 4 * CPL; i++) s = (int32_t)__builtin_amdgcn_udot4(q.w[i], q.w[i], (uint32_t)s, false);
            q.qq = group_sum<T>(s);
        }
    } else {
        constexpr int PL = QueryRegs<KIND, CPL, QB>::PLANES;
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
                if (ch < a.meta_chunk) v = load16(base + 16 + (size_t)p * a.qplane_stride + (size_t)ch * 16);
                q.w[(p * CPL + j) * 4 + 0] = v.x;
                q.w[(p * CPL + j) * 4 + 1] = v.y;
                q.w[(p * CPL + j) * 4 + 2] = v.z;
                q.w[(p * CPL + j) * 4 + 3] = v.w;
            }
        }
#pragma unroll
        for (int j = 0; j < CPL; j++) q.cmask[j] = (lig + T * j) < a.meta_chunk ? 0xFFFFFFFFu : 0u;
    }
}

// Distance of the query to up to G*U records; result keys go to cand_key[].
template <int KIND, int T, int CPL, int QB, int U>
__device__ __forceinline__ void eval_batch(const QueryRegs<KIND, CPL, QB>& q, const BeamArgs& a, int s0, int n_new,
                                           const uint32_t* cand_id, uint64_t* cand_key, int g, int lig) {
    constexpr int G = 64 / T;
    uint4 data[U][CPL];
    uint32_t ids[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
        int c = s0 + u * G + g;
        ids[u] = (c < n_new) ? cand_id[c] : JX_NONE_ID;
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
#pragma unroll
        for (int j = 0; j < CPL; j++) {
            int ch = lig + T * j;
            data[u][j] = make_uint4(0, 0, 0, 0);
            if (ids[u] != JX_NONE_ID && ch < a.nch)
                data[u][j] = load16(a.recs + (size_t)ids[u] * (size_t)a.rec_stride + (size_t)ch * 16);
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
            // <u,q_int> and sum(u), then five float32 operations in a fixed order.
            uint32_t I = 0, S = 0;
            float m_add = 0.f, m_rescale = 0.f;
            const int mj = a.meta_chunk / T, ml = a.meta_chunk % T;
            writer = (lig == ml);
#pragma unroll
            for (int j = 0; j < CPL; j++) {
                uint4 v = data[u][j];
                if (j == mj) {
                    m_add = __uint_as_float(v.x);
                    m_rescale = __uint_as_float(v.y);
                }
                v.x &= q.cmask[j];
                v.y &= q.cmask[j];
                v.z &= q.cmask[j];
                v.w &= q.cmask[j];
                if constexpr (KIND == K_RQ4) {
                    uint32_t ih = 0, il = 0;
                    const uint32_t* qh = &q.w[(0 * CPL + j) * 4];
                    const uint32_t* ql = &q.w[(1 * CPL + j) * 4];
                    ih = __builtin_amdgcn_udot8(v.x, qh[0], ih, false);
                    ih = __builtin_amdgcn_udot8(v.y, qh[1], ih, false);
                    ih = __builtin_amdgcn_udot8(v.z, qh[2], ih, false);
                    ih = __builtin_amdgcn_udot8(v.w, qh[3], ih, false);
                    il = __builtin_amdgcn_udot8(v.x, ql[0], il, false);
                    il = __builtin_amdgcn_udot8(v.y, ql[1], il, false);
                    il = __builtin_amdgcn_udot8(v.z, ql[2], il, false);
                    il = __builtin_amdgcn_udot8(v.w, ql[3], il, false);
                    I += (QB == 8) ? (16u * ih + il) : il;
                    S = __builtin_amdgcn_udot8(v.x, 0x11111111u, S, false);
                    S = __builtin_amdgcn_udot8(v.y, 0x11111111u, S, false);
                    S = __builtin_amdgcn_udot8(v.z, 0x11111111u, S, false);
                    S = __builtin_amdgcn_udot8(v.w, 0x11111111u, S, false);
                } else {
#pragma unroll
                    for (int b = 0; b < QB; b++) {
                        const uint32_t* qp = &q.w[(b * CPL + j) * 4];
                        uint32_t cnt = __builtin_popcount(v.x & qp[0]) + __builtin_popcount(v.y & qp[1]) +
                                       __builtin_popcount(v.z & qp[2]) + __builtin_popcount(v.w & qp[3]);
                        I += cnt << b;
                    }
                    S += __builtin_popcount(v.x) + __builtin_popcount(v.y) + __builtin_popcount(v.z) +
                         __builtin_popcount(v.w);
                }
            }
            I = group_sum<T>(I);
            S = group_sum<T>(S);
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

template <int KIND, int T, int CPL, int NREG, int QB>
__global__ void __launch_bounds__(JX_BEAM_WPB * 64) beam_search_kernel(BeamArgs a) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);  // records in flight per lane group
    constexpr int FCAP = NREG * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = threadIdx.x >> 6;
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const int64_t qi = (int64_t)blockIdx.x * JX_BEAM_WPB + wave;
    if (qi >= a.nq) return;  // whole wavefront leaves; there is no block-level barrier below

    const int H = 1 << a.hash_log2;
    const size_t per_wave = (size_t)FCAP * 8 + 64 * 8 + 64 * 4 + (size_t)H * 4;
    unsigned char* my = smem + per_wave * wave;
    uint64_t* fr = reinterpret_cast<uint64_t*>(my);
    uint64_t* cand_key = fr + FCAP;
    uint32_t* cand_id = reinterpret_cast<uint32_t*>(cand_key + 64);
    uint32_t* tab = cand_id + 64;

    for (int i = lane; i < H; i += 64) tab[i] = JX_NONE_ID;

    QueryRegs<KIND, CPL, QB> q;
    load_query<KIND, T, CPL, QB>(q, a, qi, lig);

    uint64_t fk[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) fk[r] = JX_EMPTY_KEY;
    int count = 0;
    const int L = a.L;
    uint32_t hops = 0, evals = 0;

    // seed: the entry vertex
    if (lane == 0) {
        cand_id[0] = a.entry;
        tab[(a.entry * 0x9E3779B1u) >> (32 - a.hash_log2)] = a.entry;
    }
    wave_sync();
    eval_batch<KIND, T, CPL, QB, 1>(q, a, 0, 1, cand_id, cand_key, g, lig);
    wave_sync();
    if (lane == 0) fk[0] = cand_key[0];
    count = 1;
    evals = 1;

    for (;;) {
        // ---- 1. closest unexpanded entry
        int sel_r = -1, sel_lane = 0;
#pragma unroll
        for (int r = 0; r < NREG; r++) {
            uint64_t m = ballot((fk[r] & 1ull) == 0ull);
            if (sel_r < 0 && m != 0ull) {
                sel_r = r;
                sel_lane = __builtin_ctzll(m);
            }
        }
        if (sel_r < 0) break;
        uint32_t u = 0;
#pragma unroll
        for (int r = 0; r < NREG; r++) {
            if (r == sel_r) {
                u = key_id(readlane64(fk[r], sel_lane));
                if (lane == sel_lane) fk[r] |= 1ull;
            }
        }
        hops++;
        const uint32_t* row = a.adj + (size_t)u * (size_t)a.R;
        for (int rb = 0; rb < a.R; rb += 64) {
            // ---- 2. adjacency row (coalesced)
            uint32_t v = JX_NONE_ID;
            if (rb + lane < a.R) v = row[rb + lane];
            bool is_new = false;
            // ---- 3. visited filter
            if (v != JX_NONE_ID) {
                uint32_t h = (v * 0x9E3779B1u) >> (32 - a.hash_log2);
                is_new = tab[h] != v;
                if (is_new) tab[h] = v;
            }
            uint64_t nm = ballot(is_new);
            if (ballot(v != JX_NONE_ID) == 0ull) break;  // rows are filled from the left
            const int n_new = __builtin_popcountll(nm);
            if (n_new == 0) continue;
            if (is_new) cand_id[prefix_count(nm)] = v;
            wave_sync();
            // ---- 4./5. gather + distances
            for (int s0 = 0; s0 < n_new; s0 += G * U)
                eval_batch<KIND, T, CPL, QB, U>(q, a, s0, n_new, cand_id, cand_key, g, lig);
            evals += n_new;
            wave_sync();
            uint64_t ck = lane < n_new ? cand_key[lane] : JX_EMPTY_KEY;
            wave_sync();
            // ---- 6. merge into the sorted frontier
            bool beats = lane < n_new;
            if (count >= L) {
                uint64_t worst = 0;
#pragma unroll
                for (int r = 0; r < NREG; r++)
                    if (r == (L - 1) / 64) worst = readlane64(fk[r], (L - 1) % 64);
                beats = beats && ((ck | 1ull) < (worst | 1ull));
            }
            uint64_t sm = ballot(beats);
            if (sm == 0ull) continue;
            uint32_t shift[NREG];
#pragma unroll
            for (int r = 0; r < NREG; r++) shift[r] = 0;
            uint32_t crank = 0, my_rank = 0;
            bool my_dup = false;
            int n_ins = 0;
            while (sm) {
                const int j = __builtin_ctzll(sm);
                sm &= sm - 1;
                const uint64_t s = readlane64(ck, j) | 1ull;
                uint32_t below = 0;
                bool dup = false;
#pragma unroll
                for (int r = 0; r < NREG; r++) {
                    const uint64_t f = fk[r] | 1ull;
                    below += (uint32_t)__builtin_popcountll(ballot(f < s));
                    dup = dup || (ballot(f == s) != 0ull);
                }
                if (dup) {  // id already in the frontier (the table forgot it)
                    if (lane == j) my_dup = true;
                    continue;
                }
#pragma unroll
                for (int r = 0; r < NREG; r++) shift[r] += (s < (fk[r] | 1ull)) ? 1u : 0u;
                crank += (s < (ck | 1ull)) ? 1u : 0u;
                if (lane == j) my_rank = below;
                n_ins++;
            }
            if (n_ins == 0) continue;
#pragma unroll
            for (int r = 0; r < NREG; r++) {
                uint32_t np = (uint32_t)(r * 64 + lane) + shift[r];
                if (np < (uint32_t)FCAP) fr[np] = fk[r];
            }
            if (beats && !my_dup) {
                uint32_t np = my_rank + crank;
                if (np < (uint32_t)FCAP) fr[np] = ck;
            }
            wave_sync();
#pragma unroll
            for (int r = 0; r < NREG; r++) {
                fk[r] = fr[r * 64 + lane];
                if (r * 64 + lane >= L) fk[r] = JX_EMPTY_KEY;  // truncate to the beam width
            }
            wave_sync();
            count = count + n_ins < L ? count + n_ins : L;
        }
    }

    // ---- results: the first out_k frontier entries
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        int p = r * 64 + lane;
        if (p < a.out_k) {
            uint64_t k = fk[r];
            bool valid = (p < count);
            uint32_t dc = key_dist(k);
            float d;
            if constexpr (KIND == K_U8)
                d = (float)dc;
            else
                d = ordered_to_f32(dc);
            a.out_ids[qi * a.out_k + p] = valid ? key_id(k) : JX_NONE_ID;
            a.out_dist[qi * a.out_k + p] = valid ? d : __builtin_inff();
        }
    }
    if (a.stats && lane == 0) {
        atomicAdd(&a.stats[0], (unsigned long long)hops);
        atomicAdd(&a.stats[1], (unsigned long long)evals);
    }
}

// ------------------------------------------------------------------ launch

template <int KIND, int T, int CPL, int QB>
static hipError_t launch_nreg(const BeamArgs& a, hipStream_t st) {
    const int nreg = (a.L + 63) / 64;
    const int H = 1 << a.hash_log2;
    dim3 grid((unsigned)((a.nq + JX_BEAM_WPB - 1) / JX_BEAM_WPB)), block(JX_BEAM_WPB * 64);
#define JX_LAUNCH(NR)                                                                                   \
    {                                                                                                   \
        size_t sh = ((size_t)(NR) * 64 * 8 + 64 * 8 + 64 * 4 + (size_t)H * 4) * JX_BEAM_WPB;            \
        auto kern = beam_search_kernel<KIND, T, CPL, NR, QB>;                                           \
        if (sh > 48 * 1024) {                                                                           \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh); \
            if (e != hipSuccess) return e;                                                              \
        }                                                                                               \
        hipLaunchKernelGGL(kern, grid, block, sh, st, a);                                               \
        return hipGetLastError();                                                                       \
    }
    if (nreg <= 1) JX_LAUNCH(1)
    if (nreg <= 2) JX_LAUNCH(2)
    if (nreg <= 4) JX_LAUNCH(4)
    JX_LAUNCH(8)
#undef JX_LAUNCH
}

template <int KIND, int QB>
static hipError_t launch_shape(const BeamArgs& a, hipStream_t st) {
    const int nch = a.nch;
    if (nch <= 8) return launch_nreg<KIND, 8, 1, QB>(a, st);
    if (nch <= 16) return launch_nreg<KIND, 16, 1, QB>(a, st);
    if (nch <= 32) return launch_nreg<KIND, 32, 1, QB>(a, st);
    if (nch <= 64) return launch_nreg<KIND, 64, 1, QB>(a, st);
    if constexpr (KIND == K_RQ1) {
        return hipErrorInvalidValue;
    } else {
        if (nch <= 128) return launch_nreg<KIND, 64, 2, QB>(a, st);
        if constexpr (KIND == K_RQ4) {
            return hipErrorInvalidValue;
        } else {
            if (nch <= 256) return launch_nreg<KIND, 64, 4, QB>(a, st);
            if (nch <= 384) return launch_nreg<KIND, 64, 6, QB>(a, st);
            return hipErrorInvalidValue;
        }
    }
}

hipError_t launch_beam_search(int kind, int qbits, const BeamArgs& a, hipStream_t st) {
    if (a.nq <= 0) return hipSuccess;
    switch (kind) {
        case K_U8: return launch_shape<K_U8, 0>(a, st);
        case K_F32: return launch_shape<K_F32, 0>(a, st);
        case K_RQ4: return qbits == 8 ? launch_shape<K_RQ4, 8>(a, st) : launch_shape<K_RQ4, 4>(a, st);
        case K_RQ1: return qbits == 8 ? launch_shape<K_RQ1, 8>(a, st) : launch_shape<K_RQ1, 4>(a, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace jx
