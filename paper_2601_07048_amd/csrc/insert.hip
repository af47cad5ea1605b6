// Batch insertion (Alg. 4 with the changes of Sec. 4.3 / 4.5): everything that
// follows the candidate search.
//
//   entry point   : column means (two-stage, fixed order, double) and the
//                   point nearest to the mean
//   forward prune : one wavefront per new point runs robustPrune (Alg. 3) on
//                   its final frontier, writes adjacency row, emits reverse
//                   edges (target, distance, source) to the kept neighbours only
//   sort          : stable LSD radix sort (8-bit digits) of the unified edge
//                   buffer on the 64-bit key (target << 32 | distance bits);
//                   stability leaves equal keys in emission order = ascending
//                   source id, so the order is (target, distance, source)
//   reverse merge : one wavefront per touched target: append if the row still
//                   fits, else robustPrune(row U new edges) with the existing
//                   neighbours' distances recomputed.  A row is written by
//                   exactly one wavefront: no locks (Sec. 3.3).
//
// robustPrune walks two sorted lists -- the target's existing neighbours (LDS)
// and the new candidates (global memory, already sorted) -- as one merged
// sequence.  Each time the closest live candidate p* is selected, all remaining
// live candidates p' get d(p*,p') computed (T lanes per vector, as in
// beamSearch) and are discarded when alpha * d(p*,p') <= d(p,p'), evaluated in
// float32 as one multiply and one compare.
#include "jx_distance.h"

namespace jx {

#ifndef INS_WPB
#define INS_WPB 1      // wavefronts per workgroup (they never cooperate: a slot is free as soon as its wavefront ends)
#endif
#define INS_RA JX_MAX_R

// ------------------------------------------------------------------ entry point

template <int DT>
__device__ __forceinline__ double elem_f64(const void* vecs, size_t i) {
    if (DT == JX_U8) return (double)reinterpret_cast<const uint8_t*>(vecs)[i];
    if (DT == JX_F16) return (double)(float)reinterpret_cast<const _Float16*>(vecs)[i];
    return (double)reinterpret_cast<const float*>(vecs)[i];
}

template <int DT>
__global__ void __launch_bounds__(256) col_partial_kernel(const void* vecs, long long n, int d, int nblk, double* partial) {
    const long long per = (n + nblk - 1) / nblk;
    const long long r0 = (long long)blockIdx.x * per;
    const long long r1 = r0 + per < n ? r0 + per : n;
    for (int j = threadIdx.x; j < d; j += 256) {
        double s = 0.0;
        for (long long i = r0; i < r1; i++) {
            s += elem_f64<DT>(vecs, (size_t)i * d + j);
        }
        partial[(size_t)blockIdx.x * d + j] = s;
    }
}

__global__ void mean_finalize_kernel(const double* partial, int nblk, int d, long long n, float* mean) {
    int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= d) return;
    double s = 0.0;
    for (int b = 0; b < nblk; b++) s += partial[(size_t)b * d + j];
    mean[j] = (float)(s / (double)n);
}

template <int DT>
__global__ void __launch_bounds__(256) dist_to_mean_kernel(const void* vecs, long long n, int d, const float* mean, double* out) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = lane_id();
    double s = 0.0;
    for (int j = lane; j < d; j += 64) {
        double v = elem_f64<DT>(vecs, (size_t)i * d + j);
        double t = v - (double)mean[j];
        s += t * t;
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += shfl_xor(s, m);
    if (lane == 0) out[i] = s;
}

// single workgroup: smallest (distance, id)
__global__ void __launch_bounds__(1024) argmin_kernel(const double* dist, long long n, uint32_t* out_id) {
    __shared__ double sd[1024];
    __shared__ long long si[1024];
    double bd = __builtin_inf();
    long long bi = 0x7FFFFFFFFFFFFFFFLL;
    for (long long i = threadIdx.x; i < n; i += 1024) {
        double v = dist[i];
        if (v < bd || (v == bd && i < bi)) {
            bd = v;
            bi = i;
        }
    }
    sd[threadIdx.x] = bd;
    si[threadIdx.x] = bi;
    __syncthreads();
    for (int s = 512; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            double od = sd[threadIdx.x + s];
            long long oi = si[threadIdx.x + s];
            if (od < sd[threadIdx.x] || (od == sd[threadIdx.x] && oi < si[threadIdx.x])) {
                sd[threadIdx.x] = od;
                si[threadIdx.x] = oi;
            }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) *out_id = (uint32_t)si[0];
}

// ------------------------------------------------------------------ robustPrune

struct PruneLds {
    uint64_t a_key[INS_RA];   // existing neighbours sorted by (distance, id); key = distance bits << 32 | id
    union {
        struct {
            uint64_t a_tmp[INS_RA];
            uint64_t cand_key[64];
        };
        uint32_t gram_scratch[128 + 128 * 4];  // MFMA path: squared norms, then the discard relation
    };
    uint32_t cand_id[64];
    uint32_t cand_src[64];
    uint32_t sel_id[INS_RA];
    uint32_t sel_dist[INS_RA];
    uint8_t a_dead[INS_RA];
};

template <int KIND>
__device__ __forceinline__ float code_to_dist(uint32_t code) {
    if constexpr (KIND == K_U8)
        return (float)code;
    else
        return ordered_to_f32(code);
}

// Candidate list B in global memory: ids and non-negative float distance bits
// with element strides, plus one discard byte per element.
struct BList {
    const uint32_t* ids;
    const uint32_t* dbits;
    int id_stride, d_stride;
    int n;
    uint8_t* dead;
};

// Evaluate d(pivot, c) for the live elements of one 64-wide chunk and discard
// those with alpha * d(pivot,c) <= d(p,c).
// CACHED: the candidates' vectors sit in an LDS cache, slot i = position i of
// list A; the record "id" handed to the distance provider is then the slot.
template <int KIND, int T, int CPL, bool IS_A, bool CACHED = false>
__device__ __forceinline__ void kill_chunk(const QueryRegs<KIND, CPL, 0>& q, const DistSrc& ds, PruneLds* L, const BList& B,
                                           int c0, int n, float alpha, int g, int lig, int lane) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    const int i = c0 + lane;
    bool alive = false;
    uint32_t id = JX_NONE_ID;
    if (i < n) {
        if (IS_A) {
            alive = L->a_dead[i] == 0;
            id = CACHED ? (uint32_t)i : (uint32_t)L->a_key[i];
        } else {
            alive = B.dead[i] == 0;
            id = B.ids[(size_t)i * B.id_stride];
        }
    }
    const uint64_t am = ballot(alive);
    const int n_alive = __builtin_popcountll(am);
    if (n_alive == 0) return;
    if (alive) {
        int slot = prefix_count(am);
        L->cand_id[slot] = id;
        L->cand_src[slot] = (uint32_t)i;
    }
    wave_sync();
    for (int s0 = 0; s0 < n_alive; s0 += G * U)
        eval_batch<KIND, T, CPL, 0, U>(q, ds, s0, n_alive, L->cand_id, L->cand_key, g, lig);
    wave_sync();
    if (lane < n_alive) {
        const uint32_t src = L->cand_src[lane];
        const float d1 = code_to_dist<KIND>(key_dist(L->cand_key[lane]));
        float d2;
        if (IS_A)
            d2 = __uint_as_float((uint32_t)(L->a_key[src] >> 32));
        else
            d2 = __uint_as_float(B.dbits[(size_t)src * B.d_stride]);
        if (__fmul_rn(alpha, d1) <= d2) {
            if (IS_A)
                L->a_dead[src] = 1;
            else
                B.dead[src] = 1;
        }
    }
    __threadfence_block();
    wave_sync();
}

// Alg. 3 over the merged sequence of A (LDS, nA entries) and B.  Returns the
// number of selected ids (L->sel_id / L->sel_dist, selection order).
template <int KIND, int T, int CPL, bool CACHED = false>
__device__ __forceinline__ int robust_prune_wave(const DistSrc& ds, PruneLds* L, int nA, const BList& B, int R, float alpha) {
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    int iA = 0, iB = 0, nsel = 0;
    QueryRegs<KIND, CPL, 0> q;
    while (nsel < R) {
        while (iA < nA && L->a_dead[iA]) iA++;
        while (iB < B.n) {
            const int i = iB + lane;
            const bool alive = i < B.n && B.dead[i] == 0;
            const uint64_t m = ballot(alive);
            if (m) {
                iB += __builtin_ctzll(m);
                break;
            }
            iB += 64;
        }
        const bool hasA = iA < nA, hasB = iB < B.n;
        if (!hasA && !hasB) break;
        uint64_t kA = JX_EMPTY_KEY, kB = JX_EMPTY_KEY;
        if (hasA) kA = L->a_key[iA];
        if (hasB) kB = ((uint64_t)B.dbits[(size_t)iB * B.d_stride] << 32) | B.ids[(size_t)iB * B.id_stride];
        const bool takeA = kA < kB;
        const uint64_t kp = takeA ? kA : kB;
        const uint32_t pid = (CACHED && takeA) ? (uint32_t)iA : (uint32_t)kp;  // record to load as the pivot
        if (takeA) iA++; else iB++;
        if (lane == 0) {
            L->sel_id[nsel] = (uint32_t)kp;
            L->sel_dist[nsel] = (uint32_t)(kp >> 32);
        }
        nsel++;
        if (nsel >= R) break;
        load_query<KIND, T, CPL, 0>(q, ds, (int64_t)pid, lig);
        for (int c0 = iA; c0 < nA; c0 += 64) kill_chunk<KIND, T, CPL, true, CACHED>(q, ds, L, B, c0, nA, alpha, g, lig, lane);
        for (int c0 = iB; c0 < B.n; c0 += 64) kill_chunk<KIND, T, CPL, false, false>(q, ds, L, B, c0, B.n, alpha, g, lig, lane);
    }
    wave_sync();
    return nsel;
}


// robustPrune for the common small case on uint8 vectors of exactly 128 bytes:
// up to 128 candidates, already merged and sorted in L->a_key, their vectors
// cached in LDS (slot i = position i, the cache covers whole tiles of 32 slots).
//
// The discard relation "i discards j" (alpha * d(i,j) <= d(p,j), i before j)
// does not depend on the order of selection, so it is computed for all pairs at
// once: d(i,j) = ||x_i||^2 + ||x_j||^2 - 2 <x_i,x_j> and the Gram matrix is a
// dense contraction done on the matrix cores (int8 MFMA 32x32x16 on the
// vectors shifted by -128, which leaves distances unchanged and exact).  Each
// accumulator element gives one ballot = one 32-column stripe of the relation
// for two rows.  The sequential part of Alg. 3 is then a scalar walk over
// bit masks: take the first live candidate, clear everything it discards.
typedef int i32x16_t __attribute__((ext_vector_type(16)));

__device__ __forceinline__ int prune_cached_u8_mfma(PruneLds* L, const unsigned char* vc, int M, int R, float alpha) {
    const int lane = lane_id();
    const int col = lane & 31, half = lane >> 5;
    const int nt = (M + 31) >> 5;  // tiles of 32 slots
    uint32_t* nrm = L->gram_scratch;         // [128] squared norms of the shifted vectors
    uint32_t* kmat = L->gram_scratch + 128;  // [128][4] discard relation, row i = mask over j
    // ---- norms: 4 lanes per slot (32 bytes each), 16 slots per step
    {
        const int sb = lane & 15, part = lane >> 4;
        for (int s0 = 0; s0 < nt * 32; s0 += 16) {
            const unsigned char* cv = vc + (size_t)(s0 + sb) * 128 + part * 32;
            uint4 c0 = *reinterpret_cast<const uint4*>(cv), c1 = *reinterpret_cast<const uint4*>(cv + 16);
            c0.x ^= 0x80808080u; c0.y ^= 0x80808080u; c0.z ^= 0x80808080u; c0.w ^= 0x80808080u;
            c1.x ^= 0x80808080u; c1.y ^= 0x80808080u; c1.z ^= 0x80808080u; c1.w ^= 0x80808080u;
            int32_t nn = 0;
            nn = __builtin_amdgcn_sdot4((int)c0.x, (int)c0.x, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c0.y, (int)c0.y, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c0.z, (int)c0.z, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c0.w, (int)c0.w, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c1.x, (int)c1.x, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c1.y, (int)c1.y, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c1.z, (int)c1.z, nn, false);
            nn = __builtin_amdgcn_sdot4((int)c1.w, (int)c1.w, nn, false);
            nn += shfl_xor(nn, 16);
            nn += shfl_xor(nn, 32);
            if (part == 0) nrm[s0 + sb] = (uint32_t)nn;
        }
    }
    wave_sync();
    // ---- discard relation, tile by tile (rows ti <= columns tj)
    for (int ti = 0; ti < nt; ti++) {
        long af[8];
#pragma unroll
        for (int ks = 0; ks < 8; ks++)
            af[ks] = *reinterpret_cast<const long*>(vc + (size_t)(ti * 32 + col) * 128 + ks * 16 + half * 8) ^ (long)0x8080808080808080ULL;
        for (int tj = ti; tj < nt; tj++) {
            i32x16_t acc;
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] = 0;
#pragma unroll
            for (int ks = 0; ks < 8; ks++) {
                const long bf = *reinterpret_cast<const long*>(vc + (size_t)(tj * 32 + col) * 128 + ks * 16 + half * 8) ^ (long)0x8080808080808080ULL;
                acc = __builtin_amdgcn_mfma_i32_32x32x16_i8(af[ks], bf, acc, 0, 0, 0);
            }
            const int j = tj * 32 + col;
            const uint32_t nj = nrm[j];
            const float d2 = j < M ? __uint_as_float((uint32_t)(L->a_key[j] >> 32)) : 0.f;
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int i = ti * 32 + 8 * (e >> 2) + 4 * half + (e & 3);
                const uint32_t dij = nrm[i] + nj - 2u * (uint32_t)acc[e];
                const bool kill = j < M && (__fmul_rn(alpha, (float)dij) <= d2);
                const uint64_t km = ballot(kill);
                if (lane == 0) {
                    const int r0 = ti * 32 + 8 * (e >> 2) + (e & 3);
                    kmat[r0 * 4 + tj] = (uint32_t)km;
                    kmat[(r0 + 4) * 4 + tj] = (uint32_t)(km >> 32);
                }
            }
        }
    }
    wave_sync();
    // ---- Alg. 3 on bit masks
    uint64_t alive0 = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
    uint64_t alive1 = M <= 64 ? 0ull : (M >= 128 ? ~0ull : ((1ull << (M - 64)) - 1ull));
    int nsel = 0;
    while (nsel < R) {
        int i;
        if (alive0) {
            i = __builtin_ctzll(alive0);
            alive0 &= alive0 - 1;
        } else if (alive1) {
            i = 64 + __builtin_ctzll(alive1);
            alive1 &= alive1 - 1;
        } else {
            break;
        }
        const uint64_t kp = L->a_key[i];
        if (lane == 0) {
            L->sel_id[nsel] = (uint32_t)kp;
            L->sel_dist[nsel] = (uint32_t)(kp >> 32);
        }
        nsel++;
        // words of columns left of the row's own tile were never written and are
        // not needed: every slot before i is already selected or discarded
        const int ti = i >> 5;
        uint32_t w[4];
#pragma unroll
        for (int t = 0; t < 4; t++) w[t] = (t >= ti && t < nt) ? kmat[i * 4 + t] : 0u;
        alive0 &= ~(((uint64_t)w[1] << 32) | w[0]);
        alive1 &= ~(((uint64_t)w[3] << 32) | w[2]);
    }
    wave_sync();
    return nsel;
}

// robustPrune of a row that is mostly the output of an earlier robustPrune call
// (uint8 vectors of 128 bytes, all M <= 128 candidates merged and sorted in
// L->a_key, their vectors cached in LDS, L->a_dead[i] = 1 marks the entries that
// were NOT selected together by that call: appended since, or new).
//
// Two entries that one call selected, i before j, satisfy "i does not discard j":
// otherwise j would not have been selected.  Distances on uint8 data are exact
// integers and alpha is fixed, so the same test gives the same answer now, and
// only pairs with a marked entry have to be evaluated.  Marked entries are taken
// in sorted order; when one is reached every earlier entry has its final state,
// because only marked entries before it could have discarded anything.  An entry
// beyond the R-th selected one is never output, so neither what it discards nor
// whether it is discarded matters.
template <int T, int CPL>
__device__ __forceinline__ int prune_cached_u8_incremental(const DistSrc& cds, PruneLds* L, int M, int R, float alpha) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    uint64_t dm[2], alive[2];
    dm[0] = ballot(lane < M && L->a_dead[lane] != 0);
    dm[1] = ballot(lane + 64 < M && L->a_dead[lane + 64] != 0);
    alive[0] = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
    alive[1] = M <= 64 ? 0ull : (M >= 128 ? ~0ull : ((1ull << (M - 64)) - 1ull));
    QueryRegs<K_U8, CPL, 0> q;
    while (dm[0] | dm[1]) {
        int t;
        if (dm[0]) {
            t = __builtin_ctzll(dm[0]);
            dm[0] &= dm[0] - 1ull;
        } else {
            t = 64 + __builtin_ctzll(dm[1]);
            dm[1] &= dm[1] - 1ull;
        }
        if (((alive[t >> 6] >> (t & 63)) & 1ull) == 0ull) continue;  // discarded by an earlier marked entry
        const float dvt = __uint_as_float((uint32_t)(L->a_key[t] >> 32));
        load_query<K_U8, T, CPL, 0>(q, cds, (int64_t)t, lig);
        uint64_t rk[2] = {0ull, 0ull}, ck[2] = {0ull, 0ull};
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int c0 = h * 64;
            if (c0 >= M) break;
            const int nn = M - c0 < 64 ? M - c0 : 64;
            if (lane < nn) L->cand_id[lane] = (uint32_t)(c0 + lane);
            wave_sync();
            for (int s0 = 0; s0 < nn; s0 += G * U)
                eval_batch<K_U8, T, CPL, 0, U>(q, cds, s0, nn, L->cand_id, L->cand_key, g, lig);
            wave_sync();
            const int j = c0 + lane;
            bool rkill = false, ckill = false;
            if (lane < nn) {
                const float d1 = (float)key_dist(L->cand_key[lane]);
                const float dvj = __uint_as_float((uint32_t)(L->a_key[j] >> 32));
                rkill = j > t && __fmul_rn(alpha, d1) <= dvj;  // t discards j
                ckill = j < t && __fmul_rn(alpha, d1) <= dvt;  // j, if selected, discards t
            }
            rk[h] = ballot(rkill);
            ck[h] = ballot(ckill);
            wave_sync();
        }
        if ((ck[0] & alive[0]) | (ck[1] & alive[1])) {
            alive[t >> 6] &= ~(1ull << (t & 63));
        } else {
            alive[0] &= ~rk[0];
            alive[1] &= ~rk[1];
        }
    }
    const int n0 = __builtin_popcountll(alive[0]);
#pragma unroll
    for (int h = 0; h < 2; h++) {
        const int j = h * 64 + lane;
        if (j < M && ((alive[h] >> lane) & 1ull)) {
            const int pos = (h ? n0 : 0) + __builtin_popcountll(alive[h] & ((1ull << lane) - 1ull));
            if (pos < R) {
                const uint64_t k = L->a_key[j];
                L->sel_id[pos] = (uint32_t)k;
                L->sel_dist[pos] = (uint32_t)(k >> 32);
            }
        }
    }
    wave_sync();
    const int total = n0 + __builtin_popcountll(alive[1]);
    return total < R ? total : R;
}


template <int KIND, int T, int CPL>
__global__ void __launch_bounds__(INS_WPB * 64) forward_prune_kernel(InsertArgs a) {
    __shared__ PruneLds lds[INS_WPB];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const long long i = (long long)blockIdx.x * INS_WPB + wave;
    if (i >= a.B) return;
    PruneLds* L = &lds[wave];
    long long xid = a.id_base + i;
    if (xid >= a.id_skip) xid++;
    BList B;
    B.ids = a.cand_ids + (size_t)i * a.L;
    B.dbits = a.cand_dist + (size_t)i * a.L;
    B.id_stride = 1;
    B.d_stride = 1;
    B.dead = a.dead + (size_t)i * a.L;
    // lists longer than 128: the block-row Gram-matrix kernel has run first and marks what it has done
    if (a.gram && a.L > 128 && B.dead[0] == 0xFF) return;
    // the frontier is filled from the left: count its valid entries
    int nB = 0;
    for (int c0 = 0; c0 < a.L; c0 += 64) {
        const int j = c0 + lane;
        const bool valid = j < a.L && B.ids[j] != JX_NONE_ID;
        if (j < a.L) B.dead[j] = 0;
        nB += __builtin_popcountll(ballot(valid));
    }
    B.n = nB;
    if (a.gram && nB <= 128) return;  // served by the Gram-matrix kernel
    __threadfence_block();
    wave_sync();
    int nsel;
    if (KIND == K_U8 && a.ds.rec_stride == 128 && nB <= 128 && (long long)((nB + 31) & ~31) * 128 <= a.vec_cache_bytes) {
        // the frontier is already sorted: cache its vectors in LDS and use the Gram-matrix form
        extern __shared__ __align__(16) unsigned char vcache[];
        unsigned char* vc = vcache + (size_t)wave * a.vec_cache_bytes;
        for (int j = lane; j < nB; j += 64) L->a_key[j] = ((uint64_t)B.dbits[j] << 32) | B.ids[j];
        for (int c = lane; c < nB * 8; c += 64) {
            const int sl = c >> 3, ch = c & 7;
            *reinterpret_cast<uint4*>(vc + (size_t)sl * 128 + ch * 16) =
                load16(a.ds.recs + (size_t)B.ids[sl] * 128 + (size_t)ch * 16);
        }
        __threadfence_block();
        wave_sync();
        nsel = prune_cached_u8_mfma(L, vc, nB, a.R, a.alpha);
    } else {
        nsel = robust_prune_wave<KIND, T, CPL>(a.ds, L, 0, B, a.R, a.alpha);
    }
    uint32_t* row = a.adj + (size_t)xid * a.R;
    for (int j = lane; j < a.R; j += 64) {
        const bool on = j < nsel;
        const uint32_t v = on ? L->sel_id[j] : JX_NONE_ID;
        row[j] = v;
        a.keys[(size_t)i * a.R + j] = on ? (((uint64_t)v << 32) | L->sel_dist[j]) : JX_EMPTY_KEY;
        a.vals[(size_t)i * a.R + j] = on ? (uint32_t)xid : JX_NONE_ID;
    }
    if (a.clean && lane == 0) a.clean[xid] = (uint8_t)(nsel < 255 ? nsel : 255);
}

template <int KIND, int T, int CPL>
__global__ void __launch_bounds__(INS_WPB * 64) reverse_merge_kernel(InsertArgs a) {
    __shared__ PruneLds lds[INS_WPB];
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int g = lane / T, lig = lane % T;
    PruneLds* L = &lds[wave];
    extern __shared__ __align__(16) unsigned char vcache[];  // INS_WPB x vec_cache_bytes
    const long long nseg = *a.nseg;
    const long long total = a.E ? a.E : a.B * a.R;
    for (long long s = (long long)blockIdx.x * INS_WPB + wave; s < nseg; s += (long long)gridDim.x * INS_WPB) {
        const uint32_t head = a.heads[s];
        if (head & 0x80000000u) continue;  // merged by the Gram-matrix kernel, which marks what it has done
        const long long lo = head;
        const uint32_t v = (uint32_t)(a.keys[lo] >> 32);
        if (v == JX_NONE_ID) continue;  // tail of empty keys
        // segment length
        int m = 0;
        for (long long c0 = lo; c0 < total; c0 += 64) {
            const long long j = c0 + lane;
            const bool same = j < total && (uint32_t)(a.keys[j] >> 32) == v;
            const uint64_t sm = ballot(same);
            m += __builtin_popcountll(sm);
            if (sm != ~0ull) break;
        }
        uint32_t* row = a.adj + (size_t)v * a.R;
        int deg = 0;
        for (int rb = 0; rb < a.R; rb += 64) {
            const bool on = rb + lane < a.R && row[rb + lane] != JX_NONE_ID;
            deg += __builtin_popcountll(ballot(on));
        }
        if (a.force_prune) deg = 0;  // consolidation: the segment holds the whole candidate set
        int nclean = (a.clean && !a.force_prune) ? (int)a.clean[v] : 0;
        if (nclean > deg) nclean = deg;
        if (!a.force_prune && deg + m <= a.R) {
            for (int j = lane; j < m; j += 64) row[deg + j] = a.vals[lo + j];
            continue;
        }
        // distances from v to its existing neighbours, then sort them
        QueryRegs<KIND, CPL, 0> q;
        load_query<KIND, T, CPL, 0>(q, a.ds, (int64_t)v, lig);
        for (int c0 = 0; c0 < deg; c0 += 64) {
            const int nn = deg - c0 < 64 ? deg - c0 : 64;
            if (lane < nn) L->cand_id[lane] = row[c0 + lane];
            wave_sync();
            for (int s0 = 0; s0 < nn; s0 += G * U)
                eval_batch<KIND, T, CPL, 0, U>(q, a.ds, s0, nn, L->cand_id, L->cand_key, g, lig);
            wave_sync();
            if (lane < nn) {
                const uint64_t k = L->cand_key[lane];
                const float dd = code_to_dist<KIND>(key_dist(k));
                L->a_tmp[c0 + lane] = ((uint64_t)__float_as_uint(dd) << 32) | (uint64_t)key_id(k);
            }
            wave_sync();
        }
        // Small case (the usual one: a full row plus a few new edges): merge both
        // lists into one, pull all candidate vectors into LDS once, and run the
        // selection loop on the cache -- no global load on its critical path.
        const int M = deg + m;
        const bool cached = M <= INS_RA && (long long)M * a.ds.rec_stride <= a.vec_cache_bytes;
        if (cached) {
            for (int j = lane; j < m; j += 64)
                L->a_tmp[deg + j] = ((uint64_t)reinterpret_cast<const uint32_t*>(a.keys + lo + j)[0] << 32) | a.vals[lo + j];
            wave_sync();
        }
        const int nsort = cached ? M : deg;
        // few entries besides those one earlier call selected together: only their pairs need evaluating
        const bool incremental = KIND == K_U8 && cached && a.ds.rec_stride == 128 && M <= 128 && M - nclean <= 12 && nclean > 0;
        for (int j = lane; j < nsort; j += 64) {
            const uint64_t k = L->a_tmp[j];
            int rank = 0;
            for (int t = 0; t < nsort; t++) rank += (L->a_tmp[t] < k) ? 1 : 0;
            L->a_key[rank] = k;
            if (incremental)
                L->a_dead[rank] = j >= nclean ? 1 : 0;
            else
                L->a_dead[j] = 0;
        }
        int nsel;
        if (cached) {
            wave_sync();
            unsigned char* vc = vcache + (size_t)wave * a.vec_cache_bytes;
            const int nch = a.ds.nch;
            for (int c = lane; c < M * nch; c += 64) {
                const int sl = c / nch, ch = c - sl * nch;
                const uint32_t id = (uint32_t)L->a_key[sl];
                *reinterpret_cast<uint4*>(vc + (size_t)sl * a.ds.rec_stride + ch * 16) =
                    load16(a.ds.recs + (size_t)id * (size_t)a.ds.rec_stride + (size_t)ch * 16);
            }
            DistSrc cds = a.ds;
            cds.recs = vc;
            cds.qrecs = vc;
            BList none;
            none.ids = nullptr;
            none.dbits = nullptr;
            none.id_stride = none.d_stride = 1;
            none.n = 0;
            none.dead = nullptr;
            __threadfence_block();
            wave_sync();
            if constexpr (KIND == K_U8) {
                if (incremental)
                    nsel = prune_cached_u8_incremental<T, CPL>(cds, L, M, a.R, a.alpha);
                else if (a.ds.rec_stride == 128 && M <= 128 && (long long)((M + 31) & ~31) * 128 <= a.vec_cache_bytes)
                    nsel = prune_cached_u8_mfma(L, vc, M, a.R, a.alpha);
                else
                    nsel = robust_prune_wave<KIND, T, CPL, true>(cds, L, M, none, a.R, a.alpha);
            } else
                nsel = robust_prune_wave<KIND, T, CPL, true>(cds, L, M, none, a.R, a.alpha);
        } else {
            BList B;
            B.ids = a.vals + lo;
            B.dbits = reinterpret_cast<const uint32_t*>(a.keys + lo);
            B.id_stride = 1;
            B.d_stride = 2;
            B.dead = a.dead + lo;
            // A hub (the entry point, vertices near it) can receive thousands of reverse edges in one batch, and every
            // selection of the loop below passes over all live candidates.  Alg. 3 visits candidates in (distance, id)
            // order, stops at R selections, and what happens to a candidate depends on earlier ones only: prune a
            // prefix of the sorted new edges first; if the R-th selection comes no later than the last included new
            // edge, the excluded ones could not have mattered and the result is exact.  Otherwise take four times as many.
            int mp = m < 512 ? m : 512;
            for (;;) {
                B.n = mp;
                for (int j = lane; j < mp; j += 64) B.dead[j] = 0;
                for (int j = lane; j < deg; j += 64) L->a_dead[j] = 0;
                __threadfence_block();
                wave_sync();
                nsel = robust_prune_wave<KIND, T, CPL, false>(a.ds, L, deg, B, a.R, a.alpha);
                if (mp == m) break;
                const uint64_t tau = ((uint64_t)B.dbits[(size_t)(mp - 1) * 2] << 32) | B.ids[mp - 1];
                if (nsel >= a.R && (((uint64_t)L->sel_dist[nsel - 1] << 32) | L->sel_id[nsel - 1]) <= tau) break;
                mp = (long long)mp * 4 < m ? mp * 4 : m;
            }
        }
        for (int j = lane; j < a.R; j += 64) row[j] = j < nsel ? L->sel_id[j] : JX_NONE_ID;
        if (a.clean && lane == 0) a.clean[v] = (uint8_t)(nsel < 255 ? nsel : 255);
        wave_sync();
    }
}

// Reverse-edge merge, lean form for the case that dominates streaming inserts into uint8 indices of 128-byte
// vectors: the row overflows, all but a few (LEAN_ND) of its candidates were selected together by the row's previous
// robustPrune call (see prune_cached_u8_incremental for why their pairs need no test), and everything fits 128
// slots.  One pass over the candidates' vectors in global memory yields d(v,c) and d(x,c) for every entry x that
// is appended or new (v and those entries sit in registers); ranks come from merging them into the sorted prefix;
// Alg. 3 is the same walk over the marked entries.  No vector cache in LDS, so five times as many wavefronts are
// resident as in the general kernel, which then finds these segments marked as done (bit 31 of the head).
#define LEAN_ND 12  // marked entries per row the lean kernel accepts (taken four at a time)
struct LeanLds {
    uint64_t key[128];      // (float bits of d(v,c), id), candidate order: the row, then the new edges
    uint64_t skey[128];     // the same, sorted
    uint32_t id[128];
    uint32_t dd[LEAN_ND][128];  // d(marked entry k, candidate j), candidate order
    uint8_t orig[128];      // candidate index of sorted position p
    uint8_t flag[128];      // sorted position p: 0 = selected by the previous call, else 1 + index of the marked entry
};

__global__ void __launch_bounds__(64) reverse_merge_u8_lean_kernel(InsertArgs a) {
    __shared__ LeanLds lds;
    LeanLds* F = &lds;
    const int lane = lane_id();
    const int g = lane >> 2, lig = lane & 3;
    const long long nseg = *a.nseg;
    const long long total = a.E ? a.E : a.B * a.R;
    const uint8_t* recs = a.ds.recs;
    for (long long s = blockIdx.x; s < nseg; s += gridDim.x) {
        const uint32_t head = a.heads[s];
        if (head & 0x80000000u) continue;
        const long long lo = head;
        const uint32_t v = (uint32_t)(a.keys[lo] >> 32);
        if (v == JX_NONE_ID) continue;
        int m = 0;
        for (long long c0 = lo; c0 < total; c0 += 64) {
            const long long j = c0 + lane;
            const bool same = j < total && (uint32_t)(a.keys[j] >> 32) == v;
            const uint64_t sm = ballot(same);
            m += __builtin_popcountll(sm);
            if (sm != ~0ull) break;
        }
        uint32_t* row = a.adj + (size_t)v * a.R;
        int deg = 0;
        for (int rb = 0; rb < a.R; rb += 64) {
            const bool on = rb + lane < a.R && row[rb + lane] != JX_NONE_ID;
            deg += __builtin_popcountll(ballot(on));
        }
        if (deg + m <= a.R) {  // the row still fits: append in (distance, source) order
            for (int j = lane; j < m; j += 64) row[deg + j] = a.vals[lo + j];
            if (lane == 0) const_cast<uint32_t*>(a.heads)[s] = head | 0x80000000u;
            continue;
        }
        int nclean = (int)a.clean[v];
        if (nclean > deg) nclean = deg;
        const int M = deg + m, nd = M - nclean;
        if (nclean == 0 || M > 128 || nd > LEAN_ND) continue;
        wave_sync();  // the previous segment's reads of the LDS arrays are done
        for (int j = lane; j < M; j += 64) F->id[j] = j < deg ? row[j] : a.vals[lo + (j - deg)];
        wave_sync();
        auto sq = [](const uint4 (&x)[2]) {
            uint32_t t = 0;
            t = __builtin_amdgcn_udot4(x[0].x, x[0].x, t, false);
            t = __builtin_amdgcn_udot4(x[0].y, x[0].y, t, false);
            t = __builtin_amdgcn_udot4(x[0].z, x[0].z, t, false);
            t = __builtin_amdgcn_udot4(x[0].w, x[0].w, t, false);
            t = __builtin_amdgcn_udot4(x[1].x, x[1].x, t, false);
            t = __builtin_amdgcn_udot4(x[1].y, x[1].y, t, false);
            t = __builtin_amdgcn_udot4(x[1].z, x[1].z, t, false);
            t = __builtin_amdgcn_udot4(x[1].w, x[1].w, t, false);
            return t;
        };
        auto dot = [](const uint4 (&x)[2], const uint4 (&y)[2]) {
            uint32_t t = 0;
            t = __builtin_amdgcn_udot4(x[0].x, y[0].x, t, false);
            t = __builtin_amdgcn_udot4(x[0].y, y[0].y, t, false);
            t = __builtin_amdgcn_udot4(x[0].z, y[0].z, t, false);
            t = __builtin_amdgcn_udot4(x[0].w, y[0].w, t, false);
            t = __builtin_amdgcn_udot4(x[1].x, y[1].x, t, false);
            t = __builtin_amdgcn_udot4(x[1].y, y[1].y, t, false);
            t = __builtin_amdgcn_udot4(x[1].z, y[1].z, t, false);
            t = __builtin_amdgcn_udot4(x[1].w, y[1].w, t, false);
            return t;
        };
        // v and four marked entries at a time sit in registers, 32 bytes per lane of each 4-lane group; every group
        // of four takes one pass over the candidates (16 per step, two steps in flight)
        uint4 qv[2];
        {
            const uint8_t* pv = recs + (size_t)v * 128 + lig * 32;
            qv[0] = load16(pv);
            qv[1] = load16(pv + 16);
        }
        const uint32_t qqv = group_sum<4>(sq(qv));
        for (int kb = 0; kb < nd; kb += 4) {
            const int nk = nd - kb < 4 ? nd - kb : 4;
            uint4 qd[4][2];
            uint32_t qqd[4];
#pragma unroll
            for (int k = 0; k < 4; k++) {
                const uint32_t idk = F->id[nclean + kb + (k < nk ? k : 0)];
                const uint8_t* pk = recs + (size_t)idk * 128 + lig * 32;
                qd[k][0] = load16(pk);
                qd[k][1] = load16(pk + 16);
            }
#pragma unroll
            for (int k = 0; k < 4; k++) qqd[k] = group_sum<4>(sq(qd[k]));
            for (int c0 = 0; c0 < M; c0 += 32) {
                uint4 x[2][2];
                int jj[2];
#pragma unroll
                for (int u = 0; u < 2; u++) {
                    jj[u] = c0 + 16 * u + g;
                    const uint32_t id = F->id[jj[u] < M ? jj[u] : M - 1];
                    const uint8_t* px = recs + (size_t)id * 128 + lig * 32;
                    x[u][0] = load16(px);
                    x[u][1] = load16(px + 16);
                }
#pragma unroll
                for (int u = 0; u < 2; u++) {
                    if (c0 + 16 * u >= M) break;  // wave-uniform
                    const uint32_t aa = dot(x[u], x[u]);
                    uint32_t dv = 0;
                    if (kb == 0) dv = (uint32_t)group_sum<4>((int32_t)aa - 2 * (int32_t)dot(x[u], qv)) + qqv;
                    uint32_t dk[4];
#pragma unroll
                    for (int k = 0; k < 4; k++) {
                        dk[k] = 0;
                        if (k < nk) dk[k] = (uint32_t)group_sum<4>((int32_t)aa - 2 * (int32_t)dot(x[u], qd[k])) + qqd[k];
                    }
                    if (lig == 0 && jj[u] < M) {
                        if (kb == 0) F->key[jj[u]] = ((uint64_t)__float_as_uint((float)dv) << 32) | (uint64_t)F->id[jj[u]];
#pragma unroll
                        for (int k = 0; k < 4; k++)
                            if (k < nk) F->dd[kb + k][jj[u]] = dk[k];
                    }
                }
            }
        }
        wave_sync();
        // ranks: the prefix is sorted already and every marked entry is merged into it.  Prefix entry: own index +
        // marked entries below it; marked entry: prefix entries below it + marked entries below it
        uint64_t kj[2];
        int rank[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int j = h * 64 + lane;
            kj[h] = j < M ? F->key[j] : JX_EMPTY_KEY;
            rank[h] = j < nclean ? j : 0;
        }
        for (int k = 0; k < nd; k++) {
            const uint64_t kt = F->key[nclean + k];
            const int below = __builtin_popcountll(ballot(lane < nclean && kj[0] < kt)) +
                              __builtin_popcountll(ballot(64 + lane < nclean && kj[1] < kt));
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int j = h * 64 + lane;
                rank[h] += (kt < kj[h]) ? 1 : 0;
                if (j == nclean + k) rank[h] += below;
            }
        }
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int j = h * 64 + lane;
            if (j < M) {
                F->skey[rank[h]] = kj[h];
                F->orig[rank[h]] = (uint8_t)j;
                F->flag[rank[h]] = j >= nclean ? (uint8_t)(1 + j - nclean) : (uint8_t)0;
            }
        }
        wave_sync();
        // Alg. 3 over the marked entries, sorted space
        uint64_t sk[2], dm[2], alive[2];
        float dvp[2];
        int og[2];
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int p = h * 64 + lane;
            sk[h] = p < M ? F->skey[p] : JX_EMPTY_KEY;
            dvp[h] = __uint_as_float((uint32_t)(sk[h] >> 32));
            og[h] = p < M ? (int)F->orig[p] : 0;
            dm[h] = ballot(p < M && F->flag[p] != 0);
        }
        alive[0] = M >= 64 ? ~0ull : ((1ull << M) - 1ull);
        alive[1] = M <= 64 ? 0ull : (M >= 128 ? ~0ull : ((1ull << (M - 64)) - 1ull));
        while (dm[0] | dm[1]) {
            int t;
            if (dm[0]) {
                t = __builtin_ctzll(dm[0]);
                dm[0] &= dm[0] - 1ull;
            } else {
                t = 64 + __builtin_ctzll(dm[1]);
                dm[1] &= dm[1] - 1ull;
            }
            if (((alive[t >> 6] >> (t & 63)) & 1ull) == 0ull) continue;
            const int k = (int)F->flag[t] - 1;
            const float dvt = __uint_as_float((uint32_t)(F->skey[t] >> 32));
            uint64_t rk[2], ck[2];
#pragma unroll
            for (int h = 0; h < 2; h++) {
                const int p = h * 64 + lane;
                const float d1 = (float)F->dd[k][og[h]];
                const float ad = __fmul_rn(a.alpha, d1);
                rk[h] = ballot(p < M && p > t && ad <= dvp[h]);
                ck[h] = ballot(p < M && p < t && ad <= dvt);
            }
            if ((ck[0] & alive[0]) | (ck[1] & alive[1])) {
                alive[t >> 6] &= ~(1ull << (t & 63));
            } else {
                alive[0] &= ~rk[0];
                alive[1] &= ~rk[1];
            }
        }
        const int n0 = __builtin_popcountll(alive[0]);
        const int tot = n0 + __builtin_popcountll(alive[1]);
        const int nsel = tot < a.R ? tot : a.R;
#pragma unroll
        for (int h = 0; h < 2; h++) {
            const int p = h * 64 + lane;
            if (p < M && ((alive[h] >> lane) & 1ull)) {
                const int pos = (h ? n0 : 0) + __builtin_popcountll(alive[h] & ((1ull << lane) - 1ull));
                if (pos < a.R) row[pos] = (uint32_t)sk[h];
            }
        }
        for (int j = nsel + lane; j < a.R; j += 64) row[j] = JX_NONE_ID;
        if (lane == 0) {
            a.clean[v] = (uint8_t)(nsel < 255 ? nsel : 255);
            const_cast<uint32_t*>(a.heads)[s] = head | 0x80000000u;
        }
    }
}

// Forward robustPrune, lean form for uint8 vectors of 128 bytes and frontiers of at most 128 entries.  The
// selection loop of Alg. 3 has one dependent memory round trip per selected neighbour; here up to four pivots --
// the next live candidates in order -- are taken per round: one pass over the live candidates behind the first
// pivot loads every vector once and tests it against all four (the pivots sit in registers), then the pivots are
// resolved in order: a pivot that is still live is selected and discards what it discards, one that an earlier
// pivot discarded is skipped (its tests were wasted).  Every test is the pairwise test of Alg. 3 on exact
// integers, so the result is the sequential algorithm's.
template <int MAXC>
struct FwdLds {
    uint32_t id[MAXC];
    float dx[MAXC];        // d(x, candidate)
    uint32_t sel_id[MAXC];
    uint32_t sel_dist[MAXC];
    uint16_t cand[MAXC];   // live candidates behind the first pivot, compacted
    uint8_t kb[MAXC];      // bit i: pivot i discards this candidate
};

// The rounds described above on the candidates F->id / F->dx (sorted by (distance, id); alive = one bit per
// candidate).  Returns the number of selected neighbours, F->sel_id / F->sel_dist in selection order.
template <int MAXC>
__device__ __forceinline__ int multi_pivot_prune_u8(FwdLds<MAXC>* F, const uint8_t* recs, uint64_t (&alive)[MAXC / 64], const int R,
                                                    const float alpha) {
    constexpr int NW = MAXC / 64;
    const int lane = lane_id();
    const int g = lane >> 2, lig = lane & 3;
    auto dot = [](const uint4 (&x)[2], const uint4 (&y)[2]) {
        uint32_t t = 0;
        t = __builtin_amdgcn_udot4(x[0].x, y[0].x, t, false);
        t = __builtin_amdgcn_udot4(x[0].y, y[0].y, t, false);
        t = __builtin_amdgcn_udot4(x[0].z, y[0].z, t, false);
        t = __builtin_amdgcn_udot4(x[0].w, y[0].w, t, false);
        t = __builtin_amdgcn_udot4(x[1].x, y[1].x, t, false);
        t = __builtin_amdgcn_udot4(x[1].y, y[1].y, t, false);
        t = __builtin_amdgcn_udot4(x[1].z, y[1].z, t, false);
        t = __builtin_amdgcn_udot4(x[1].w, y[1].w, t, false);
        return t;
    };
    auto any_alive = [&]() {
        uint64_t m = 0;
#pragma unroll
        for (int w = 0; w < NW; w++) m |= alive[w];
        return m != 0ull;
    };
    int nsel = 0;
    while (nsel < R && any_alive()) {
        // ---- pivots: the next live candidates, as many as may still be selected, at most four
        int t[4], np = 0;
        {
            uint64_t m[NW];
#pragma unroll
            for (int w = 0; w < NW; w++) m[w] = alive[w];
            const int room = R - nsel < 4 ? R - nsel : 4;
#pragma unroll
            for (int k = 0; k < 4; k++) {
                t[k] = 0;
                if (k < room) {
                    bool found = false;
#pragma unroll
                    for (int w = 0; w < NW; w++) {
                        if (!found && m[w]) {
                            t[k] = 64 * w + __builtin_ctzll(m[w]);
                            m[w] &= m[w] - 1ull;
                            np = k + 1;
                            found = true;
                        }
                    }
                }
            }
        }
        // ---- live candidates behind the first pivot
        int n_alive = 0;
#pragma unroll
        for (int h = 0; h < NW; h++) {
            const int j = h * 64 + lane;
            const bool on = ((alive[h] >> lane) & 1ull) && j > t[0];
            const uint64_t m = ballot(on);
            if (on) F->cand[n_alive + prefix_count(m)] = (uint16_t)j;
            n_alive += __builtin_popcountll(m);
        }
        if (n_alive == 0 || nsel + 1 >= R) {
            // the last neighbour there is, or the last one there is room for: nothing left to discard
            if (lane == 0) {
                F->sel_id[nsel] = F->id[t[0]];
                F->sel_dist[nsel] = __float_as_uint(F->dx[t[0]]);
            }
            nsel++;
            break;
        }
        wave_sync();
        uint4 qd[4][2];
        uint32_t qqd[4];
#pragma unroll
        for (int k = 0; k < 4; k++) {
            const uint32_t idk = F->id[t[k < np ? k : 0]];
            const uint8_t* pk = recs + (size_t)idk * 128 + lig * 32;
            qd[k][0] = load16(pk);
            qd[k][1] = load16(pk + 16);
        }
#pragma unroll
        for (int k = 0; k < 4; k++) qqd[k] = group_sum<4>(dot(qd[k], qd[k]));
        for (int c0 = 0; c0 < n_alive; c0 += 32) {
            uint4 x[2][2];
            int jj[2], jc[2];
#pragma unroll
            for (int u = 0; u < 2; u++) {
                jj[u] = c0 + 16 * u + g;
                jc[u] = (int)F->cand[jj[u] < n_alive ? jj[u] : n_alive - 1];
                const uint8_t* px = recs + (size_t)F->id[jc[u]] * 128 + lig * 32;
                x[u][0] = load16(px);
                x[u][1] = load16(px + 16);
            }
#pragma unroll
            for (int u = 0; u < 2; u++) {
                if (c0 + 16 * u >= n_alive) break;  // wave-uniform
                const uint32_t aa = dot(x[u], x[u]);
                uint32_t bits = 0;
                const float dxc = F->dx[jc[u]];
#pragma unroll
                for (int k = 0; k < 4; k++) {
                    if (k < np) {
                        const uint32_t dk = (uint32_t)group_sum<4>((int32_t)aa - 2 * (int32_t)dot(x[u], qd[k])) + qqd[k];
                        if (jc[u] > t[k] && __fmul_rn(alpha, (float)dk) <= dxc) bits |= 1u << k;
                    }
                }
                if (lig == 0 && jj[u] < n_alive) F->kb[jc[u]] = (uint8_t)bits;
            }
        }
        wave_sync();
        uint64_t K[4][NW];
#pragma unroll
        for (int h = 0; h < NW; h++) {
            const int j = h * 64 + lane;
            const bool on = ((alive[h] >> lane) & 1ull) && j > t[0];
            const uint32_t b = on ? (uint32_t)F->kb[j] : 0u;
#pragma unroll
            for (int k = 0; k < 4; k++) K[k][h] = ballot((b >> k) & 1u);
        }
        // ---- resolve the pivots in order
#pragma unroll
        for (int k = 0; k < 4; k++) {
            if (k < np && nsel < R) {
                const int tk = t[k];
                bool live = false;
#pragma unroll
                for (int w = 0; w < NW; w++)
                    if (w == (tk >> 6)) live = (alive[w] >> (tk & 63)) & 1ull;
                if (live) {
                    if (lane == 0) {
                        F->sel_id[nsel] = F->id[tk];
                        F->sel_dist[nsel] = __float_as_uint(F->dx[tk]);
                    }
                    nsel++;
#pragma unroll
                    for (int w = 0; w < NW; w++) {
                        if (w == (tk >> 6)) alive[w] &= ~(1ull << (tk & 63));
                        alive[w] &= ~K[k][w];
                    }
                }
            }
        }
        wave_sync();
    }
    wave_sync();
    return nsel;
}

// N = 128 (final frontiers of L_build <= 128) or 512 (expansion lists)
template <int N>
__global__ void __launch_bounds__(64) forward_prune_u8_lean_kernel(InsertArgs a) {
    __shared__ FwdLds<N> lds;
    FwdLds<N>* F = &lds;
    const int lane = lane_id();
    const long long i = blockIdx.x;
    if (i >= a.B) return;
    long long xid = a.id_base + i;
    if (xid >= a.id_skip) xid++;
    const uint32_t* ids = a.cand_ids + (size_t)i * a.L;
    const uint32_t* dbits = a.cand_dist + (size_t)i * a.L;
    uint64_t alive[N / 64];
#pragma unroll
    for (int h = 0; h < N / 64; h++) {
        const int j = h * 64 + lane;
        uint32_t id = JX_NONE_ID;
        if (j < a.L) id = ids[j];
        const bool valid = id != JX_NONE_ID;
        if (valid) {
            F->id[j] = id;
            F->dx[j] = __uint_as_float(dbits[j]);
        }
        alive[h] = ballot(valid);  // the frontier is filled from the left
    }
    wave_sync();
    const int nsel = multi_pivot_prune_u8<N>(F, a.ds.recs, alive, a.R, a.alpha);
    uint32_t* row = a.adj + (size_t)xid * a.R;
    for (int j = lane; j < a.R; j += 64) {
        const bool on = j < nsel;
        const uint32_t v = on ? F->sel_id[j] : JX_NONE_ID;
        row[j] = v;
        a.keys[(size_t)i * a.R + j] = on ? (((uint64_t)v << 32) | F->sel_dist[j]) : JX_EMPTY_KEY;
        a.vals[(size_t)i * a.R + j] = on ? (uint32_t)xid : JX_NONE_ID;
    }
    if (a.clean && lane == 0) a.clean[xid] = (uint8_t)(nsel < 255 ? nsel : 255);
}

// The same rounds for consolidation after deletions (Sec. 4.6): the segment holds the whole candidate set of its
// vertex, sorted by (distance, id); sets of at most 512 are pruned here and marked, larger ones are left to the
// general kernel.
__global__ void __launch_bounds__(64) consol_prune_u8_lean_kernel(InsertArgs a) {
    __shared__ FwdLds<512> lds;
    FwdLds<512>* F = &lds;
    const int lane = lane_id();
    const long long nseg = *a.nseg;
    const long long total = a.E ? a.E : a.B * a.R;
    for (long long s = blockIdx.x; s < nseg; s += gridDim.x) {
        const uint32_t head = a.heads[s];
        if (head & 0x80000000u) continue;
        const long long lo = head;
        const uint32_t v = (uint32_t)(a.keys[lo] >> 32);
        if (v == JX_NONE_ID) continue;
        int m = 0;
        for (long long c0 = lo; c0 < total; c0 += 64) {
            const long long j = c0 + lane;
            const bool same = j < total && (uint32_t)(a.keys[j] >> 32) == v;
            const uint64_t sm = ballot(same);
            m += __builtin_popcountll(sm);
            if (sm != ~0ull) break;
        }
        if (m > 512) continue;
        wave_sync();  // the previous segment's reads of the LDS arrays are done
        uint64_t alive[8];
#pragma unroll
        for (int h = 0; h < 8; h++) {
            const int j = h * 64 + lane;
            const bool valid = j < m;
            if (valid) {
                F->id[j] = a.vals[lo + j];
                F->dx[j] = __uint_as_float((uint32_t)a.keys[lo + j]);
            }
            alive[h] = ballot(valid);
        }
        wave_sync();
        const int nsel = multi_pivot_prune_u8<512>(F, a.ds.recs, alive, a.R, a.alpha);
        uint32_t* row = a.adj + (size_t)v * a.R;
        for (int j = lane; j < a.R; j += 64) row[j] = j < nsel ? F->sel_id[j] : JX_NONE_ID;
        if (lane == 0) {
            if (a.clean) a.clean[v] = (uint8_t)(nsel < 255 ? nsel : 255);
            const_cast<uint32_t*>(a.heads)[s] = head | 0x80000000u;
        }
    }
}

// ------------------------------------------------------------------ radix sort

#define RS_ITEMS 16
#define RS_TILE (256 * RS_ITEMS)

// exclusive prefix sum of `total` counters, single workgroup
__global__ void __launch_bounds__(1024) radix_scan_kernel(uint32_t* table, long long total) {
    __shared__ uint32_t ws[16];
    __shared__ uint32_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (long long c0 = 0; c0 < total; c0 += 1024) {
        const long long i = c0 + threadIdx.x;
        const uint32_t v = i < total ? table[i] : 0u;
        uint32_t x = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            uint32_t o = __shfl_up(x, s, 64);
            if (lane >= s) x += o;
        }
        if (lane == 63) ws[wave] = x;
        __syncthreads();
        uint32_t woff = 0;
        for (int w = 0; w < wave; w++) woff += ws[w];
        const uint32_t carry = carry_s;
        if (i < total) table[i] = carry + woff + x - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = carry + woff + x;
        __syncthreads();
    }
}

// 8-bit digits.  A tile of 4,096 keys is sorted on the digit inside LDS by two stable 4-bit passes (every thread
// counts the 16 keys it holds per nibble value; an exclusive scan over the counters in nibble-major, thread-minor
// order gives each key its rank), then written out run by run.
__global__ void __launch_bounds__(256) radix_hist8_kernel(const uint64_t* keys, long long n, int shift, uint32_t* table, int ntiles) {
    __shared__ uint32_t cnt[256];
    cnt[threadIdx.x] = 0;
    __syncthreads();
    const long long base = (long long)blockIdx.x * RS_TILE;
#pragma unroll
    for (int e = 0; e < RS_ITEMS; e++) {
        const long long i = base + e * 256 + threadIdx.x;
        if (i < n) atomicAdd(&cnt[(keys[i] >> shift) & 255], 1u);
    }
    __syncthreads();
    table[(size_t)threadIdx.x * ntiles + blockIdx.x] = cnt[threadIdx.x];
}

// one workgroup per digit: exclusive prefix sum over the tiles of its row, row total to table[256 * ntiles + digit]
__global__ void __launch_bounds__(1024) radix_rowscan8_kernel(uint32_t* table, int ntiles) {
    __shared__ uint32_t ws[16];
    __shared__ uint32_t carry_s;
    uint32_t* row = table + (size_t)blockIdx.x * ntiles;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c0 = 0; c0 < ntiles; c0 += 1024) {
        const int i = c0 + threadIdx.x;
        const uint32_t v = i < ntiles ? row[i] : 0u;
        uint32_t x = v;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            uint32_t o = __shfl_up(x, s, 64);
            if (lane >= s) x += o;
        }
        if (lane == 63) ws[wave] = x;
        __syncthreads();
        uint32_t woff = 0;
        for (int w = 0; w < wave; w++) woff += ws[w];
        const uint32_t carry = carry_s;
        if (i < ntiles) row[i] = carry + woff + x - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = carry + woff + x;
        __syncthreads();
    }
    if (threadIdx.x == 0) table[(size_t)256 * ntiles + blockIdx.x] = carry_s;
}

// exclusive scan of psum[256] in place by the first wavefront (4 entries per lane); callers synchronise around it
__device__ __forceinline__ void scan256_wave0(uint32_t* psum, int t) {
    if (t < 64) {
        uint32_t a0 = psum[4 * t], a1 = psum[4 * t + 1], a2 = psum[4 * t + 2], a3 = psum[4 * t + 3];
        uint32_t tot = a0 + a1 + a2 + a3, x = tot;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            uint32_t o = __shfl_up(x, s, 64);
            if (t >= s) x += o;
        }
        uint32_t ex = x - tot;
        psum[4 * t] = ex;
        psum[4 * t + 1] = ex + a0;
        psum[4 * t + 2] = ex + a0 + a1;
        psum[4 * t + 3] = ex + a0 + a1 + a2;
    }
}

__global__ void __launch_bounds__(256) radix_scatter8_kernel(const uint64_t* keys, const uint32_t* vals, uint64_t* keys_out,
                                                            uint32_t* vals_out, long long n, int shift,
                                                            const uint32_t* table, int ntiles) {
    __shared__ uint64_t sk[RS_TILE];
    __shared__ uint32_t sv[RS_TILE];
    __shared__ uint16_t hist[16 * 256];  // [digit][thread]
    __shared__ uint32_t psum[256];
    __shared__ uint32_t gbase[256];
    __shared__ uint16_t dstart[256];
    const int t = threadIdx.x;
    const long long tile0 = (long long)blockIdx.x * RS_TILE;
    const int cnt = (int)(n - tile0 < (long long)RS_TILE ? n - tile0 : (long long)RS_TILE);
    // where each digit's run of this tile starts in the output: digits below it, then the tiles before this one
    psum[t] = table[(size_t)256 * ntiles + t];
    __syncthreads();
    scan256_wave0(psum, t);
    __syncthreads();
    gbase[t] = psum[t] + table[(size_t)t * ntiles + blockIdx.x];
    uint64_t k[RS_ITEMS];
    uint32_t v[RS_ITEMS];
#pragma unroll
    for (int e = 0; e < RS_ITEMS; e++) {
        const long long i = tile0 + (long long)t * RS_ITEMS + e;
        k[e] = i < n ? keys[i] : JX_EMPTY_KEY;  // padding carries the largest digit and comes last in the tile: it stays last
        v[e] = i < n ? vals[i] : 0u;
    }
    __syncthreads();
#pragma unroll
    for (int half = 0; half < 2; half++) {
        const int sh = shift + 4 * half;
#pragma unroll
        for (int d = 0; d < 16; d++) hist[d * 256 + t] = 0;
#pragma unroll
        for (int e = 0; e < RS_ITEMS; e++) hist[((k[e] >> sh) & 15) * 256 + t]++;
        __syncthreads();
        uint32_t loc[16];
        uint32_t sum = 0;
#pragma unroll
        for (int e = 0; e < 16; e++) {
            loc[e] = sum;
            sum += hist[t * 16 + e];
        }
        psum[t] = sum;
        __syncthreads();
        scan256_wave0(psum, t);
        __syncthreads();
        const uint32_t off = psum[t];
#pragma unroll
        for (int e = 0; e < 16; e++) hist[t * 16 + e] = (uint16_t)(off + loc[e]);
        __syncthreads();
#pragma unroll
        for (int e = 0; e < RS_ITEMS; e++) {
            const int d = (int)((k[e] >> sh) & 15);
            const uint32_t r = hist[d * 256 + t];
            hist[d * 256 + t] = (uint16_t)(r + 1);
            sk[r] = k[e];
            sv[r] = v[e];
        }
        __syncthreads();
        if (half == 0) {
#pragma unroll
            for (int e = 0; e < RS_ITEMS; e++) {
                k[e] = sk[t * RS_ITEMS + e];
                v[e] = sv[t * RS_ITEMS + e];
            }
            __syncthreads();
        }
    }
    for (int i = t; i < cnt; i += 256) {
        const int d = (int)((sk[i] >> shift) & 255);
        if (i == 0 || (int)((sk[i - 1] >> shift) & 255) != d) dstart[d] = (uint16_t)i;
    }
    __syncthreads();
    for (int i = t; i < cnt; i += 256) {
        const uint64_t key = sk[i];
        const int d = (int)((key >> shift) & 255);
        const size_t pos = (size_t)gbase[d] + (size_t)(i - dstart[d]);
        keys_out[pos] = key;
        vals_out[pos] = sv[i];
    }
}

__global__ void __launch_bounds__(1024) segment_heads_kernel(const uint64_t* keys, long long n, uint32_t* heads, uint32_t* nseg) {
    __shared__ uint32_t woff[17];
    const int lane = lane_id(), wave = threadIdx.x >> 6;
    // 4 consecutive keys per thread
    const long long i0 = ((long long)blockIdx.x * 1024 + threadIdx.x) * 4;
    bool is_head[4];
    int mine = 0;
    uint32_t prev = JX_NONE_ID;
    if (i0 > 0 && i0 < n) prev = (uint32_t)(keys[i0 - 1] >> 32);
#pragma unroll
    for (int e = 0; e < 4; e++) {
        const long long i = i0 + e;
        uint32_t t = JX_NONE_ID;
        if (i < n) t = (uint32_t)(keys[i] >> 32);
        is_head[e] = t != JX_NONE_ID && (i == 0 || t != prev);
        mine += is_head[e] ? 1 : 0;
        prev = t;
    }
    // one atomic per workgroup (same-address atomics serialise; the order of the list does not matter)
    uint32_t x = (uint32_t)mine;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        uint32_t o = __shfl_up(x, s, 64);
        if (lane >= s) x += o;
    }
    if (lane == 63) woff[wave] = x;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint32_t tot = 0;
        for (int w = 0; w < 16; w++) {
            const uint32_t c = woff[w];
            woff[w] = tot;
            tot += c;
        }
        woff[16] = tot ? atomicAdd(nseg, tot) : 0u;
    }
    __syncthreads();
    uint32_t pos = woff[16] + woff[wave] + x - (uint32_t)mine;
#pragma unroll
    for (int e = 0; e < 4; e++)
        if (is_head[e]) heads[pos++] = (uint32_t)(i0 + e);
}

// ------------------------------------------------------------------ launchers

hipError_t launch_entry_point(const void* vecs, int dtype, long long n, int d, double* partial, float* mean, double* dist,
                              uint32_t* out_id, hipStream_t st) {
    int nblk = (int)((n + 255) / 256);
    if (nblk > 512) nblk = 512;
    if (nblk < 1) nblk = 1;
    if (dtype == JX_U8)
        hipLaunchKernelGGL(col_partial_kernel<JX_U8>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    else if (dtype == JX_F16)
        hipLaunchKernelGGL(col_partial_kernel<JX_F16>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    else
        hipLaunchKernelGGL(col_partial_kernel<JX_F32>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    hipLaunchKernelGGL(mean_finalize_kernel, dim3((d + 255) / 256), dim3(256), 0, st, partial, nblk, d, n, mean);
    if (dtype == JX_U8)
        hipLaunchKernelGGL(dist_to_mean_kernel<JX_U8>, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, vecs, n, d, mean, dist);
    else if (dtype == JX_F16)
        hipLaunchKernelGGL(dist_to_mean_kernel<JX_F16>, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, vecs, n, d, mean, dist);
    else
        hipLaunchKernelGGL(dist_to_mean_kernel<JX_F32>, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, vecs, n, d, mean, dist);
    hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(1024), 0, st, dist, n, out_id);
    return hipGetLastError();
}

// column means only (two-stage, fixed order): the RaBitQ centroid
hipError_t launch_column_mean(const void* vecs, int dtype, long long n, int d, double* partial, float* mean, hipStream_t st) {
    int nblk = (int)((n + 255) / 256);
    if (nblk > 512) nblk = 512;
    if (nblk < 1) nblk = 1;
    if (dtype == JX_U8)
        hipLaunchKernelGGL(col_partial_kernel<JX_U8>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    else if (dtype == JX_F16)
        hipLaunchKernelGGL(col_partial_kernel<JX_F16>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    else
        hipLaunchKernelGGL(col_partial_kernel<JX_F32>, dim3(nblk), dim3(256), 0, st, vecs, n, d, nblk, partial);
    hipLaunchKernelGGL(mean_finalize_kernel, dim3((d + 255) / 256), dim3(256), 0, st, partial, nblk, d, n, mean);
    return hipGetLastError();
}

int entry_point_partial_blocks(long long n) {
    long long nblk = (n + 255) / 256;
    return (int)(nblk > 512 ? 512 : (nblk < 1 ? 1 : nblk));
}

template <int KIND, int T, int CPL>
static hipError_t launch_prune_pair(bool forward, const InsertArgs& a, hipStream_t st) {
    if (forward) {
        dim3 grid((unsigned)((a.B + INS_WPB - 1) / INS_WPB));
        const size_t sh = (size_t)INS_WPB * a.vec_cache_bytes;
        if (sh > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute((const void*)forward_prune_kernel<KIND, T, CPL>,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL((forward_prune_kernel<KIND, T, CPL>), grid, dim3(INS_WPB * 64), sh, st, a);
    } else {
        long long want = ((a.E ? a.E : a.B * a.R) + INS_WPB - 1) / INS_WPB;
        const long long cap = 16384 / INS_WPB;  // persistent wavefronts, segments dealt round-robin
        unsigned grid = (unsigned)(want < cap ? (want < 1 ? 1 : want) : cap);
        hipLaunchKernelGGL((reverse_merge_kernel<KIND, T, CPL>), dim3(grid), dim3(INS_WPB * 64),
                           (size_t)INS_WPB * a.vec_cache_bytes, st, a);
    }
    return hipGetLastError();
}

template <int KIND>
static hipError_t launch_prune_shape(bool forward, const InsertArgs& a, hipStream_t st) {
    // same record-to-lane mapping as beamSearch: 2 chunks per lane up to 64 chunks
    const int nch = a.ds.nch;
    if (nch <= 8) return launch_prune_pair<KIND, 4, 2>(forward, a, st);
    if (nch <= 16) return launch_prune_pair<KIND, 8, 2>(forward, a, st);
    if (nch <= 32) return launch_prune_pair<KIND, 16, 2>(forward, a, st);
    if (nch <= 64) return launch_prune_pair<KIND, 32, 2>(forward, a, st);
    if (nch <= 128) return launch_prune_pair<KIND, 64, 2>(forward, a, st);
    if (nch <= 256) return launch_prune_pair<KIND, 64, 4>(forward, a, st);
    if (nch <= 384) return launch_prune_pair<KIND, 64, 6>(forward, a, st);
    return hipErrorInvalidValue;
}

hipError_t launch_forward_prune(int dtype, const InsertArgs& a, hipStream_t st) {
    if (a.gram) {
        hipError_t e = launch_forward_prune_gram(dtype, a, st);
        if (e != hipSuccess || a.L <= 128) return e;  // wider frontiers: the list-based kernel takes the rest
    }
    if (dtype == JX_U8 && !a.gram && a.ds.rec_stride == 128 && a.ds.nch == 8 && a.L <= 512) {
        if (a.L <= 128)
            hipLaunchKernelGGL(forward_prune_u8_lean_kernel<128>, dim3((unsigned)a.B), dim3(64), 0, st, a);
        else
            hipLaunchKernelGGL(forward_prune_u8_lean_kernel<512>, dim3((unsigned)a.B), dim3(64), 0, st, a);
        return hipGetLastError();
    }
    if (dtype == JX_U8) return launch_prune_shape<K_U8>(true, a, st);
    if (dtype == JX_F16) return launch_prune_shape<K_F16>(true, a, st);
    return launch_prune_shape<K_F32>(true, a, st);
}

hipError_t launch_reverse_merge(int dtype, const InsertArgs& a, hipStream_t st) {
    if (a.gram) {
        hipError_t e = launch_reverse_merge_gram(dtype, a, st);
        if (e != hipSuccess) return e;
    }
    if (dtype == JX_U8 && a.force_prune && a.ds.rec_stride == 128 && a.ds.nch == 8) {
        // consolidation: candidate sets of at most 512 take the multi-pivot form
        const long long want = a.E ? a.E : a.B * a.R;
        const unsigned grid = (unsigned)(want < 8192 ? (want < 1 ? 1 : want) : 8192);
        hipLaunchKernelGGL(consol_prune_u8_lean_kernel, dim3(grid), dim3(64), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (dtype == JX_U8 && a.clean && !a.force_prune && a.ds.rec_stride == 128 && a.ds.nch == 8) {
        // overflowing rows that are almost entirely their previous prune's output: lean kernel first
        const long long want = a.E ? a.E : a.B * a.R;
        const unsigned grid = (unsigned)(want < 8192 ? (want < 1 ? 1 : want) : 8192);
        hipLaunchKernelGGL(reverse_merge_u8_lean_kernel, dim3(grid), dim3(64), 0, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (dtype == JX_U8) return launch_prune_shape<K_U8>(false, a, st);
    if (dtype == JX_F16) return launch_prune_shape<K_F16>(false, a, st);
    return launch_prune_shape<K_F32>(false, a, st);
}

// Sorts n (key, value) pairs on key bits [0, nbits), stable.  The result is in
// keys_a/vals_a again (an even number of passes is always run).
hipError_t launch_radix_sort(uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b, long long n, int nbits,
                             uint32_t* table, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int ntiles = (int)((n + RS_TILE - 1) / RS_TILE);
    // an even number of 8-bit passes (the result has to end in keys_a / vals_a; a pass over bits beyond nbits only
    // copies).  With 4-bit digits the same sort took 14 passes of 162 us at 6.4M keys; these take 80 us each: the
    // tile leaves LDS sorted, so the global writes are runs
    int passes = (nbits + 7) / 8;
    if (passes & 1) passes++;
    if (passes > 8) passes = 8;
    uint64_t *ki = keys_a, *ko = keys_b;
    uint32_t *vi = vals_a, *vo = vals_b;
    for (int p = 0; p < passes; p++) {
        const int shift = 8 * p;
        hipLaunchKernelGGL(radix_hist8_kernel, dim3(ntiles), dim3(256), 0, st, ki, n, shift, table, ntiles);
        hipLaunchKernelGGL(radix_rowscan8_kernel, dim3(256), dim3(1024), 0, st, table, ntiles);
        hipLaunchKernelGGL(radix_scatter8_kernel, dim3(ntiles), dim3(256), 0, st, ki, vi, ko, vo, n, shift, table, ntiles);
        uint64_t* tk = ki; ki = ko; ko = tk;
        uint32_t* tv = vi; vi = vo; vo = tv;
    }
    return hipGetLastError();
}

hipError_t launch_scan_u32(uint32_t* data, long long n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(radix_scan_kernel, dim3(1), dim3(1024), 0, st, data, n);
    return hipGetLastError();
}

hipError_t launch_argmin(const double* dist, long long n, uint32_t* out_id, hipStream_t st) {
    hipLaunchKernelGGL(argmin_kernel, dim3(1), dim3(1024), 0, st, dist, n, out_id);
    return hipGetLastError();
}

hipError_t launch_segment_heads(const uint64_t* keys, long long n, uint32_t* heads, uint32_t* nseg, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(segment_heads_kernel, dim3((unsigned)((n + 4095) / 4096)), dim3(1024), 0, st, keys, n, heads, nseg);
    return hipGetLastError();
}

}  // namespace jx
