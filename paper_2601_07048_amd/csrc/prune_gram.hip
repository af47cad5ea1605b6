// robustPrune (Alg. 3) for float32 / binary16 vectors as a dense contraction.
//
// Whether candidate i discards candidate j (alpha * d(i,j) <= d(p,j)) does not
// depend on the order in which Alg. 3 selects, so all pair distances of one
// prune are computed at once from the Gram matrix of its candidate vectors,
//     d(i,j) = G_ii + G_jj - 2 G_ij,   G = X X^T,
// on the matrix cores, and every candidate vector is read exactly once (the
// selection-centric form reads the surviving candidates again for every
// selected neighbour: 20-30 times the bytes for 2-6 KB vectors).
//
// One wavefront per prune, up to 128 candidates = 4 blocks of 32 rows.  Operand
// fragments go straight from global memory into the MFMA operand registers: a
// lane (row r = lane % 32, half h = lane / 32) loads the 64 contiguous bytes
// h*64 .. h*64+63 of each 128-byte piece of its row, and the k-th 16-byte
// load is the operand of the k-th MFMA step for the A side (row block bi) and
// the B side (row block bj) alike; since both sides use the same assignment of
// vector coordinates to MFMA k-slots, any such assignment sums every
// coordinate exactly once.
//   float32 : v_mfma_f32_32x32x2f32 on rows centred at the pruned vertex p
//             (x_j - x_p: distances are translation invariant and the
//             cancellation in G_ii + G_jj - 2 G_ij then involves local
//             magnitudes only); G_jj is d(p,j) itself.
//   binary16: v_mfma_f32_32x32x16_f16 on the stored values (products exact,
//             float32 accumulation, as in the binary16 distance provider);
//             where d(p,.) is not known beforehand p joins as one more row.
// The upper triangle of tiles is enough for candidates in any order: element
// (i,j), i in an earlier block than j, yields both "i discards j" and "j
// discards i" (two ballots per accumulator register = two 32-column stripes of
// bit masks).  Alg. 3 itself is then a walk over the candidates in (distance,
// id) order on 128-bit masks.
#include "jx_distance.h"

namespace jx {

typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
typedef int gi32x16_t __attribute__((ext_vector_type(16)));
typedef int gi32x4_t __attribute__((ext_vector_type(4)));

// accumulator of a tile: float32, or int32 for uint8 vectors (v_mfma_i32_32x32x32_i8 on the values shifted by -128:
// distances are translation invariant and everything stays an exact integer)
template <int DT> struct GAcc { typedef f32x16_t type; };
template <> struct GAcc<JX_U8> { typedef gi32x16_t type; };

__device__ __forceinline__ uint4 shift128(uint4 x) {
    x.x ^= 0x80808080u;
    x.y ^= 0x80808080u;
    x.z ^= 0x80808080u;
    x.w ^= 0x80808080u;
    return x;
}
// d(i,j) from G_ii, G_jj (held as raw bits in the float arrays) and G_ij, as the float the alpha test uses
template <int DT, typename A>
__device__ __forceinline__ float gram_dist(float ni, float nj, A gij) {
    if constexpr (DT == JX_U8)
        return (float)(uint32_t)(__float_as_int(ni) + __float_as_int(nj) - 2 * (int)gij);
    else
        return fmaxf((ni + nj) - 2.f * (float)gij, 0.f);
}
template <int DT, typename A>
__device__ __forceinline__ float gram_store(A g) {
    if constexpr (DT == JX_U8)
        return __int_as_float((int)g);
    else
        return (float)g;
}

#ifndef GP_WPB
#define GP_WPB 1  // wavefronts per workgroup (independent of each other)
#endif
#define GP_MAX 128

struct GramLds {
    uint64_t key[GP_MAX];
    uint32_t id[GP_MAX];
    float dp[GP_MAX];   // d(p, j)
    float nrm[GP_MAX];  // G_jj
    float gv[GP_MAX];   // G_jp (binary16, p as extra row)
    uint32_t kill[GP_MAX * 4];  // row i: mask over j of "i discards j", words of column blocks >= block(i)
    uint32_t kb[GP_MAX * 4];    // row i: mask over j of "j discards i", words of column blocks > block(i)
    uint32_t sel_id[GP_MAX];
    uint32_t sel_dist[GP_MAX];
    uint8_t order[GP_MAX];      // rank in (distance, id) order -> candidate slot
};

__host__ __device__ constexpr int gp_tile(int nt, int bi, int bj) { return bi * nt - bi * (bi - 1) / 2 + (bj - bi); }

// Preconditions: L->id[0..M) holds the candidates; with have_dp also L->dp[0..M), the candidates being in
// (distance, id) order.  M + (binary16 && !have_dp ? 1 : 0) <= 32 * NT.  Returns the number selected
// (L->sel_id / L->sel_dist, distance bits as float32).
template <int DT, int NT>
__device__ __forceinline__ int gram_prune_wave(const uint8_t* recs, size_t stride, int vec_bytes, GramLds* L, int M, uint32_t p,
                                               bool have_dp, int R, float alpha) {
    constexpr int NTILE = NT * (NT + 1) / 2;
    const int lane = lane_id(), col = lane & 31, half = lane >> 5;
    const bool extra = (DT != JX_F32) && !have_dp;
    const int Mx = M + (extra ? 1 : 0);
    const uint8_t* rp[NT];
    bool rv[NT];
    const uint8_t* pp = recs + (size_t)p * stride;
#pragma unroll
    for (int b = 0; b < NT; b++) {
        const int i = b * 32 + col;
        rv[b] = i < Mx;
        const uint32_t id = i < M ? L->id[i] : p;
        rp[b] = recs + (size_t)id * stride;
    }
    typename GAcc<DT>::type acc[NTILE];
#pragma unroll
    for (int t = 0; t < NTILE; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[t][e] = 0;

    for (int p0 = 0; p0 < vec_bytes; p0 += 128) {
        const int off = p0 + half * 64;
        if constexpr (DT == JX_U8) {
            uint4 f[NT][4];
#pragma unroll
            for (int b = 0; b < NT; b++)
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int o = off + s * 16;
                    f[b][s] = make_uint4(0, 0, 0, 0);  // rows and bytes beyond the data: zero after the shift
                    if (rv[b] && o < vec_bytes) f[b][s] = shift128(load16(rp[b] + o));
                }
#pragma unroll
            for (int s = 0; s < 4; s++)
#pragma unroll
                for (int bi = 0; bi < NT; bi++)
#pragma unroll
                    for (int bj = bi; bj < NT; bj++)
                        acc[gp_tile(NT, bi, bj)] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                            __builtin_bit_cast(gi32x4_t, f[bi][s]), __builtin_bit_cast(gi32x4_t, f[bj][s]),
                            acc[gp_tile(NT, bi, bj)], 0, 0, 0);
        } else if constexpr (DT == JX_F32) {
            float f[NT][16];
            float c[16];
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const int o = off + s * 16;
                uint4 x = make_uint4(0, 0, 0, 0);
                if (o < vec_bytes) x = load16(pp + o);
                c[4 * s + 0] = __uint_as_float(x.x);
                c[4 * s + 1] = __uint_as_float(x.y);
                c[4 * s + 2] = __uint_as_float(x.z);
                c[4 * s + 3] = __uint_as_float(x.w);
            }
#pragma unroll
            for (int b = 0; b < NT; b++)
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int o = off + s * 16;
                    uint4 x = make_uint4(0, 0, 0, 0);
                    if (o < vec_bytes) x = load16(rp[b] + o);  // rows beyond the last candidate point at p: they centre to zero
                    f[b][4 * s + 0] = __uint_as_float(x.x) - c[4 * s + 0];
                    f[b][4 * s + 1] = __uint_as_float(x.y) - c[4 * s + 1];
                    f[b][4 * s + 2] = __uint_as_float(x.z) - c[4 * s + 2];
                    f[b][4 * s + 3] = __uint_as_float(x.w) - c[4 * s + 3];
                }
#pragma unroll
            for (int e = 0; e < 16; e++)
#pragma unroll
                for (int bi = 0; bi < NT; bi++)
#pragma unroll
                    for (int bj = bi; bj < NT; bj++)
                        acc[gp_tile(NT, bi, bj)] =
                            __builtin_amdgcn_mfma_f32_32x32x2f32(f[bi][e], f[bj][e], acc[gp_tile(NT, bi, bj)], 0, 0, 0);
        } else {
            uint4 f[NT][4];
#pragma unroll
            for (int b = 0; b < NT; b++)
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int o = off + s * 16;
                    f[b][s] = make_uint4(0, 0, 0, 0);
                    if (rv[b] && o < vec_bytes) f[b][s] = load16(rp[b] + o);
                }
#pragma unroll
            for (int s = 0; s < 4; s++)
#pragma unroll
                for (int bi = 0; bi < NT; bi++)
#pragma unroll
                    for (int bj = bi; bj < NT; bj++)
                        acc[gp_tile(NT, bi, bj)] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                            __builtin_bit_cast(f16x8_t, f[bi][s]), __builtin_bit_cast(f16x8_t, f[bj][s]),
                            acc[gp_tile(NT, bi, bj)], 0, 0, 0);
        }
    }

    // Accumulator layout of the 32x32 tiles: register e of lane (col, half) holds row 8*(e/4) + 4*half + e%4, column col.
    // ---- G_jj from the diagonal tiles
    {
        const int hcol = (col >> 2) & 1, ecol = ((col >> 3) << 2) | (col & 3);
#pragma unroll
        for (int b = 0; b < NT; b++) {
            float dv = 0.f;
#pragma unroll
            for (int e = 0; e < 16; e++)
                if (e == ecol) dv = gram_store<DT>(acc[gp_tile(NT, b, b)][e]);
            if (half == hcol) L->nrm[b * 32 + col] = dv;
        }
    }
    // ---- binary16 without known distances: column of the extra row p (slot M)
    if (extra) {
        const int bv = M >> 5, cv = M & 31;
#pragma unroll
        for (int bi = 0; bi < NT; bi++)
#pragma unroll
            for (int bj = bi; bj < NT; bj++)
                if (bj == bv && col == cv) {
#pragma unroll
                    for (int e = 0; e < 16; e++)
                        L->gv[bi * 32 + 8 * (e >> 2) + 4 * half + (e & 3)] = gram_store<DT>(acc[gp_tile(NT, bi, bj)][e]);
                }
    }
    wave_sync();
    if (!have_dp) {
        for (int j = lane; j < M; j += 64) {
            float d;
            if constexpr (DT == JX_F32)
                d = L->nrm[j];
            else if constexpr (DT == JX_U8)
                d = gram_dist<DT>(L->nrm[M], L->nrm[j], __float_as_int(L->gv[j]));
            else
                d = gram_dist<DT>(L->nrm[M], L->nrm[j], L->gv[j]);
            L->dp[j] = d;
            L->key[j] = ((uint64_t)__float_as_uint(d) << 32) | L->id[j];
        }
        wave_sync();
        for (int j = lane; j < M; j += 64) {
            const uint64_t k = L->key[j];
            int rank = 0;
            for (int t = 0; t < M; t++) {
                const uint64_t o = L->key[t];
                rank += (o < k || (o == k && t < j)) ? 1 : 0;
            }
            L->order[rank] = (uint8_t)j;
        }
    } else {
        for (int j = lane; j < M; j += 64) L->order[j] = (uint8_t)j;
    }
    wave_sync();
    // ---- the discard relation, tile by tile
#pragma unroll
    for (int bi = 0; bi < NT; bi++)
#pragma unroll
        for (int bj = bi; bj < NT; bj++) {
            const int j = bj * 32 + col;
            const float nj = L->nrm[j];
            const float dpj = L->dp[j < M ? j : 0];
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int r0 = bi * 32 + 8 * (e >> 2) + (e & 3);
                const int i = r0 + 4 * half;
                const float ni = L->nrm[i];
                const float dpi = L->dp[i < M ? i : 0];
                const float dij = gram_dist<DT>(ni, nj, acc[gp_tile(NT, bi, bj)][e]);
                const float ad = __fmul_rn(alpha, dij);
                const bool ok = i < M && j < M && i != j;
                const uint64_t m1 = ballot(ok && ad <= dpj);
                if (lane == 0) {
                    L->kill[r0 * 4 + bj] = (uint32_t)m1;
                    L->kill[(r0 + 4) * 4 + bj] = (uint32_t)(m1 >> 32);
                }
                if (bi != bj) {
                    const uint64_t m2 = ballot(ok && ad <= dpi);
                    if (lane == 0) {
                        L->kb[r0 * 4 + bj] = (uint32_t)m2;
                        L->kb[(r0 + 4) * 4 + bj] = (uint32_t)(m2 >> 32);
                    }
                }
            }
        }
    wave_sync();
    // ---- Alg. 3: candidates in (distance, id) order; a candidate is gone if a selected one discards it
    uint32_t A[4], S[4];
#pragma unroll
    for (int t = 0; t < 4; t++) {
        const int rem = M - 32 * t;
        A[t] = rem >= 32 ? 0xFFFFFFFFu : (rem <= 0 ? 0u : ((1u << rem) - 1u));
        S[t] = 0u;
    }
    int nsel = 0;
    for (int r = 0; r < M && nsel < R; r++) {
        const int c = L->order[r];
        const int w = c >> 5;
        const uint32_t bit = 1u << (c & 31);
        uint32_t aw = 0u;
#pragma unroll
        for (int t = 0; t < 4; t++)
            if (t == w) aw = A[t];
        if (!(aw & bit)) continue;
        const uint32_t cid = L->id[c];
        if (cid == p) continue;
        bool gone = false;
#pragma unroll
        for (int t = 1; t < NT; t++)
            if (t > w) gone = gone || (L->kb[c * 4 + t] & S[t]) != 0u;
        if (gone) continue;
        if (lane == 0) {
            L->sel_id[nsel] = cid;
            L->sel_dist[nsel] = __float_as_uint(L->dp[c]);
        }
        nsel++;
#pragma unroll
        for (int t = 0; t < NT; t++) {
            if (t == w) S[t] |= bit;
            if (t >= w) A[t] &= ~L->kill[c * 4 + t];
        }
    }
    wave_sync();
    return nsel;
}

// ---- forward prune of the final frontier of each new point (Alg. 4 step 2)
template <int DT, int NT>
__global__ void __launch_bounds__(GP_WPB * 64) forward_prune_gram_kernel(InsertArgs a) {
    __shared__ GramLds lds[GP_WPB];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const long long i = (long long)blockIdx.x * GP_WPB + wave;
    if (i >= a.B) return;
    GramLds* L = &lds[wave];
    long long xid = a.id_base + i;
    if (xid >= a.id_skip) xid++;
    const uint32_t* ids = a.cand_ids + (size_t)i * a.L;
    const uint32_t* dbits = a.cand_dist + (size_t)i * a.L;
    int nB = 0;
    for (int c0 = 0; c0 < a.L; c0 += 64) {
        const int j = c0 + lane;
        const bool valid = j < a.L && ids[j] != JX_NONE_ID;  // the frontier is filled from the left
        nB += __builtin_popcountll(ballot(valid));
    }
    if (nB > GP_MAX) return;  // left to the list-based kernel
    const int nt = nB <= 64 ? 2 : (nB + 31) >> 5;
    if (nt != NT) return;  // another instantiation's share
    for (int j = lane; j < nB; j += 64) {
        L->id[j] = ids[j];
        L->dp[j] = __uint_as_float(dbits[j]);
    }
    wave_sync();
    const int nsel = gram_prune_wave<DT, NT>(a.ds.recs, (size_t)a.ds.rec_stride, a.ds.nch * 16, L, nB, (uint32_t)xid, true, a.R, a.alpha);
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

// ---- reverse-edge merge (Alg. 4 step 3): the targets whose row overflows and whose candidates fit 128 slots
template <int DT, int NT>
__global__ void __launch_bounds__(GP_WPB * 64) reverse_merge_gram_kernel(InsertArgs a) {
    __shared__ GramLds lds[GP_WPB];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    GramLds* L = &lds[wave];
    const long long nseg = *a.nseg;
    const long long total = a.E ? a.E : a.B * a.R;
    for (long long s = (long long)blockIdx.x * GP_WPB + wave; s < nseg; s += (long long)gridDim.x * GP_WPB) {
        const uint32_t head = a.heads[s];
        if (head & 0x80000000u) continue;  // already merged by another instantiation
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
        if (a.force_prune) deg = 0;
        if (!a.force_prune && deg + m <= a.R) continue;  // appended by the list-based kernel
        const int M = deg + m;
        const int Mx = M + (DT != JX_F32 ? 1 : 0);
        if (Mx > GP_MAX) continue;  // left to the list-based kernel
        const int nt = Mx <= 64 ? 2 : (Mx + 31) >> 5;
        if (nt != NT) continue;
        for (int j = lane; j < deg; j += 64) L->id[j] = row[j];
        for (int j = lane; j < m; j += 64) L->id[deg + j] = a.vals[lo + j];
        wave_sync();
        const int nsel = gram_prune_wave<DT, NT>(a.ds.recs, (size_t)a.ds.rec_stride, a.ds.nch * 16, L, M, v, false, a.R, a.alpha);
        for (int j = lane; j < a.R; j += 64) row[j] = j < nsel ? L->sel_id[j] : JX_NONE_ID;
        if (a.clean && lane == 0) a.clean[v] = (uint8_t)(nsel < 255 ? nsel : 255);
        // the row has changed, so degree and overflow can no longer be derived from it: mark the segment as done
        if (lane == 0) const_cast<uint32_t*>(a.heads)[s] = head | 0x80000000u;
        wave_sync();
    }
}


// ---- more than 128 candidates: the same contraction, one block row of tiles at a time --------------------------
// Eight 32-row blocks make 36 upper-triangle tiles, too many accumulators for one pass, and only the bit masks of
// the relation have to survive a tile.  So the wavefront walks the block rows: for block row bi it accumulates the
// tiles (bi, bi .. nb-1) over the whole vector length, turns them into mask words, and moves on; a block is read
// (nb - bi) + 1 times instead of once, still far less than the list-based form reads.  G_jj (and G_jp for
// binary16) are needed for columns of later blocks, so a first pass over the vectors computes them with plain
// fused multiply-adds.
// Beyond 256 candidates only a prefix is taken: Alg. 3 visits candidates in (distance, id) order and stops at R
// selections, and what happens to a candidate depends on earlier ones only.  The pool is the existing neighbours
// plus the closest new candidates (the new list arrives sorted) up to 256 rows; if the walk selects R neighbours
// before it meets a pool member beyond the last included new candidate, the excluded ones could not have mattered
// and the result is exact.  Otherwise the segment is left to the list-based kernel.
#define GB_MAX 256
#define GB_NB 8

struct GramBigLds {
    uint64_t key[GB_MAX];
    uint32_t id[GB_MAX];
    float dp[GB_MAX];
    float nrm[GB_MAX];
    uint32_t kill[GB_MAX * GB_NB];
    uint32_t kb[GB_MAX * GB_NB];
    uint32_t sel_id[GB_MAX];
    uint32_t sel_dist[GB_MAX];  // float bits of d(p, selected), selection order
    uint16_t order[GB_MAX];
};

// L->id[0..M): n_fixed existing neighbours, then new candidates, ascending, whose distances to p are the low words of
// new_keys[0..M-n_fixed) (edge keys) or, if new_keys is null, new_dbits[0..M-n_fixed) (float bits).  truncated: further
// new candidates exist beyond the pool.  Returns the number selected, or -1 if the pool did not suffice.
template <int DT>
__device__ __forceinline__ int gram_prune_big(const uint8_t* recs, size_t stride, int vec_bytes, GramBigLds* L, int M, uint32_t p,
                                              int R, float alpha, int n_fixed, const uint64_t* new_keys, bool truncated,
                                              const uint32_t* new_dbits = nullptr) {
    const int lane = lane_id(), col = lane & 31, half = lane >> 5;
    const int nb = (M + 31) >> 5;
    const uint8_t* pp = recs + (size_t)p * stride;
    // ---- pass 1: d(p, j) and G_jj.  float32: rows centred at p, so both are the same number
    float npp = 0.f;
    int ipp = 0;
    if constexpr (DT != JX_F32) {
        for (int p0 = half * 64; p0 < vec_bytes; p0 += 128)
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const int o = p0 + s * 16;
                if (o < vec_bytes) {
                    if constexpr (DT == JX_F16) {
                        const uint4 x = load16(pp + o);
                        npp = hdot2(x.x, x.x, npp);
                        npp = hdot2(x.y, x.y, npp);
                        npp = hdot2(x.z, x.z, npp);
                        npp = hdot2(x.w, x.w, npp);
                    } else {
                        const uint4 x = shift128(load16(pp + o));
                        ipp = __builtin_amdgcn_sdot4((int)x.x, (int)x.x, ipp, false);
                        ipp = __builtin_amdgcn_sdot4((int)x.y, (int)x.y, ipp, false);
                        ipp = __builtin_amdgcn_sdot4((int)x.z, (int)x.z, ipp, false);
                        ipp = __builtin_amdgcn_sdot4((int)x.w, (int)x.w, ipp, false);
                    }
                }
            }
        npp += shfl_xor(npp, 32);
        ipp += shfl_xor(ipp, 32);
    }
    for (int b = 0; b < nb; b++) {
        const int i = b * 32 + col;
        const uint8_t* rp = recs + (size_t)(i < M ? L->id[i] : p) * stride;
        float nn = 0.f, np = 0.f;
        int inn = 0, inp = 0;
        for (int p0 = half * 64; p0 < vec_bytes; p0 += 128)
#pragma unroll
            for (int s = 0; s < 4; s++) {
                const int o = p0 + s * 16;
                if (o < vec_bytes) {
                    uint4 x = load16(rp + o), c = load16(pp + o);
                    if constexpr (DT == JX_F32) {
                        const float d0 = __uint_as_float(x.x) - __uint_as_float(c.x), d1 = __uint_as_float(x.y) - __uint_as_float(c.y);
                        const float d2 = __uint_as_float(x.z) - __uint_as_float(c.z), d3 = __uint_as_float(x.w) - __uint_as_float(c.w);
                        nn = fmaf(d0, d0, nn);
                        nn = fmaf(d1, d1, nn);
                        nn = fmaf(d2, d2, nn);
                        nn = fmaf(d3, d3, nn);
                    } else if constexpr (DT == JX_F16) {
                        nn = hdot2(x.x, x.x, nn);
                        nn = hdot2(x.y, x.y, nn);
                        nn = hdot2(x.z, x.z, nn);
                        nn = hdot2(x.w, x.w, nn);
                        np = hdot2(x.x, c.x, np);
                        np = hdot2(x.y, c.y, np);
                        np = hdot2(x.z, c.z, np);
                        np = hdot2(x.w, c.w, np);
                    } else {
                        x = shift128(x);
                        c = shift128(c);
                        inn = __builtin_amdgcn_sdot4((int)x.x, (int)x.x, inn, false);
                        inn = __builtin_amdgcn_sdot4((int)x.y, (int)x.y, inn, false);
                        inn = __builtin_amdgcn_sdot4((int)x.z, (int)x.z, inn, false);
                        inn = __builtin_amdgcn_sdot4((int)x.w, (int)x.w, inn, false);
                        inp = __builtin_amdgcn_sdot4((int)x.x, (int)c.x, inp, false);
                        inp = __builtin_amdgcn_sdot4((int)x.y, (int)c.y, inp, false);
                        inp = __builtin_amdgcn_sdot4((int)x.z, (int)c.z, inp, false);
                        inp = __builtin_amdgcn_sdot4((int)x.w, (int)c.w, inp, false);
                    }
                }
            }
        nn += shfl_xor(nn, 32);
        np += shfl_xor(np, 32);
        inn += shfl_xor(inn, 32);
        inp += shfl_xor(inp, 32);
        if (half == 0) {
            float d = nn, nstore = nn;
            if constexpr (DT == JX_F16) d = fmaxf(npp + nn - 2.f * np, 0.f);
            if constexpr (DT == JX_U8) {
                d = (float)(uint32_t)(ipp + inn - 2 * inp);
                nstore = __int_as_float(inn);
            }
            L->nrm[i] = i < M ? nstore : 0.f;
            // a new candidate keeps the distance it was sorted by
            if (i >= n_fixed && i < M)
                d = __uint_as_float(new_keys ? (uint32_t)(new_keys[i - n_fixed] & 0xFFFFFFFFull) : new_dbits[i - n_fixed]);
            L->dp[i] = d;
            if (i < M) L->key[i] = ((uint64_t)__float_as_uint(d) << 32) | L->id[i];
        }
    }
    wave_sync();
    for (int j = lane; j < M; j += 64) {
        const uint64_t k = L->key[j];
        int rank = 0;
        for (int t = 0; t < M; t++) {
            const uint64_t o = L->key[t];
            rank += (o < k || (o == k && t < j)) ? 1 : 0;
        }
        L->order[rank] = (uint16_t)j;
    }
    // ---- pass 2: block rows of the Gram matrix -> mask words
    for (int bi = 0; bi < nb; bi++) {
        typename GAcc<DT>::type acc[GB_NB];
#pragma unroll
        for (int t = 0; t < GB_NB; t++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[t][e] = 0;
        const uint8_t* rp[GB_NB];
        bool rv[GB_NB];
#pragma unroll
        for (int t = 0; t < GB_NB; t++) {
            const int i = (bi + t) * 32 + col;
            rv[t] = i < M;
            rp[t] = recs + (size_t)(i < M ? L->id[i] : p) * stride;
        }
        for (int p0 = 0; p0 < vec_bytes; p0 += 128) {
            const int off = p0 + half * 64;
            if constexpr (DT == JX_F32) {
                float c[16], fa[16];
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int o = off + s * 16;
                    uint4 x = make_uint4(0, 0, 0, 0), y = x;
                    if (o < vec_bytes) {
                        x = load16(pp + o);
                        y = load16(rp[0] + o);
                    }
                    c[4 * s + 0] = __uint_as_float(x.x);
                    c[4 * s + 1] = __uint_as_float(x.y);
                    c[4 * s + 2] = __uint_as_float(x.z);
                    c[4 * s + 3] = __uint_as_float(x.w);
                    fa[4 * s + 0] = __uint_as_float(y.x) - c[4 * s + 0];
                    fa[4 * s + 1] = __uint_as_float(y.y) - c[4 * s + 1];
                    fa[4 * s + 2] = __uint_as_float(y.z) - c[4 * s + 2];
                    fa[4 * s + 3] = __uint_as_float(y.w) - c[4 * s + 3];
                }
#pragma unroll
                for (int t = 0; t < GB_NB; t++) {
                    if (bi + t >= nb) break;  // uniform
                    float fb[16];
                    if (t == 0) {
#pragma unroll
                        for (int e = 0; e < 16; e++) fb[e] = fa[e];
                    } else {
#pragma unroll
                        for (int s = 0; s < 4; s++) {
                            const int o = off + s * 16;
                            uint4 y = make_uint4(0, 0, 0, 0);
                            if (o < vec_bytes) y = load16(rp[t] + o);  // rows beyond M point at p and centre to zero
                            fb[4 * s + 0] = __uint_as_float(y.x) - c[4 * s + 0];
                            fb[4 * s + 1] = __uint_as_float(y.y) - c[4 * s + 1];
                            fb[4 * s + 2] = __uint_as_float(y.z) - c[4 * s + 2];
                            fb[4 * s + 3] = __uint_as_float(y.w) - c[4 * s + 3];
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 16; e++) acc[t] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[e], fb[e], acc[t], 0, 0, 0);
                }
            } else {
                uint4 fa[4];
#pragma unroll
                for (int s = 0; s < 4; s++) {
                    const int o = off + s * 16;
                    fa[s] = make_uint4(0, 0, 0, 0);
                    if (rv[0] && o < vec_bytes) fa[s] = DT == JX_U8 ? shift128(load16(rp[0] + o)) : load16(rp[0] + o);
                }
#pragma unroll
                for (int t = 0; t < GB_NB; t++) {
                    if (bi + t >= nb) break;  // uniform
                    uint4 fb[4];
#pragma unroll
                    for (int s = 0; s < 4; s++) {
                        const int o = off + s * 16;
                        fb[s] = fa[s];
                        if (t > 0) {
                            fb[s] = make_uint4(0, 0, 0, 0);
                            if (rv[t] && o < vec_bytes) fb[s] = DT == JX_U8 ? shift128(load16(rp[t] + o)) : load16(rp[t] + o);
                        }
                    }
#pragma unroll
                    for (int s = 0; s < 4; s++) {
                        if constexpr (DT == JX_U8)
                            acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(gi32x4_t, fa[s]),
                                                                           __builtin_bit_cast(gi32x4_t, fb[s]), acc[t], 0, 0, 0);
                        else
                            acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, fa[s]),
                                                                            __builtin_bit_cast(f16x8_t, fb[s]), acc[t], 0, 0, 0);
                    }
                }
            }
        }
        // masks of this block row
#pragma unroll
        for (int t = 0; t < GB_NB; t++) {
            if (bi + t >= nb) break;
            const int bj = bi + t;
            const int j = bj * 32 + col;
            const float nj = L->nrm[j], dpj = L->dp[j];
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int r0 = bi * 32 + 8 * (e >> 2) + (e & 3);
                const int i = r0 + 4 * half;
                const float ni = L->nrm[i], dpi = L->dp[i];
                const float dij = gram_dist<DT>(ni, nj, acc[t][e]);
                const float ad = __fmul_rn(alpha, dij);
                const bool ok = i < M && j < M && i != j;
                const uint64_t m1 = ballot(ok && ad <= dpj);
                if (lane == 0) {
                    L->kill[r0 * GB_NB + bj] = (uint32_t)m1;
                    L->kill[(r0 + 4) * GB_NB + bj] = (uint32_t)(m1 >> 32);
                }
                if (t > 0) {
                    const uint64_t m2 = ballot(ok && ad <= dpi);
                    if (lane == 0) {
                        L->kb[r0 * GB_NB + bj] = (uint32_t)m2;
                        L->kb[(r0 + 4) * GB_NB + bj] = (uint32_t)(m2 >> 32);
                    }
                }
            }
        }
    }
    wave_sync();
    // ---- Alg. 3 on 256-bit masks
    const uint64_t tau = truncated ? L->key[M - 1] : JX_EMPTY_KEY;  // the last new candidate of the pool
    uint32_t A[GB_NB], S[GB_NB];
#pragma unroll
    for (int t = 0; t < GB_NB; t++) {
        const int rem = M - 32 * t;
        A[t] = rem >= 32 ? 0xFFFFFFFFu : (rem <= 0 ? 0u : ((1u << rem) - 1u));
        S[t] = 0u;
    }
    int nsel = 0;
    bool short_pool = truncated;  // cleared when R neighbours are found inside the prefix
    for (int r = 0; r < M; r++) {
        if (nsel >= R) {
            short_pool = false;
            break;
        }
        const int c = L->order[r];
        if (truncated && L->key[c] > tau) break;  // beyond the prefix with room left: excluded candidates would matter
        const int w = c >> 5;
        const uint32_t bit = 1u << (c & 31);
        uint32_t aw = 0u;
#pragma unroll
        for (int t = 0; t < GB_NB; t++)
            if (t == w) aw = A[t];
        if (!(aw & bit)) continue;
        const uint32_t cid = L->id[c];
        if (cid == p) continue;
        bool gone = false;
#pragma unroll
        for (int t = 1; t < GB_NB; t++)
            if (t > w && t < nb) gone = gone || (L->kb[c * GB_NB + t] & S[t]) != 0u;
        if (gone) continue;
        if (lane == 0) {
            L->sel_id[nsel] = cid;
            L->sel_dist[nsel] = __float_as_uint(L->dp[c]);
        }
        nsel++;
#pragma unroll
        for (int t = 0; t < GB_NB; t++) {
            if (t == w) S[t] |= bit;
            if (t >= w && t < nb) A[t] &= ~L->kill[c * GB_NB + t];
        }
    }
    wave_sync();
    if (nsel >= R) short_pool = false;
    return short_pool ? -1 : nsel;
}

// ---- forward prune of candidate lists of 129 .. 256 entries, or of the closest 256 of a longer list (expansion
// lists as candidate sets hold 150 - 200 vertices).  Every point of the batch gets a mark in a.dead[i * a.L]: 0xFF =
// row and reverse edges written here, 0 = left to the list-based kernel (which also owns lists of at most 128, the
// one-pass kernels' share).
template <int DT>
__global__ void __launch_bounds__(GP_WPB * 64) forward_prune_gram_big_kernel(InsertArgs a) {
    extern __shared__ __align__(16) unsigned char gb_dyn[];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    GramBigLds* L = reinterpret_cast<GramBigLds*>(gb_dyn) + wave;
    const long long i = (long long)blockIdx.x * GP_WPB + wave;
    if (i >= a.B) return;
    long long xid = a.id_base + i;
    if (xid >= a.id_skip) xid++;
    const uint32_t* ids = a.cand_ids + (size_t)i * a.L;
    const uint32_t* dbits = a.cand_dist + (size_t)i * a.L;
    int nB = 0;
    for (int c0 = 0; c0 < a.L; c0 += 64) {
        const int j = c0 + lane;
        const bool valid = j < a.L && ids[j] != JX_NONE_ID;  // the list is filled from the left
        nB += __builtin_popcountll(ballot(valid));
    }
    if (lane == 0) a.dead[(size_t)i * a.L] = 0;
    if (nB <= GP_MAX) return;
    const int M = nB < GB_MAX ? nB : GB_MAX;
    for (int j = lane; j < M; j += 64) L->id[j] = ids[j];
    wave_sync();
    const int nsel = gram_prune_big<DT>(a.ds.recs, (size_t)a.ds.rec_stride, a.ds.nch * 16, L, M, (uint32_t)xid, a.R, a.alpha, 0, nullptr,
                                        M < nB, dbits);
    if (nsel < 0) return;  // the closest 256 did not yield R neighbours
    uint32_t* row = a.adj + (size_t)xid * a.R;
    for (int j = lane; j < a.R; j += 64) {
        const bool on = j < nsel;
        const uint32_t v = on ? L->sel_id[j] : JX_NONE_ID;
        row[j] = v;
        a.keys[(size_t)i * a.R + j] = on ? (((uint64_t)v << 32) | L->sel_dist[j]) : JX_EMPTY_KEY;
        a.vals[(size_t)i * a.R + j] = on ? (uint32_t)xid : JX_NONE_ID;
    }
    if (a.clean && lane == 0) a.clean[xid] = (uint8_t)(nsel < 255 ? nsel : 255);
    if (lane == 0) a.dead[(size_t)i * a.L] = 0xFF;
}

template <int DT>
__global__ void __launch_bounds__(GP_WPB * 64) reverse_merge_gram_big_kernel(InsertArgs a) {
    extern __shared__ __align__(16) unsigned char gb_dyn[];
    const int wave = threadIdx.x >> 6, lane = lane_id();
    GramBigLds* L = reinterpret_cast<GramBigLds*>(gb_dyn) + wave;
    const long long nseg = *a.nseg;
    const long long total = a.E ? a.E : a.B * a.R;
    for (long long s = (long long)blockIdx.x * GP_WPB + wave; s < nseg; s += (long long)gridDim.x * GP_WPB) {
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
        if (a.force_prune) deg = 0;
        if (!a.force_prune && deg + m <= a.R) continue;
        if (deg + m + (DT != JX_F32 ? 1 : 0) <= GP_MAX) continue;  // the one-pass kernels' share
        if (deg > GB_MAX - 64) continue;                             // too little room for new candidates: list-based kernel
        const int mp = m < GB_MAX - deg ? m : GB_MAX - deg;          // new candidates in the pool (the closest ones)
        const int M = deg + mp;
        for (int j = lane; j < deg; j += 64) L->id[j] = row[j];
        for (int j = lane; j < mp; j += 64) L->id[deg + j] = a.vals[lo + j];
        wave_sync();
        const int nsel = gram_prune_big<DT>(a.ds.recs, (size_t)a.ds.rec_stride, a.ds.nch * 16, L, M, v, a.R, a.alpha, deg, a.keys + lo,
                                            mp < m);
        if (nsel < 0) continue;  // the prefix did not yield R neighbours: left to the list-based kernel
        for (int j = lane; j < a.R; j += 64) row[j] = j < nsel ? L->sel_id[j] : JX_NONE_ID;
        if (a.clean && lane == 0) a.clean[v] = (uint8_t)(nsel < 255 ? nsel : 255);
        if (lane == 0) const_cast<uint32_t*>(a.heads)[s] = head | 0x80000000u;
        wave_sync();
    }
}

template <int DT>
static hipError_t launch_forward_gram_dt(const InsertArgs& a, hipStream_t st) {
    dim3 grid((unsigned)((a.B + GP_WPB - 1) / GP_WPB)), block(GP_WPB * 64);
    hipLaunchKernelGGL((forward_prune_gram_kernel<DT, 2>), grid, block, 0, st, a);
    if (a.L > 64) hipLaunchKernelGGL((forward_prune_gram_kernel<DT, 3>), grid, block, 0, st, a);
    if (a.L > 96) hipLaunchKernelGGL((forward_prune_gram_kernel<DT, 4>), grid, block, 0, st, a);
    if (a.L > GP_MAX) {  // longer lists (expansion lists): block-row form on the closest 256
        const size_t sh = sizeof(GramBigLds) * GP_WPB;
        hipError_t e = hipFuncSetAttribute((const void*)forward_prune_gram_big_kernel<DT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((forward_prune_gram_big_kernel<DT>), grid, block, sh, st, a);
    }
    return hipGetLastError();
}

template <int DT>
static hipError_t launch_reverse_gram_dt(const InsertArgs& a, hipStream_t st) {
    long long want = ((a.E ? a.E : a.B * a.R) + GP_WPB - 1) / GP_WPB;
    const long long cap = 8192 / GP_WPB;  // persistent wavefronts, segments dealt round-robin
    dim3 grid((unsigned)(want < cap ? (want < 1 ? 1 : want) : cap)), block(GP_WPB * 64);
    hipLaunchKernelGGL((reverse_merge_gram_kernel<DT, 2>), grid, block, 0, st, a);
    hipLaunchKernelGGL((reverse_merge_gram_kernel<DT, 3>), grid, block, 0, st, a);
    hipLaunchKernelGGL((reverse_merge_gram_kernel<DT, 4>), grid, block, 0, st, a);
    {   // 129 .. 256 candidates: few and long, 27 KB of LDS per wavefront
        const size_t sh = sizeof(GramBigLds) * GP_WPB;
        hipError_t e = hipFuncSetAttribute((const void*)reverse_merge_gram_big_kernel<DT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((reverse_merge_gram_big_kernel<DT>), dim3(grid.x < 4096 / GP_WPB ? grid.x : 4096 / GP_WPB), block, sh, st, a);
    }
    return hipGetLastError();
}

hipError_t launch_forward_prune_gram(int dtype, const InsertArgs& a, hipStream_t st) {
    if (a.B <= 0) return hipSuccess;
    if (dtype == JX_U8) return launch_forward_gram_dt<JX_U8>(a, st);
    return dtype == JX_F16 ? launch_forward_gram_dt<JX_F16>(a, st) : launch_forward_gram_dt<JX_F32>(a, st);
}

hipError_t launch_reverse_merge_gram(int dtype, const InsertArgs& a, hipStream_t st) {
    if (dtype == JX_U8) return launch_reverse_gram_dt<JX_U8>(a, st);
    return dtype == JX_F16 ? launch_reverse_gram_dt<JX_F16>(a, st) : launch_reverse_gram_dt<JX_F32>(a, st);
}

}  // namespace jx
