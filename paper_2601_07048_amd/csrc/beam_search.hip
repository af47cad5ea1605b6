// beamSearch kernel (Alg. 1 / Alg. 2 of the paper, fused as in Sec. 4.1 and
// App. B): one wavefront serves one query for its whole life.
//
// Per expansion ("hop") the wavefront
//   1. picks the closest unexpanded frontier entry u (ballot over registers),
//   2. reads adjacency row adj[u] with one coalesced 4R-byte load,
//   3. drops ids it has seen before with a small table in LDS: sets of two
//      16-bit tags of a permuted id (set and tag together name the id exactly),
//      or full ids when the index is too large for that.  A table that only
//      ever forgets has no false positives, so the frontier sequence equals
//      that of an exact visited set -- the filter changes the number of distance
//      evaluations, never the result,
//   4. gathers the surviving neighbours' records (vector or RaBitQ code) with
//      16-byte loads, T lanes per record, several records in flight per lane,
//   5. reduces the partial distances inside each T-lane group,
//   6. merges the new (distance,id) keys into the sorted frontier, which lives
//      in registers (one key per lane per 64 entries): every candidate that
//      beats the current worst entry is broadcast once, every lane counts how
//      many candidates precede its entries, and one LDS scatter/gather applies
//      the permutation.  Keys are 64-bit (ordered distance, id, expanded flag),
//      so the order is the strict total order (distance, id).
#include <stdio.h>
#include "jx_distance.h"

namespace jx {

// Tuning constants (compile-time; the values are the optima measured on gfx950 at N = 1M, 10,000 queries):
// 16-byte loads in flight per lane for the exact uint8, 1-bit and 4-bit kernels, and the
// waves per SIMD the small exact kernels are held to.
#ifndef JX_UMAX_EXACT
#define JX_UMAX_EXACT 8
#endif
#ifndef JX_UMAX_RQ1
#define JX_UMAX_RQ1 8
#endif
#ifndef JX_UMAX_RQ4
#define JX_UMAX_RQ4 8
#endif
#ifndef JX_WPE_EXACT
#define JX_WPE_EXACT 6
#endif

template <int KIND, int T, int CPL, int NREG, int QB>
__global__ void __launch_bounds__(JX_BEAM_WPB * 64) __attribute__((amdgpu_waves_per_eu(((KIND <= K_F32 || KIND == K_F16) && NREG <= 2 && CPL <= 2) ? JX_WPE_EXACT : 1, 8)))
beam_search_kernel(BeamArgs a) {
    constexpr int G = 64 / T;
    constexpr int UMAX = (KIND == K_RQ1) ? JX_UMAX_RQ1 : ((KIND == K_U8) ? JX_UMAX_EXACT : ((KIND == K_RQ4) ? JX_UMAX_RQ4 : 8));  // 16-byte loads in flight per lane (the 1-bit path keeps its bit planes in registers)
    constexpr int U0 = (UMAX / CPL) > 0 ? (UMAX / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);  // records in flight per lane group
    constexpr int FCAP = NREG * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = threadIdx.x >> 6;
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const int64_t qi = (int64_t)blockIdx.x * JX_BEAM_WPB + wave;
    if (qi >= a.nq) return;  // whole wavefront leaves; there is no block-level barrier below

    const int H = a.hash_slots;
    const int tag_bits = a.tag_bits;  // > 0: 16-bit entries (slot and tag together name the id exactly)
    const uint32_t id_mask = tag_bits ? ((1u << (tag_bits + 30 - __builtin_clz((uint32_t)H))) - 1u) : 0u;  // H / 2 sets
    const size_t per_wave = (size_t)FCAP * 8 + 64 * 8 + 64 * 4 + (size_t)H * (tag_bits ? 2 : 4);
    unsigned char* my = smem + per_wave * wave;
    uint64_t* fr = reinterpret_cast<uint64_t*>(my);
    uint64_t* cand_key = fr + FCAP;
    uint32_t* cand_id = reinterpret_cast<uint32_t*>(cand_key + 64);
    uint32_t* tab = cand_id + 64;

    for (int i = lane; i < (tag_bits ? H / 2 : H); i += 64) tab[i] = JX_NONE_ID;
    for (int i = lane; i < FCAP; i += 64) fr[i] = JX_EMPTY_KEY;

    QueryRegs<KIND, CPL, QB> q;
    load_query<KIND, T, CPL, QB>(q, a.ds, qi + (qi >= a.q_skip ? 1 : 0), lig);

    uint64_t fk[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) fk[r] = JX_EMPTY_KEY;
    int count = 0;
    const int L = a.L;
    const bool full = a.ds.nch == T * CPL;  // wave-uniform: no chunk slot is idle
    uint32_t hops = 0, evals = 0;

    // seed: the entry vertex
    if (lane == 0) {
        cand_id[0] = a.entry;
        if (tag_bits) {
            const uint32_t h = (a.entry * 0x9E3779B1u) & id_mask;
            tab[h >> tag_bits] = 0xFFFF0000u | (h & ((1u << tag_bits) - 1u));
        } else if (H) {
            tab[__umulhi(a.entry * 0x9E3779B1u, (uint32_t)H)] = a.entry;
        }
    }
    wave_sync();
    eval_batch<KIND, T, CPL, QB, 1>(q, a.ds, 0, 1, cand_id, cand_key, g, lig);
    wave_sync();
    if (lane == 0) {
        fk[0] = cand_key[0];
        fr[0] = cand_key[0];
    }
    wave_sync();
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
                if (tag_bits) {
                    // ids below 2^b, b = log2(sets) + tag_bits: multiplying by an odd constant permutes them, so the
                    // set (high bits) and the tag (low bits) of the product identify the id.  Two tags per set in one
                    // 32-bit word, most recent first: one LDS read finds both, one write installs the new one
                    const uint32_t h = (v * 0x9E3779B1u) & id_mask;
                    const uint32_t tag = h & ((1u << tag_bits) - 1u);
                    const uint32_t w = tab[h >> tag_bits];
                    is_new = (w & 0xFFFFu) != tag && (w >> 16) != tag;
                    if (is_new) tab[h >> tag_bits] = (w << 16) | tag;
                } else if (H) {
                    uint32_t h = __umulhi(v * 0x9E3779B1u, (uint32_t)H);
                    is_new = tab[h] != v;
                    if (is_new) tab[h] = v;
                } else {
                    // no filter (Alg. 2 as printed): every neighbour is evaluated; one that is still in the frontier
                    // is recognised by the merge, one that has left it cannot come back (its key is above the worst)
                    is_new = true;
                }
            }
            uint64_t nm = ballot(is_new);
            if (ballot(v != JX_NONE_ID) == 0ull) break;  // rows are filled from the left
            const int n_new = __builtin_popcountll(nm);
            if (n_new == 0) continue;
            if (is_new) cand_id[prefix_count(nm)] = v;
            wave_sync();
            // ---- 4./5. gather + distances
            if (full) {
                for (int s0 = 0; s0 < n_new; s0 += G * U)
                    eval_batch<KIND, T, CPL, QB, U, true>(q, a.ds, s0, n_new, cand_id, cand_key, g, lig);
            } else {
                for (int s0 = 0; s0 < n_new; s0 += G * U)
                    eval_batch<KIND, T, CPL, QB, U, false>(q, a.ds, s0, n_new, cand_id, cand_key, g, lig);
            }
            evals += n_new;
            wave_sync();
            uint64_t ck = lane < n_new ? cand_key[lane] : JX_EMPTY_KEY;
            wave_sync();
            // ---- 6. merge into the sorted frontier
            // fr[] mirrors the frontier (flags aside) and is sorted, unused slots
            // hold the largest key: every candidate finds its rank among the
            // frontier entries by binary search, all candidates at once.
            const uint64_t ckm = ck | 1ull;
            bool beats = lane < n_new;
            if (count >= L) beats = beats && (ckm < (fr[L - 1] | 1ull));
            if (ballot(beats) == 0ull) continue;  // nothing enters the frontier (the common case late in a search)
            uint32_t pos = 0;
#pragma unroll
            for (int step = FCAP / 2; step >= 1; step >>= 1)
                if ((fr[pos + step - 1] | 1ull) < ckm) pos += step;
            // an id that is already in the frontier (the table forgot it) is dropped
            beats = beats && ((fr[pos] | 1ull) != ckm);
            uint64_t sm = ballot(beats);
            if (sm == 0ull) continue;
            const int n_ins = __builtin_popcountll(sm);
            uint32_t shift[NREG];
#pragma unroll
            for (int r = 0; r < NREG; r++) shift[r] = 0;
            uint32_t crank = 0;
            while (sm) {
                const int j = __builtin_ctzll(sm);
                sm &= sm - 1;
                const uint64_t s = readlane64(ckm, j);
#pragma unroll
                for (int r = 0; r < NREG; r++) shift[r] += (s < (fk[r] | 1ull)) ? 1u : 0u;
                crank += (s < ckm) ? 1u : 0u;
            }
            wave_sync();  // all binary-search reads of fr[] are done
#pragma unroll
            for (int r = 0; r < NREG; r++) {
                uint32_t np = (uint32_t)(r * 64 + lane) + shift[r];
                if (np < (uint32_t)FCAP) fr[np] = fk[r];
            }
            if (beats) {
                uint32_t np = pos + crank;
                if (np < (uint32_t)FCAP) fr[np] = ck;
            }
            wave_sync();
#pragma unroll
            for (int r = 0; r < NREG; r++) {
                fk[r] = fr[r * 64 + lane];
                if (r * 64 + lane >= L) {  // truncate to the beam width
                    fk[r] = JX_EMPTY_KEY;
                    fr[r * 64 + lane] = JX_EMPTY_KEY;
                }
            }
            wave_sync();
            count = count + n_ins < L ? count + n_ins : L;
        }
    }

    // ---- results: the first out_k frontier entries that are not logically
    // deleted (Sec. 4.6: deleted vertices are traversed but never returned)
    int base_pos = 0;
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        const int p = r * 64 + lane;
        const uint64_t k = fk[r];
        const uint32_t id = key_id(k);
        bool keep = p < count;
        if (keep && a.deleted) keep = a.deleted[id] == 0;
        const uint64_t km = ballot(keep);
        const int pos = base_pos + prefix_count(km);
        if (keep && pos < a.out_k) {
            const uint32_t dc = key_dist(k);
            float d;
            if constexpr (KIND == K_U8)
                d = (float)dc;
            else
                d = ordered_to_f32(dc);
            a.out_ids[qi * a.out_k + pos] = id;
            a.out_dist[qi * a.out_k + pos] = d;
        }
        base_pos += __builtin_popcountll(km);
    }
    for (int p = base_pos + lane; p < a.out_k; p += 64) {
        a.out_ids[qi * a.out_k + p] = JX_NONE_ID;
        a.out_dist[qi * a.out_k + p] = __builtin_inff();
    }
    if (a.stats && lane == 0) {
        atomicAdd(&a.stats[0], (unsigned long long)hops);
        atomicAdd(&a.stats[1], (unsigned long long)evals);
    }
}

// ------------------------------------------------------------------ two expansions per round
//
// A search over a 10,000-query batch lasts about two query lifetimes, and a lifetime is a chain of dependent
// expansions: select, row, filter, gather, merge.  This variant overlaps two links of the chain without changing
// the sequence Alg. 1 prescribes.  Besides the closest unexpanded entry u1 it takes the second closest, u2, reads
// both rows, filters row(u1) and then row(u2) through the visited table (in that order: what the sequential search
// would do if u2 came next), and gathers both candidate lists in one batch.  The candidates of u1 are merged; if u2
// is still the closest unexpanded entry -- no candidate of u1 overtook or evicted it, the usual case -- its
// expansion has happened exactly as it would have, and its candidates are merged too.  Otherwise the table words
// that row(u2) changed are restored, its candidates are dropped, and the search goes on from the merged frontier.
// Frontier sequence, results and the expansion / evaluation counts are those of the one-at-a-time search; a
// dropped list costs its gather.

// candidates ck (lane < n) into the sorted frontier (registers fk, mirror fr): the merge step of the kernel above
template <int NREG>
__device__ __forceinline__ void frontier_merge(uint64_t (&fk)[NREG], uint64_t* fr, int& count, const int L, const uint64_t ck,
                                               const int n, const int lane) {
    constexpr int FCAP = NREG * 64;
    const uint64_t ckm = ck | 1ull;
    bool beats = lane < n;
    if (count >= L) beats = beats && (ckm < (fr[L - 1] | 1ull));
    if (ballot(beats) == 0ull) return;
    uint32_t pos = 0;
#pragma unroll
    for (int step = FCAP / 2; step >= 1; step >>= 1)
        if ((fr[pos + step - 1] | 1ull) < ckm) pos += step;
    beats = beats && ((fr[pos] | 1ull) != ckm);
    uint64_t sm = ballot(beats);
    if (sm == 0ull) return;
    const int n_ins = __builtin_popcountll(sm);
    uint32_t shift[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) shift[r] = 0;
    uint32_t crank = 0;
    while (sm) {
        const int j = __builtin_ctzll(sm);
        sm &= sm - 1;
        const uint64_t s = readlane64(ckm, j);
#pragma unroll
        for (int r = 0; r < NREG; r++) shift[r] += (s < (fk[r] | 1ull)) ? 1u : 0u;
        crank += (s < ckm) ? 1u : 0u;
    }
    wave_sync();
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        uint32_t np = (uint32_t)(r * 64 + lane) + shift[r];
        if (np < (uint32_t)FCAP) fr[np] = fk[r];
    }
    if (beats) {
        uint32_t np = pos + crank;
        if (np < (uint32_t)FCAP) fr[np] = ck;
    }
    wave_sync();
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        fk[r] = fr[r * 64 + lane];
        if (r * 64 + lane >= L) {
            fk[r] = JX_EMPTY_KEY;
            fr[r * 64 + lane] = JX_EMPTY_KEY;
        }
    }
    wave_sync();
    count = count + n_ins < L ? count + n_ins : L;
}

// rows of at most 64 entries only (the launcher checks)
template <int KIND, int T, int CPL, int NREG, int QB>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(((KIND <= K_F32 || KIND == K_F16) && NREG <= 2 && CPL <= 2) ? JX_WPE_EXACT : 1, 8)))
beam_search_pair_kernel(BeamArgs a) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    constexpr int FCAP = NREG * 64;
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const int64_t qi = blockIdx.x;
    if (qi >= a.nq) return;

    const int H = a.hash_slots;
    const int tag_bits = a.tag_bits;
    const uint32_t id_mask = tag_bits ? ((1u << (tag_bits + 30 - __builtin_clz((uint32_t)H))) - 1u) : 0u;
    uint64_t* fr = reinterpret_cast<uint64_t*>(smem);
    uint64_t* cand_key = fr + FCAP;                                     // [128]
    uint32_t* cand_id = reinterpret_cast<uint32_t*>(cand_key + 128);    // [128]
    uint32_t* tab = cand_id + 128;

    for (int i = lane; i < (tag_bits ? H / 2 : H); i += 64) tab[i] = JX_NONE_ID;
    for (int i = lane; i < FCAP; i += 64) fr[i] = JX_EMPTY_KEY;

    QueryRegs<KIND, CPL, QB> q;
    load_query<KIND, T, CPL, QB>(q, a.ds, qi + (qi >= a.q_skip ? 1 : 0), lig);

    uint64_t fk[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) fk[r] = JX_EMPTY_KEY;
    int count = 0;
    const int L = a.L;
    const bool full = a.ds.nch == T * CPL;
    uint32_t hops = 0, evals = 0;

    if (lane == 0) {
        cand_id[0] = a.entry;
        if (tag_bits) {
            const uint32_t h = (a.entry * 0x9E3779B1u) & id_mask;
            tab[h >> tag_bits] = 0xFFFF0000u | (h & ((1u << tag_bits) - 1u));
        } else {
            tab[__umulhi(a.entry * 0x9E3779B1u, (uint32_t)H)] = a.entry;
        }
    }
    wave_sync();
    eval_batch<KIND, T, CPL, QB, 1>(q, a.ds, 0, 1, cand_id, cand_key, g, lig);
    wave_sync();
    if (lane == 0) {
        fk[0] = cand_key[0];
        fr[0] = cand_key[0];
    }
    wave_sync();
    count = 1;
    evals = 1;

    // visited filter: true if v has not been seen; installs it; slot / old word returned for a possible restore
    auto filter = [&](const uint32_t v, uint32_t& slot, uint32_t& old) -> bool {
        bool is_new = false;
        slot = 0;
        old = 0;
        if (v != JX_NONE_ID) {
            if (tag_bits) {
                const uint32_t h = (v * 0x9E3779B1u) & id_mask;
                const uint32_t tag = h & ((1u << tag_bits) - 1u);
                slot = h >> tag_bits;
                old = tab[slot];
                is_new = (old & 0xFFFFu) != tag && (old >> 16) != tag;
                if (is_new) tab[slot] = (old << 16) | tag;
            } else {
                slot = __umulhi(v * 0x9E3779B1u, (uint32_t)H);
                old = tab[slot];
                is_new = old != v;
                if (is_new) tab[slot] = v;
            }
        }
        return is_new;
    };

    for (;;) {
        // ---- the two closest unexpanded entries
        uint64_t um[NREG];
#pragma unroll
        for (int r = 0; r < NREG; r++) um[r] = ballot((fk[r] & 1ull) == 0ull);
        int r1 = -1, l1 = 0;
#pragma unroll
        for (int r = 0; r < NREG; r++)
            if (r1 < 0 && um[r] != 0ull) {
                r1 = r;
                l1 = __builtin_ctzll(um[r]);
                um[r] &= um[r] - 1ull;
            }
        if (r1 < 0) break;
        int r2 = -1, l2 = 0;
#pragma unroll
        for (int r = 0; r < NREG; r++)
            if (r2 < 0 && um[r] != 0ull) {
                r2 = r;
                l2 = __builtin_ctzll(um[r]);
            }
        uint32_t u1 = 0;
        uint64_t key2 = JX_EMPTY_KEY;
#pragma unroll
        for (int r = 0; r < NREG; r++) {
            if (r == r1) {
                u1 = readlane32((uint32_t)fk[r], l1) >> 1;
                if (lane == l1) fk[r] |= 1ull;
            }
            if (r == r2) key2 = readlane64(fk[r], l2);
        }
        const bool have2 = r2 >= 0;
        // ---- both rows, both filters (row 1 first), one gather
        uint32_t v1 = JX_NONE_ID, v2 = JX_NONE_ID;
        if (lane < a.R) v1 = a.adj[(size_t)u1 * (size_t)a.R + lane];
        if (have2 && lane < a.R) v2 = a.adj[(size_t)key_id(key2) * (size_t)a.R + lane];
        uint32_t slot1, old1, slot2, old2;
        const bool new1 = filter(v1, slot1, old1);
        const uint64_t nm1 = ballot(new1);
        const bool new2 = filter(v2, slot2, old2);
        const uint64_t nm2 = ballot(new2);
        const int n1 = __builtin_popcountll(nm1), n2 = __builtin_popcountll(nm2);
        uint64_t ck1 = JX_EMPTY_KEY, ck2 = JX_EMPTY_KEY;
        if (n1 + n2 > 0) {
            if (new1) cand_id[prefix_count(nm1)] = v1;
            if (new2) cand_id[n1 + prefix_count(nm2)] = v2;
            wave_sync();
            const int ntot = n1 + n2;
            if (full) {
                for (int s0 = 0; s0 < ntot; s0 += G * U)
                    eval_batch<KIND, T, CPL, QB, U, true>(q, a.ds, s0, ntot, cand_id, cand_key, g, lig);
            } else {
                for (int s0 = 0; s0 < ntot; s0 += G * U)
                    eval_batch<KIND, T, CPL, QB, U, false>(q, a.ds, s0, ntot, cand_id, cand_key, g, lig);
            }
            wave_sync();
            if (lane < n1) ck1 = cand_key[lane];
            if (lane < n2) ck2 = cand_key[n1 + lane];
            wave_sync();
        }
        // ---- expansion of u1
        hops++;
        evals += n1;
        if (n1 > 0) frontier_merge<NREG>(fk, fr, count, L, ck1, n1, lane);
        if (!have2) continue;
        // ---- is u2 what comes next?
        int rn = -1, ln = 0;
#pragma unroll
        for (int r = 0; r < NREG; r++) {
            const uint64_t m = ballot((fk[r] & 1ull) == 0ull);
            if (rn < 0 && m != 0ull) {
                rn = r;
                ln = __builtin_ctzll(m);
            }
        }
        bool ok = false;
#pragma unroll
        for (int r = 0; r < NREG; r++) {
            if (r == rn) {
                ok = readlane64(fk[r], ln) == key2;
                if (ok && lane == ln) fk[r] |= 1ull;
            }
        }
        if (ok) {
            hops++;
            evals += n2;
            if (n2 > 0) frontier_merge<NREG>(fk, fr, count, L, ck2, n2, lane);
        } else {
            if (new2) tab[slot2] = old2;  // as if row(u2) had never been looked at
            wave_sync();
        }
    }

    int base_pos = 0;
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        const int p = r * 64 + lane;
        const uint64_t k = fk[r];
        const uint32_t id = key_id(k);
        bool keep = p < count;
        if (keep && a.deleted) keep = a.deleted[id] == 0;
        const uint64_t km = ballot(keep);
        const int pos = base_pos + prefix_count(km);
        if (keep && pos < a.out_k) {
            const uint32_t dc = key_dist(k);
            float d;
            if constexpr (KIND == K_U8)
                d = (float)dc;
            else
                d = ordered_to_f32(dc);
            a.out_ids[qi * a.out_k + pos] = id;
            a.out_dist[qi * a.out_k + pos] = d;
        }
        base_pos += __builtin_popcountll(km);
    }
    for (int p = base_pos + lane; p < a.out_k; p += 64) {
        a.out_ids[qi * a.out_k + p] = JX_NONE_ID;
        a.out_dist[qi * a.out_k + p] = __builtin_inff();
    }
    if (a.stats && lane == 0) {
        atomicAdd(&a.stats[0], (unsigned long long)hops);
        atomicAdd(&a.stats[1], (unsigned long long)evals);
    }
}

// ------------------------------------------------------------------ launch

// largest batch that takes two expansions per round: beyond it the machine is full several times over and a search is
// bound by bandwidth, not by the lifetime of a query
static constexpr long long PAIR_MAX_QUERIES = 32768;

template <int KIND, int T, int CPL, int QB>
static hipError_t launch_nreg(const BeamArgs& a, hipStream_t st, char* name) {
    const int nreg = (a.L + 63) / 64;
    const int H = a.hash_slots;
    dim3 grid((unsigned)((a.nq + JX_BEAM_WPB - 1) / JX_BEAM_WPB)), block(JX_BEAM_WPB * 64);
    if constexpr (CPL <= 2 && (KIND == K_U8 || KIND == K_RQ4 || KIND == K_RQ1)) {
        // batches that do not fill the machine several times over are bound by the lifetime of a query: two
        // expansions per round (JX_FLAG_NO_PAIR switches it off).  Not for float vectors: their searches are bound by
        // bandwidth, and the dropped second lists cost 12 % at d = 200, L = 128.
        // measured: +2..6 % for records of one 128-byte line from L = 64 (-3 % at L = 32); -8..-11 % for the 496- and
        // 208-byte records of d = 960 / 1536 codes, whose searches run at 7 TB/s and pay for every dropped list
        if (nreg <= 2 && a.L >= 64 && a.R <= 64 && a.ds.rec_stride <= 128 && a.nq <= PAIR_MAX_QUERIES && H > 0 &&
            !(a.flags & JX_FLAG_NO_PAIR)) {
            const size_t sh = (size_t)nreg * 64 * 8 + 128 * 8 + 128 * 4 + (size_t)H * (a.tag_bits ? 2 : 4);
            dim3 pgrid((unsigned)a.nq), pblock(64);
            if (name) snprintf(name, 96, "beam_search_pair_kernel<%d,%d,%d,%d,%d>", KIND, T, CPL, nreg <= 1 ? 1 : 2, QB);
            if (nreg <= 1)
                hipLaunchKernelGGL((beam_search_pair_kernel<KIND, T, CPL, 1, QB>), pgrid, pblock, sh, st, a);
            else
                hipLaunchKernelGGL((beam_search_pair_kernel<KIND, T, CPL, 2, QB>), pgrid, pblock, sh, st, a);
            return hipGetLastError();
        }
    }
#define JX_LAUNCH(NR)                                                                                   \
    {                                                                                                   \
        size_t sh = ((size_t)(NR) * 64 * 8 + 64 * 8 + 64 * 4 + (size_t)H * (a.tag_bits ? 2 : 4)) * JX_BEAM_WPB; \
        auto kern = beam_search_kernel<KIND, T, CPL, NR, QB>;                                           \
        if (sh > 48 * 1024) {                                                                           \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh); \
            if (e != hipSuccess) return e;                                                              \
        }                                                                                               \
        if (name) snprintf(name, 96, "beam_search_kernel<%d,%d,%d,%d,%d>", KIND, T, CPL, NR, QB);       \
        hipLaunchKernelGGL(kern, grid, block, sh, st, a);                                               \
        return hipGetLastError();                                                                       \
    }
    if (nreg <= 1) JX_LAUNCH(1)
    if (nreg <= 2) JX_LAUNCH(2)
    if (nreg <= 4) JX_LAUNCH(4)
    JX_LAUNCH(8)
#undef JX_LAUNCH
}

// Record-to-lane mapping.  Default: two 16-byte chunks per lane for records of at most 64 chunks -- a record is then
// covered by half as many lanes as it has chunks, so twice as many candidates share one instruction and the in-group
// reduction is one step shorter (1-bit codes with B_q = 8: one chunk per lane, the eight bit planes of a second
// chunk would not fit the registers); larger records: all 64 lanes, 2 to 6 chunks each.  JX_FLAG_LANES_WIDE: one
// chunk per lane.  JX_FLAG_LANES_NARROW: four chunks per lane (uint8 records of at most 8 chunks, float32 records of
// at most 32).
template <int KIND, int QB>
static hipError_t launch_shape(const BeamArgs& a, hipStream_t st, char* name) {
    const int nch = a.ds.nch;
    const bool wide = (a.flags & JX_FLAG_LANES_WIDE) != 0, narrow = (a.flags & JX_FLAG_LANES_NARROW) != 0;
    if constexpr (KIND == K_U8) {
        if (narrow && nch <= 8) return launch_nreg<KIND, 2, 4, QB>(a, st, name);
    }
    if constexpr (KIND == K_F32) {
        if (narrow && nch <= 32) return launch_nreg<KIND, 8, 4, QB>(a, st, name);
    }
    const bool two = !wide && nch <= 64 && !(KIND == K_RQ1 && (QB == 8 || nch > 16));
    if (two) {
        if constexpr (KIND == K_RQ1) {
            // 8 lanes x 2 chunks with the four bit planes of both chunks in registers (measured 10 % faster than
            // 16 x 1 at L = 64..128)
            return launch_nreg<KIND, 8, 2, QB>(a, st, name);
        } else {
            if (nch <= 8) return launch_nreg<KIND, 4, 2, QB>(a, st, name);
            if (nch <= 16) return launch_nreg<KIND, 8, 2, QB>(a, st, name);
            if (nch <= 32) return launch_nreg<KIND, 16, 2, QB>(a, st, name);
            return launch_nreg<KIND, 32, 2, QB>(a, st, name);
        }
    }
    if (nch <= 8) return launch_nreg<KIND, 8, 1, QB>(a, st, name);
    if (nch <= 16) return launch_nreg<KIND, 16, 1, QB>(a, st, name);
    if (nch <= 32) return launch_nreg<KIND, 32, 1, QB>(a, st, name);
    if (nch <= 64) return launch_nreg<KIND, 64, 1, QB>(a, st, name);
    if constexpr (KIND == K_RQ1) {
        return hipErrorInvalidValue;
    } else {
        if (nch <= 128) return launch_nreg<KIND, 64, 2, QB>(a, st, name);
        if constexpr (KIND == K_RQ4) {
            return hipErrorInvalidValue;
        } else {
            if (nch <= 256) return launch_nreg<KIND, 64, 4, QB>(a, st, name);
            if (nch <= 384) return launch_nreg<KIND, 64, 6, QB>(a, st, name);
            return hipErrorInvalidValue;
        }
    }
}

hipError_t launch_beam_search(int kind, int qbits, const BeamArgs& a, hipStream_t st, char* kernel_name) {
    if (kernel_name) kernel_name[0] = 0;
    if (a.nq <= 0) return hipSuccess;
    switch (kind) {
        case K_U8: return launch_shape<K_U8, 0>(a, st, kernel_name);
        case K_F32: return launch_shape<K_F32, 0>(a, st, kernel_name);
        case K_F16: return launch_shape<K_F16, 0>(a, st, kernel_name);
        case K_RQ4: return qbits == 8 ? launch_shape<K_RQ4, 8>(a, st, kernel_name) : launch_shape<K_RQ4, 4>(a, st, kernel_name);
        case K_RQ1: return qbits == 8 ? launch_shape<K_RQ1, 8>(a, st, kernel_name) : launch_shape<K_RQ1, 4>(a, st, kernel_name);
    }
    return hipErrorInvalidValue;
}

}  // namespace jx
