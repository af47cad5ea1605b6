// beamSearch kernels shared by the translation units that launch them (beam_search.hip: the production
// instances; beam_variants.hip: the ablation instances).
#pragma once
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
#ifndef JX_WPE_RQ1
#define JX_WPE_RQ1 5  // wavefronts per SIMD the 1-bit kernel with its query planes in LDS is held to (96 VGPRs)
#endif
#ifndef JX_WPE_EXACT
#define JX_WPE_EXACT 6
#endif

// Results of one query: the first out_k frontier entries that are not logically deleted (Sec. 4.6: deleted vertices
// are traversed but never returned), then padding; the expansion and evaluation counters.
template <int KIND, int NREG>
__device__ __forceinline__ void write_results(const BeamArgs& a, const int64_t qi, const uint64_t (&fk)[NREG], const int count,
                                              const int lane, const uint32_t hops, const uint32_t evals) {
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
        // 64 stripes of counters, one 128-byte line each: ten thousand same-address atomics would serialise
        unsigned long long* sp = a.stats + (size_t)(qi & 63) * 16;
        atomicAdd(&sp[0], (unsigned long long)hops);
        atomicAdd(&sp[1], (unsigned long long)evals);
    }
}

// Entries of the LDS mirror of the frontier: the binary search wants a power of two
template <int NREG>
constexpr int mirror_entries() {
    int m = 64;
    while (m < NREG * 64) m *= 2;
    return m;
}

// Merge step: candidates ck (one per lane, lane < n) into the sorted frontier (registers fk: entry p in lane p % 64,
// register p / 64; mirror fr in LDS, unused slots hold the largest key).  Every candidate finds its rank among the
// frontier entries by binary search in the mirror, all candidates at once (this also recognises an id that is in
// the frontier already).  A candidate that lands in register r (rank / 64 == r) precedes every entry of the higher
// registers and none of the lower ones, so only register r's lanes have to compare against it: the candidates are
// broadcast one by one per register, which makes the step cost O(inserted) instead of O(inserted x registers).
// One LDS scatter / gather applies the permutation; the tail beyond L is dropped.
template <int NREG>
__device__ __forceinline__ void frontier_merge(uint64_t (&fk)[NREG], uint64_t* fr, int& count, uint64_t& worst, const int L,
                                               const uint64_t ck, const int n, const int lane) {
    constexpr int FCAP = NREG * 64;
    constexpr int MIR = mirror_entries<NREG>();
    const uint64_t ckm = ck | 1ull;
    // worst = entry L - 1 of the frontier with the flag bit set (all ones while the frontier is not full): kept in
    // a register from merge to merge, so that the usual expansion, which inserts nothing, reads no LDS here
    bool beats = lane < n && ckm < worst;
    if (ballot(beats) == 0ull) return;  // nothing enters the frontier (the common case late in a search)
    uint32_t pos = 0;
#pragma unroll
    for (int step = MIR / 2; step >= 1; step >>= 1)
        if ((fr[pos + step - 1] | 1ull) < ckm) pos += step;
    // an id that is already in the frontier (the visited table forgot it) is dropped
    beats = beats && ((fr[pos] | 1ull) != ckm);
    const uint64_t sm = ballot(beats);
    if (sm == 0ull) return;
    const int n_ins = __builtin_popcountll(sm);
    uint32_t shift[NREG];
    uint32_t crank = 0, below = 0;
#pragma unroll
    for (int r = 0; r < NREG; r++) {
        uint64_t m = NREG == 1 ? sm : ballot(beats && (pos >> 6) == (uint32_t)r);
        shift[r] = below;  // candidates of the lower registers precede every entry of this one
        below += (uint32_t)__builtin_popcountll(m);
        const uint64_t mine = fk[r] | 1ull;
        while (m) {
            const int j = __builtin_ctzll(m);
            m &= m - 1;
            const uint64_t s = readlane64(ckm, j);
            shift[r] += (s < mine) ? 1u : 0u;
            crank += (s < ckm) ? 1u : 0u;  // over all registers' loops: rank among the inserted candidates
        }
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
    worst = fr[L - 1] | 1ull;
}

// The expansion list of one query (Alg. 1's set V; what Alg. 4 hands to robustPrune), kept in LDS in expansion order:
// sort its first n entries by key = (distance, id) -- a bitonic network over cap (a power of two) slots, padded with
// the largest key, four compare-exchanges per lane and stage at cap = 512 -- then write the ids and distances of the
// entries that are not logically deleted to out_ids / out_dist [qi][out_k], padded with JX_NONE / +inf.
template <int KIND>
__device__ __forceinline__ void write_visited(const BeamArgs& a, const int64_t qi, uint64_t* vis, const int n, const int lane) {
    const int cap = a.vis_cap;
    for (int i = n + lane; i < cap; i += 64) vis[i] = JX_EMPTY_KEY;
    wave_sync();
    for (int k = 2; k <= cap; k <<= 1) {
        for (int j = k >> 1; j >= 1; j >>= 1) {
            for (int p = lane; p < cap / 2; p += 64) {
                const int i = ((p & ~(j - 1)) << 1) | (p & (j - 1));  // p with a zero bit inserted at bit log2(j)
                const int m = i | j;
                const uint64_t x = vis[i], y = vis[m];
                const bool up = (i & k) == 0;
                if ((x > y) == up) {
                    vis[i] = y;
                    vis[m] = x;
                }
            }
            wave_sync();
        }
    }
    int base_pos = 0;
    for (int p0 = 0; p0 < cap; p0 += 64) {
        const uint64_t k = vis[p0 + lane];
        const uint32_t id = key_id(k);
        bool keep = p0 + lane < n;
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
}

// One query per wavefront, WPB wavefronts (queries) per workgroup; TILED selects the element-strided loads of the
// load ablation (jx_distance.h); VIS returns the expansion list instead of the frontier (BeamArgs::vis_cap).
template <int KIND, int T, int CPL, int NREG, int QB, int WPB, bool TILED, bool VIS = false>
__device__ __forceinline__ void beam_search_body(const BeamArgs& a) {
    constexpr int G = 64 / T;
    constexpr int UMAX = (KIND == K_RQ1) ? JX_UMAX_RQ1 : ((KIND == K_U8) ? JX_UMAX_EXACT : ((KIND == K_RQ4) ? JX_UMAX_RQ4 : 8));  // 16-byte loads in flight per lane (the 1-bit path keeps its bit planes in registers)
    constexpr int U0 = (UMAX / CPL) > 0 ? (UMAX / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);  // records in flight per lane group
    constexpr int FCAP = mirror_entries<NREG>();  // entries of the LDS mirror of the frontier
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = threadIdx.x >> 6;
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const int64_t qi = (int64_t)blockIdx.x * WPB + wave;
    if (qi >= a.nq) return;  // whole wavefront leaves; there is no block-level barrier below

    const int H = a.hash_slots;
    const int tag_bits = a.tag_bits;  // > 0: 16-bit entries (slot and tag together name the id exactly)
    const uint32_t id_mask = tag_bits ? ((1u << (tag_bits + 30 - __builtin_clz((uint32_t)H))) - 1u) : 0u;  // H / 2 sets
    constexpr int QL = query_lds_bytes<KIND, T, CPL, QB>();  // query bit planes kept in LDS (jx_distance.h)
    const size_t per_wave = (size_t)QL + (size_t)FCAP * 8 + 64 * 8 + 64 * 4 + (size_t)H * (tag_bits ? 2 : 4) + (VIS ? (size_t)a.vis_cap * 8 : 0);
    unsigned char* my = smem + per_wave * wave;
    uint64_t* fr = reinterpret_cast<uint64_t*>(my + QL);
    uint64_t* cand_key = fr + FCAP;
    uint32_t* cand_id = reinterpret_cast<uint32_t*>(cand_key + 64);
    uint32_t* tab = cand_id + 64;
    uint64_t* vis = reinterpret_cast<uint64_t*>(my + per_wave) - (VIS ? a.vis_cap : 0);  // behind the table (8-byte aligned)

    for (int i = lane; i < (tag_bits ? H / 2 : H); i += 64) tab[i] = JX_NONE_ID;
    for (int i = lane; i < FCAP; i += 64) fr[i] = JX_EMPTY_KEY;

    QueryRegs<KIND, CPL, QB> q;
    load_query<KIND, T, CPL, QB, TILED>(q, a.ds, qi + (qi >= a.q_skip ? 1 : 0), lig, reinterpret_cast<uint4*>(my));

    uint64_t fk[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) fk[r] = JX_EMPTY_KEY;
    int count = 0;
    uint64_t worst = JX_EMPTY_KEY;  // see frontier_merge
    const int L = a.L;
    const bool full = (sep_meta<KIND, CPL>() ? a.ds.meta_chunk : a.ds.nch) == T * CPL;  // wave-uniform: no chunk slot is idle
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
    eval_batch<KIND, T, CPL, QB, 1, false, TILED>(q, a.ds, 0, 1, cand_id, cand_key, g, lig);
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
                const uint64_t ukey = readlane64(fk[r], sel_lane);
                u = key_id(ukey);
                if (lane == sel_lane) fk[r] |= 1ull;
                if constexpr (VIS) {
                    if (lane == 0 && hops < (uint32_t)a.vis_cap) vis[hops] = ukey | 1ull;
                }
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
                    eval_batch<KIND, T, CPL, QB, U, true, TILED>(q, a.ds, s0, n_new, cand_id, cand_key, g, lig);
            } else {
                for (int s0 = 0; s0 < n_new; s0 += G * U)
                    eval_batch<KIND, T, CPL, QB, U, false, TILED>(q, a.ds, s0, n_new, cand_id, cand_key, g, lig);
            }
            evals += n_new;
            wave_sync();
            uint64_t ck = lane < n_new ? cand_key[lane] : JX_EMPTY_KEY;
            wave_sync();
            // ---- 6. merge into the sorted frontier
            frontier_merge<NREG>(fk, fr, count, worst, L, ck, n_new, lane);
        }
    }

    if constexpr (VIS) {
        write_visited<KIND>(a, qi, vis, (int)(hops < (uint32_t)a.vis_cap ? hops : (uint32_t)a.vis_cap), lane);
        if (a.stats && lane == 0) {
            unsigned long long* sp = a.stats + (size_t)(qi & 63) * 16;
            atomicAdd(&sp[0], (unsigned long long)hops);
            atomicAdd(&sp[1], (unsigned long long)evals);
        }
    } else {
        write_results<KIND, NREG>(a, qi, fk, count, lane, hops, evals);
    }
}

template <int KIND, int T, int CPL, int NREG, int QB>
__global__ void __launch_bounds__(JX_BEAM_WPB * 64) __attribute__((amdgpu_waves_per_eu(((KIND <= K_F32 || KIND == K_F16) && NREG <= 2 && CPL <= 2) ? JX_WPE_EXACT : ((query_in_lds<KIND, CPL, QB>() && NREG <= 4) ? JX_WPE_RQ1 : 1), 8)))
beam_search_kernel(BeamArgs a) {
    beam_search_body<KIND, T, CPL, NREG, QB, JX_BEAM_WPB, false>(a);
}

// Ablation instances (exact distances): WPB queries per workgroup, element-strided ("tiled") loads.
template <int KIND, int T, int CPL, int NREG, int WPB, bool TILED>
__global__ void __launch_bounds__(WPB * 64) __attribute__((amdgpu_waves_per_eu((NREG <= 2 && CPL <= 2) ? JX_WPE_EXACT : 1, 8)))
beam_search_variant_kernel(BeamArgs a) {
    beam_search_body<KIND, T, CPL, NREG, 0, WPB, TILED>(a);
}

// Insertion with the expansion list as candidate set (exact distances; see BeamArgs::vis_cap)
template <int KIND, int T, int CPL, int NREG>
__global__ void __launch_bounds__(64) beam_search_visited_kernel(BeamArgs a) {
    beam_search_body<KIND, T, CPL, NREG, 0, 1, false, true>(a);
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

// rows of at most 64 entries only (the launcher checks)
template <int KIND, int T, int CPL, int NREG, int QB>
__global__ void __launch_bounds__(64) __attribute__((amdgpu_waves_per_eu(((KIND <= K_F32 || KIND == K_F16) && NREG <= 2 && CPL <= 2) ? JX_WPE_EXACT : 1, 8)))
beam_search_pair_kernel(BeamArgs a) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    constexpr int FCAP = mirror_entries<NREG>();
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
    uint64_t worst = JX_EMPTY_KEY;  // see frontier_merge
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
        if (n1 > 0) frontier_merge<NREG>(fk, fr, count, worst, L, ck1, n1, lane);
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
            if (n2 > 0) frontier_merge<NREG>(fk, fr, count, worst, L, ck2, n2, lane);
        } else {
            if (new2) tab[slot2] = old2;  // as if row(u2) had never been looked at
            wave_sync();
        }
    }

    write_results<KIND, NREG>(a, qi, fk, count, lane, hops, evals);
}

}  // namespace jx
