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
#include "beam_kernels.h"

namespace jx {

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
        if (nreg <= 4 && a.L >= 64 && a.R <= 64 && a.ds.rec_stride <= 128 && a.nq <= PAIR_MAX_QUERIES && H > 0 &&
            !(a.flags & JX_FLAG_NO_PAIR)) {
            const int pn = nreg <= 1 ? 1 : (nreg <= 2 ? 2 : 4);
            const size_t sh = (size_t)pn * 64 * 8 + 128 * 8 + 128 * 4 + (size_t)H * (a.tag_bits ? 2 : 4);
            dim3 pgrid((unsigned)a.nq), pblock(64);
            if (name) snprintf(name, 96, "beam_search_pair_kernel<%d,%d,%d,%d,%d>", KIND, T, CPL, pn, QB);
            if (pn == 1)
                hipLaunchKernelGGL((beam_search_pair_kernel<KIND, T, CPL, 1, QB>), pgrid, pblock, sh, st, a);
            else if (pn == 2)
                hipLaunchKernelGGL((beam_search_pair_kernel<KIND, T, CPL, 2, QB>), pgrid, pblock, sh, st, a);
            else
                hipLaunchKernelGGL((beam_search_pair_kernel<KIND, T, CPL, 4, QB>), pgrid, pblock, sh, st, a);
            return hipGetLastError();
        }
    }
#define JX_LAUNCH(NR)                                                                                   \
    {                                                                                                   \
        size_t sh = ((size_t)query_lds_bytes<KIND, T, CPL, QB>() + (size_t)mirror_entries<NR>() * 8 + 64 * 8 + 64 * 4 + (size_t)H * (a.tag_bits ? 2 : 4)) * JX_BEAM_WPB; \
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
    if constexpr (KIND == K_RQ1 || KIND == K_RQ4) {
        // code searches run wide beams (L = 192, 384 are sweep points): 3 and 6 frontier registers per lane
        if (nreg == 3) JX_LAUNCH(3)
    }
    if (nreg <= 4) JX_LAUNCH(4)
    if constexpr (KIND == K_RQ1 || KIND == K_RQ4) {
        if (nreg <= 6) JX_LAUNCH(6)
    }
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
    if constexpr (KIND == K_RQ1 && QB == 4) {
        // 9 to 12 code chunks (1-bit codes of d = 1536: 208-byte records): 4 lanes x 3 code chunks, meta chunk read
        // by every lane -- 16 records per pass and no idle chunk slot
        if (!wide && !narrow && a.ds.meta_chunk > 8 && a.ds.meta_chunk <= 12) return launch_nreg<KIND, 4, 3, QB>(a, st, name);
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
    if (a.vis_cap) return launch_beam_visited(kind, a, st, kernel_name);
    if (a.flags & (JX_FLAG_TILED_LOADS | JX_FLAG_QPW_2 | JX_FLAG_QPW_4 | JX_FLAG_WAVES_2 | JX_FLAG_WAVES_4))
        return launch_beam_variant(kind, a, st, kernel_name);
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
