// Ablation instances of the beamSearch kernel (Sec. 6.5 "Ablation study"; App. Block-Size, Tile Size and Load
// microbenchmarks), selected through the JX_FLAG_* switches of the C ABI.  Every instance returns exactly what the
// production kernels return (the parity tests run them against the CPU oracle); they exist to be timed.
//   JX_FLAG_TILED_LOADS  element-strided 4-byte loads instead of 16-byte chunks (Sec. 4.4)
//   JX_FLAG_QPW_2 / _4   two / four queries (wavefronts) per workgroup
//   JX_FLAG_WAVES_2 / _4 two / four wavefronts share one query (Sec. 4.1: larger blocks for larger vectors): wavefront
//                        0 owns the frontier and the visited table, all wavefronts evaluate distances
#include <stdio.h>
#include "beam_kernels.h"

namespace jx {

// W wavefronts per query.  Wavefront 0 selects, reads the row, filters and merges; the distance evaluations of an
// expansion are dealt to the W wavefronts in batches of G * U candidates.  Rows of at most 64 entries.
template <int KIND, int T, int CPL, int NREG, int W>
__global__ void __launch_bounds__(W * 64) beam_search_team_kernel(BeamArgs a) {
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    constexpr int MIR = mirror_entries<NREG>();
    extern __shared__ __align__(16) unsigned char smem[];
    const int wave = threadIdx.x >> 6;
    const int lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const int64_t qi = blockIdx.x;
    if (qi >= a.nq) return;  // the whole workgroup leaves

    const int H = a.hash_slots;
    const int tag_bits = a.tag_bits;
    const uint32_t id_mask = tag_bits ? ((1u << (tag_bits + 30 - __builtin_clz((uint32_t)H))) - 1u) : 0u;
    uint64_t* fr = reinterpret_cast<uint64_t*>(smem);
    uint64_t* cand_key = fr + MIR;
    uint32_t* cand_id = reinterpret_cast<uint32_t*>(cand_key + 64);
    int* ctrl = reinterpret_cast<int*>(cand_id + 64);  // [0]: candidates of this expansion, -1 = the search is over
    uint32_t* tab = reinterpret_cast<uint32_t*>(ctrl + 4);

    for (int i = threadIdx.x; i < (tag_bits ? H / 2 : H); i += W * 64) tab[i] = JX_NONE_ID;
    for (int i = threadIdx.x; i < MIR; i += W * 64) fr[i] = JX_EMPTY_KEY;

    QueryRegs<KIND, CPL, 0> q;
    load_query<KIND, T, CPL, 0>(q, a.ds, qi + (qi >= a.q_skip ? 1 : 0), lig);

    uint64_t fk[NREG];
#pragma unroll
    for (int r = 0; r < NREG; r++) fk[r] = JX_EMPTY_KEY;
    int count = 0;
    uint64_t worst = JX_EMPTY_KEY;
    const int L = a.L;
    uint32_t hops = 0, evals = 0;

    __syncthreads();
    if (wave == 0) {
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
        eval_batch<KIND, T, CPL, 0, 1>(q, a.ds, 0, 1, cand_id, cand_key, g, lig);
        wave_sync();
        if (lane == 0) {
            fk[0] = cand_key[0];
            fr[0] = cand_key[0];
        }
        wave_sync();
        count = 1;
        evals = 1;
    }

    for (;;) {
        if (wave == 0) {
            int sel_r = -1, sel_lane = 0;
#pragma unroll
            for (int r = 0; r < NREG; r++) {
                uint64_t m = ballot((fk[r] & 1ull) == 0ull);
                if (sel_r < 0 && m != 0ull) {
                    sel_r = r;
                    sel_lane = __builtin_ctzll(m);
                }
            }
            int n_new = -1;
            if (sel_r >= 0) {
                uint32_t u = 0;
#pragma unroll
                for (int r = 0; r < NREG; r++) {
                    if (r == sel_r) {
                        u = key_id(readlane64(fk[r], sel_lane));
                        if (lane == sel_lane) fk[r] |= 1ull;
                    }
                }
                hops++;
                uint32_t v = JX_NONE_ID;
                if (lane < a.R) v = a.adj[(size_t)u * (size_t)a.R + lane];
                bool is_new = false;
                if (v != JX_NONE_ID) {
                    if (tag_bits) {
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
                        is_new = true;
                    }
                }
                const uint64_t nm = ballot(is_new);
                n_new = __builtin_popcountll(nm);
                if (is_new) cand_id[prefix_count(nm)] = v;
            }
            if (lane == 0) ctrl[0] = n_new;
        }
        __syncthreads();
        const int n_new = ctrl[0];
        if (n_new < 0) break;  // every wavefront reads the same value: the barriers stay matched
        for (int s0 = wave * G * U; s0 < n_new; s0 += W * G * U)
            eval_batch<KIND, T, CPL, 0, U, false>(q, a.ds, s0, n_new, cand_id, cand_key, g, lig);
        __syncthreads();
        if (wave == 0 && n_new > 0) {
            evals += n_new;
            const uint64_t ck = lane < n_new ? cand_key[lane] : JX_EMPTY_KEY;
            wave_sync();
            frontier_merge<NREG>(fk, fr, count, worst, L, ck, n_new, lane);
        }
    }
    if (wave == 0) write_results<KIND, NREG>(a, qi, fk, count, lane, hops, evals);
}

// ------------------------------------------------------------------ launch

template <int KIND, int T, int CPL, int WPB, bool TILED>
static hipError_t launch_variant(const BeamArgs& a, hipStream_t st, char* name) {
    const int nreg = (a.L + 63) / 64;
    const int H = a.hash_slots;
    dim3 grid((unsigned)((a.nq + WPB - 1) / WPB)), block(WPB * 64);
#define JX_LAUNCH(NR)                                                                                              \
    {                                                                                                              \
        size_t sh = ((size_t)mirror_entries<NR>() * 8 + 64 * 8 + 64 * 4 + (size_t)H * (a.tag_bits ? 2 : 4)) * WPB; \
        auto kern = beam_search_variant_kernel<KIND, T, CPL, NR, WPB, TILED>;                                      \
        if (sh > 48 * 1024) {                                                                                      \
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh); \
            if (e != hipSuccess) return e;                                                                         \
        }                                                                                                          \
        if (name) snprintf(name, 96, "beam_search_variant_kernel<%d,%d,%d,%d,%d,%s>", KIND, T, CPL, NR, WPB, TILED ? "true" : "false"); \
        hipLaunchKernelGGL(kern, grid, block, sh, st, a);                                                          \
        return hipGetLastError();                                                                                  \
    }
    if (nreg <= 1) JX_LAUNCH(1)
    if (nreg <= 2) JX_LAUNCH(2)
    if (nreg <= 4) JX_LAUNCH(4)
#undef JX_LAUNCH
    return hipErrorInvalidValue;
}

template <int KIND, int T, int CPL, int W>
static hipError_t launch_team(const BeamArgs& a, hipStream_t st, char* name) {
    const int nreg = (a.L + 63) / 64;
    const int H = a.hash_slots;
    dim3 grid((unsigned)a.nq), block(W * 64);
#define JX_LAUNCH(NR)                                                                                              \
    {                                                                                                              \
        size_t sh = (size_t)mirror_entries<NR>() * 8 + 64 * 8 + 64 * 4 + 16 + (size_t)H * (a.tag_bits ? 2 : 4);    \
        if (name) snprintf(name, 96, "beam_search_team_kernel<%d,%d,%d,%d,%d>", KIND, T, CPL, NR, W);              \
        hipLaunchKernelGGL((beam_search_team_kernel<KIND, T, CPL, NR, W>), grid, block, sh, st, a);                \
        return hipGetLastError();                                                                                  \
    }
    if (nreg <= 1) JX_LAUNCH(1)
    if (nreg <= 2) JX_LAUNCH(2)
    if (nreg <= 4) JX_LAUNCH(4)
#undef JX_LAUNCH
    return hipErrorInvalidValue;
}

// ------------------------------------------------------------------ expansion list as output (JX_CAND_VISITED)

template <int KIND, int T, int CPL>
static hipError_t launch_visited_shape(const BeamArgs& a, hipStream_t st, char* name) {
    const int nreg = (a.L + 63) / 64;
    const size_t tail = 64 * 8 + 64 * 4 + (size_t)a.hash_slots * (a.tag_bits ? 2 : 4) + (size_t)a.vis_cap * 8;
    if (name) snprintf(name, 96, "beam_search_visited_kernel<%d,%d,%d,%d>", KIND, T, CPL, nreg <= 1 ? 1 : 2);
    if (nreg <= 1)
        hipLaunchKernelGGL((beam_search_visited_kernel<KIND, T, CPL, 1>), dim3((unsigned)a.nq), dim3(64), mirror_entries<1>() * 8 + tail, st, a);
    else
        hipLaunchKernelGGL((beam_search_visited_kernel<KIND, T, CPL, 2>), dim3((unsigned)a.nq), dim3(64), mirror_entries<2>() * 8 + tail, st, a);
    return hipGetLastError();
}

// Offered for the record shapes of the five workload configurations -- uint8 vectors of at most 128 bytes, float32
// vectors of at most 512 bytes or of 2,049 to 6,144 bytes -- with L_build <= 128.
bool visited_list_offered(int kind, int nch, int L, int R) {
    (void)R;
    if (L > 128) return false;
    if (kind == K_U8) return nch <= 8;
    if (kind == K_F32) return nch <= 32 || (nch > 128 && nch <= 384);
    return false;
}

hipError_t launch_beam_visited(int kind, const BeamArgs& a, hipStream_t st, char* kernel_name) {
    const int nch = a.ds.nch;
    if (!visited_list_offered(kind, nch, a.L, a.R) || a.vis_cap < 64 || a.vis_cap > 512 || (a.vis_cap & (a.vis_cap - 1)))
        return hipErrorInvalidValue;
    if (kind == K_U8) return launch_visited_shape<K_U8, 4, 2>(a, st, kernel_name);
    if (nch <= 32) return launch_visited_shape<K_F32, 16, 2>(a, st, kernel_name);
    if (nch <= 256) return launch_visited_shape<K_F32, 64, 4>(a, st, kernel_name);
    return launch_visited_shape<K_F32, 64, 6>(a, st, kernel_name);
}

// Instances exist for the shapes the ablation measures: 128-byte uint8 vectors, float32 vectors of at most 512 bytes
// (tiled loads) and of 2,049 to 6,144 bytes (tiled loads, wavefront teams), beam widths up to 256.  Anything else:
// hipErrorInvalidValue, which the C ABI reports as a failed launch.
hipError_t launch_beam_variant(int kind, const BeamArgs& a, hipStream_t st, char* kernel_name) {
    const int nch = a.ds.nch;
    const uint32_t f = a.flags;
    const int nsel = ((f & JX_FLAG_TILED_LOADS) ? 1 : 0) + ((f & (JX_FLAG_QPW_2 | JX_FLAG_QPW_4)) ? 1 : 0) +
                     ((f & (JX_FLAG_WAVES_2 | JX_FLAG_WAVES_4)) ? 1 : 0);
    if (nsel != 1 || a.L > 256) return hipErrorInvalidValue;  // one axis at a time
    if (f & JX_FLAG_TILED_LOADS) {
        if (kind == K_U8 && nch <= 8) return launch_variant<K_U8, 4, 2, 1, true>(a, st, kernel_name);
        if (kind == K_F32 && nch <= 32) return launch_variant<K_F32, 16, 2, 1, true>(a, st, kernel_name);
        if (kind == K_F32 && nch > 128 && nch <= 256) return launch_variant<K_F32, 64, 4, 1, true>(a, st, kernel_name);
        return hipErrorInvalidValue;
    }
    if (f & (JX_FLAG_QPW_2 | JX_FLAG_QPW_4)) {
        if (kind != K_U8 || nch > 8) return hipErrorInvalidValue;
        if (f & JX_FLAG_QPW_4) return launch_variant<K_U8, 4, 2, 4, false>(a, st, kernel_name);
        return launch_variant<K_U8, 4, 2, 2, false>(a, st, kernel_name);
    }
    if (kind != K_F32 || a.R > 64) return hipErrorInvalidValue;
    const bool four = (f & JX_FLAG_WAVES_4) != 0;
    if (nch > 128 && nch <= 256) return four ? launch_team<K_F32, 64, 4, 4>(a, st, kernel_name) : launch_team<K_F32, 64, 4, 2>(a, st, kernel_name);
    if (nch > 256 && nch <= 384) return four ? launch_team<K_F32, 64, 6, 4>(a, st, kernel_name) : launch_team<K_F32, 64, 6, 2>(a, st, kernel_name);
    return hipErrorInvalidValue;
}

}  // namespace jx
