// Batch deletion (Sec. 4.6, the algorithm of FreshDiskANN): mark, consolidate.
//
//   mark         one byte per vertex; deleted vertices stay in the graph and are
//                traversed, the search kernel drops them from every output.
//   consolidate  for every live vertex v that points to a deleted vertex the
//                candidate set is (live neighbours of v) U (live neighbours of
//                each deleted neighbour), v excluded.  The work is arranged as
//                flat, regular passes instead of one irregular task per vertex:
//                count -> prefix sum -> emit (v, candidate) pairs -> sort by
//                (v, candidate) -> drop repeated pairs and compute d(v, c) ->
//                stable sort by (v, distance), which keeps equal distances in
//                candidate-id order -> robustPrune per segment (the reverse-merge
//                kernel with the existing row ignored) -> empty the deleted rows.
//                New rows only depend on the rows of v itself and of deleted
//                vertices, which are not rewritten until the end, so slices of
//                vertices can be processed one after the other.
#include "jx_distance.h"

namespace jx {

__global__ void mark_deleted_kernel(uint8_t* deleted, const uint32_t* ids, long long n, long long nvert,
                                    unsigned long long* counter) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t id = ids[i];
    if (id >= (unsigned long long)nvert) return;  // unknown ids are ignored
    // byte-wide exchange through the containing word keeps repeated ids from being counted twice
    uint32_t* w = reinterpret_cast<uint32_t*>(deleted + (id & ~3u));
    const uint32_t bit = 1u << (8 * (id & 3u));
    const uint32_t old = atomicOr(w, bit);
    if (!(old & bit)) atomicAdd(counter, 1ull);
}

hipError_t launch_mark_deleted(uint8_t* deleted, const uint32_t* ids, long long n, long long nvert, unsigned long long* counter,
                               hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(mark_deleted_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, deleted, ids, n, nvert, counter);
    return hipGetLastError();
}

// one wavefront per vertex; R <= 256
__global__ void __launch_bounds__(256) consol_count_kernel(ConsolArgs a) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= a.n) return;
    const int lane = lane_id();
    uint32_t total = 0;
    bool hit = false;
    if (!a.deleted[v]) {
        const uint32_t* row = a.adj + (size_t)v * a.R;
        for (int rb = 0; rb < a.R; rb += 64) {
            const uint32_t u = rb + lane < a.R ? row[rb + lane] : JX_NONE_ID;
            const bool valid = u != JX_NONE_ID;
            const bool dead = valid && a.deleted[u] != 0;
            total += (uint32_t)__builtin_popcountll(ballot(valid && !dead));
            uint64_t dm = ballot(dead);
            hit = hit || dm != 0ull;
            while (dm) {
                const int j = __builtin_ctzll(dm);
                dm &= dm - 1;
                const uint32_t du = readlane32(u, j);
                const uint32_t* ru = a.adj + (size_t)du * a.R;
                for (int rc = 0; rc < a.R; rc += 64) {
                    const uint32_t w = rc + lane < a.R ? ru[rc + lane] : JX_NONE_ID;
                    const bool ok = w != JX_NONE_ID && w != (uint32_t)v && a.deleted[w] == 0;
                    total += (uint32_t)__builtin_popcountll(ballot(ok));
                }
            }
        }
    }
    if (lane == 0) a.cnt[v] = hit ? total : 0u;
}

hipError_t launch_consol_count(const ConsolArgs& a, hipStream_t st) {
    if (a.n <= 0) return hipSuccess;
    hipLaunchKernelGGL(consol_count_kernel, dim3((unsigned)((a.n + 3) / 4)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// same walk as the count kernel, writing (v << 32 | candidate) keys
__global__ void __launch_bounds__(256) consol_emit_kernel(ConsolArgs a) {
    const long long v = a.v0 + (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= a.v1) return;
    const int lane = lane_id();
    if (a.cnt[v] == 0u) return;  // deleted itself, or no deleted neighbour
    uint32_t pos = a.offs[v - a.v0];
    const uint32_t* row = a.adj + (size_t)v * a.R;
    for (int rb = 0; rb < a.R; rb += 64) {
        const uint32_t u = rb + lane < a.R ? row[rb + lane] : JX_NONE_ID;
        const bool valid = u != JX_NONE_ID;
        const bool dead = valid && a.deleted[u] != 0;
        const uint64_t lm = ballot(valid && !dead);
        if (valid && !dead) {
            const uint32_t p = pos + (uint32_t)prefix_count(lm);
            a.keys[p] = ((uint64_t)(uint32_t)v << 32) | u;
            a.vals[p] = 0u;
        }
        pos += (uint32_t)__builtin_popcountll(lm);
        uint64_t dm = ballot(dead);
        while (dm) {
            const int j = __builtin_ctzll(dm);
            dm &= dm - 1;
            const uint32_t du = readlane32(u, j);
            const uint32_t* ru = a.adj + (size_t)du * a.R;
            for (int rc = 0; rc < a.R; rc += 64) {
                const uint32_t w = rc + lane < a.R ? ru[rc + lane] : JX_NONE_ID;
                const bool ok = w != JX_NONE_ID && w != (uint32_t)v && a.deleted[w] == 0;
                const uint64_t om = ballot(ok);
                if (ok) {
                    const uint32_t p = pos + (uint32_t)prefix_count(om);
                    a.keys[p] = ((uint64_t)(uint32_t)v << 32) | w;
                    a.vals[p] = 0u;
                }
                pos += (uint32_t)__builtin_popcountll(om);
            }
        }
    }
}

hipError_t launch_consol_emit(const ConsolArgs& a, hipStream_t st) {
    const long long nv = a.v1 - a.v0;
    if (nv <= 0) return hipSuccess;
    hipLaunchKernelGGL(consol_emit_kernel, dim3((unsigned)((nv + 3) / 4)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// sorted (v, candidate) pairs -> (v << 32 | distance bits, candidate); a repeated pair gets the empty key.
// 8 lanes per pair, chunks strided over the lanes.
template <int KIND>
__global__ void __launch_bounds__(256) consol_dist_kernel(ConsolArgs a, uint64_t* keys_out, uint32_t* vals_out) {
    const int lane = lane_id();
    const int g = lane >> 3, lig = lane & 7;
    const long long i = ((long long)blockIdx.x * 4 + (threadIdx.x >> 6)) * 8 + g;
    const bool in = i < a.E;
    const uint64_t k = in ? a.keys[i] : JX_EMPTY_KEY;
    const bool dup = in && i > 0 && a.keys[i - 1] == k;
    const uint32_t v = (uint32_t)(k >> 32), c = (uint32_t)k;
    uint32_t acc_u = 0;
    float acc_f = 0.f;
    if (in && !dup) {
        const uint8_t* pv = a.ds.recs + (size_t)v * (size_t)a.ds.rec_stride;
        const uint8_t* pc = a.ds.recs + (size_t)c * (size_t)a.ds.rec_stride;
        for (int ch = lig; ch < a.ds.nch; ch += 8) {
            const uint4 x = load16(pv + (size_t)ch * 16), y = load16(pc + (size_t)ch * 16);
            const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
            for (int t = 0; t < 4; t++) {
                if constexpr (KIND == K_U8) {
                    acc_u = __builtin_amdgcn_udot4(xs[t], xs[t], acc_u, false);
                    acc_u = __builtin_amdgcn_udot4(ys[t], ys[t], acc_u, false);
                    acc_u -= 2u * __builtin_amdgcn_udot4(xs[t], ys[t], 0u, false);
                } else if constexpr (KIND == K_F16) {
                    const half2_t hx = __builtin_bit_cast(half2_t, xs[t]), hy = __builtin_bit_cast(half2_t, ys[t]);
                    const float d0 = (float)hx.x - (float)hy.x, d1 = (float)hx.y - (float)hy.y;
                    acc_f = fmaf(d0, d0, acc_f);
                    acc_f = fmaf(d1, d1, acc_f);
                } else {
                    const float df = __uint_as_float(xs[t]) - __uint_as_float(ys[t]);
                    acc_f = fmaf(df, df, acc_f);
                }
            }
        }
    }
    float dist;
    if constexpr (KIND == K_U8) {
        dist = (float)group_sum<8>(acc_u);
    } else {
        dist = fmaxf(group_sum<8>(acc_f), 0.f);
    }
    if (in && lig == 0) {
        keys_out[i] = dup ? JX_EMPTY_KEY : (((uint64_t)v << 32) | __float_as_uint(dist));
        vals_out[i] = dup ? JX_NONE_ID : c;
    }
}

hipError_t launch_consol_dist(int dtype, const ConsolArgs& a, uint64_t* keys_out, uint32_t* vals_out, hipStream_t st) {
    if (a.E <= 0) return hipSuccess;
    dim3 grid((unsigned)((a.E + 31) / 32)), block(256);
    if (dtype == JX_U8)
        hipLaunchKernelGGL(consol_dist_kernel<K_U8>, grid, block, 0, st, a, keys_out, vals_out);
    else if (dtype == JX_F16)
        hipLaunchKernelGGL(consol_dist_kernel<K_F16>, grid, block, 0, st, a, keys_out, vals_out);
    else
        hipLaunchKernelGGL(consol_dist_kernel<K_F32>, grid, block, 0, st, a, keys_out, vals_out);
    return hipGetLastError();
}

__global__ void clear_deleted_rows_kernel(uint32_t* adj, int R, long long n, const uint8_t* deleted) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n * R) return;
    if (deleted[i / R]) adj[i] = JX_NONE_ID;
}

hipError_t launch_clear_deleted_rows(uint32_t* adj, int R, long long n, const uint8_t* deleted, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(clear_deleted_rows_kernel, dim3((unsigned)((n * R + 255) / 256)), dim3(256), 0, st, adj, R, n, deleted);
    return hipGetLastError();
}

// squared distance (double) of every live vertex to vertex `target`; deleted vertices get +inf
template <int DT>
__global__ void __launch_bounds__(256) dist_to_vertex_kernel(const void* vecs, long long n, int d, uint32_t target,
                                                            const uint8_t* deleted, double* out) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = lane_id();
    double s = 0.0;
    for (int j = lane; j < d; j += 64) {
        double a, b;
        if (DT == JX_U8) {
            a = (double)reinterpret_cast<const uint8_t*>(vecs)[(size_t)i * d + j];
            b = (double)reinterpret_cast<const uint8_t*>(vecs)[(size_t)target * d + j];
        } else if (DT == JX_F16) {
            a = (double)(float)reinterpret_cast<const _Float16*>(vecs)[(size_t)i * d + j];
            b = (double)(float)reinterpret_cast<const _Float16*>(vecs)[(size_t)target * d + j];
        } else {
            a = (double)reinterpret_cast<const float*>(vecs)[(size_t)i * d + j];
            b = (double)reinterpret_cast<const float*>(vecs)[(size_t)target * d + j];
        }
        const double t = a - b;
        s += t * t;
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += shfl_xor(s, m);
    if (lane == 0) out[i] = deleted[i] ? __builtin_inf() : s;
}

hipError_t launch_nearest_live(const void* vecs, int dtype, long long n, int d, uint32_t target, const uint8_t* deleted,
                               double* dist, uint32_t* out_id, hipStream_t st) {
    dim3 grid((unsigned)((n + 3) / 4)), block(256);
    if (dtype == JX_U8)
        hipLaunchKernelGGL(dist_to_vertex_kernel<JX_U8>, grid, block, 0, st, vecs, n, d, target, deleted, dist);
    else if (dtype == JX_F16)
        hipLaunchKernelGGL(dist_to_vertex_kernel<JX_F16>, grid, block, 0, st, vecs, n, d, target, deleted, dist);
    else
        hipLaunchKernelGGL(dist_to_vertex_kernel<JX_F32>, grid, block, 0, st, vecs, n, d, target, deleted, dist);
    return launch_argmin(dist, n, out_id, st);
}

// ---- compaction (third phase of Sec. 4.6): order-preserving renaming of the live vertices ----

// flag[v] = 1 for live vertices (scanned into the renaming afterwards); err is set if a live row names a deleted vertex
__global__ void __launch_bounds__(256) compact_flags_kernel(const uint32_t* adj, int R, long long n, const uint8_t* deleted,
                                                           uint32_t* flag, uint32_t* err) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v > n) return;
    const int lane = lane_id();
    if (v == n) {  // one slot past the end receives the total
        if (lane == 0) flag[n] = 0u;
        return;
    }
    const bool live = deleted[v] == 0;
    if (lane == 0) flag[v] = live ? 1u : 0u;
    if (!live) return;
    bool bad = false;
    for (int j = lane; j < R; j += 64) {
        const uint32_t u = adj[(size_t)v * R + j];
        if (u != JX_NONE_ID && deleted[u]) bad = true;
    }
    if (bad) atomicOr(err, 1u);
}

// adj[i] = map[adj[i]] in place; the public renaming gets NONE for removed vertices
__global__ void compact_rename_kernel(uint32_t* adj, long long n_entries, const uint32_t* map, const uint8_t* deleted, long long n,
                                      uint32_t* public_map) {
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_entries) {
        const uint32_t u = adj[i];
        if (u != JX_NONE_ID) adj[i] = map[u];
    }
    if (public_map && i < n) public_map[i] = deleted[i] ? JX_NONE_ID : map[i];
}

// live records of vertices [c0, c1) -> staging, packed in order; UNIT = uint4 or uint32_t
template <typename UNIT>
__global__ void __launch_bounds__(256) compact_gather_kernel(const uint8_t* base, int rec_bytes, long long c0, long long c1,
                                                            const uint32_t* map, const uint8_t* deleted, uint8_t* staging) {
    const long long v = c0 + (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= c1 || deleted[v]) return;
    const int lane = lane_id();
    const size_t slot = (size_t)(map[v] - map[c0]);
    const UNIT* src = reinterpret_cast<const UNIT*>(base + (size_t)v * rec_bytes);
    UNIT* dst = reinterpret_cast<UNIT*>(staging + slot * rec_bytes);
    for (int b = lane; b < rec_bytes / (int)sizeof(UNIT); b += 64) dst[b] = src[b];
}

// staging -> base[map[c0] ...]; the number of records is read on the device (map[c1] - map[c0])
template <typename UNIT>
__global__ void __launch_bounds__(256) compact_scatter_kernel(uint8_t* base, int rec_bytes, long long c0, long long c1,
                                                             const uint32_t* map, const uint8_t* staging) {
    const size_t units = (size_t)(map[c1] - map[c0]) * (size_t)(rec_bytes / (int)sizeof(UNIT));
    UNIT* dst = reinterpret_cast<UNIT*>(base + (size_t)map[c0] * rec_bytes);
    const UNIT* src = reinterpret_cast<const UNIT*>(staging);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < units; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

hipError_t launch_compact_flags(const uint32_t* adj, int R, long long n, const uint8_t* deleted, uint32_t* flag, uint32_t* err,
                                hipStream_t st) {
    hipLaunchKernelGGL(compact_flags_kernel, dim3((unsigned)((n + 1 + 3) / 4)), dim3(256), 0, st, adj, R, n, deleted, flag, err);
    return hipGetLastError();
}

hipError_t launch_compact_rename(uint32_t* adj, int R, long long n, const uint32_t* map, const uint8_t* deleted,
                                 uint32_t* public_map, hipStream_t st) {
    const long long ne = n * R;
    hipLaunchKernelGGL(compact_rename_kernel, dim3((unsigned)((ne + 255) / 256)), dim3(256), 0, st, adj, ne, map, deleted, n,
                       public_map);
    return hipGetLastError();
}

// Moves the live records of one array to their new places, slice by slice through the staging buffer: the
// destination of a slice ends where its sources begin at the latest, and its own sources are all in the staging
// buffer before the first of them is overwritten.
template <typename UNIT>
static void compact_records_units(uint8_t* base, int rec_bytes, long long n, const uint32_t* map, const uint8_t* deleted,
                                  uint8_t* staging, long long slice, hipStream_t st) {
    for (long long c0 = 0; c0 < n; c0 += slice) {
        const long long c1 = c0 + slice < n ? c0 + slice : n;
        hipLaunchKernelGGL(compact_gather_kernel<UNIT>, dim3((unsigned)((c1 - c0 + 3) / 4)), dim3(256), 0, st, base, rec_bytes, c0,
                           c1, map, deleted, staging);
        hipLaunchKernelGGL(compact_scatter_kernel<UNIT>, dim3(2048), dim3(256), 0, st, base, rec_bytes, c0, c1, map, staging);
    }
}

// Moves the live records of one array to their new places, slice by slice through the staging buffer: the
// destination of a slice ends where its sources begin at the latest, and its own sources are all in the staging
// buffer before the first of them is overwritten.
hipError_t launch_compact_records(uint8_t* base, int rec_bytes, long long n, const uint32_t* map, const uint8_t* deleted,
                                  uint8_t* staging, long long staging_bytes, hipStream_t st) {
    if (rec_bytes % 4) return hipErrorInvalidValue;
    long long slice = staging_bytes / rec_bytes;
    if (slice < 1) return hipErrorInvalidValue;
    if (slice > (1LL << 24)) slice = 1LL << 24;  // keeps the gather grid within range
    if (rec_bytes % 16 == 0)
        compact_records_units<uint4>(base, rec_bytes, n, map, deleted, staging, slice, st);
    else
        compact_records_units<uint32_t>(base, rec_bytes, n, map, deleted, staging, slice, st);
    return hipGetLastError();
}

}  // namespace jx
