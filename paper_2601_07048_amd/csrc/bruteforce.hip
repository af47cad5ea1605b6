// Exhaustive k-nearest-neighbour search: the recall ground truth (Sec. 6.1).
//
// A 256-thread workgroup owns a tile of 64 queries and streams a slice of the
// base set through LDS in tiles of 64 vectors.  Each thread accumulates a 4x4
// block of the 64x64 distance tile (uint8: packed dot products, the distance is
// ||a||^2 + ||q||^2 - 2<a,q> in exact integers; float32: sum of squared
// differences; binary16: packed half dot products in float32 and the same
// norm form, clamped at 0).  A wavefront then folds each row of the tile into that query's
// sorted top-k list in LDS; only candidates that beat the current k-th key do
// any work.  A second kernel merges the per-slice lists.
#include "jx_distance.h"

namespace jx {

#define BF_TQ 64
#define BF_TB 64
#define BF_KS 16  // dwords of the vector dimension per slab

template <int DT>
__global__ void __launch_bounds__(256) bruteforce_tile_kernel(BfArgs a) {
    __shared__ uint32_t Qs[BF_KS][BF_TQ + 1];
    __shared__ uint32_t Bs[BF_KS][BF_TB + 1];
    __shared__ uint32_t Dt[BF_TQ][BF_TB + 1];
    __shared__ uint32_t qn[BF_TQ], bn[BF_TB];
    extern __shared__ __align__(16) unsigned char dyn[];
    uint64_t* topk = reinterpret_cast<uint64_t*>(dyn);  // [BF_TQ][k]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tx = tid & 15, ty = tid >> 4;
    const int k = a.k;
    const long long q0 = (long long)blockIdx.x * BF_TQ;
    const int dw = (DT == JX_U8) ? a.d / 4 : (DT == JX_F16 ? a.d / 2 : a.d);  // dwords per vector
    const long long per = (a.n + a.nsplit - 1) / a.nsplit;
    const long long b_begin = (long long)blockIdx.y * per;
    const long long b_end = b_begin + per < a.n ? b_begin + per : a.n;
    const uint32_t* Q = reinterpret_cast<const uint32_t*>(a.queries);
    const uint32_t* B = reinterpret_cast<const uint32_t*>(a.base);

    for (int i = tid; i < BF_TQ * k; i += 256) topk[i] = JX_EMPTY_KEY;
    __syncthreads();

    for (long long b0 = b_begin; b0 < b_end; b0 += BF_TB) {
        uint32_t acc_u[4][4];
        float acc_f[4][4];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                acc_u[i][j] = 0;
                acc_f[i][j] = 0.f;
            }
        uint32_t nacc = 0;  // threads 0..63: ||b||^2, threads 64..127: ||q||^2
        float naccf = 0.f;
        for (int ks = 0; ks < dw; ks += BF_KS) {
            // stage one slab of both tiles, transposed to [kk][row]
#pragma unroll
            for (int t = 0; t < 4; t++) {
                int idx = tid + t * 256;
                int row = idx / BF_KS, kk = idx % BF_KS;
                uint32_t qv = 0, bv = 0;
                if (ks + kk < dw) {
                    if (q0 + row < a.nq) qv = Q[(size_t)(q0 + row) * dw + ks + kk];
                    if (b0 + row < b_end) bv = B[(size_t)(b0 + row) * dw + ks + kk];
                }
                Qs[kk][row] = qv;
                Bs[kk][row] = bv;
            }
            __syncthreads();
            if (DT != JX_F32 && tid < 128) {
#pragma unroll
                for (int kk = 0; kk < BF_KS; kk++) {
                    uint32_t v = tid < 64 ? Bs[kk][tid] : Qs[kk][tid - 64];
                    if (DT == JX_U8)
                        nacc = __builtin_amdgcn_udot4(v, v, nacc, false);
                    else
                        naccf = hdot2(v, v, naccf);
                }
            }
#pragma unroll
            for (int kk = 0; kk < BF_KS; kk++) {
                uint32_t qv[4], bv[4];
#pragma unroll
                for (int i = 0; i < 4; i++) {
                    qv[i] = Qs[kk][ty * 4 + i];
                    bv[i] = Bs[kk][tx * 4 + i];
                }
#pragma unroll
                for (int i = 0; i < 4; i++)
#pragma unroll
                    for (int j = 0; j < 4; j++) {
                        if (DT == JX_U8) {
                            acc_u[i][j] = __builtin_amdgcn_udot4(qv[i], bv[j], acc_u[i][j], false);
                        } else if (DT == JX_F16) {
                            acc_f[i][j] = hdot2(qv[i], bv[j], acc_f[i][j]);
                        } else {
                            float df = __uint_as_float(qv[i]) - __uint_as_float(bv[j]);
                            acc_f[i][j] = fmaf(df, df, acc_f[i][j]);
                        }
                    }
            }
            __syncthreads();
        }
        if (DT != JX_F32) {
            const uint32_t nv = (DT == JX_U8) ? nacc : __float_as_uint(naccf);
            if (tid < 64) bn[tid] = nv;
            else if (tid < 128) qn[tid - 64] = nv;
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                uint32_t code;
                if (DT == JX_U8)
                    code = qn[ty * 4 + i] + bn[tx * 4 + j] - 2u * acc_u[i][j];
                else if (DT == JX_F16)
                    code = f32_to_ordered(fmaxf(__uint_as_float(qn[ty * 4 + i]) + __uint_as_float(bn[tx * 4 + j]) - 2.f * acc_f[i][j], 0.f));
                else
                    code = f32_to_ordered(acc_f[i][j]);
                Dt[ty * 4 + i][tx * 4 + j] = code;
            }
        __syncthreads();
        // fold the tile into the per-query lists: wave w owns rows 16w..16w+15
        for (int rr = 0; rr < 16; rr++) {
            const int row = wave * 16 + rr;
            if (q0 + row >= a.nq) break;
            uint64_t* list = topk + (size_t)row * k;
            const long long bid = b0 + lane;
            uint64_t key = JX_EMPTY_KEY;
            if (bid < b_end) key = ((uint64_t)Dt[row][lane] << 32) | (uint64_t)(uint32_t)bid;
            uint64_t thr = list[k - 1];
            uint64_t sm = ballot(key < thr);
            while (sm) {
                const int j = __builtin_ctzll(sm);
                sm &= sm - 1;
                const uint64_t s = readlane64(key, j);
                if (!(s < list[k - 1])) continue;  // the threshold may have tightened meanwhile
                // entries e = lane, lane+64 (k <= 128)
                uint64_t cur0 = lane < k ? list[lane] : 0, cur1 = lane + 64 < k ? list[lane + 64] : 0;
                uint64_t prev0 = (lane >= 1 && lane - 1 < k) ? list[lane - 1] : 0;
                uint64_t prev1 = (lane + 63 < k) ? list[lane + 63] : 0;
                wave_sync();
                if (lane < k) {
                    uint64_t nv = cur0;
                    if (s < cur0) nv = (lane >= 1 && s < prev0) ? prev0 : s;
                    list[lane] = nv;
                }
                if (lane + 64 < k) {
                    uint64_t nv = cur1;
                    if (s < cur1) nv = (s < prev1) ? prev1 : s;
                    list[lane + 64] = nv;
                }
                wave_sync();
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < BF_TQ * k; i += 256) {
        int row = i / k, e = i % k;
        if (q0 + row < a.nq) a.partial[((size_t)(q0 + row) * a.nsplit + blockIdx.y) * k + e] = topk[i];
    }
}

// One wavefront per query: k rounds of "take the smallest remaining key".
template <int DT>
__global__ void __launch_bounds__(64) bruteforce_merge_kernel(BfArgs a) {
    extern __shared__ __align__(16) unsigned char dyn[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(dyn);
    const long long qi = blockIdx.x;
    const int lane = threadIdx.x;
    const int m = a.nsplit * a.k;
    const uint64_t* src = a.partial + (size_t)qi * m;
    for (int i = lane; i < m; i += 64) keys[i] = src[i];
    wave_sync();
    for (int r = 0; r < a.k; r++) {
        uint64_t best = JX_EMPTY_KEY;
        int bi = -1;
        for (int i = lane; i < m; i += 64) {
            uint64_t v = keys[i];
            if (v < best) {
                best = v;
                bi = i;
            }
        }
        uint64_t wbest = best;
#pragma unroll
        for (int s = 1; s < 64; s <<= 1) {
            uint64_t o = shfl_xor(wbest, s);
            wbest = o < wbest ? o : wbest;
        }
        if (wbest != JX_EMPTY_KEY && best == wbest && bi >= 0) keys[bi] = JX_EMPTY_KEY;  // ids are unique
        wave_sync();
        if (lane == 0) {
            bool valid = wbest != JX_EMPTY_KEY;
            uint32_t code = (uint32_t)(wbest >> 32);
            float dist = (DT == JX_U8) ? (float)code : ordered_to_f32(code);
            a.out_ids[qi * a.k + r] = valid ? (uint32_t)wbest : JX_NONE_ID;
            a.out_dist[qi * a.k + r] = valid ? dist : __builtin_inff();
        }
    }
}

hipError_t launch_bruteforce(const BfArgs& a, hipStream_t st) {
    if (a.nq <= 0) return hipSuccess;
    dim3 grid((unsigned)((a.nq + BF_TQ - 1) / BF_TQ), (unsigned)a.nsplit);
    size_t sh = (size_t)BF_TQ * a.k * 8;
    size_t shm = (size_t)a.nsplit * a.k * 8;
    if (a.dtype == JX_U8) {
        auto kt = bruteforce_tile_kernel<JX_U8>;
        (void)hipFuncSetAttribute((const void*)kt, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(kt, grid, dim3(256), sh, st, a);
        auto km = bruteforce_merge_kernel<JX_U8>;
        (void)hipFuncSetAttribute((const void*)km, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(km, dim3((unsigned)a.nq), dim3(64), shm, st, a);
    } else if (a.dtype == JX_F16) {
        auto kt = bruteforce_tile_kernel<JX_F16>;
        (void)hipFuncSetAttribute((const void*)kt, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(kt, grid, dim3(256), sh, st, a);
        auto km = bruteforce_merge_kernel<JX_F16>;
        (void)hipFuncSetAttribute((const void*)km, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(km, dim3((unsigned)a.nq), dim3(64), shm, st, a);
    } else {
        auto kt = bruteforce_tile_kernel<JX_F32>;
        (void)hipFuncSetAttribute((const void*)kt, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(kt, grid, dim3(256), sh, st, a);
        auto km = bruteforce_merge_kernel<JX_F32>;
        (void)hipFuncSetAttribute((const void*)km, hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipLaunchKernelGGL(km, dim3((unsigned)a.nq), dim3(64), shm, st, a);
    }
    return hipGetLastError();
}

// ------------------------------------------------------------------ utilities

__global__ void fill_u32_kernel(uint32_t* p, long long n, uint32_t v) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

hipError_t launch_fill_u32(uint32_t* p, long long n, uint32_t v, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    long long blocks = (n + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(fill_u32_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

__global__ void row_degrees_kernel(const uint32_t* adj, long long n, int R, uint32_t* deg) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const uint32_t* row = adj + (size_t)i * R;
    int g = 0;
    while (g < R && row[g] != JX_NONE_ID) g++;
    deg[i] = (uint32_t)g;
}

// adjacency table handed in from outside: every entry must be a vertex id below n or the padding value, a row must
// be filled from the left (the kernels stop at the first padding entry) and must not name a vertex twice (two lanes
// would pass the visited filter of beamSearch in the same instruction and the frontier merge would rank the two
// equal keys alike).  One wavefront per row, the row staged in LDS; counts the offending entries.
__global__ void __launch_bounds__(256) validate_adj_kernel(const uint32_t* adj, long long n, int R, uint32_t* bad) {
    __shared__ uint32_t rows[4][JX_MAX_R];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long r = (long long)blockIdx.x * 4 + wave;
    if (r >= n) return;  // whole wavefront; no workgroup barrier below
    const uint32_t* row = adj + (size_t)r * R;
    uint32_t* mine = rows[wave];
    uint32_t nbad = 0;
    for (int e = lane; e < R; e += 64) mine[e] = row[e];
    wave_sync();
    for (int e = lane; e < R; e += 64) {
        const uint32_t v = mine[e];
        if (v == JX_NONE_ID) continue;
        bool wrong = v >= (unsigned long long)n || (e > 0 && mine[e - 1] == JX_NONE_ID);
        for (int j = 0; j < e && !wrong; j++) wrong = mine[j] == v;
        nbad += wrong ? 1u : 0u;
    }
    if (nbad) atomicAdd(bad, nbad);
}

hipError_t launch_validate_adj(const uint32_t* adj, long long n, int R, uint32_t* bad, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (R > JX_MAX_R) return hipErrorInvalidValue;
    hipLaunchKernelGGL(validate_adj_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, adj, n, R, bad);
    return hipGetLastError();
}

hipError_t launch_row_degrees(const uint32_t* adj, long long n, int R, uint32_t* deg, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(row_degrees_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, adj, n, R, deg);
    return hipGetLastError();
}

// Maximum-inner-product search as L2 search (Sec. 6.3, Text2Image): one extra coordinate sqrt(M^2 - |x|^2) for base
// vectors (M >= every |x|), 0 for queries; then |x' - q'|^2 = M^2 + |q|^2 - 2<x,q>.  One wavefront per row, squared
// norm accumulated in double; dim_out >= dim + 1, the rest is zero padding.
__global__ void __launch_bounds__(256) mips_augment_kernel(const float* in, long long n, int dim, float max_norm, int is_query,
                                                          float* out, int dim_out, float* norm_out) {
    const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int lane = threadIdx.x & 63;
    const float* x = in + (size_t)i * dim;
    float* y = out ? out + (size_t)i * dim_out : nullptr;
    double s = 0.0;
    for (int j = lane; j < dim; j += 64) {
        const float v = x[j];
        s += (double)v * (double)v;
        if (y) y[j] = v;
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += __shfl_xor(s, m, 64);
    if (norm_out && lane == 0) norm_out[i] = (float)sqrt(s);
    if (!y) return;
    if (lane == 0) {
        const double rest = (double)max_norm * (double)max_norm - s;
        y[dim] = is_query ? 0.f : (float)sqrt(rest > 0.0 ? rest : 0.0);
    }
    for (int j = dim + 1 + lane; j < dim_out; j += 64) y[j] = 0.f;
}

hipError_t launch_mips_augment(const float* in, long long n, int dim, float max_norm, int is_query, float* out, int dim_out,
                               float* norm_out, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(mips_augment_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, in, n, dim, max_norm, is_query, out,
                       dim_out, norm_out);
    return hipGetLastError();
}

// Calibration: independent gathers of whole records in a given id order, T = rec_bytes / 16 lanes per record,
// eight 16-byte loads in flight per lane; nothing depends on a loaded value except the final checksum.
template <int T>
__global__ void __launch_bounds__(256) gather_probe_kernel(const uint8_t* table, const uint32_t* ids, long long n_ids,
                                                          uint32_t* sink) {
    constexpr int G = 64 / T;
    const int lane = threadIdx.x & 63, g = lane / T, lig = lane % T;
    const long long wave = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const long long nwaves = (long long)gridDim.x * 4;
    uint32_t acc = 0;
    for (long long base = wave * (8 * G); base < n_ids; base += nwaves * (8 * G)) {
        uint4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) {
            long long i = base + u * G + g;
            if (i >= n_ids) i = n_ids - 1;
            v[u] = *reinterpret_cast<const uint4*>(table + (size_t)ids[i] * (size_t)(T * 16) + (size_t)lig * 16);
        }
#pragma unroll
        for (int u = 0; u < 8; u++) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

hipError_t launch_gather_probe(const uint8_t* table, int rec_bytes, const uint32_t* ids, long long n_ids, int blocks,
                               uint32_t* sink, hipStream_t st) {
    dim3 grid((unsigned)blocks), block(256);
    switch (rec_bytes) {
        case 64: hipLaunchKernelGGL(gather_probe_kernel<4>, grid, block, 0, st, table, ids, n_ids, sink); break;
        case 128: hipLaunchKernelGGL(gather_probe_kernel<8>, grid, block, 0, st, table, ids, n_ids, sink); break;
        case 256: hipLaunchKernelGGL(gather_probe_kernel<16>, grid, block, 0, st, table, ids, n_ids, sink); break;
        case 512: hipLaunchKernelGGL(gather_probe_kernel<32>, grid, block, 0, st, table, ids, n_ids, sink); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace jx
