// RaBitQ pipeline (Sec. 5.1): rotation GEMM on the matrix cores, encoder,
// integer query records, exact re-rank.
//
//   rotate      out = (in - c) P^T   float32 MFMA (32x32x2), 128x128 tile per
//               workgroup, 64x64 per wavefront, K staged through LDS in slabs
//               of 32; the centroid is subtracted while staging.
//   encode      one wavefront per vector: 1-bit codes via ballot, 4-bit codes
//               with the max-abs grid scale; data_add, data_rescale in double.
//   query prep  one wavefront per query: min/max, B_q-bit integer query,
//               nibble planes (4-bit codes) or bit planes (1-bit codes).
//   rerank      one wavefront per query: exact float32 squared L2 of the first
//               `rerank` frontier entries against the original query, sorted by
//               (distance, id).
#include "jx_distance.h"

namespace jx {

typedef float f32x16 __attribute__((ext_vector_type(16)));

#define GT 128
#define GK 32
#define GLD 36  // padded LDS row (floats)

// IN: storage type of the input rows (JX_F32, JX_F16, JX_U8); all three convert to float32 exactly
template <int IN>
__global__ void __launch_bounds__(256) rotate_gemm_kernel(const void* __restrict__ in_v, long long n, int d,
                                                          const float* __restrict__ P, const float* __restrict__ c,
                                                          float* __restrict__ out) {
    __shared__ __align__(16) float As[GT][GLD];
    __shared__ __align__(16) float Bs[GT][GLD];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const long long m0 = (long long)blockIdx.y * GT;
    const int n0 = blockIdx.x * GT;
    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

    for (int k0 = 0; k0 < d; k0 += GK) {
#pragma unroll
        for (int t = 0; t < 4; t++) {
            const int idx = tid + t * 256;
            const int row = idx >> 3, c4 = (idx & 7) * 4;
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (k0 + c4 < d) {
                if (m0 + row < n) {
                    float4 v;
                    if (IN == JX_F16) {
                        const _Float16* hp = reinterpret_cast<const _Float16*>(in_v) + (size_t)(m0 + row) * d + k0 + c4;
                        v = make_float4((float)hp[0], (float)hp[1], (float)hp[2], (float)hp[3]);
                    } else if (IN == JX_U8) {
                        const uint8_t* bp = reinterpret_cast<const uint8_t*>(in_v) + (size_t)(m0 + row) * d + k0 + c4;
                        v = make_float4((float)bp[0], (float)bp[1], (float)bp[2], (float)bp[3]);
                    } else {
                        v = *reinterpret_cast<const float4*>(reinterpret_cast<const float*>(in_v) + (size_t)(m0 + row) * d + k0 + c4);
                    }
                    const float4 cc = *reinterpret_cast<const float4*>(c + k0 + c4);
                    a = make_float4(v.x - cc.x, v.y - cc.y, v.z - cc.z, v.w - cc.w);
                }
                if (n0 + row < d) b = *reinterpret_cast<const float4*>(P + (size_t)(n0 + row) * d + k0 + c4);
            }
            *reinterpret_cast<float4*>(&As[row][c4]) = a;
            *reinterpret_cast<float4*>(&Bs[row][c4]) = b;
        }
        __syncthreads();
#pragma unroll
        for (int s8 = 0; s8 < GK / 8; s8++) {
            float4 af[2], bf[2];
#pragma unroll
            for (int s = 0; s < 2; s++) {
                af[s] = *reinterpret_cast<const float4*>(&As[wm * 64 + s * 32 + (lane & 31)][8 * s8 + 4 * (lane >> 5)]);
                bf[s] = *reinterpret_cast<const float4*>(&Bs[wn * 64 + s * 32 + (lane & 31)][8 * s8 + 4 * (lane >> 5)]);
            }
#pragma unroll
            for (int mi = 0; mi < 2; mi++)
#pragma unroll
                for (int ni = 0; ni < 2; ni++) {
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi].x, bf[ni].x, acc[mi][ni], 0, 0, 0);
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi].y, bf[ni].y, acc[mi][ni], 0, 0, 0);
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi].z, bf[ni].z, acc[mi][ni], 0, 0, 0);
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[mi].w, bf[ni].w, acc[mi][ni], 0, 0, 0);
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int mi = 0; mi < 2; mi++)
#pragma unroll
        for (int ni = 0; ni < 2; ni++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const long long row = m0 + wm * 64 + mi * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
                const int col = n0 + wn * 64 + ni * 32 + (lane & 31);
                if (row < n && col < d) out[(size_t)row * d + col] = acc[mi][ni][e];
            }
}

hipError_t launch_rotate(const void* in, int in_dtype, long long n, int d, const float* P, const float* c, float* out,
                         hipStream_t st) {
    if (n <= 0) return hipSuccess;
    dim3 grid((unsigned)((d + GT - 1) / GT), (unsigned)((n + GT - 1) / GT));
    if (in_dtype == JX_F16)
        hipLaunchKernelGGL(rotate_gemm_kernel<JX_F16>, grid, dim3(256), 0, st, in, n, d, P, c, out);
    else if (in_dtype == JX_U8)
        hipLaunchKernelGGL(rotate_gemm_kernel<JX_U8>, grid, dim3(256), 0, st, in, n, d, P, c, out);
    else
        hipLaunchKernelGGL(rotate_gemm_kernel<JX_F32>, grid, dim3(256), 0, st, in, n, d, P, c, out);
    return hipGetLastError();
}

// ------------------------------------------------------------------ encoder

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v += shfl_xor(v, m);
    return v;
}
__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v = fmaxf(v, shfl_xor(v, m));
    return v;
}
__device__ __forceinline__ float wave_min_f32(float v) {
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) v = fminf(v, shfl_xor(v, m));
    return v;
}

// Code layout: 1-bit: coordinate i is bit i%32 of dword i/32.  4-bit: coordinate i
// is nibble i%8 of dword i/8 (so even coordinates sit in low nibbles of a byte).
__global__ void __launch_bounds__(256) encode_kernel(EncodeArgs a) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= a.n) return;
    const int lane = lane_id();
    const float* r = a.rot + (size_t)v * a.d;
    uint8_t* code = a.codes + (size_t)v * a.code_stride;
    double l2 = 0.0, ip = 0.0;
    if (a.bits == 1) {
        for (int c0 = 0; c0 < a.d; c0 += 64) {
            const int i = c0 + lane;
            const float x = i < a.d ? r[i] : -1.0f;
            const bool pos = i < a.d && x >= 0.0f;
            const uint64_t m = ballot(pos);
            if (i < a.d) {
                l2 += (double)x * (double)x;
                ip += 0.5 * fabs((double)x);
            }
            if (lane == 0) *reinterpret_cast<uint32_t*>(code + c0 / 8) = (uint32_t)m;
            if (lane == 1 && c0 + 32 < a.d) *reinterpret_cast<uint32_t*>(code + c0 / 8 + 4) = (uint32_t)(m >> 32);
        }
    } else {
        const int half = 1 << (a.bits - 1);
        float amax = 0.f;
        for (int i = lane; i < a.d; i += 64) amax = fmaxf(amax, fabsf(r[i]));
        amax = wave_max_f32(amax);
        const float t = amax > 0.f ? __fdiv_rn((float)half - 0.5f, amax) : 0.f;
        const double cb = ((double)(1 << a.bits) - 1.0) * 0.5;
        // 32 / bits consecutive coordinates per lane -> one dword (field i % per of dword i / per)
        const int per = 32 / a.bits;
        for (int c0 = 0; c0 < a.d; c0 += 64 * per) {
            const int i0 = c0 + lane * per;
            if (i0 < a.d) {
                uint32_t w = 0;
                for (int j = 0; j < per; j++) {
                    const float x = r[i0 + j];
                    float lvf = floorf(__fmul_rn(t, fabsf(x)));
                    int lv = (int)lvf;
                    lv = lv > half - 1 ? half - 1 : (lv < 0 ? 0 : lv);
                    const int u = x >= 0.0f ? half + lv : half - 1 - lv;
                    w |= (uint32_t)u << (a.bits * j);
                    l2 += (double)x * (double)x;
                    ip += ((double)u - cb) * (double)x;
                }
                *reinterpret_cast<uint32_t*>(code + (size_t)i0 * a.bits / 8) = w;
            }
        }
    }
    l2 = wave_sum_f64(l2);
    ip = wave_sum_f64(ip);
    for (int b = a.code_bytes + lane * 4; b < a.pad_to; b += 256) *reinterpret_cast<uint32_t*>(code + b) = 0u;
    if (lane == 0) {
        float* m = reinterpret_cast<float*>(a.meta + (size_t)v * a.meta_stride);
        m[0] = l2 > 0.0 ? (float)l2 : 0.f;
        m[1] = l2 > 0.0 ? (float)(-2.0 * l2 / ip) : 0.f;
        for (int b = 0; b < a.meta_pad; b += 4) m[2 + b / 4] = 0.f;
    }
}

// ---- max-cosine rule (m > 1): the grid point whose direction is closest to r.
// One workgroup per vector.  The grid scale t steps coordinate i to level j at the breakpoint t = j/|r_i|
// (j = 1 .. 2^(m-1)-1); after the breakpoints <= t have been applied,
//     <xbar,|r|> = l1/2 + sum_j PrefA[cnt_j(t)],   ||xbar||^2 = d/4 + sum_j 2j cnt_j(t),
// where cnt_j(t) counts the level-j breakpoints <= t and PrefA are prefix sums of the magnitudes in descending
// order.  So only the d magnitudes are sorted (bitonic network in LDS); the level-j breakpoints j/|r|_(p) are then
// already ascending in p, their quotients are tabulated once in double (comparisons are on the very values the
// definition compares), and every breakpoint evaluates its cosine with one binary search per level: the state at
// the end of its group of equal t.  The largest cosine wins, the smallest t among equals, and t -> 0+ competes.  The
// level of a coordinate is then the number of its own breakpoints that are <= t.
#define MC_CAP 8192   // breakpoints per vector
#define MC_DMAX 4096  // dimensions

__device__ __forceinline__ double block_scan_incl(double v, double* ws, int tid) {
    // inclusive scan over the 256 threads of the workgroup
    const int lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
        double o = __shfl_up(v, s, 64);
        if (lane >= s) v += o;
    }
    if (lane == 63) ws[wave] = v;
    __syncthreads();
    double off = 0.0;
    for (int w = 0; w < wave; w++) off += ws[w];
    __syncthreads();
    return v + off;
}

__global__ void __launch_bounds__(256) encode_maxcos_kernel(EncodeArgs a) {
    extern __shared__ __align__(16) unsigned char dyn[];
    const int half = 1 << (a.bits - 1), nl = half - 1;
    int dpad = 256;
    while (dpad < a.d) dpad <<= 1;
    float* sa = reinterpret_cast<float*>(dyn);                          // [dpad] magnitudes, descending
    double* pref = reinterpret_cast<double*>(dyn + (size_t)dpad * 4);   // [dpad + 1] prefix sums of sa
    double* Q = pref + dpad + 2;                                        // [nl][d] quotients j / sa[p]
    __shared__ double ws[8];
    __shared__ double red_c[256], red_t[256];
    __shared__ int s_npos;
    __shared__ double s_l1, s_l2, s_ip, s_best_t;
    const int tid = threadIdx.x;
    const long long v = blockIdx.x;
    const float* r = a.rot + (size_t)v * a.d;
    uint8_t* code = a.codes + (size_t)v * a.code_stride;

    // ---- sums, magnitudes
    double l1 = 0.0, l2 = 0.0;
    for (int i = tid; i < a.d; i += 256) {
        const double x = fabs((double)r[i]);
        l1 += x;
        l2 += x * x;
    }
    int npos_t = 0;
    for (int e = tid; e < dpad; e += 256) {
        const float x = e < a.d ? fabsf(r[e]) : 0.f;
        sa[e] = x;
        npos_t += x > 0.f ? 1 : 0;
    }
    {   // block sums (fixed order)
        const double t1 = block_scan_incl(l1, ws, tid);
        if (tid == 255) s_l1 = t1;
        const double t2 = block_scan_incl(l2, ws, tid);
        if (tid == 255) s_l2 = t2;
        const double t3 = block_scan_incl((double)npos_t, ws, tid);
        if (tid == 255) s_npos = (int)t3;
    }
    __syncthreads();
    // ---- bitonic sort, descending
    for (int k = 2; k <= dpad; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int e = tid; e < dpad / 2; e += 256) {
                const int lo = ((e & ~(j - 1)) << 1) | (e & (j - 1));
                const int hi = lo | j;
                const bool down = (lo & k) == 0;
                const float xl = sa[lo], xh = sa[hi];
                if ((xl < xh) == down) {
                    sa[lo] = xh;
                    sa[hi] = xl;
                }
            }
            __syncthreads();
        }
    }
    const int npos = s_npos;  // the zeros sit behind the npos positive magnitudes
    // ---- prefix sums (thread t owns dpad/256 consecutive entries) and the quotient lists
    {
        const int PER = dpad / 256, e0 = tid * PER;
        double loc = 0.0;
        for (int e = e0; e < e0 + PER; e++) loc += (double)sa[e];
        double run = block_scan_incl(loc, ws, tid) - loc;
        if (tid == 0) pref[0] = 0.0;
        for (int e = e0; e < e0 + PER; e++) {
            run += (double)sa[e];
            pref[e + 1] = run;
        }
    }
    for (int e = tid; e < nl * npos; e += 256) {
        const int j = e / npos + 1, p = e - (j - 1) * npos;
        Q[(size_t)(j - 1) * a.d + p] = (double)j / (double)sa[p];
    }
    __syncthreads();
    // ---- every breakpoint evaluates the cosine at the end of its group of equal t
    const double ip0 = 0.5 * s_l1, nn0 = 0.25 * (double)a.d;
    double best = -1.0, best_t = __builtin_inf();
    for (int e = tid; e < nl * npos; e += 256) {
        const int j = e / npos, p = e - j * npos;
        const double t = Q[(size_t)j * a.d + p];
        double ip = ip0, nn = nn0;
        for (int jj = 0; jj < nl; jj++) {
            const double* q = Q + (size_t)jj * a.d;
            int lo = 0, hi = npos;  // number of level-(jj+1) breakpoints <= t
            while (lo < hi) {
                const int mid = (lo + hi) >> 1;
                if (q[mid] <= t)
                    lo = mid + 1;
                else
                    hi = mid;
            }
            ip += pref[lo];
            nn += 2.0 * (double)(jj + 1) * (double)lo;
        }
        const double c = ip / sqrt(nn);
        if (c > best || (c == best && t < best_t)) {
            best = c;
            best_t = t;
        }
    }
    red_c[tid] = best;
    red_t[tid] = best_t;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) {
            const double oc = red_c[tid + s], ot = red_t[tid + s];
            if (oc > red_c[tid] || (oc == red_c[tid] && ot < red_t[tid])) {
                red_c[tid] = oc;
                red_t[tid] = ot;
            }
        }
        __syncthreads();
    }
    if (tid == 0) {
        // the all-zero-level grid (t -> 0+) competes too; a later cosine must be strictly larger
        const double c0 = ip0 / sqrt(nn0);
        s_best_t = (npos > 0 && nl > 0 && red_c[0] > c0) ? red_t[0] : 0.0;
    }
    __syncthreads();
    const double bt = s_best_t;
    // ---- codes: 32 / bits consecutive coordinates per thread -> one dword
    const double cb = ((double)(1 << a.bits) - 1.0) * 0.5;
    const int per = 32 / a.bits;
    double ip = 0.0;
    for (int i0 = tid * per; i0 < a.d; i0 += 256 * per) {
        uint32_t w = 0;
        for (int j = 0; j < per; j++) {
            const float x = r[i0 + j];
            const double ax = fabs((double)x);
            int lv = 0;
            if (ax > 0.0)
                while (lv + 1 < half && (double)(lv + 1) / ax <= bt) lv++;
            const int u = x >= 0.0f ? half + lv : half - 1 - lv;
            w |= (uint32_t)u << (a.bits * j);
            ip += ((double)u - cb) * (double)x;
        }
        *reinterpret_cast<uint32_t*>(code + (size_t)i0 * a.bits / 8) = w;
    }
    const double tip = block_scan_incl(ip, ws, tid);
    if (tid == 255) s_ip = tip;
    __syncthreads();
    for (int b = a.code_bytes + tid * 4; b < a.pad_to; b += 1024) *reinterpret_cast<uint32_t*>(code + b) = 0u;
    if (tid == 0) {
        float* m = reinterpret_cast<float*>(a.meta + (size_t)v * a.meta_stride);
        m[0] = s_l2 > 0.0 ? (float)s_l2 : 0.f;
        m[1] = s_l2 > 0.0 ? (float)(-2.0 * s_l2 / s_ip) : 0.f;
        for (int b = 0; b < a.meta_pad; b += 4) m[2 + b / 4] = 0.f;
    }
}

hipError_t launch_encode(const EncodeArgs& a, hipStream_t st) {
    if (a.n <= 0) return hipSuccess;
    if (a.bits > 1 && a.rule == JX_RULE_MAXCOS) {
        const int nl = (1 << (a.bits - 1)) - 1;
        if ((a.bits != 4 && a.bits != 2) || a.d * nl > MC_CAP || a.d > MC_DMAX) return hipErrorInvalidValue;
        int dpad = 256;
        while (dpad < a.d) dpad <<= 1;
        const size_t sh = (size_t)dpad * 4 + (size_t)(dpad + 2) * 8 + (size_t)nl * a.d * 8;
        hipError_t e = hipFuncSetAttribute((const void*)encode_maxcos_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sh);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(encode_maxcos_kernel, dim3((unsigned)a.n), dim3(256), sh, st, a);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(encode_kernel, dim3((unsigned)((a.n + 3) / 4)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// 2-bit and 8-bit codes are searched as two planes of the 1-bit / 4-bit provider: u = lo + 2^f hi with f = 1 / 4.
// Natural packing (field i % per of dword i / per) <-> planes ([lo plane][hi plane], each plane_bytes long, a plane
// packed as 1-bit / 4-bit codes are).  Two natural dwords make one dword of each plane.
__device__ __forceinline__ uint32_t even_bits(uint32_t x) {  // bits 0,2,4,.. -> bits 0..15
    x &= 0x55555555u;
    x = (x | (x >> 1)) & 0x33333333u;
    x = (x | (x >> 2)) & 0x0F0F0F0Fu;
    x = (x | (x >> 4)) & 0x00FF00FFu;
    x = (x | (x >> 8)) & 0x0000FFFFu;
    return x;
}
__device__ __forceinline__ uint32_t spread_bits(uint32_t x) {  // bits 0..15 -> bits 0,2,4,..
    x &= 0x0000FFFFu;
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    x = (x | (x << 2)) & 0x33333333u;
    x = (x | (x << 1)) & 0x55555555u;
    return x;
}
__device__ __forceinline__ uint32_t low_nibbles(uint32_t x) {  // low nibble of each byte -> bits 0..15
    x &= 0x0F0F0F0Fu;
    x = (x | (x >> 4)) & 0x00FF00FFu;
    x = (x | (x >> 8)) & 0x0000FFFFu;
    return x;
}
__device__ __forceinline__ uint32_t spread_nibbles(uint32_t x) {  // nibbles 0..3 -> low nibble of bytes 0..3
    x &= 0x0000FFFFu;
    x = (x | (x << 8)) & 0x00FF00FFu;
    x = (x | (x << 4)) & 0x0F0F0F0Fu;
    return x;
}
__device__ __forceinline__ void split_pair(int bits, uint32_t n0, uint32_t n1, uint32_t* lo, uint32_t* hi) {
    if (bits == 2) {
        *lo = even_bits(n0) | (even_bits(n1) << 16);
        *hi = even_bits(n0 >> 1) | (even_bits(n1 >> 1) << 16);
    } else {
        *lo = low_nibbles(n0) | (low_nibbles(n1) << 16);
        *hi = low_nibbles(n0 >> 4) | (low_nibbles(n1 >> 4) << 16);
    }
}
__device__ __forceinline__ void join_pair(int bits, uint32_t lo, uint32_t hi, uint32_t* n0, uint32_t* n1) {
    if (bits == 2) {
        *n0 = spread_bits(lo) | (spread_bits(hi) << 1);
        *n1 = spread_bits(lo >> 16) | (spread_bits(hi >> 16) << 1);
    } else {
        *n0 = spread_nibbles(lo) | (spread_nibbles(hi) << 4);
        *n1 = spread_nibbles(lo >> 16) | (spread_nibbles(hi >> 16) << 4);
    }
}

// in place: natural codes at the start of each record -> two planes; one wavefront per record, staged in LDS
__global__ void __launch_bounds__(256) planarize_kernel(uint8_t* recs, long long n, int code_stride, int code_bytes, int plane_bytes,
                                                       int bits) {
    extern __shared__ __align__(16) uint32_t stage[];  // 4 x code_bytes / 4
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const int lane = lane_id();
    uint32_t* mine = stage + (size_t)(threadIdx.x >> 6) * (code_bytes / 4);
    uint32_t* rec = reinterpret_cast<uint32_t*>(recs + (size_t)v * code_stride);
    const int nd = code_bytes / 4;  // natural dwords (even: dim % 32 == 0)
    for (int k = lane; k < nd; k += 64) mine[k] = rec[k];
    wave_sync();
    for (int k = lane; k < plane_bytes / 4; k += 64) {  // dword k of each plane, zero beyond the codes
        uint32_t lo = 0, hi = 0;
        if (2 * k + 1 < nd) split_pair(bits, mine[2 * k], mine[2 * k + 1], &lo, &hi);
        rec[k] = lo;
        rec[plane_bytes / 4 + k] = hi;
    }
}

hipError_t launch_planarize(uint8_t* recs, long long n, int code_stride, int code_bytes, int plane_bytes, int bits, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(planarize_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), (size_t)4 * code_bytes, st, recs, n, code_stride,
                       code_bytes, plane_bytes, bits);
    return hipGetLastError();
}

// records -> unpadded codes + meta
__global__ void __launch_bounds__(256) unpack_records_kernel(const uint8_t* recs, long long n, int code_stride, int code_bytes,
                                                            int meta_off, uint8_t* codes, float* meta, int planar_bits,
                                                            int plane_bytes) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const int lane = lane_id();
    const uint8_t* rec = recs + (size_t)v * code_stride;
    if (planar_bits) {  // two planes -> natural packing
        const uint32_t* pl = reinterpret_cast<const uint32_t*>(rec);
        uint32_t* out = reinterpret_cast<uint32_t*>(codes + (size_t)v * code_bytes);
        for (int k = lane; 2 * k + 1 < code_bytes / 4; k += 64) {
            uint32_t n0, n1;
            join_pair(planar_bits, pl[k], pl[plane_bytes / 4 + k], &n0, &n1);
            out[2 * k] = n0;
            out[2 * k + 1] = n1;
        }
    } else
    for (int b = lane * 4; b < code_bytes; b += 256)
        *reinterpret_cast<uint32_t*>(codes + (size_t)v * code_bytes + b) = *reinterpret_cast<const uint32_t*>(rec + b);
    if (lane < 2) meta[2 * v + lane] = reinterpret_cast<const float*>(rec + meta_off)[lane];
}

hipError_t launch_unpack_records(const uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off,
                                 uint8_t* codes, float* meta, int planar_bits, int plane_bytes, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(unpack_records_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, recs, n, code_stride, code_bytes,
                       meta_off, codes, meta, planar_bits, plane_bytes);
    return hipGetLastError();
}

// unpadded codes + meta -> records (padding zeroed)
__global__ void __launch_bounds__(256) pack_records_kernel(uint8_t* recs, long long n, int code_stride, int code_bytes,
                                                          int meta_off, const uint8_t* codes, const float* meta) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const int lane = lane_id();
    uint8_t* rec = recs + (size_t)v * code_stride;
    for (int b = lane * 4; b < code_stride; b += 256) {
        uint32_t w = 0;
        if (b < code_bytes) w = *reinterpret_cast<const uint32_t*>(codes + (size_t)v * code_bytes + b);
        else if (b == meta_off) w = __float_as_uint(meta[2 * v]);
        else if (b == meta_off + 4) w = __float_as_uint(meta[2 * v + 1]);
        *reinterpret_cast<uint32_t*>(rec + b) = w;
    }
}

hipError_t launch_pack_records(uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off,
                               const uint8_t* codes, const float* meta, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(pack_records_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, recs, n, code_stride, code_bytes,
                       meta_off, codes, meta);
    return hipGetLastError();
}

// Sum of the code units of every record (codes in their natural packing: fields of `bits` bits), stored as a
// uint32 behind the two floats of the meta chunk: the estimator's sum(u) term then costs the search kernel nothing.
__global__ void __launch_bounds__(256) code_sums_kernel(uint8_t* recs, long long n, int code_stride, int code_bytes,
                                                       int meta_off, int bits) {
    const long long v = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (v >= n) return;
    const int lane = lane_id();
    uint8_t* rec = recs + (size_t)v * code_stride;
    uint32_t s = 0;
    for (int b = lane * 4; b < code_bytes; b += 256) {
        const uint32_t w = *reinterpret_cast<const uint32_t*>(rec + b);
        if (bits == 1)
            s += (uint32_t)__builtin_popcount(w);
        else if (bits == 2)
            s += (uint32_t)__builtin_popcount(w & 0x55555555u) + 2u * (uint32_t)__builtin_popcount(w & 0xAAAAAAAAu);
        else if (bits == 4)
            s += __builtin_amdgcn_udot8(w, 0x11111111u, 0u, false);
        else
            s += __builtin_amdgcn_udot4(w, 0x01010101u, 0u, false);
    }
#pragma unroll
    for (int m = 1; m < 64; m <<= 1) s += shfl_xor(s, m);
    if (lane == 0) *reinterpret_cast<uint32_t*>(rec + meta_off + 8) = s;
}

hipError_t launch_code_sums(uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off, int bits, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(code_sums_kernel, dim3((unsigned)((n + 3) / 4)), dim3(256), 0, st, recs, n, code_stride, code_bytes,
                       meta_off, bits);
    return hipGetLastError();
}

// ------------------------------------------------------------------ query records

__global__ void __launch_bounds__(256) query_prep_kernel(QueryPrepArgs a) {
    const long long qi = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (qi >= a.nq) return;
    const int lane = lane_id();
    const float* q = a.rot + (size_t)qi * a.d;
    uint8_t* rec = a.qrecs + (size_t)qi * a.qrec_stride;
    float lo = __builtin_inff(), hi = -__builtin_inff();
    double s = 0.0, s2 = 0.0;
    for (int i = lane; i < a.d; i += 64) {
        const float x = q[i];
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
        s += (double)x;
        s2 += (double)x * (double)x;
    }
    lo = wave_min_f32(lo);
    hi = wave_max_f32(hi);
    s = wave_sum_f64(s);
    s2 = wave_sum_f64(s2);
    const float levels = (float)((1 << a.qbits) - 1);
    const float delta = __fdiv_rn(__fsub_rn(hi, lo), levels);
    const double cb = ((double)(1 << a.bits) - 1.0) * 0.5;
    if (lane == 0) {
        float* hdr = reinterpret_cast<float*>(rec);
        hdr[0] = lo;
        hdr[1] = delta;
        hdr[2] = (float)s2;
        hdr[3] = (float)(cb * s);
    }
    const bool nib = a.bits >= 4;  // 4- and 8-bit codes: nibble planes; 1- and 2-bit codes: bit planes
    const int nplanes = nib ? 2 : a.qbits;
    // zero the padding of each plane (planes are whole 16-byte chunks)
    const int written = nib ? a.d / 2 : a.d / 8;
    for (int p = 0; p < nplanes; p++)
        for (int b = written + lane * 4; b < a.plane_stride; b += 256)
            *reinterpret_cast<uint32_t*>(rec + 16 + (size_t)p * a.plane_stride + b) = 0u;
    auto quant = [&](float x) -> uint32_t {
        if (!(delta > 0.f)) return 0u;
        float t = __fdiv_rn(__fsub_rn(x, lo), delta);
        t = floorf(__fadd_rn(t, 0.5f));
        t = t < 0.f ? 0.f : (t > levels ? levels : t);
        return (uint32_t)t;
    };
    if (nib) {
        // nibble planes: dword k holds coordinates 8k..8k+7; plane 0 = high nibbles, plane 1 = low nibbles
        for (int c0 = 0; c0 < a.d; c0 += 512) {
            const int i0 = c0 + lane * 8;
            if (i0 < a.d) {
                uint32_t wh = 0, wl = 0;
#pragma unroll
                for (int j = 0; j < 8; j++) {
                    const uint32_t v = quant(q[i0 + j]);
                    wh |= (v >> 4) << (4 * j);
                    wl |= (v & 15u) << (4 * j);
                }
                *reinterpret_cast<uint32_t*>(rec + 16 + i0 / 2) = wh;
                *reinterpret_cast<uint32_t*>(rec + 16 + a.plane_stride + i0 / 2) = wl;
            }
        }
    } else {
        // bit planes: plane b, dword k, bit j = bit b of q_int[32k + j]
        for (int c0 = 0; c0 < a.d; c0 += 64) {
            const int i = c0 + lane;
            const uint32_t v = i < a.d ? quant(q[i]) : 0u;
            for (int b = 0; b < a.qbits; b++) {
                const uint64_t m = ballot(((v >> b) & 1u) != 0u);
                if (lane == 0) *reinterpret_cast<uint32_t*>(rec + 16 + (size_t)b * a.plane_stride + c0 / 8) = (uint32_t)m;
                if (lane == 1 && c0 + 32 < a.d)
                    *reinterpret_cast<uint32_t*>(rec + 16 + (size_t)b * a.plane_stride + c0 / 8 + 4) = (uint32_t)(m >> 32);
            }
        }
    }
}

hipError_t launch_query_prep(const QueryPrepArgs& a, hipStream_t st) {
    if (a.nq <= 0) return hipSuccess;
    hipLaunchKernelGGL(query_prep_kernel, dim3((unsigned)((a.nq + 3) / 4)), dim3(256), 0, st, a);
    return hipGetLastError();
}

// ------------------------------------------------------------------ exact re-rank

struct RerankLds {
    uint64_t key[JX_MAX_L];
    uint64_t cand_key[64];
    uint32_t cand_id[64];
};

template <int KIND, int T, int CPL>
__global__ void __launch_bounds__(256) rerank_kernel(RerankArgs a) {
    __shared__ RerankLds lds[4];
    constexpr int G = 64 / T;
    constexpr int U0 = (8 / CPL) > 0 ? (8 / CPL) : 1;
    constexpr int U = U0 < (64 / G) ? U0 : (64 / G);
    const int wave = threadIdx.x >> 6, lane = lane_id();
    const int g = lane / T, lig = lane % T;
    const long long qi = (long long)blockIdx.x * 4 + wave;
    if (qi >= a.nq) return;
    RerankLds* L = &lds[wave];
    QueryRegs<KIND, CPL, 0> q;
    load_query<KIND, T, CPL, 0>(q, a.ds, qi, lig);
    const uint32_t* cand = a.cand + (size_t)qi * a.cand_stride;
    int m = 0;
    for (int c0 = 0; c0 < a.rr; c0 += 64) {
        const int j = c0 + lane;
        const uint32_t id = j < a.rr ? cand[j] : JX_NONE_ID;
        const uint64_t vm = ballot(id != JX_NONE_ID);
        const int nn = __builtin_popcountll(vm);
        if (nn == 0) break;  // the frontier is filled from the left
        if (id != JX_NONE_ID) L->cand_id[prefix_count(vm)] = id;
        wave_sync();
        for (int s0 = 0; s0 < nn; s0 += G * U) eval_batch<KIND, T, CPL, 0, U>(q, a.ds, s0, nn, L->cand_id, L->cand_key, g, lig);
        wave_sync();
        if (lane < nn) L->key[m + lane] = L->cand_key[lane] | 1ull;
        m += nn;
        wave_sync();
    }
    // rank sort by (distance, id); write the first k, pad what is left
    for (int j = m + lane; j < a.k; j += 64) {
        a.out_ids[qi * a.k + j] = JX_NONE_ID;
        a.out_dist[qi * a.k + j] = __builtin_inff();
    }
    for (int j = lane; j < m; j += 64) {
        const uint64_t kj = L->key[j];
        int rank = 0;
        for (int t = 0; t < m; t++) rank += (L->key[t] < kj) ? 1 : 0;
        if (rank < a.k) {
            a.out_ids[qi * a.k + rank] = key_id(kj);
            const uint32_t dc = key_dist(kj);
            a.out_dist[qi * a.k + rank] = (KIND == K_U8) ? (float)dc : ordered_to_f32(dc);
        }
    }
    if (a.stats && lane == 0) atomicAdd(&a.stats[(size_t)(qi & 63) * 16 + 2], (unsigned long long)m);
}

template <int KIND>
static hipError_t launch_rerank_shape(const RerankArgs& a, hipStream_t st) {
    dim3 grid((unsigned)((a.nq + 3) / 4)), block(256);
    const int nch = a.ds.nch;
#define JX_RR(T, C)                                                             \
    {                                                                           \
        hipLaunchKernelGGL((rerank_kernel<KIND, T, C>), grid, block, 0, st, a); \
        return hipGetLastError();                                               \
    }
    if (nch <= 8) JX_RR(4, 2)
    if (nch <= 16) JX_RR(8, 2)
    if (nch <= 32) JX_RR(16, 2)
    if (nch <= 64) JX_RR(32, 2)
    if (nch <= 128) JX_RR(64, 2)
    if (nch <= 256) JX_RR(64, 4)
    if (nch <= 384) JX_RR(64, 6)
#undef JX_RR
    return hipErrorInvalidValue;
}

hipError_t launch_rerank(int dtype, const RerankArgs& a, hipStream_t st) {
    if (a.nq <= 0) return hipSuccess;
    if (dtype == JX_U8) return launch_rerank_shape<K_U8>(a, st);
    if (dtype == JX_F16) return launch_rerank_shape<K_F16>(a, st);
    return launch_rerank_shape<K_F32>(a, st);
}

}  // namespace jx
