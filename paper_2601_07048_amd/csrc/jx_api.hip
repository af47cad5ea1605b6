// C ABI of libjx (see include/jx.h): argument checks, arena layout, phase
// orchestration.  Every step of the path runs in the HIP kernels; nothing here
// computes on the host except the tiny amount of control that needs a count.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <new>
#include "jx_internal.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

#define JX_HIP(expr)                                                                         \
    do {                                                                                     \
        hipError_t e__ = (expr);                                                             \
        if (e__ != hipSuccess) return fail(JX_EHIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

inline int64_t align256(int64_t x) { return (x + 255) & ~(int64_t)255; }

struct Layout {
    int64_t vecs, adj, codes, P, centroid, stats, work, work_bytes, total;
    int vec_bytes, code_bytes, meta_chunk, code_stride;
};

int check_params(const jx_params* p) {
    if (!p) return fail(JX_EINVAL, "params is NULL");
    if (p->dtype != JX_U8 && p->dtype != JX_F32) return fail(JX_EINVAL, "dtype must be JX_U8 or JX_F32");
    if (p->dim <= 0) return fail(JX_EINVAL, "dim must be positive");
    if (p->dtype == JX_U8 && p->dim % 16) return fail(JX_EINVAL, "uint8 dim must be a multiple of 16");
    if (p->dtype == JX_F32 && p->dim % 4) return fail(JX_EINVAL, "float32 dim must be a multiple of 4");
    int vb = p->dim * (p->dtype == JX_U8 ? 1 : 4);
    if (vb > 384 * 16) return fail(JX_EINVAL, "vectors larger than 6144 bytes are not supported");
    if (p->R < 1 || p->R > JX_MAX_R) return fail(JX_EINVAL, "R out of range");
    if (p->L_build < 1 || p->L_build > JX_MAX_L) return fail(JX_EINVAL, "L_build out of range");
    if (!(p->alpha >= 1.0f)) return fail(JX_EINVAL, "alpha must be >= 1");
    if (p->cand_mode != JX_CAND_FRONTIER) return fail(JX_EINVAL, "only JX_CAND_FRONTIER is supported");
    if (p->capacity < 1 || p->capacity > 0x7FFFFFFELL) return fail(JX_EINVAL, "capacity out of range");
    if (p->max_batch < 1) return fail(JX_EINVAL, "max_batch must be positive");
    if (p->quant_bits != 0 && p->quant_bits != 1 && p->quant_bits != 4)
        return fail(JX_EINVAL, "quant_bits must be 0, 1 or 4");
    if (p->quant_bits && p->dtype != JX_F32) return fail(JX_EINVAL, "RaBitQ needs float32 data");
    if (p->quant_bits && p->dim % 32) return fail(JX_EINVAL, "RaBitQ needs dim to be a multiple of 32");
    if (!(p->batch_growth >= 0.0f) || p->batch_growth > 1.0f) return fail(JX_EINVAL, "batch_growth must be in [0, 1]");
    return JX_OK;
}

// Workspace of the insert phase for internal batches of at most B points.
struct InsertWork {
    int64_t cand_ids, cand_dist, keys0, keys1, vals0, vals1, heads, dead, table, counters, partial, mean, dist, total;
};

int64_t insert_work(const jx_params* p, int64_t B, InsertWork* w) {
    int64_t off = 0;
    const int64_t E = B * p->R;
    auto take = [&](int64_t bytes) { int64_t o = off; off += align256(bytes); return o; };
    w->cand_ids = take(B * p->L_build * 4);
    w->cand_dist = take(B * p->L_build * 4);
    w->keys0 = take(E * 8);
    w->keys1 = take(E * 8);
    w->vals0 = take(E * 4);
    w->vals1 = take(E * 4);
    w->heads = take(E * 4);
    w->dead = take(B * (p->R > p->L_build ? p->R : p->L_build));
    w->table = take(16 * (E / 4096 + 2) * 4);
    w->counters = take(256);
    w->partial = take((int64_t)512 * p->dim * 8);
    w->mean = take((int64_t)p->dim * 4);
    w->dist = take(p->capacity * 8);
    w->total = off;
    return off;
}

void layout(const jx_params* p, Layout* L) {
    L->vec_bytes = p->dim * (p->dtype == JX_U8 ? 1 : 4);
    L->code_bytes = p->quant_bits ? p->dim * p->quant_bits / 8 : 0;
    L->meta_chunk = (L->code_bytes + 15) / 16;
    L->code_stride = p->quant_bits ? (L->meta_chunk + 1) * 16 : 0;
    int64_t off = 0;
    L->vecs = off;
    off += align256((int64_t)p->capacity * L->vec_bytes);
    L->adj = off;
    off += align256((int64_t)p->capacity * p->R * 4);
    L->codes = off;
    off += align256((int64_t)p->capacity * L->code_stride);
    L->P = off;
    off += align256(p->quant_bits ? (int64_t)p->dim * p->dim * 4 : 0);
    L->centroid = off;
    off += align256((int64_t)p->dim * 4);
    L->stats = off;
    off += 256;
    // workspace: the larger of the insert phase and the query phase, at least 64 MiB
    const int64_t B = p->max_batch;
    InsertWork iw;
    int64_t ins = insert_work(p, B, &iw);
    int64_t qry = align256(B * p->dim * 4)                              // rotated queries
                  + align256(B * ((int64_t)p->dim + 64) * 2)            // integer query records
                  + align256(B * JX_MAX_L * 4) * 2;                     // frontier ids / distances for re-rank
    int64_t w = ins > qry ? ins : qry;
    if (w < (64 << 20)) w = 64 << 20;
    L->work = off;
    L->work_bytes = w;
    off += align256(w);
    L->total = off;
}

}  // namespace
namespace {
int64_t batch_cap(const jx_params& p, int64_t linked) {
    const float gr = p.batch_growth > 0.0f ? p.batch_growth : 0.25f;
    int64_t c = (int64_t)floor((double)gr * (double)linked);
    return c < 1 ? 1 : c;
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

int hash_log2_for(int L) {
    int h = 9;
    while ((1 << h) < 4 * L && h < 12) h++;
    return h;
}

}  // namespace

#pragma GCC visibility push(default)
extern "C" {

const char* jx_strerror(int code) {
    switch (code) {
        case JX_OK: return "ok";
        case JX_EINVAL: return "invalid argument";
        case JX_ECAPACITY: return "capacity exceeded";
        case JX_ESTATE: return "index is not in a state that allows this call";
        case JX_EHIP: return "HIP runtime error";
    }
    return "unknown error";
}

const char* jx_last_error(void) { return g_err; }

int64_t jx_arena_bytes(const jx_params* p) {
    int rc = check_params(p);
    if (rc) return rc;
    Layout L;
    layout(p, &L);
    return L.total;
}

int jx_create(const jx_params* p, void* d_arena, int64_t arena_bytes, void* stream, jx_index** out) {
    int rc = check_params(p);
    if (rc) return rc;
    if (!d_arena || !out) return fail(JX_EINVAL, "arena or out is NULL");
    if (((uintptr_t)d_arena) & 255) return fail(JX_EINVAL, "arena must be 256-byte aligned");
    Layout L;
    layout(p, &L);
    if (arena_bytes < L.total) return fail(JX_ECAPACITY, "arena holds %lld bytes, %lld needed", (long long)arena_bytes, (long long)L.total);
    jx_index* x = new (std::nothrow) jx_index();
    if (!x) return fail(JX_EINVAL, "out of host memory");
    memset(x, 0, sizeof *x);
    x->p = *p;
    x->n = 0;
    x->entry = JX_NONE;
    x->vec_bytes = L.vec_bytes;
    x->d_arena = (uint8_t*)d_arena;
    x->arena_bytes = arena_bytes;
    x->d_vecs = x->d_arena + L.vecs;
    x->d_adj = (uint32_t*)(x->d_arena + L.adj);
    x->d_codes = x->d_arena + L.codes;
    x->d_P = (float*)(x->d_arena + L.P);
    x->d_centroid = (float*)(x->d_arena + L.centroid);
    x->d_stats = (unsigned long long*)(x->d_arena + L.stats);
    x->d_work = x->d_arena + L.work;
    x->work_bytes = L.work_bytes;
    x->code_bytes = L.code_bytes;
    x->meta_chunk = L.meta_chunk;
    x->code_stride = L.code_stride;
    hipError_t e = jx::launch_fill_u32(x->d_adj, (long long)p->capacity * p->R, JX_NONE, as_stream(stream));
    if (e != hipSuccess) {
        delete x;
        return fail(JX_EHIP, "fill adjacency: %s", hipGetErrorString(e));
    }
    *out = x;
    return JX_OK;
}

int jx_destroy(jx_index* idx) {
    delete idx;
    return JX_OK;
}

int jx_size(const jx_index* idx, int64_t* n, uint32_t* entry_id) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (n) *n = idx->n;
    if (entry_id) *entry_id = idx->entry;
    return JX_OK;
}

int jx_import_graph(jx_index* idx, const void* d_vecs, int64_t n, const uint32_t* d_adj, uint32_t entry_id, void* stream) {
    if (!idx || !d_vecs || !d_adj) return fail(JX_EINVAL, "NULL argument");
    if (n < 1 || n > idx->p.capacity) return fail(JX_ECAPACITY, "n = %lld exceeds capacity", (long long)n);
    if (entry_id >= (uint64_t)n) return fail(JX_EINVAL, "entry id out of range");
    hipStream_t st = as_stream(stream);
    JX_HIP(hipMemcpyAsync(idx->d_vecs, d_vecs, (size_t)n * idx->vec_bytes, hipMemcpyDeviceToDevice, st));
    JX_HIP(hipMemcpyAsync(idx->d_adj, d_adj, (size_t)n * idx->p.R * 4, hipMemcpyDeviceToDevice, st));
    if (n < idx->n) JX_HIP(jx::launch_fill_u32(idx->d_adj + (size_t)n * idx->p.R, (idx->n - n) * idx->p.R, JX_NONE, st));
    idx->n = n;
    idx->entry = entry_id;
    idx->quantized = 0;
    return JX_OK;
}

int jx_export_graph(jx_index* idx, uint32_t* d_adj, uint32_t* d_deg, void* stream) {
    if (!idx || !d_adj) return fail(JX_EINVAL, "NULL argument");
    hipStream_t st = as_stream(stream);
    if (idx->n == 0) return JX_OK;
    JX_HIP(hipMemcpyAsync(d_adj, idx->d_adj, (size_t)idx->n * idx->p.R * 4, hipMemcpyDeviceToDevice, st));
    if (d_deg) JX_HIP(jx::launch_row_degrees(idx->d_adj, idx->n, idx->p.R, d_deg, st));
    return JX_OK;
}

static int search_common(jx_index* idx, const void* d_queries, int64_t nq, int32_t out_k, int32_t L, int32_t mode,
                         uint32_t* d_out_ids, float* d_out_dist, jx_stats* h_stats, hipStream_t st) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (nq < 0) return fail(JX_EINVAL, "nq < 0");
    if (nq > 0 && (!d_queries || !d_out_ids || !d_out_dist)) return fail(JX_EINVAL, "NULL argument");
    if (L < 1 || L > JX_MAX_L) return fail(JX_EINVAL, "L must be in [1, %d]", JX_MAX_L);
    if (out_k < 1 || out_k > L) return fail(JX_EINVAL, "k must be in [1, L]");
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    if (mode != JX_EXACT && mode != JX_RABITQ) return fail(JX_EINVAL, "unknown mode");
    if (mode == JX_RABITQ) return fail(JX_ESTATE, "index is not quantised");
    if (nq == 0) return JX_OK;
    if (h_stats) JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_stats, 16, 0u, st));
    jx::BeamArgs a;
    memset(&a, 0, sizeof a);
    a.adj = idx->d_adj;
    a.R = idx->p.R;
    a.ds.recs = idx->d_vecs;
    a.ds.rec_stride = idx->vec_bytes;
    a.ds.nch = idx->vec_bytes / 16;
    a.ds.meta_chunk = 0;
    a.ds.qrecs = (const uint8_t*)d_queries;
    a.ds.qrec_stride = idx->vec_bytes;
    a.nq = nq;
    a.q_skip = 0x7FFFFFFFFFFFFFFFLL;
    a.L = L;
    a.entry = idx->entry;
    a.hash_log2 = hash_log2_for(L);
    a.out_ids = d_out_ids;
    a.out_dist = d_out_dist;
    a.out_k = out_k;
    a.stats = h_stats ? idx->d_stats : nullptr;
    JX_HIP(jx::launch_beam_search(idx->p.dtype == JX_U8 ? 0 : 1, 0, a, st));
    if (h_stats) {
        unsigned long long hs[2];
        JX_HIP(hipMemcpyAsync(hs, idx->d_stats, sizeof hs, hipMemcpyDeviceToHost, st));
        JX_HIP(hipStreamSynchronize(st));
        memset(h_stats, 0, sizeof *h_stats);
        h_stats->hops = hs[0];
        h_stats->dist_evals = hs[1];
        h_stats->adj_bytes = hs[0] * 4ull * idx->p.R;
        h_stats->vec_bytes = hs[1] * (unsigned long long)idx->vec_bytes;
    }
    return JX_OK;
}

int jx_search(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, int32_t L, int32_t mode, int32_t rerank,
              uint32_t* d_out_ids, float* d_out_dist, jx_stats* h_stats, void* stream) {
    if (rerank != 0 && (rerank < k || rerank > L)) return fail(JX_EINVAL, "rerank must be 0 or in [k, L]");
    return search_common(idx, d_queries, nq, k, L, mode, d_out_ids, d_out_dist, h_stats, as_stream(stream));
}

int jx_beam_frontier(jx_index* idx, const void* d_queries, int64_t nq, int32_t L, int32_t mode, uint32_t* d_out_ids,
                     float* d_out_dist, jx_stats* h_stats, void* stream) {
    return search_common(idx, d_queries, nq, L, L, mode, d_out_ids, d_out_dist, h_stats, as_stream(stream));
}

int jx_bruteforce(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, uint32_t* d_out_ids, float* d_out_dist,
                  void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (nq > 0 && (!d_queries || !d_out_ids || !d_out_dist)) return fail(JX_EINVAL, "NULL argument");
    if (k < 1 || k > JX_MAX_BF_K) return fail(JX_EINVAL, "k must be in [1, %d]", JX_MAX_BF_K);
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    if (nq <= 0) return JX_OK;
    hipStream_t st = as_stream(stream);
    // split the base set so that the grid has at least ~2048 workgroups, and
    // slice the queries so that the per-slice partial lists fit the workspace
    int64_t tiles_b = (idx->n + 63) / 64;
    int64_t nqt = (nq + 63) / 64;
    int64_t nsplit = (2048 + nqt - 1) / nqt;
    if (nsplit > 64) nsplit = 64;
    if (nsplit > tiles_b) nsplit = tiles_b;
    if (nsplit < 1) nsplit = 1;
    int64_t per_q = nsplit * k * 8;
    int64_t slice = idx->work_bytes / per_q;
    slice = (slice / 64) * 64;
    if (slice < 64) return fail(JX_ECAPACITY, "workspace too small for brute force");
    for (int64_t q0 = 0; q0 < nq; q0 += slice) {
        int64_t m = nq - q0 < slice ? nq - q0 : slice;
        jx::BfArgs a;
        memset(&a, 0, sizeof a);
        a.base = idx->d_vecs;
        a.queries = (const uint8_t*)d_queries + (size_t)q0 * idx->vec_bytes;
        a.dtype = idx->p.dtype;
        a.d = idx->p.dim;
        a.n = idx->n;
        a.nq = m;
        a.k = k;
        a.nsplit = (int)nsplit;
        a.partial = (uint64_t*)idx->d_work;
        a.out_ids = d_out_ids + (size_t)q0 * k;
        a.out_dist = d_out_dist + (size_t)q0 * k;
        JX_HIP(jx::launch_bruteforce(a, st));
    }
    return JX_OK;
}

static int run_subbatch(jx_index* idx, const InsertWork& w, int64_t pos0, int64_t B, int64_t first, int64_t id_skip,
                        int64_t n_after, hipStream_t st) {
    uint8_t* W = idx->d_work;
    const jx_params& p = idx->p;
    jx::DistSrc ds;
    memset(&ds, 0, sizeof ds);
    ds.recs = idx->d_vecs;
    ds.rec_stride = idx->vec_bytes;
    ds.nch = idx->vec_bytes / 16;
    ds.qrecs = idx->d_vecs;
    ds.qrec_stride = idx->vec_bytes;
    const int64_t id_base = first + pos0;
    // 1. candidate generation: beamSearch from the entry point on the graph as it stands
    jx::BeamArgs b;
    memset(&b, 0, sizeof b);
    b.adj = idx->d_adj;
    b.R = p.R;
    b.ds = ds;
    b.ds.qrecs = idx->d_vecs + (size_t)id_base * idx->vec_bytes;
    b.nq = B;
    b.q_skip = id_skip >= id_base ? id_skip - id_base : 0;
    b.L = p.L_build;
    b.entry = idx->entry;
    b.hash_log2 = hash_log2_for(p.L_build);
    b.out_ids = (uint32_t*)(W + w.cand_ids);
    b.out_dist = (float*)(W + w.cand_dist);
    b.out_k = p.L_build;
    b.stats = nullptr;
    JX_HIP(jx::launch_beam_search(p.dtype == JX_U8 ? 0 : 1, 0, b, st));
    // 2. robustPrune of the frontier, new rows, reverse edges
    jx::InsertArgs a;
    memset(&a, 0, sizeof a);
    a.ds = ds;
    a.adj = idx->d_adj;
    a.R = p.R;
    a.L = p.L_build;
    a.alpha = p.alpha;
    a.B = B;
    a.id_base = id_base;
    a.id_skip = id_skip;
    a.cand_ids = (const uint32_t*)(W + w.cand_ids);
    a.cand_dist = (const uint32_t*)(W + w.cand_dist);
    a.dead = W + w.dead;
    a.keys = (uint64_t*)(W + w.keys0);
    a.vals = (uint32_t*)(W + w.vals0);
    a.heads = (const uint32_t*)(W + w.heads);
    a.nseg = (const uint32_t*)(W + w.counters);
    JX_HIP(jx::launch_forward_prune(p.dtype, a, st));
    // 3. one global sort by (target, distance, source)
    int tbits = 1;
    while (((int64_t)1 << tbits) <= n_after) tbits++;
    const int64_t E = B * p.R;
    JX_HIP(jx::launch_radix_sort((uint64_t*)(W + w.keys0), (uint32_t*)(W + w.vals0), (uint64_t*)(W + w.keys1),
                                 (uint32_t*)(W + w.vals1), E, 32 + tbits, (uint32_t*)(W + w.table), st));
    // 4. per target: append or robustPrune
    JX_HIP(jx::launch_fill_u32((uint32_t*)(W + w.counters), 16, 0u, st));
    JX_HIP(jx::launch_segment_heads((const uint64_t*)(W + w.keys0), E, (uint32_t*)(W + w.heads), (uint32_t*)(W + w.counters), st));
    JX_HIP(jx::launch_reverse_merge(p.dtype, a, st));
    return JX_OK;
}

int jx_insert(jx_index* idx, const void* d_vecs, int64_t n, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (n < 0) return fail(JX_EINVAL, "n < 0");
    if (n == 0) return JX_OK;
    if (!d_vecs) return fail(JX_EINVAL, "d_vecs is NULL");
    const jx_params& p = idx->p;
    const int64_t first = idx->n;
    if (first + n > p.capacity) return fail(JX_ECAPACITY, "%lld + %lld points exceed the capacity %lld", (long long)first, (long long)n, (long long)p.capacity);
    if (idx->quantized) return fail(JX_ESTATE, "insert into a quantised index is not available in this build");
    // the internal batch schedule: min(remaining, max(1, floor(batch_growth * linked)))
    {
        int64_t linked = first == 0 ? 1 : first, rem = first == 0 ? n - 1 : n, maxB = 0;
        while (rem > 0) {
            int64_t B = rem < batch_cap(p, linked) ? rem : batch_cap(p, linked);
            if (B > maxB) maxB = B;
            linked += B;
            rem -= B;
        }
        if (maxB > p.max_batch) return fail(JX_ECAPACITY, "an internal batch of %lld points exceeds max_batch = %lld", (long long)maxB, (long long)p.max_batch);
    }
    hipStream_t st = as_stream(stream);
    InsertWork w;
    insert_work(&p, p.max_batch, &w);
    if (w.total > idx->work_bytes) return fail(JX_ECAPACITY, "workspace too small");
    uint8_t* W = idx->d_work;
    JX_HIP(hipMemcpyAsync(idx->d_vecs + (size_t)first * idx->vec_bytes, d_vecs, (size_t)n * idx->vec_bytes, hipMemcpyDeviceToDevice, st));
    int64_t id_skip = 0x7FFFFFFFFFFFFFFFLL;
    int64_t m = n, linked = first;
    if (first == 0) {
        // entry point: the point nearest to the mean of this first call; it joins alone
        JX_HIP(jx::launch_entry_point(idx->d_vecs, p.dtype, n, p.dim, (double*)(W + w.partial), (float*)(W + w.mean),
                                      (double*)(W + w.dist), (uint32_t*)(W + w.counters) + 32, st));
        uint32_t e = 0;
        JX_HIP(hipMemcpyAsync(&e, (uint32_t*)(W + w.counters) + 32, 4, hipMemcpyDeviceToHost, st));
        JX_HIP(hipStreamSynchronize(st));
        if (e >= (uint64_t)n) return fail(JX_EHIP, "entry point selection returned %u", e);
        idx->entry = e;
        id_skip = e;
        m = n - 1;
        linked = 1;
    }
    int64_t pos = 0;
    while (pos < m) {
        int64_t B = m - pos < batch_cap(p, linked) ? m - pos : batch_cap(p, linked);
        int rc = run_subbatch(idx, w, pos, B, first, id_skip, first + n, st);
        if (rc) return rc;
        pos += B;
        linked += B;
    }
    idx->n = first + n;
    return JX_OK;
}

int jx_quantize(jx_index* idx, int32_t bits, const float* d_rotation, const float* d_centroid, int32_t query_bits,
                int32_t rule, void* stream) {
    (void)idx; (void)bits; (void)d_rotation; (void)d_centroid; (void)query_bits; (void)rule; (void)stream;
    return fail(JX_ESTATE, "jx_quantize: not available in this build");
}

int jx_export_codes(jx_index* idx, uint8_t* d_codes, float* d_meta, float* d_centroid, void* stream) {
    (void)idx; (void)d_codes; (void)d_meta; (void)d_centroid; (void)stream;
    return fail(JX_ESTATE, "index is not quantised");
}

int jx_rotate(jx_index* idx, const float* d_in, int64_t n, float* d_out, void* stream) {
    (void)idx; (void)d_in; (void)n; (void)d_out; (void)stream;
    return fail(JX_ESTATE, "index is not quantised");
}

int jx_encode_rotated(jx_index* idx, const float* d_rot, int64_t n, uint8_t* d_codes, float* d_meta, void* stream) {
    (void)idx; (void)d_rot; (void)n; (void)d_codes; (void)d_meta; (void)stream;
    return fail(JX_ESTATE, "index is not quantised");
}

}  // extern "C"
#pragma GCC visibility pop
