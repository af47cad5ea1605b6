// C ABI of libjx (see include/jx.h): argument checks, arena layout, phase
// orchestration.  Every step of the path runs in the HIP kernels; nothing here
// computes on the host except the tiny amount of control that needs a count.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <mutex>
#include <new>
#include <vector>
#include "jx_internal.h"

// Scratch of jx_bruteforce_static: one copy per GPU, held from the moment the code object is loaded until the
// process ends.  Host code never uses this name as an address (it is only the host-side handle of the symbol); the
// device address is looked up once per device with hipGetSymbolAddress, see static_scratch().
static __device__ __align__(256) unsigned char scratch[JX_STATIC_SCRATCH_BYTES];

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
    int64_t vecs, adj, codes, P, centroid, stats, stripes, deleted, clean, work, work_bytes, total;
    int vec_bytes, code_bytes, meta_chunk, code_stride, plane_chunks, plane_shift;
};

int elem_bytes(int dtype) { return dtype == JX_U8 ? 1 : (dtype == JX_F16 ? 2 : 4); }

// distance provider of the exact path for a storage type (0 uint8, 1 float32, 4 binary16)
int exact_kind(int dtype) { return dtype == JX_U8 ? 0 : (dtype == JX_F16 ? 4 : 1); }

int check_params(const jx_params* p) {
    if (!p) return fail(JX_EINVAL, "params is NULL");
    if (p->dtype != JX_U8 && p->dtype != JX_F32 && p->dtype != JX_F16)
        return fail(JX_EINVAL, "dtype must be JX_U8, JX_F32 or JX_F16");
    if (p->dim <= 0) return fail(JX_EINVAL, "dim must be positive");
    if (p->dtype == JX_U8 && p->dim % 16) return fail(JX_EINVAL, "uint8 dim must be a multiple of 16");
    if (p->dtype == JX_F32 && p->dim % 4) return fail(JX_EINVAL, "float32 dim must be a multiple of 4");
    if (p->dtype == JX_F16 && p->dim % 8) return fail(JX_EINVAL, "binary16 dim must be a multiple of 8");
    int vb = p->dim * elem_bytes(p->dtype);
    if (vb > 384 * 16) return fail(JX_EINVAL, "vectors larger than 6144 bytes are not supported");
    if (p->R < 1 || p->R > JX_MAX_R) return fail(JX_EINVAL, "R out of range");
    if (p->L_build < 1 || p->L_build > JX_MAX_L) return fail(JX_EINVAL, "L_build out of range");
    if (!(p->alpha >= 1.0f)) return fail(JX_EINVAL, "alpha must be >= 1");
    if (p->cand_mode != JX_CAND_FRONTIER && p->cand_mode != JX_CAND_VISITED) return fail(JX_EINVAL, "unknown cand_mode");
    if (p->cand_mode == JX_CAND_VISITED && !jx::visited_list_offered(exact_kind(p->dtype), vb / 16, p->L_build, p->R))
        return fail(JX_EINVAL, "JX_CAND_VISITED is offered for L_build <= 128 on uint8 vectors of at most 128 bytes and float32 vectors of at most 512 or of 2049..6144 bytes");
    if (p->capacity < 1 || p->capacity > 0x7FFFFFFELL) return fail(JX_EINVAL, "capacity out of range");
    if (p->max_batch < 1) return fail(JX_EINVAL, "max_batch must be positive");
    if ((int64_t)p->max_batch * p->R >= 0x7FFFFFFFLL) return fail(JX_EINVAL, "max_batch * R must stay below 2^31");
    if (p->quant_bits != 0 && p->quant_bits != 1 && p->quant_bits != 2 && p->quant_bits != 4 && p->quant_bits != 8)
        return fail(JX_EINVAL, "quant_bits must be 0, 1, 2, 4 or 8");
    if (p->quant_bits && p->dim % 32) return fail(JX_EINVAL, "RaBitQ needs dim to be a multiple of 32");
    if (!(p->batch_growth >= 0.0f) || p->batch_growth > 1.0f) return fail(JX_EINVAL, "batch_growth must be in [0, 1]");
    if (p->flags & ~JX_FLAG_ALL) return fail(JX_EINVAL, "unknown bits in flags");
    return JX_OK;
}

// Workspace of the insert phase for internal batches of at most B points.
struct InsertWork {
    int64_t cand_ids, cand_dist, keys0, keys1, vals0, vals1, heads, dead, table, counters, partial, mean, dist, total;
};

// candidates per new point that beamSearch hands to robustPrune: the frontier, or the expansion list
int cand_len(const jx_params* p) { return p->cand_mode == JX_CAND_VISITED ? jx::visited_cap(p->L_build) : p->L_build; }

int64_t insert_work(const jx_params* p, int64_t B, InsertWork* w) {
    int64_t off = 0;
    const int64_t E = B * p->R;
    const int64_t Lc = cand_len(p);
    auto take = [&](int64_t bytes) { int64_t o = off; off += align256(bytes); return o; };
    w->cand_ids = take(B * Lc * 4);
    w->cand_dist = take(B * Lc * 4);
    w->keys0 = take(E * 8);
    w->keys1 = take(E * 8);
    w->vals0 = take(E * 4);
    w->vals1 = take(E * 4);
    w->heads = take(E * 4);
    w->dead = take(B * (p->R > Lc ? p->R : Lc));
    w->table = take((256 * (E / 4096 + 2) + 256) * 4);  // radix sort: [digit][tile] counters and one total per digit
    w->counters = take(256);
    w->partial = take((int64_t)512 * p->dim * 8);
    w->mean = take((int64_t)p->dim * 4);
    w->dist = take(p->capacity * 8);  // entry-point distances (double), or consolidation counts + offsets
    w->total = off;
    return off;
}

// Workspace of the query phase (RaBitQ mode) for slices of at most B queries.
struct QueryWork {
    int64_t rot, qrecs, fr_ids, fr_dist, total;
    int plane_stride, qrec_stride_max;
};

int64_t query_work(const jx_params* p, int64_t B, int plane_chunks, QueryWork* w) {
    int64_t off = 0;
    auto take = [&](int64_t bytes) { int64_t o = off; off += align256(bytes); return o; };
    w->plane_stride = plane_chunks * 16;
    w->qrec_stride_max = 16 + (p->quant_bits >= 4 ? 2 : 8) * w->plane_stride;
    if (!p->quant_bits) {
        w->rot = w->qrecs = w->fr_ids = w->fr_dist = 0;
        w->total = 0;
        return 0;
    }
    w->rot = take(B * p->dim * 4);
    w->qrecs = take(B * (int64_t)w->qrec_stride_max);
    w->fr_ids = take(B * JX_MAX_L * 4);
    w->fr_dist = take(B * JX_MAX_L * 4);
    w->total = off;
    return off;
}

void layout(const jx_params* p, Layout* L) {
    L->vec_bytes = p->dim * elem_bytes(p->dtype);
    // 1- and 4-bit codes are one plane; 2- and 8-bit codes are stored as a low and a high plane of the 1-bit /
    // 4-bit kind (u = lo + 2 hi, u = lo + 16 hi), each padded to whole 16-byte chunks
    L->code_bytes = p->quant_bits ? p->dim * p->quant_bits / 8 : 0;
    const int fam = p->quant_bits <= 2 ? 1 : 4;
    const int ncp = (p->quant_bits == 2 || p->quant_bits == 8) ? 2 : 1;
    L->plane_chunks = p->quant_bits ? (p->dim * fam / 8 + 15) / 16 : 0;
    L->plane_shift = ncp == 2 ? fam : 0;
    L->meta_chunk = ncp * L->plane_chunks;
    // records start on 128-byte lines: a gather then touches ceil(record / 128) lines, the fewest any layout allows
    L->code_stride = p->quant_bits ? ((L->meta_chunk + 1) * 16 + 127) / 128 * 128 : 0;
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
    L->stripes = off;
    off += 64 * 16 * 8;
    L->deleted = off;
    off += align256((int64_t)p->capacity + 4);
    L->clean = off;
    off += align256((int64_t)p->capacity + 4);
    // workspace: the larger of the insert phase and the query phase, at least 64 MiB
    const int64_t B = p->max_batch;
    InsertWork iw;
    int64_t ins = insert_work(p, B, &iw);
    QueryWork qw;
    int64_t qry = query_work(p, B, L->plane_chunks, &qw);
    int64_t qnt = align256((int64_t)512 * p->dim * 8) + align256((int64_t)p->dim * 4 * 1024);  // centroid + >= 1024 rotated rows
    if (p->quant_bits && qnt > qry) qry = qnt;
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

// How robustPrune is computed: 0 = list-based kernels, 1 / 2 = Gram-matrix kernels for float32 / binary16 data (the
// default for float data), 3 = Gram-matrix kernels for uint8 data (JX_FLAG_GRAM_U8)
int gram_mode(const jx_index* idx) {
    if (idx->flags & JX_FLAG_NO_GRAM) return 0;
    if (idx->p.dtype == JX_U8) return (idx->flags & JX_FLAG_GRAM_U8) ? 3 : 0;
    return idx->p.dtype == JX_F16 ? 2 : 1;
}

// Rows of uint8 indices remember how many leading entries one robustPrune call selected together, which lets the
// next prune of the row skip the pairs among them
bool incremental_prune(const jx_index* idx) { return !(idx->flags & JX_FLAG_NO_INCR_PRUNE); }

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// split of the base set used by the brute-force kernels: at least ~2048 workgroups, at most 64 partial lists per query
int64_t bruteforce_nsplit(int64_t n, int64_t nq) {
    int64_t tiles_b = (n + 63) / 64;
    int64_t nqt = (nq + 63) / 64;
    int64_t nsplit = (2048 + nqt - 1) / nqt;
    if (nsplit > 64) nsplit = 64;
    if (nsplit > tiles_b) nsplit = tiles_b;
    if (nsplit < 1) nsplit = 1;
    return nsplit;
}

// Device address of `scratch` on the current device, resolved on first use per device and kept.
int static_scratch(unsigned char** out) {
    static std::mutex mu;
    static unsigned char* ptr[64] = {nullptr};
    int dev = -1;
    JX_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return fail(JX_EHIP, "device ordinal %d out of range", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!ptr[dev]) {
        void* p = nullptr;
        JX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(JX_EHIP, "hipGetSymbolAddress returned a null address");
        ptr[dev] = (unsigned char*)p;
    }
    *out = ptr[dev];
    return JX_OK;
}

// Visited table of beamSearch for beam width L on n vertices.  While ids fit slots x 2^15 the table holds 16-bit
// tags (see BeamArgs::tag_bits): twice the slots in the same LDS, 16 % fewer repeated distance evaluations at L = 96.
// 1,024 32-bit / 2,048 16-bit slots at least: measured optimum against the LDS footprint for L <= 256 and records of
// at most 256 bytes; twice / four times that for larger records (below).
// JX_FLAG_VISITED_IDS keeps full ids; JX_FLAG_VISITED_NONE (slots = 0) switches the filter off.
void visited_table_for(uint32_t flags, int L, int64_t n, int rec_bytes, int* slots, int* tag_bits) {
    *tag_bits = 0;
    if (flags & JX_FLAG_VISITED_NONE) {
        *slots = 0;
        return;
    }
    int id_bits = 1;
    while (((int64_t)1 << id_bits) < n) id_bits++;
    int h = 1024;
    while (h < 4 * L && h < 4096) h *= 2;
    // the table only ever forgets, so its size trades LDS (resident queries) against re-evaluated neighbours; a
    // re-evaluation costs a record's bytes, so larger records buy a larger table (measured at N = 1M, L = 128:
    // 496-byte code records -8 % evaluations / -5 % kernel time at 2x; 3,840- and 6,144-byte vectors -12..-17 %
    // evaluations / -11..-17 % at 4x; 8x loses to occupancy, and records of at most 256 bytes lose at 2x already)
    if (rec_bytes > 1024)
        h *= 4;
    else if (rec_bytes > 256)
        h *= 2;
    *slots = h;
    if (!(flags & JX_FLAG_VISITED_IDS)) {
        int h16 = 2 * h, lg = 0;
        while ((2 << lg) < h16) lg++;  // log2 of the number of sets (two entries each)
        int tb = id_bits - lg;
        if (tb < 1) tb = 1;
        if (tb <= 15) {
            *slots = h16;
            *tag_bits = tb;
        }
    }
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
    x->d_stripes = (unsigned long long*)(x->d_arena + L.stripes);
    x->d_deleted = x->d_arena + L.deleted;
    x->d_clean = x->d_arena + L.clean;
    x->d_work = x->d_arena + L.work;
    x->work_bytes = L.work_bytes;
    x->code_bytes = L.code_bytes;
    x->meta_chunk = L.meta_chunk;
    x->plane_chunks = L.plane_chunks;
    x->plane_shift = L.plane_shift;
    x->code_stride = L.code_stride;
    x->flags = p->flags;
    hipError_t e = jx::launch_fill_u32(x->d_adj, (long long)p->capacity * p->R, JX_NONE, as_stream(stream));
    if (e == hipSuccess) e = jx::launch_fill_u32((uint32_t*)x->d_stats, 64, 0u, as_stream(stream));
    if (e == hipSuccess) e = jx::launch_fill_u32((uint32_t*)x->d_deleted, (p->capacity + 3) / 4, 0u, as_stream(stream));
    if (e == hipSuccess) e = jx::launch_fill_u32((uint32_t*)x->d_clean, (p->capacity + 3) / 4, 0u, as_stream(stream));
    if (e != hipSuccess) {
        delete x;
        return fail(JX_EHIP, "arena initialisation: %s", hipGetErrorString(e));
    }
    *out = x;
    return JX_OK;
}

int jx_destroy(jx_index* idx) {
    delete idx;
    return JX_OK;
}

int jx_set_flags(jx_index* idx, uint32_t flags) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (flags & ~JX_FLAG_ALL) return fail(JX_EINVAL, "unknown bits in flags");
    idx->flags = flags;
    idx->p.flags = flags;
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
    {   // a table with ids out of range or with a repeated id in a row would send the search kernels out of bounds:
        // check it before it is installed
        uint32_t* d_bad = (uint32_t*)(idx->d_stats + 10);
        uint32_t bad = 0;
        JX_HIP(jx::launch_fill_u32(d_bad, 1, 0u, st));
        JX_HIP(jx::launch_validate_adj(d_adj, n, idx->p.R, d_bad, st));
        JX_HIP(hipMemcpyAsync(&bad, d_bad, 4, hipMemcpyDeviceToHost, st));
        JX_HIP(hipStreamSynchronize(st));
        if (bad) return fail(JX_EINVAL, "%u adjacency entries are out of range, follow a padding entry or repeat an id of their row", bad);
    }
    JX_HIP(hipMemcpyAsync(idx->d_vecs, d_vecs, (size_t)n * idx->vec_bytes, hipMemcpyDeviceToDevice, st));
    JX_HIP(hipMemcpyAsync(idx->d_adj, d_adj, (size_t)n * idx->p.R * 4, hipMemcpyDeviceToDevice, st));
    if (n < idx->n) JX_HIP(jx::launch_fill_u32(idx->d_adj + (size_t)n * idx->p.R, (idx->n - n) * idx->p.R, JX_NONE, st));
    JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_clean, (idx->p.capacity + 3) / 4, 0u, st));  // nothing is known about foreign rows
    if (idx->any_delete) {
        JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_deleted, (idx->p.capacity + 3) / 4, 0u, st));
        JX_HIP(jx::launch_fill_u32((uint32_t*)(idx->d_stats + 8), 2, 0u, st));
        idx->any_delete = 0;
    }
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

// Stage timer used when the caller asks for jx_stats: events on the launch stream.
struct StageTimer {
    bool on;
    hipStream_t st;
    hipEvent_t ev[2];
    float acc[4];
    int rc;
    StageTimer(bool enable, hipStream_t s) : on(enable), st(s), rc(0) {
        acc[0] = acc[1] = acc[2] = acc[3] = 0.f;
        if (on && (hipEventCreate(&ev[0]) != hipSuccess || hipEventCreate(&ev[1]) != hipSuccess)) on = false;
    }
    ~StageTimer() {
        if (on) {
            (void)hipEventDestroy(ev[0]);
            (void)hipEventDestroy(ev[1]);
        }
    }
    void begin() {
        if (on) (void)hipEventRecord(ev[0], st);
    }
    // closes the stage; synchronises (stats calls block anyway)
    void end(int stage) {
        if (!on) return;
        (void)hipEventRecord(ev[1], st);
        (void)hipEventSynchronize(ev[1]);
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ev[0], ev[1]) == hipSuccess) acc[stage] += ms;
    }
};

static void fill_exact_src(const jx_index* idx, jx::DistSrc* ds, const void* queries) {
    memset(ds, 0, sizeof *ds);
    ds->recs = idx->d_vecs;
    ds->rec_stride = idx->vec_bytes;
    ds->nch = idx->vec_bytes / 16;
    ds->qrecs = (const uint8_t*)queries;
    ds->qrec_stride = idx->vec_bytes;
}

static int search_common(jx_index* idx, const void* d_queries, int64_t nq, int32_t out_k, int32_t L, int32_t mode,
                         int32_t rerank, uint32_t* d_out_ids, float* d_out_dist, jx_stats* h_stats, hipStream_t st) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (nq < 0) return fail(JX_EINVAL, "nq < 0");
    if (nq > 0 && (!d_queries || !d_out_ids || !d_out_dist)) return fail(JX_EINVAL, "NULL argument");
    if (L < 1 || L > JX_MAX_L) return fail(JX_EINVAL, "L must be in [1, %d]", JX_MAX_L);
    if (out_k < 1 || out_k > L) return fail(JX_EINVAL, "k must be in [1, L]");
    if (rerank != 0 && (rerank < out_k || rerank > L)) return fail(JX_EINVAL, "rerank must be 0 or in [k, L]");
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    if (idx->entry == JX_NONE) return fail(JX_ESTATE, "every vertex has been deleted");
    if (mode != JX_EXACT && mode != JX_RABITQ) return fail(JX_EINVAL, "unknown mode");
    if (mode == JX_RABITQ && !idx->quantized) return fail(JX_ESTATE, "index is not quantised");
    if (nq == 0) return JX_OK;
    const jx_params& p = idx->p;
    if (h_stats) JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_stripes, 64 * 16 * 2, 0u, st));
    jx::BeamArgs a;
    memset(&a, 0, sizeof a);
    a.adj = idx->d_adj;
    a.R = p.R;
    a.q_skip = 0x7FFFFFFFFFFFFFFFLL;
    a.L = L;
    a.entry = idx->entry;
    visited_table_for(idx->flags, L, idx->n, mode == JX_EXACT ? idx->vec_bytes : idx->code_stride, &a.hash_slots, &a.tag_bits);
    a.flags = idx->flags;
    a.stats = h_stats ? idx->d_stripes : nullptr;
    a.deleted = idx->any_delete ? idx->d_deleted : nullptr;
    StageTimer tm(h_stats != nullptr, st);
    char kname[96] = "";
    if (mode == JX_EXACT) {
        // distances are already exact: a re-rank would change nothing
        fill_exact_src(idx, &a.ds, d_queries);
        a.nq = nq;
        a.out_ids = d_out_ids;
        a.out_dist = d_out_dist;
        a.out_k = out_k;
        tm.begin();
        JX_HIP(jx::launch_beam_search(exact_kind(p.dtype), 0, a, st, kname));
        tm.end(2);
    } else {
        QueryWork qw;
        query_work(&p, p.max_batch, idx->plane_chunks, &qw);
        uint8_t* W = idx->d_work;
        const int nplanes = idx->quantized >= 4 ? 2 : idx->qbits;
        const int qrec_stride = 16 + nplanes * qw.plane_stride;
        for (int64_t q0 = 0; q0 < nq; q0 += p.max_batch) {
            const int64_t m = nq - q0 < p.max_batch ? nq - q0 : p.max_batch;
            const uint8_t* qs = (const uint8_t*)d_queries + (size_t)q0 * idx->vec_bytes;
            tm.begin();
            JX_HIP(jx::launch_rotate(qs, p.dtype, m, p.dim, idx->d_P, idx->d_centroid, (float*)(W + qw.rot), st));
            tm.end(0);
            jx::QueryPrepArgs qp;
            memset(&qp, 0, sizeof qp);
            qp.rot = (const float*)(W + qw.rot);
            qp.nq = m;
            qp.d = p.dim;
            qp.bits = idx->quantized;
            qp.qbits = idx->qbits;
            qp.qrecs = W + qw.qrecs;
            qp.qrec_stride = qrec_stride;
            qp.plane_stride = qw.plane_stride;
            tm.begin();
            JX_HIP(jx::launch_query_prep(qp, st));
            tm.end(1);
            memset(&a.ds, 0, sizeof a.ds);
            a.ds.recs = idx->d_codes;
            a.ds.rec_stride = idx->code_stride;
            a.ds.nch = idx->meta_chunk + 1;
            a.ds.meta_chunk = idx->meta_chunk;
            a.ds.qrecs = W + qw.qrecs;
            a.ds.qrec_stride = qrec_stride;
            a.ds.qplane_stride = qw.plane_stride;
            a.ds.plane_chunks = idx->plane_chunks;
            a.ds.plane_shift = idx->plane_shift;
            a.nq = m;
            if (rerank) {
                a.out_ids = (uint32_t*)(W + qw.fr_ids);
                a.out_dist = (float*)(W + qw.fr_dist);
                a.out_k = rerank;
            } else {
                a.out_ids = d_out_ids + (size_t)q0 * out_k;
                a.out_dist = d_out_dist + (size_t)q0 * out_k;
                a.out_k = out_k;
            }
            tm.begin();
            JX_HIP(jx::launch_beam_search(idx->quantized >= 4 ? 2 : 3, idx->qbits, a, st, kname));
            tm.end(2);
            if (rerank) {
                jx::RerankArgs r;
                memset(&r, 0, sizeof r);
                fill_exact_src(idx, &r.ds, qs);
                r.nq = m;
                r.cand = (const uint32_t*)(W + qw.fr_ids);
                r.cand_stride = rerank;
                r.rr = rerank;
                r.k = out_k;
                r.out_ids = d_out_ids + (size_t)q0 * out_k;
                r.out_dist = d_out_dist + (size_t)q0 * out_k;
                r.stats = h_stats ? idx->d_stripes : nullptr;
                tm.begin();
                JX_HIP(jx::launch_rerank(p.dtype, r, st));
                tm.end(3);
            }
        }
    }
    if (h_stats) {
        unsigned long long stripes[64 * 16], hs[3] = {0, 0, 0};
        JX_HIP(hipMemcpyAsync(stripes, idx->d_stripes, sizeof stripes, hipMemcpyDeviceToHost, st));
        JX_HIP(hipStreamSynchronize(st));
        for (int i = 0; i < 64; i++)
            for (int c = 0; c < 3; c++) hs[c] += stripes[i * 16 + c];
        memset(h_stats, 0, sizeof *h_stats);
        h_stats->hops = hs[0];
        h_stats->dist_evals = hs[1];
        h_stats->adj_bytes = hs[0] * 4ull * p.R;
        h_stats->vec_bytes = hs[1] * (unsigned long long)(mode == JX_EXACT ? idx->vec_bytes : (idx->meta_chunk + 1) * 16);
        h_stats->rerank_bytes = hs[2] * (unsigned long long)idx->vec_bytes;
        h_stats->rotate_ms = tm.acc[0];
        h_stats->prep_ms = tm.acc[1];
        h_stats->beam_ms = tm.acc[2];
        h_stats->rerank_ms = tm.acc[3];
        memcpy(h_stats->beam_kernel, kname, sizeof kname);
    }
    return JX_OK;
}

int jx_search(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, int32_t L, int32_t mode, int32_t rerank,
              uint32_t* d_out_ids, float* d_out_dist, jx_stats* h_stats, void* stream) {
    return search_common(idx, d_queries, nq, k, L, mode, rerank, d_out_ids, d_out_dist, h_stats, as_stream(stream));
}

int jx_beam_frontier(jx_index* idx, const void* d_queries, int64_t nq, int32_t L, int32_t mode, uint32_t* d_out_ids,
                     float* d_out_dist, jx_stats* h_stats, void* stream) {
    return search_common(idx, d_queries, nq, L, L, mode, 0, d_out_ids, d_out_dist, h_stats, as_stream(stream));
}

int jx_bruteforce(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, uint32_t* d_out_ids, float* d_out_dist,
                  void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (nq > 0 && (!d_queries || !d_out_ids || !d_out_dist)) return fail(JX_EINVAL, "NULL argument");
    if (k < 1 || k > JX_MAX_BF_K) return fail(JX_EINVAL, "k must be in [1, %d]", JX_MAX_BF_K);
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    if (nq <= 0) return JX_OK;
    hipStream_t st = as_stream(stream);
    // split the base set, and slice the queries so that the per-slice partial lists fit the workspace
    const int64_t nsplit = bruteforce_nsplit(idx->n, nq);
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

int jx_bruteforce_static(const void* d_base, int64_t n, int32_t dim, int32_t dtype, const void* d_queries, int64_t nq,
                         int32_t k, uint32_t* d_out_ids, float* d_out_dist, void* stream) {
    if (dtype != JX_U8 && dtype != JX_F32 && dtype != JX_F16) return fail(JX_EINVAL, "dtype must be JX_U8, JX_F32 or JX_F16");
    if (dim <= 0 || (dtype == JX_U8 && dim % 16) || (dtype == JX_F32 && dim % 4) || (dtype == JX_F16 && dim % 8))
        return fail(JX_EINVAL, "dim must be a positive multiple of 16 (uint8), 4 (float32) or 8 (binary16)");
    if (n < 1 || n > 0x7FFFFFFELL) return fail(JX_EINVAL, "n out of range");
    if (k < 1 || k > JX_MAX_BF_K) return fail(JX_EINVAL, "k must be in [1, %d]", JX_MAX_BF_K);
    if (nq < 0) return fail(JX_EINVAL, "nq < 0");
    if (nq == 0) return JX_OK;
    if (!d_base || !d_queries || !d_out_ids || !d_out_dist) return fail(JX_EINVAL, "NULL argument");
    const int64_t nsplit = bruteforce_nsplit(n, nq);
    const int64_t need = nq * nsplit * k * 8;
    if (need > (int64_t)JX_STATIC_SCRATCH_BYTES)
        return fail(JX_ECAPACITY, "nq * nsplit * k * 8 = %lld * %lld * %d * 8 = %lld bytes of partial lists exceed the static scratch of %lld bytes",
                    (long long)nq, (long long)nsplit, (int)k, (long long)need, (long long)JX_STATIC_SCRATCH_BYTES);
    unsigned char* sc = nullptr;
    int rc = static_scratch(&sc);
    if (rc) return rc;
    jx::BfArgs a;
    memset(&a, 0, sizeof a);
    a.base = d_base;
    a.queries = d_queries;
    a.dtype = dtype;
    a.d = dim;
    a.n = n;
    a.nq = nq;
    a.k = k;
    a.nsplit = (int)nsplit;
    a.partial = (uint64_t*)sc;  // every list the merge reads is written by the tile kernel first: nothing to clear
    a.out_ids = d_out_ids;
    a.out_dist = d_out_dist;
    JX_HIP(jx::launch_bruteforce(a, as_stream(stream)));
    return JX_OK;
}

static int encode_range(jx_index* idx, int64_t first, int64_t count, hipStream_t st);

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
    visited_table_for(idx->flags, p.L_build, n_after, idx->vec_bytes, &b.hash_slots, &b.tag_bits);
    b.flags = idx->flags;
    const int Lc = cand_len(&p);
    b.out_ids = (uint32_t*)(W + w.cand_ids);
    b.out_dist = (float*)(W + w.cand_dist);
    b.out_k = Lc;
    b.vis_cap = p.cand_mode == JX_CAND_VISITED ? Lc : 0;
    b.stats = nullptr;
    b.deleted = idx->any_delete ? idx->d_deleted : nullptr;  // new points never link to deleted vertices
    JX_HIP(jx::launch_beam_search(exact_kind(p.dtype), 0, b, st));
    // 2. robustPrune of the frontier, new rows, reverse edges
    jx::InsertArgs a;
    memset(&a, 0, sizeof a);
    a.ds = ds;
    a.adj = idx->d_adj;
    a.R = p.R;
    a.L = Lc;
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
    a.clean = incremental_prune(idx) ? idx->d_clean : nullptr;
    // forward prune: no LDS vector cache.  A whole frontier (128 x 128 bytes per wavefront) would leave room for
    // one workgroup per CU only, and the Gram-matrix form then measured slower (47 ms against 32 ms per 1M inserts)
    a.vec_cache_bytes = 0;
    a.gram = gram_mode(idx);
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
    // LDS room per wavefront for the vectors of a full row plus up to 32 new edges (96 x 128 bytes);
    // larger merges take the path that reads from global memory
    a.vec_cache_bytes = 12288;
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
    if (first > 0 && idx->entry == JX_NONE) return fail(JX_ESTATE, "every vertex has been deleted");
    if (first + n > p.capacity) return fail(JX_ECAPACITY, "%lld + %lld points exceed the capacity %lld", (long long)first, (long long)n, (long long)p.capacity);
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
    if (idx->quantized) return encode_range(idx, first, n, st);  // new points get codes with the frozen P and c
    return JX_OK;
}

// rotate + encode vectors [first, first+count) of the store into their records
static int encode_range(jx_index* idx, int64_t first, int64_t count, hipStream_t st) {
    const jx_params& p = idx->p;
    uint8_t* W = idx->d_work;
    const int64_t part = align256((int64_t)512 * p.dim * 8);
    int64_t slice = (idx->work_bytes - part) / ((int64_t)p.dim * 4);
    if (slice < 1) return fail(JX_ECAPACITY, "workspace too small to encode");
    float* rot = (float*)(W + part);
    for (int64_t s0 = 0; s0 < count; s0 += slice) {
        const int64_t m = count - s0 < slice ? count - s0 : slice;
        const uint8_t* src = idx->d_vecs + (size_t)(first + s0) * idx->vec_bytes;
        JX_HIP(jx::launch_rotate(src, p.dtype, m, p.dim, idx->d_P, idx->d_centroid, rot, st));
        jx::EncodeArgs e;
        memset(&e, 0, sizeof e);
        e.rot = rot;
        e.n = m;
        e.d = p.dim;
        e.bits = idx->quantized;
        e.rule = idx->rule;
        e.codes = idx->d_codes + (size_t)(first + s0) * idx->code_stride;
        e.code_stride = idx->code_stride;
        e.code_bytes = idx->code_bytes;
        e.pad_to = idx->meta_chunk * 16;
        e.meta = e.codes + (size_t)idx->meta_chunk * 16;
        e.meta_stride = idx->code_stride;
        e.meta_pad = 8;
        JX_HIP(jx::launch_encode(e, st));
        JX_HIP(jx::launch_code_sums(e.codes, m, idx->code_stride, idx->code_bytes, idx->meta_chunk * 16, idx->quantized, st));
        if (idx->plane_shift)
            JX_HIP(jx::launch_planarize(e.codes, m, idx->code_stride, idx->code_bytes, idx->plane_chunks * 16, idx->quantized, st));
    }
    return JX_OK;
}

int jx_quantize(jx_index* idx, int32_t bits, const float* d_rotation, const float* d_centroid, int32_t query_bits,
                int32_t rule, void* stream) {
    if (!idx || !d_rotation) return fail(JX_EINVAL, "NULL argument");
    const jx_params& p = idx->p;
    if (!p.quant_bits) return fail(JX_ESTATE, "the index was created with quant_bits = 0");
    if (bits != p.quant_bits) return fail(JX_EINVAL, "bits must equal params.quant_bits (%d)", p.quant_bits);
    if (query_bits != 4 && query_bits != 8) return fail(JX_EINVAL, "query_bits must be 4 or 8");
    const bool maxcos_offered = (bits == 2 || bits == 4) && p.dim * ((1 << (bits - 1)) - 1) <= 8192 && p.dim <= 4096;
    if (rule == JX_RULE_DEFAULT) rule = maxcos_offered ? JX_RULE_MAXCOS : JX_RULE_MAXABS;
    if (rule != JX_RULE_MAXABS && rule != JX_RULE_MAXCOS) return fail(JX_EINVAL, "unknown code rule");
    if (rule == JX_RULE_MAXCOS && bits > 1 && !maxcos_offered)
        return fail(JX_EINVAL, "JX_RULE_MAXCOS supports 2- and 4-bit codes with dim * (2^(bits-1) - 1) <= 8192 and dim <= 4096; use JX_RULE_MAXABS");
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    hipStream_t st = as_stream(stream);
    JX_HIP(hipMemcpyAsync(idx->d_P, d_rotation, (size_t)p.dim * p.dim * 4, hipMemcpyDeviceToDevice, st));
    if (d_centroid) {
        JX_HIP(hipMemcpyAsync(idx->d_centroid, d_centroid, (size_t)p.dim * 4, hipMemcpyDeviceToDevice, st));
    } else {
        JX_HIP(jx::launch_column_mean(idx->d_vecs, p.dtype, idx->n, p.dim, (double*)idx->d_work, idx->d_centroid, st));
    }
    idx->quantized = bits;
    idx->qbits = query_bits;
    idx->rule = rule;
    int rc = encode_range(idx, 0, idx->n, st);
    if (rc) idx->quantized = 0;
    return rc;
}

int jx_export_codes(jx_index* idx, uint8_t* d_codes, float* d_meta, float* d_centroid, void* stream) {
    if (!idx || !d_codes || !d_meta) return fail(JX_EINVAL, "NULL argument");
    if (!idx->quantized) return fail(JX_ESTATE, "index is not quantised");
    hipStream_t st = as_stream(stream);
    JX_HIP(jx::launch_unpack_records(idx->d_codes, idx->n, idx->code_stride, idx->code_bytes, idx->meta_chunk * 16, d_codes,
                                     d_meta, idx->plane_shift ? idx->quantized : 0, idx->plane_chunks * 16, st));
    if (d_centroid)
        JX_HIP(hipMemcpyAsync(d_centroid, idx->d_centroid, (size_t)idx->p.dim * 4, hipMemcpyDeviceToDevice, st));
    return JX_OK;
}

int jx_import_codes(jx_index* idx, int32_t bits, const float* d_rotation, const float* d_centroid, int32_t query_bits,
                    const uint8_t* d_codes, const float* d_meta, void* stream) {
    if (!idx || !d_rotation || !d_centroid || !d_codes || !d_meta) return fail(JX_EINVAL, "NULL argument");
    const jx_params& p = idx->p;
    if (!p.quant_bits) return fail(JX_ESTATE, "the index was created with quant_bits = 0");
    if (bits != p.quant_bits) return fail(JX_EINVAL, "bits must equal params.quant_bits (%d)", p.quant_bits);
    if (query_bits != 4 && query_bits != 8) return fail(JX_EINVAL, "query_bits must be 4 or 8");
    if (idx->n == 0) return fail(JX_ESTATE, "index is empty");
    hipStream_t st = as_stream(stream);
    JX_HIP(hipMemcpyAsync(idx->d_P, d_rotation, (size_t)p.dim * p.dim * 4, hipMemcpyDeviceToDevice, st));
    JX_HIP(hipMemcpyAsync(idx->d_centroid, d_centroid, (size_t)p.dim * 4, hipMemcpyDeviceToDevice, st));
    JX_HIP(jx::launch_pack_records(idx->d_codes, idx->n, idx->code_stride, idx->code_bytes, idx->meta_chunk * 16, d_codes, d_meta, st));
    JX_HIP(jx::launch_code_sums(idx->d_codes, idx->n, idx->code_stride, idx->code_bytes, idx->meta_chunk * 16, bits, st));
    if (idx->plane_shift)
        JX_HIP(jx::launch_planarize(idx->d_codes, idx->n, idx->code_stride, idx->code_bytes, idx->plane_chunks * 16, bits, st));
    idx->quantized = bits;
    idx->qbits = query_bits;
    idx->rule = JX_RULE_MAXABS;
    return JX_OK;
}

int jx_rotate(jx_index* idx, const float* d_in, int64_t n, float* d_out, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (!idx->quantized) return fail(JX_ESTATE, "index is not quantised");
    if (n < 0) return fail(JX_EINVAL, "n < 0");
    if (n == 0) return JX_OK;
    if (!d_in || !d_out) return fail(JX_EINVAL, "NULL argument");
    JX_HIP(jx::launch_rotate(d_in, JX_F32, n, idx->p.dim, idx->d_P, idx->d_centroid, d_out, as_stream(stream)));
    return JX_OK;
}

int jx_encode_rotated(jx_index* idx, const float* d_rot, int64_t n, uint8_t* d_codes, float* d_meta, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (!idx->quantized) return fail(JX_ESTATE, "index is not quantised");
    if (n < 0) return fail(JX_EINVAL, "n < 0");
    if (n == 0) return JX_OK;
    if (!d_rot || !d_codes || !d_meta) return fail(JX_EINVAL, "NULL argument");
    jx::EncodeArgs e;
    memset(&e, 0, sizeof e);
    e.rot = d_rot;
    e.n = n;
    e.d = idx->p.dim;
    e.bits = idx->quantized;
    e.rule = idx->rule;
    e.codes = d_codes;
    e.code_stride = idx->code_bytes;
    e.code_bytes = idx->code_bytes;
    e.pad_to = idx->code_bytes;
    e.meta = (uint8_t*)d_meta;
    e.meta_stride = 8;
    e.meta_pad = 0;
    JX_HIP(jx::launch_encode(e, as_stream(stream)));
    return JX_OK;
}

static int read_deleted_count(jx_index* idx, hipStream_t st, int64_t* out) {
    unsigned long long c = 0;
    if (idx->any_delete) {
        JX_HIP(hipMemcpyAsync(&c, idx->d_stats + 8, sizeof c, hipMemcpyDeviceToHost, st));
        JX_HIP(hipStreamSynchronize(st));
    }
    *out = (int64_t)c;
    return JX_OK;
}

int jx_delete(jx_index* idx, const uint32_t* d_ids, int64_t n, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    if (n < 0) return fail(JX_EINVAL, "n < 0");
    if (n == 0) return JX_OK;
    if (!d_ids) return fail(JX_EINVAL, "d_ids is NULL");
    idx->any_delete = 1;
    JX_HIP(jx::launch_mark_deleted(idx->d_deleted, d_ids, n, idx->n, idx->d_stats + 8, as_stream(stream)));
    return JX_OK;
}

int jx_deleted_count(jx_index* idx, int64_t* n_deleted, void* stream) {
    if (!idx || !n_deleted) return fail(JX_EINVAL, "NULL argument");
    return read_deleted_count(idx, as_stream(stream), n_deleted);
}

int jx_consolidate(jx_index* idx, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    hipStream_t st = as_stream(stream);
    int64_t ndel = 0;
    int rc = read_deleted_count(idx, st, &ndel);
    if (rc) return rc;
    if (ndel == 0 || idx->n == 0) return JX_OK;
    const jx_params& p = idx->p;
    const int64_t n = idx->n;
    InsertWork w;
    insert_work(&p, p.max_batch, &w);
    if (w.total > idx->work_bytes) return fail(JX_ECAPACITY, "workspace too small");
    const int64_t Ecap = (int64_t)p.max_batch * p.R;
    if (Ecap > 0xFFFFFFFFLL) return fail(JX_ECAPACITY, "max_batch * R exceeds 2^32");
    uint8_t* W = idx->d_work;
    jx::ConsolArgs c;
    memset(&c, 0, sizeof c);
    fill_exact_src(idx, &c.ds, idx->d_vecs);
    c.adj = idx->d_adj;
    c.R = p.R;
    c.n = n;
    c.deleted = idx->d_deleted;
    c.cnt = (uint32_t*)(W + w.dist);
    uint32_t* d_offs = c.cnt + p.capacity;
    c.offs = d_offs;
    // 1. candidates per vertex on the graph as it stands
    JX_HIP(jx::launch_consol_count(c, st));
    std::vector<uint32_t> cnt;
    try {
        cnt.resize((size_t)n);
    } catch (...) {
        return fail(JX_EINVAL, "out of host memory");
    }
    JX_HIP(hipMemcpyAsync(cnt.data(), c.cnt, (size_t)n * 4, hipMemcpyDeviceToHost, st));
    JX_HIP(hipStreamSynchronize(st));
    for (int64_t v = 0; v < n; v++)
        if (cnt[(size_t)v] > Ecap)  // checked before any row changes
            return fail(JX_ECAPACITY, "vertex %lld has %u consolidation candidates, the edge buffer holds max_batch * R = %lld",
                        (long long)v, cnt[(size_t)v], (long long)Ecap);
    int tbits = 1;
    while (((int64_t)1 << tbits) <= n) tbits++;
    jx::InsertArgs a;
    memset(&a, 0, sizeof a);
    a.ds = c.ds;
    a.adj = idx->d_adj;
    a.R = p.R;
    a.L = p.L_build;
    a.alpha = p.alpha;
    a.dead = W + w.dead;
    a.keys = (uint64_t*)(W + w.keys1);
    a.vals = (uint32_t*)(W + w.vals1);
    a.heads = (const uint32_t*)(W + w.heads);
    a.nseg = (const uint32_t*)(W + w.counters);
    a.force_prune = 1;
    a.clean = incremental_prune(idx) ? idx->d_clean : nullptr;
    a.gram = gram_mode(idx);
    a.vec_cache_bytes = 12288;
    // 2. slices of consecutive vertices whose candidate lists fit the edge buffers; every new row is
    //    computed from its own old row and from rows of deleted vertices, none of which is rewritten here
    int64_t v0 = 0;
    while (v0 < n) {
        int64_t v1 = v0, E = 0;
        while (v1 < n && E + cnt[(size_t)v1] <= Ecap) E += cnt[(size_t)v1++];
        if (E > 0) {
            const int64_t nv = v1 - v0;
            JX_HIP(hipMemcpyAsync(d_offs, c.cnt + v0, (size_t)nv * 4, hipMemcpyDeviceToDevice, st));
            JX_HIP(jx::launch_scan_u32(d_offs, nv, st));
            c.v0 = v0;
            c.v1 = v1;
            c.E = E;
            c.keys = (uint64_t*)(W + w.keys0);
            c.vals = (uint32_t*)(W + w.vals0);
            JX_HIP(jx::launch_consol_emit(c, st));
            // (v, candidate) order brings repeated candidates together
            JX_HIP(jx::launch_radix_sort((uint64_t*)(W + w.keys0), (uint32_t*)(W + w.vals0), (uint64_t*)(W + w.keys1),
                                         (uint32_t*)(W + w.vals1), E, 32 + tbits, (uint32_t*)(W + w.table), st));
            JX_HIP(jx::launch_consol_dist(p.dtype, c, (uint64_t*)(W + w.keys1), (uint32_t*)(W + w.vals1), st));
            // (v, distance) order; the sort is stable, so equal distances stay in id order
            JX_HIP(jx::launch_radix_sort((uint64_t*)(W + w.keys1), (uint32_t*)(W + w.vals1), (uint64_t*)(W + w.keys0),
                                         (uint32_t*)(W + w.vals0), E, 32 + tbits, (uint32_t*)(W + w.table), st));
            JX_HIP(jx::launch_fill_u32((uint32_t*)(W + w.counters), 16, 0u, st));
            JX_HIP(jx::launch_segment_heads((const uint64_t*)(W + w.keys1), E, (uint32_t*)(W + w.heads),
                                            (uint32_t*)(W + w.counters), st));
            a.E = E;
            a.B = (E + p.R - 1) / p.R;
            JX_HIP(jx::launch_reverse_merge(p.dtype, a, st));
        }
        v0 = v1;
    }
    // 3. nothing points to a deleted vertex any more: empty their rows
    JX_HIP(jx::launch_clear_deleted_rows(idx->d_adj, p.R, n, idx->d_deleted, st));
    // 4. a deleted entry point hands over to the nearest live vertex
    uint8_t entry_dead = 0;
    if (idx->entry == JX_NONE) return JX_OK;
    JX_HIP(hipMemcpyAsync(&entry_dead, idx->d_deleted + idx->entry, 1, hipMemcpyDeviceToHost, st));
    JX_HIP(hipStreamSynchronize(st));
    if (entry_dead) {
        if (ndel >= n) {
            idx->entry = JX_NONE;
        } else {
            uint32_t* d_best = (uint32_t*)(W + w.counters) + 32;
            JX_HIP(jx::launch_nearest_live(idx->d_vecs, p.dtype, n, p.dim, idx->entry, idx->d_deleted, (double*)(W + w.dist),
                                           d_best, st));
            uint32_t e = JX_NONE;
            JX_HIP(hipMemcpyAsync(&e, d_best, 4, hipMemcpyDeviceToHost, st));
            JX_HIP(hipStreamSynchronize(st));
            if (e >= (uint64_t)n) return fail(JX_EHIP, "entry point selection returned %u", e);
            idx->entry = e;
        }
    }
    return JX_OK;
}

int jx_compact(jx_index* idx, uint32_t* d_old_to_new, void* stream) {
    if (!idx) return fail(JX_EINVAL, "index is NULL");
    hipStream_t st = as_stream(stream);
    const int64_t n = idx->n;
    if (n == 0) return JX_OK;
    const jx_params& p = idx->p;
    InsertWork w;
    insert_work(&p, p.max_batch, &w);
    if (w.total > idx->work_bytes) return fail(JX_ECAPACITY, "workspace too small");
    uint8_t* W = idx->d_work;
    uint32_t* map = (uint32_t*)(W + w.dist);           // [n + 1]: live vertices before v; [n] = live in total
    uint32_t* err = (uint32_t*)(W + w.counters) + 40;
    uint8_t* staging = W;                               // everything in front of the renaming
    const int64_t staging_bytes = w.dist;
    JX_HIP(jx::launch_fill_u32(err, 1, 0u, st));
    JX_HIP(jx::launch_compact_flags(idx->d_adj, p.R, n, idx->d_deleted, map, err, st));
    uint32_t herr = 0;
    JX_HIP(hipMemcpyAsync(&herr, err, 4, hipMemcpyDeviceToHost, st));
    JX_HIP(hipStreamSynchronize(st));
    if (herr) return fail(JX_ESTATE, "a live vertex still points to a deleted one: call jx_consolidate first");
    JX_HIP(jx::launch_scan_u32(map, n + 1, st));
    JX_HIP(jx::launch_compact_rename(idx->d_adj, p.R, n, map, idx->d_deleted, d_old_to_new, st));
    JX_HIP(jx::launch_compact_records(idx->d_vecs, idx->vec_bytes, n, map, idx->d_deleted, staging, staging_bytes, st));
    JX_HIP(jx::launch_compact_records((uint8_t*)idx->d_adj, p.R * 4, n, map, idx->d_deleted, staging, staging_bytes, st));
    if (idx->quantized)
        JX_HIP(jx::launch_compact_records(idx->d_codes, idx->code_stride, n, map, idx->d_deleted, staging, staging_bytes, st));
    uint32_t live = 0, new_entry = JX_NONE;
    JX_HIP(hipMemcpyAsync(&live, map + n, 4, hipMemcpyDeviceToHost, st));
    if (idx->entry != JX_NONE) JX_HIP(hipMemcpyAsync(&new_entry, map + idx->entry, 4, hipMemcpyDeviceToHost, st));
    JX_HIP(hipStreamSynchronize(st));
    if (live > (uint64_t)n) return fail(JX_EHIP, "compaction counted %u live vertices of %lld", live, (long long)n);
    if (live < (uint64_t)n) JX_HIP(jx::launch_fill_u32(idx->d_adj + (size_t)live * p.R, (n - live) * p.R, JX_NONE, st));
    JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_deleted, (n + 3) / 4, 0u, st));
    JX_HIP(jx::launch_fill_u32((uint32_t*)idx->d_clean, (n + 3) / 4, 0u, st));  // rows moved: start again from "nothing known"
    JX_HIP(jx::launch_fill_u32((uint32_t*)(idx->d_stats + 8), 2, 0u, st));
    idx->n = live;
    idx->entry = live ? new_entry : JX_NONE;
    idx->any_delete = 0;
    return JX_OK;
}

int jx_mips_augment(const float* d_in, int64_t n, int32_t dim, float max_norm, int32_t is_query, float* d_out,
                    int32_t dim_out, float* d_norms, void* stream) {
    if (n < 0) return fail(JX_EINVAL, "n < 0");
    if (n == 0) return JX_OK;
    if (!d_in || (!d_out && !d_norms)) return fail(JX_EINVAL, "NULL argument");
    if (dim < 1) return fail(JX_EINVAL, "dim must be positive");
    if (d_out && dim_out < dim + 1) return fail(JX_EINVAL, "dim_out must be at least dim + 1");
    if (d_out && !(max_norm >= 0.0f)) return fail(JX_EINVAL, "max_norm must be non-negative");
    JX_HIP(jx::launch_mips_augment(d_in, n, dim, max_norm, is_query, d_out, dim_out, d_norms, as_stream(stream)));
    return JX_OK;
}

int jx_probe_gather(const void* d_table, int64_t n_rec, int32_t rec_bytes, const uint32_t* d_ids, int64_t n_ids,
                    int32_t blocks, uint32_t* d_sink, void* stream) {
    if (!d_table || !d_ids || !d_sink) return fail(JX_EINVAL, "NULL argument");
    if (rec_bytes != 64 && rec_bytes != 128 && rec_bytes != 256 && rec_bytes != 512)
        return fail(JX_EINVAL, "rec_bytes must be 64, 128, 256 or 512");
    if (n_rec < 1 || n_ids < 1 || blocks < 1 || blocks > 65536) return fail(JX_EINVAL, "sizes out of range");
    JX_HIP(jx::launch_gather_probe((const uint8_t*)d_table, rec_bytes, d_ids, n_ids, blocks, d_sink, as_stream(stream)));
    return JX_OK;
}

}  // extern "C"
#pragma GCC visibility pop
