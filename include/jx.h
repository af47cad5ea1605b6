/*
 * jx.h -- C ABI of libjx: a single-GPU (gfx950 / MI355X) implementation of the
 * Vamana-graph approximate nearest-neighbour path of "GPU-Accelerated ANNS:
 * Quantized for Speed, Built for Change" (Jasper): batched beamSearch for
 * queries and for batch insertion, robustPrune, reverse-edge merge, RaBitQ
 * codes with estimated distances, exact re-ranking.
 *
 * General rules
 *   - Every pointer named d_* is DEVICE memory, every h_* is HOST memory.
 *   - The library never allocates or frees device memory: the caller hands in
 *     one arena (jx_arena_bytes / jx_create) and owns it, and owns every input
 *     and output buffer.  The arena must stay alive and untouched until
 *     jx_destroy.
 *   - All work is enqueued on the caller's stream (`stream` is a hipStream_t
 *     passed as void*; NULL = the default stream).  Calls return after
 *     enqueueing unless stated otherwise ("blocks" = synchronises the stream).
 *   - A handle is not thread-safe.  Inserts, quantisation and searches on one
 *     index run in phases and must not overlap (Sec. 4.5: a batch of inserts
 *     completes before queries resume, and vice versa).  One exception:
 *     jx_search calls in JX_EXACT mode with h_stats == NULL only read the index
 *     and write their own outputs, so several of them may be in flight on
 *     different streams of the device (from one host thread); JX_RABITQ
 *     searches use the index's workspace and must not overlap anything.
 *   - Ids are uint32, assigned in insertion order starting at 0; at most
 *     2^31 - 2 points.  0xFFFFFFFF (JX_NONE) marks an empty slot.
 *   - Distances are SQUARED Euclidean distances (App. B: the square root is
 *     monotone and is elided).  Results are sorted ascending by (distance, id).
 *   - Return value: 0 on success, a negative JX_E* code otherwise; nothing
 *     throws or aborts across the boundary.  jx_last_error() gives the text of
 *     the last failure on the calling thread.
 */
#ifndef JX_H
#define JX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define JX_NONE 0xFFFFFFFFu

/* element types of the stored vectors and of the queries */
#define JX_U8 0  /* uint8, distances accumulated exactly in int32 */
#define JX_F32 1 /* float32 */
#define JX_F16 2 /* IEEE binary16 storage of float data (App. D); distances accumulated in float32 */

/* search modes */
#define JX_EXACT 0  /* distances on the stored full-precision vectors */
#define JX_RABITQ 1 /* RaBitQ-estimated distances on the codes (needs jx_quantize) */

/* what beamSearch hands to robustPrune during insertion */
#define JX_CAND_FRONTIER 0 /* the final frontier F (Alg. 2's output): at most L_build candidates */
#define JX_CAND_VISITED 1  /* the expansion list V (Alg. 1's output, which Alg. 4 step 2 prunes): every vertex the
                              search expanded, F included -- the first min(512, 4 L_build rounded up to a power of
                              two) of them in expansion order.  Offered for L_build <= 128 on uint8 vectors of at
                              most 128 bytes and float32 vectors of at most 512 or of 2,049..6,144 bytes */

/* rule that picks the m-bit code for m > 1 (Sec. 5.1 says only "simple scalar
 * quantization") */
#define JX_RULE_MAXCOS 0 /* the grid point whose direction is closest to r ("extended" codes): exact sweep
                           over the breakpoints of the grid scale; 2- and 4-bit codes with dim * (2^(m-1) - 1) <= 8192, dim <= 4096 */
#define JX_RULE_MAXABS 1 /* grid scale t = (2^(m-1) - 1/2) / max_i |r_i| */
#define JX_RULE_DEFAULT (-1) /* JX_RULE_MAXCOS where it is offered for the index's dim and bits, else JX_RULE_MAXABS */

/*
 * jx_params.flags / jx_set_flags: implementation switches.  0 selects the
 * defaults, which are the measured optima on gfx950.  No switch changes a
 * result: every combination returns the same ids, distances and graphs (the
 * parity tests hold each of them to the CPU oracle); they change which kernel
 * variant does the work, and exist for the kernel-variant ablation (Sec. 6.5
 * "Ablation study"; App. Block-Size, Tile Size and Load microbenchmarks) and
 * for comparisons in the tests.  Nothing in the library reads an environment
 * variable.
 */
#define JX_FLAG_NO_PAIR (1u << 0)       /* beamSearch: never take two expansions per round */
#define JX_FLAG_NO_INCR_PRUNE (1u << 1) /* uint8 reverse merge: always prune a whole row, never only the pairs that
                                           involve entries added since the row's last prune */
#define JX_FLAG_NO_GRAM (1u << 2)       /* float data: robustPrune by the list-based kernels, not the Gram-matrix (MFMA) ones */
#define JX_FLAG_GRAM_U8 (1u << 3)       /* uint8 data: robustPrune by the Gram-matrix kernels as well */
#define JX_FLAG_VISITED_IDS (1u << 4)   /* beamSearch visited filter: direct-mapped table of full 32-bit ids (ParlayANN's
                                           table, Sec. 4.2) instead of two-way sets of 16-bit tags */
#define JX_FLAG_VISITED_NONE (1u << 5)  /* beamSearch visited filter: none -- Alg. 2 as printed: every neighbour is
                                           evaluated, the frontier's expanded bit is the only memory */
#define JX_FLAG_LANES_WIDE (1u << 6)    /* beamSearch: twice the default lanes per record (one 16-byte chunk per lane) */
#define JX_FLAG_LANES_NARROW (1u << 7)  /* beamSearch: half the default lanes per record (four chunks per lane; uint8
                                           and float32 records of at most 8 / 32 chunks) */
#define JX_FLAG_TILED_LOADS (1u << 8)   /* beamSearch, exact uint8 / float32: the "tiled" load of Sec. 4.4 -- each lane
                                           reads 4-byte elements strided over its lane group -- instead of the
                                           "chunked" 16-byte loads */
#define JX_FLAG_WAVES_2 (1u << 9)       /* beamSearch, exact float32 records of more than 64 chunks: two wavefronts */
#define JX_FLAG_WAVES_4 (1u << 10)      /* ... four wavefronts share one query's distance evaluations (Sec. 4.1: larger
                                           blocks for larger vectors) */
#define JX_FLAG_QPW_2 (1u << 11)        /* beamSearch: two */
#define JX_FLAG_QPW_4 (1u << 12)        /* ... four queries (wavefronts) per workgroup instead of one */
#define JX_FLAG_ALL ((1u << 13) - 1u)

/* error codes */
#define JX_OK 0
#define JX_EINVAL (-1)    /* bad argument: dim, k > L, L too large, NULL pointer, dtype */
#define JX_ECAPACITY (-2) /* insert beyond capacity, batch beyond max_batch, arena too small */
#define JX_ESTATE (-3)    /* search on an empty index, RaBitQ search before jx_quantize */
#define JX_EHIP (-4)      /* a HIP call failed; see jx_last_error() */

/* limits */
#define JX_MAX_L 512    /* largest beam width L / L_build */
#define JX_MAX_R 256    /* largest out-degree R */
#define JX_MAX_BF_K 128 /* largest k of jx_bruteforce */
#define JX_STATIC_SCRATCH_BYTES (16 << 20) /* device scratch of jx_bruteforce_static, held per GPU for the life of the process */

typedef struct jx_index jx_index; /* opaque, host side */

typedef struct {
    int32_t dim;       /* d.  uint8: multiple of 16; float32: multiple of 4; binary16: multiple of 8 */
    int32_t dtype;     /* JX_U8 | JX_F32 | JX_F16 (queries have the same type) */
    int32_t R;         /* maximum out-degree (Sec. 3.1), 1..JX_MAX_R */
    int32_t L_build;   /* beam width used by insertion (Alg. 4), R.. JX_MAX_L is not required; 1..JX_MAX_L */
    float alpha;       /* robustPrune factor, applied to squared distances (Alg. 3) */
    int32_t cand_mode; /* JX_CAND_FRONTIER | JX_CAND_VISITED */
    int64_t capacity;  /* maximum number of points; rows are preallocated */
    int64_t max_batch; /* largest number of points linked by one internal batch
                          and largest number of queries processed at once
                          (larger query batches are processed in slices) */
    int32_t quant_bits; /* 0: never quantised; 1, 2, 4 or 8: reserve room for RaBitQ codes of that width */
    float batch_growth; /* an internal insert batch holds at most max(1, floor(batch_growth * #linked))
                           points; 0 selects the default 0.25 */
    uint32_t flags;     /* JX_FLAG_* switches; 0 = defaults */
} jx_params;

/* Counters of one jx_search call, summed over its queries. */
typedef struct {
    uint64_t hops;         /* expansions (adjacency rows read) */
    uint64_t dist_evals;   /* distance evaluations in beamSearch */
    uint64_t adj_bytes;    /* hops * 4R */
    uint64_t vec_bytes;    /* dist_evals * bytes fetched per evaluation */
    uint64_t rerank_bytes; /* exact re-rank reads */
    /* elapsed time of each stage of the call, from HIP events recorded on the
     * caller's stream around the stage's launches (summed over query slices) */
    float rotate_ms, prep_ms, beam_ms, rerank_ms;
    /* the beamSearch kernel instance the call launched, as a profiler prints it:
     * "beam_search_kernel<KIND,T,CPL,NREG,QB>" -- distance provider (0 uint8, 1 float32, 2 4-bit codes, 3 1-bit
     * codes, 4 binary16), lanes per record, 16-byte chunks per lane, frontier registers per lane (64 entries
     * each), query bits; "beam_search_pair_kernel<...>" = two expansions per round */
    char beam_kernel[96];
} jx_stats;

/* Bytes of device memory jx_create needs for these parameters (256-aligned
 * sub-buffers: vectors, adjacency, codes, rotation, workspaces). <0: JX_EINVAL. */
int64_t jx_arena_bytes(const jx_params* p);

/* Create an empty index inside the caller's arena (device memory, at least
 * jx_arena_bytes(p) bytes, 256-byte aligned).  Enqueues a fill of the
 * adjacency table with JX_NONE on `stream`.  *out is a host object freed by
 * jx_destroy. */
int jx_create(const jx_params* p, void* d_arena, int64_t arena_bytes, void* stream, jx_index** out);

/* Frees the host object only. */
int jx_destroy(jx_index* idx);

/* Replace the index's JX_FLAG_* switches (takes effect from the next call; bits outside JX_FLAG_ALL: JX_EINVAL).
 * A debug entry point: it lets one index be searched, or a build be continued, under several kernel variants. */
int jx_set_flags(jx_index* idx, uint32_t flags);

/*
 * Batch insertion (Alg. 4 with the changes of Sec. 4.3 and 4.5).
 * d_vecs: n vectors of the index's dtype, row-major [n][dim]; they receive ids
 * [N, N+n) in the given order.  The call (1) appends them to the store, (2) on
 * the first call picks the entry point = the point of that call nearest to the
 * call's coordinate-wise mean (the paper's "medoid"), which joins the graph
 * first with an empty row, (3) links the remaining points in id order in
 * internal batches of size min(remaining, max(1, floor(batch_growth * number of
 * points already linked))) (Sec. 6.2 reports batches of 0.5 % to 32 % of the
 * index as working); each batch runs beamSearch
 * (L_build, from the entry point, exact distances) for all its points against
 * the graph as it stood before the batch, robustPrune of the final frontier
 * (Alg. 3), emission of reverse edges to the kept neighbours only, one global
 * sort by (target, distance, source), and per target either an append (row
 * still fits) or robustPrune of row U new edges.  If the index is quantised
 * the new vectors are encoded as well.
 * Errors: JX_ECAPACITY if N+n > capacity or an internal batch > max_batch.
 * Blocks only on the first call (reads the entry id back).
 */
int jx_insert(jx_index* idx, const void* d_vecs, int64_t n, void* stream);

/*
 * RaBitQ quantisation of the current base set (Sec. 5.1); any storage type (uint8 and
 * binary16 values enter the rotation as float32, exactly).
 * bits: 1, 2, 4 or 8 (must equal params.quant_bits).  d_rotation: orthogonal matrix P,
 * float32 [dim][dim] row-major, applied as r = P (v - c).  d_centroid: c
 * (float32 [dim]) or NULL = mean of the current base set.  query_bits: width
 * B_q of the integer query (4 or 8).  rule: JX_RULE_MAXCOS, JX_RULE_MAXABS or
 * JX_RULE_DEFAULT (ignored for 1-bit codes).
 * Per vector the arena holds the dim*bits/8 code bytes (2- and 8-bit codes
 * split into a low and a high plane of 1-bit / 4-bit fields), zero padding to
 * 16-byte chunks, then data_add = ||r||^2 and data_rescale = -2||r||^2/<xbar,r>
 * as two floats and the code sum as uint32, the record padded to a multiple
 * of 128 bytes.  jx_export_codes / jx_import_codes always speak the natural
 * packing: coordinate i in bits [i*bits, (i+1)*bits) of the little-endian
 * bit string.  The matrix, centroid and
 * parameters are copied into the arena and frozen; later inserts are encoded
 * with them.  dim must be a multiple of 32.
 */
int jx_quantize(jx_index* idx, int32_t bits, const float* d_rotation, const float* d_centroid, int32_t query_bits,
                int32_t rule, void* stream);

/*
 * beamSearch for a batch of queries (Alg. 1 / Alg. 2) + optional exact re-rank.
 * d_queries: [nq][dim] of the index's dtype.  k <= L <= JX_MAX_L.
 * mode JX_EXACT: distances on the stored vectors.  mode JX_RABITQ: queries are
 * centred, rotated (MFMA GEMM) and turned into integer records; beamSearch runs
 * on estimated distances.  rerank == 0: the first k frontier entries are
 * returned (distance = the estimate in RaBitQ mode).  rerank > 0 (k <= rerank
 * <= L): the first `rerank` frontier entries are re-scored with the exact
 * squared L2 against the original query, sorted by (distance, id), and the
 * first k returned.
 * d_out_ids [nq][k], d_out_dist [nq][k]; slots beyond the number of reachable
 * points hold JX_NONE / +inf.  h_stats: NULL, or a host struct that receives
 * the counters -- in that case the call BLOCKS until the stream has drained.
 * Errors: JX_ESTATE on an empty index or RaBitQ mode before jx_quantize.
 */
int jx_search(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, int32_t L, int32_t mode, int32_t rerank,
              uint32_t* d_out_ids, float* d_out_dist, jx_stats* h_stats, void* stream);

/*
 * The beamSearch stage alone: whole final frontier of every query, as used by
 * insertion (Alg. 4, step 1).  d_out_ids / d_out_dist: [nq][L]; unused slots
 * JX_NONE / +inf.  mode as in jx_search.
 */
int jx_beam_frontier(jx_index* idx, const void* d_queries, int64_t nq, int32_t L, int32_t mode, uint32_t* d_out_ids,
                     float* d_out_dist, jx_stats* h_stats, void* stream);

/* Exact k nearest neighbours of every query by exhaustive search (the recall
 * ground truth of Sec. 6.1).  k <= JX_MAX_BF_K. */
int jx_bruteforce(jx_index* idx, const void* d_queries, int64_t nq, int32_t k, uint32_t* d_out_ids,
                  float* d_out_dist, void* stream);

/*
 * jx_bruteforce for callers that cannot allocate device memory and have no
 * arena either: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same kernels and same results as jx_bruteforce, but
 * no index is needed: d_base is [n][dim] of `dtype` (JX_U8 | JX_F32 | JX_F16,
 * dim a multiple of 16 / 4 / 8), d_queries [nq][dim] of the same type, outputs
 * [nq][k], k <= JX_MAX_BF_K.  The per-query partial lists live in a scratch
 * array of JX_STATIC_SCRATCH_BYTES that is part of the library's device code
 * (one copy per GPU, resolved with hipGetSymbolAddress at the first call on
 * that GPU); the call performs no hipMalloc / hipFree and calls no allocating
 * library routine.  Limit: nq * nsplit * k * 8 <= JX_STATIC_SCRATCH_BYTES with
 * nsplit = clamp(ceil(2048 / ceil(nq / 64)), 1, min(64, ceil(n / 64))) --
 * e.g. 10,000 queries at k = 10 (nsplit 14: 11.2 MB), or any nq * k <= 32,768;
 * beyond it JX_ECAPACITY and nothing is launched.  All calls on one GPU share
 * that GPU's scratch: calls that overlap in time on one GPU (different streams
 * or threads) race; consecutive calls on one stream are safe.  Nothing has to
 * be cleared between calls: every list that is read is written first.
 */
int jx_bruteforce_static(const void* d_base, int64_t n, int32_t dim, int32_t dtype, const void* d_queries, int64_t nq,
                         int32_t k, uint32_t* d_out_ids, float* d_out_dist, void* stream);

/* Batch deletion (Sec. 4.6 and 6.4: mark, consolidate, compact; the scheme of
 * FreshDiskANN that the paper adopts).
 *
 * jx_delete marks the n vertices d_ids[n] (device) as deleted: an in-place,
 * asynchronous flag update.  Ids >= the number of points and ids already
 * marked are ignored.  From then on a deleted vertex is still traversed by
 * beamSearch (its out-edges keep the graph connected) but never appears in
 * any output: not in search results, not in the frontier returned by
 * jx_beam_frontier, not among re-rank candidates, and not among the insertion
 * candidates of later jx_insert calls.  jx_bruteforce ignores the marks.
 *
 * jx_consolidate repairs the graph, in place: every live vertex v with at
 * least one deleted out-neighbour gets as candidate set its live neighbours
 * plus the live out-neighbours (other than v) of each deleted neighbour, and
 * its row becomes robustPrune (Alg. 3, the index's alpha and R) of that set;
 * all rows are computed from the graph as it stood at the call.  The rows of
 * deleted vertices are then emptied.  If the entry point is deleted, the
 * live vertex nearest to it (distance, then id) takes its place.  Ids do
 * not change and deleted vertices stay marked (jx_compact removes them).
 * Synchronises with the stream (it needs counts on the host).
 * JX_ECAPACITY if one vertex has more than max_batch * R candidates
 * (max_batch >= R always suffices).
 *
 * jx_deleted_count returns the number of vertices marked so far
 * (synchronises with the stream).
 *
 * jx_compact (third phase) removes the deleted vertices physically: live
 * vertices keep their relative order (new id = number of live vertices with
 * a smaller old id), vectors, rows, RaBitQ records and the entry point move
 * along, the freed tail of the arena becomes insertable again and the marks
 * are cleared.  Because the renaming preserves the id order, every search
 * returns the renamed ids of what it returned before.  d_old_to_new (device,
 * [points before the call], may be NULL) receives the renaming, JX_NONE for
 * removed vertices.  JX_ESTATE, and nothing changed, if a live vertex still
 * points to a deleted one (jx_consolidate has not run since the last
 * jx_delete).  Synchronises with the stream. */
int jx_delete(jx_index* idx, const uint32_t* d_ids, int64_t n, void* stream);
int jx_consolidate(jx_index* idx, void* stream);
int jx_compact(jx_index* idx, uint32_t* d_old_to_new, void* stream);
int jx_deleted_count(jx_index* idx, int64_t* n_deleted, void* stream);

/* Maximum-inner-product data as squared-L2 data (Sec. 6.3, the Text2Image
 * set: one extra dimension restores a metric space for graph construction).
 * For n float32 rows d_in [n][dim]:
 *   d_norms [n] (may be NULL) receives |x| (accumulated in double);
 *   d_out [n][dim_out] (may be NULL; dim_out >= dim + 1) receives the row,
 *   then sqrt(max(max_norm^2 - |x|^2, 0)) for base rows (is_query = 0) or 0
 *   for query rows (is_query != 0), then zeros up to dim_out (choose dim_out
 *   as the next multiple of 4 for a JX_F32 index).
 * With max_norm >= every base norm, |x' - q'|^2 = max_norm^2 + |q|^2 - 2<x,q>,
 * so nearest neighbours in the augmented space are the largest inner
 * products.  Both buffers may be requested in one call. */
int jx_mips_augment(const float* d_in, int64_t n, int32_t dim, float max_norm, int32_t is_query, float* d_out,
                    int32_t dim_out, float* d_norms, void* stream);

/* Calibration aid for the roofline of beamSearch (Sec. 6.5 prices the kernel
 * against memory bandwidth): reads the n_ids records d_ids[i] (all < n_rec;
 * not checked on the device -- the caller guarantees it) of a table of
 * rec_bytes-byte records (64, 128, 256 or 512) with independent 16-byte
 * loads, rec_bytes/16 lanes per record, eight loads in flight per lane, from
 * `blocks` workgroups of 256 threads, and writes one checksum word per thread
 * to d_sink [blocks*256].  Gives the rate at which this GPU serves gathers of
 * that record size when nothing else limits them. */
int jx_probe_gather(const void* d_table, int64_t n_rec, int32_t rec_bytes, const uint32_t* d_ids, int64_t n_ids,
                    int32_t blocks, uint32_t* d_sink, void* stream);

/* Number of points and entry id (host values; no device work). */
int jx_size(const jx_index* idx, int64_t* n, uint32_t* entry_id);

/* Copy out the adjacency table (d_adj [N][R], JX_NONE padded) and the row
 * degrees (d_deg [N]; may be NULL). */
int jx_export_graph(jx_index* idx, uint32_t* d_adj, uint32_t* d_deg, void* stream);

/* Replace the index content by n vectors and a ready-made graph (used to
 * search a graph built elsewhere, e.g. by a reference implementation).
 * Rows must be filled from the left and padded with JX_NONE, ids must be
 * below n and no row may name a vertex twice: the table is checked on the device first (the call synchronises)
 * and JX_EINVAL leaves the index untouched. */
int jx_import_graph(jx_index* idx, const void* d_vecs, int64_t n, const uint32_t* d_adj, uint32_t entry_id,
                    void* stream);

/* Copy out codes (d_codes [N][dim*bits/8], unpadded), the two floats per
 * vector (d_meta [N][2]) and the centroid (d_centroid [dim], may be NULL). */
int jx_export_codes(jx_index* idx, uint8_t* d_codes, float* d_meta, float* d_centroid, void* stream);

/* Install codes produced elsewhere (d_codes [N][dim*bits/8] unpadded, d_meta
 * [N][2]) together with the rotation and centroid they were made with; the
 * counterpart of jx_export_codes.  Lets a test search on injected codes. */
int jx_import_codes(jx_index* idx, int32_t bits, const float* d_rotation, const float* d_centroid, int32_t query_bits,
                    const uint8_t* d_codes, const float* d_meta, void* stream);

/* Stage entry points of the RaBitQ pipeline (Sec. 5.1), used to test each
 * stage against injected inputs.
 *   jx_rotate: d_out[n][dim] = (d_in[n][dim] - c) P^T with the index's frozen
 *   P and c (the GEMM used for queries and for encoding).
 *   jx_encode_rotated: encode n already-rotated vectors into unpadded codes
 *   and meta, with the index's bits and rule. */
int jx_rotate(jx_index* idx, const float* d_in, int64_t n, float* d_out, void* stream);
int jx_encode_rotated(jx_index* idx, const float* d_rot, int64_t n, uint8_t* d_codes, float* d_meta, void* stream);

const char* jx_strerror(int code);
const char* jx_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* JX_H */
