// Host-side internals of libjx: index object, arena layout, kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "../../include/jx.h"

#ifndef JX_BEAM_WPB
#define JX_BEAM_WPB 1  // wavefronts (= queries) per workgroup of the beamSearch kernel: a slot is free again as soon as its query ends
#endif

namespace jx {

// ---- beamSearch -----------------------------------------------------------
// Where distances are taken: stored records and the records of the queries.
struct DistSrc {
    const uint8_t* recs;   // records the distances are taken on
    long long rec_stride;  // bytes between records (multiple of 16)
    int nch;               // 16-byte chunks read per record
    int meta_chunk;        // RaBitQ: chunk that holds data_add, data_rescale
    const uint8_t* qrecs;  // per-query records
    long long qrec_stride;
    int qplane_stride;     // RaBitQ: bytes between the query's planes
    int plane_chunks;      // RaBitQ: chunks per code plane (= meta_chunk for 1- and 4-bit codes, meta_chunk / 2 for
                           // 2- and 8-bit codes, which are stored as a low and a high plane)
    int plane_shift;       // RaBitQ: log2 of the weight of the high plane (1 for 2-bit, 4 for 8-bit codes, else 0)
};

struct BeamArgs {
    const uint32_t* adj;   // [N][R]
    int R;
    DistSrc ds;
    long long nq;
    long long q_skip;      // query i reads record i + (i >= q_skip); used by insertion to skip the entry point
    int L;
    uint32_t entry;
    int hash_slots;        // visited-table size (any value >= 64; slot = high word of hash * size)
    int tag_bits;          // 0: 32-bit entries hold the id.  > 0: hash_slots is a power of two, the table has hash_slots / 2
                           // sets of two 16-bit entries, every id is below (hash_slots / 2) << tag_bits, and an entry holds
                           // the low tag_bits (<= 15) of the permuted id
    uint32_t* out_ids;     // [nq][out_k]
    float* out_dist;       // [nq][out_k]
    int out_k;
    unsigned long long* stats;  // NULL, or 64 stripes of 16 counters (query i adds to stripe i % 64): [0] hops, [1] dist_evals
    const uint8_t* deleted;     // [N] 1 = logically deleted (never returned), or NULL
    uint32_t flags;             // JX_FLAG_* switches that select a kernel variant
    int vis_cap;                // > 0 (a power of two <= 512): instead of the frontier, out_ids / out_dist [nq][vis_cap]
                                // receive the expanded vertices (Alg. 1's set V), the first vis_cap of them in
                                // expansion order, sorted by (distance, id)
};
// kernel_name (may be NULL): receives the name of the instance that was launched, at most 96 bytes
hipError_t launch_beam_search(int kind, int qbits, const BeamArgs& a, hipStream_t st, char* kernel_name = nullptr);
// ablation instances (JX_FLAG_TILED_LOADS, JX_FLAG_QPW_*, JX_FLAG_WAVES_*); hipErrorInvalidValue where none exists
hipError_t launch_beam_variant(int kind, const BeamArgs& a, hipStream_t st, char* kernel_name);
// beamSearch that returns the expansion list (BeamArgs::vis_cap); instances: see visited_list_offered()
hipError_t launch_beam_visited(int kind, const BeamArgs& a, hipStream_t st, char* kernel_name);
bool visited_list_offered(int kind, int nch, int L, int R);
// length of the expansion list kept per query for beam width L: 4 L rounded up to a power of two, 64..512
inline int visited_cap(int L) {
    int c = 64;
    while (c < 4 * L && c < 512) c *= 2;
    return c;
}

// ---- batch insertion -------------------------------------------------------
struct InsertArgs {
    DistSrc ds;            // recs = qrecs = the vector store
    uint32_t* adj;
    int R, L;
    float alpha;
    long long B;           // points in this batch
    long long id_base;     // id of batch element i = id_base + i (+1 if >= id_skip)
    long long id_skip;
    const uint32_t* cand_ids;   // [B][L]
    const uint32_t* cand_dist;  // [B][L] float bits
    uint8_t* dead;              // max(B*L, B*R) bytes
    uint64_t* keys;             // [B*R] edge keys
    uint32_t* vals;             // [B*R] edge sources
    const uint32_t* heads;      // segment starts (reverse merge); bit 31 is set by a kernel that has merged the segment
    const uint32_t* nseg;       // number of segments (device)
    long long E;                // reverse merge: number of sorted edges (0 = B * R)
    int force_prune;            // consolidation: ignore the existing row, always prune the candidate segment
    int gram;                   // float data: 1 (float32) / 2 (binary16) = prunes of at most 128 candidates go to the Gram-matrix kernels
    int vec_cache_bytes;        // reverse merge: LDS bytes per wavefront for candidate vectors (0 = never cache)
    uint8_t* clean;             // [N] leading entries of each row that one robustPrune call selected together
                                // (saturated at 255; 0 = nothing known), or NULL
};

hipError_t launch_entry_point(const void* vecs, int dtype, long long n, int d, double* partial, float* mean, double* dist,
                              uint32_t* out_id, hipStream_t st);
hipError_t launch_forward_prune(int dtype, const InsertArgs& a, hipStream_t st);
hipError_t launch_reverse_merge(int dtype, const InsertArgs& a, hipStream_t st);
hipError_t launch_forward_prune_gram(int dtype, const InsertArgs& a, hipStream_t st);
hipError_t launch_reverse_merge_gram(int dtype, const InsertArgs& a, hipStream_t st);
hipError_t launch_radix_sort(uint64_t* keys_a, uint32_t* vals_a, uint64_t* keys_b, uint32_t* vals_b, long long n, int nbits,
                             uint32_t* table, hipStream_t st);
hipError_t launch_argmin(const double* dist, long long n, uint32_t* out_id, hipStream_t st);
hipError_t launch_segment_heads(const uint64_t* keys, long long n, uint32_t* heads, uint32_t* nseg, hipStream_t st);

// ---- RaBitQ -----------------------------------------------------------------
struct EncodeArgs {
    const float* rot;   // [n][d]
    long long n;
    int d, bits, rule;
    uint8_t* codes;     // record i at codes + i*code_stride
    long long code_stride;
    int code_bytes;     // d*bits/8
    int pad_to;         // bytes of the code area to zero-fill (>= code_bytes)
    uint8_t* meta;      // two floats of vector i at meta + i*meta_stride
    long long meta_stride;
    int meta_pad;       // bytes after the two floats to zero-fill
};

struct QueryPrepArgs {
    const float* rot;  // [nq][d] rotated, centred queries
    long long nq;
    int d, bits, qbits;
    uint8_t* qrecs;    // [nq][qrec_stride]: 16-byte header {lo, delta, query_add, query_sumq}, then planes
    long long qrec_stride;
    int plane_stride;  // bytes per plane (multiple of 16)
};

struct RerankArgs {
    DistSrc ds;              // recs = the float32 store, qrecs = the original queries
    long long nq;
    const uint32_t* cand;    // [nq][cand_stride] frontier ids (JX_NONE padded)
    int cand_stride, rr, k;
    uint32_t* out_ids;       // [nq][k]
    float* out_dist;
    unsigned long long* stats;  // the same stripes: [2] += number of vectors read
};

hipError_t launch_rotate(const void* in, int in_dtype, long long n, int d, const float* P, const float* c, float* out,
                         hipStream_t st);
hipError_t launch_encode(const EncodeArgs& a, hipStream_t st);
hipError_t launch_unpack_records(const uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off,
                                 uint8_t* codes, float* meta, int planar_bits, int plane_bytes, hipStream_t st);
hipError_t launch_planarize(uint8_t* recs, long long n, int code_stride, int code_bytes, int plane_bytes, int bits, hipStream_t st);
hipError_t launch_pack_records(uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off,
                               const uint8_t* codes, const float* meta, hipStream_t st);
hipError_t launch_code_sums(uint8_t* recs, long long n, int code_stride, int code_bytes, int meta_off, int bits, hipStream_t st);
hipError_t launch_query_prep(const QueryPrepArgs& a, hipStream_t st);
hipError_t launch_rerank(int dtype, const RerankArgs& a, hipStream_t st);
hipError_t launch_column_mean(const void* vecs, int dtype, long long n, int d, double* partial, float* mean, hipStream_t st);

// ---- batch deletion ---------------------------------------------------------
struct ConsolArgs {
    DistSrc ds;
    const uint32_t* adj;
    int R;
    long long n;
    const uint8_t* deleted;
    uint32_t* cnt;        // [n] candidates per vertex (0 = row untouched)
    const uint32_t* offs; // [v1 - v0] exclusive prefix of cnt over the slice
    long long v0, v1;     // vertex range of this slice
    uint64_t* keys;       // slice edge buffer
    uint32_t* vals;
    long long E;          // elements in the slice
};
hipError_t launch_mark_deleted(uint8_t* deleted, const uint32_t* ids, long long n, long long nvert, unsigned long long* counter, hipStream_t st);
hipError_t launch_consol_count(const ConsolArgs& a, hipStream_t st);
hipError_t launch_scan_u32(uint32_t* data, long long n, hipStream_t st);
hipError_t launch_consol_emit(const ConsolArgs& a, hipStream_t st);
hipError_t launch_consol_dist(int dtype, const ConsolArgs& a, uint64_t* keys_out, uint32_t* vals_out, hipStream_t st);
hipError_t launch_clear_deleted_rows(uint32_t* adj, int R, long long n, const uint8_t* deleted, hipStream_t st);
hipError_t launch_nearest_live(const void* vecs, int dtype, long long n, int d, uint32_t target, const uint8_t* deleted,
                               double* dist, uint32_t* out_id, hipStream_t st);

hipError_t launch_compact_flags(const uint32_t* adj, int R, long long n, const uint8_t* deleted, uint32_t* flag, uint32_t* err,
                                hipStream_t st);
hipError_t launch_compact_rename(uint32_t* adj, int R, long long n, const uint32_t* map, const uint8_t* deleted,
                                 uint32_t* public_map, hipStream_t st);
hipError_t launch_compact_records(uint8_t* base, int rec_bytes, long long n, const uint32_t* map, const uint8_t* deleted,
                                  uint8_t* staging, long long staging_bytes, hipStream_t st);

// ---- brute force ------------------------------------------------------------
struct BfArgs {
    const void* base;
    const void* queries;
    int dtype, d;
    long long n, nq;
    int k;
    int nsplit;
    uint32_t* norms;        // u8: [n] squared norms of the base vectors
    uint64_t* partial;      // [nq][nsplit][k]
    uint32_t* out_ids;
    float* out_dist;
};
hipError_t launch_bruteforce(const BfArgs& a, hipStream_t st);

// ---- small utilities ----------------------------------------------------------
hipError_t launch_fill_u32(uint32_t* p, long long n, uint32_t v, hipStream_t st);
hipError_t launch_mips_augment(const float* in, long long n, int dim, float max_norm, int is_query, float* out, int dim_out,
                               float* norm_out, hipStream_t st);
hipError_t launch_gather_probe(const uint8_t* table, int rec_bytes, const uint32_t* ids, long long n_ids, int blocks,
                               uint32_t* sink, hipStream_t st);
hipError_t launch_validate_adj(const uint32_t* adj, long long n, int R, uint32_t* bad, hipStream_t st);
hipError_t launch_row_degrees(const uint32_t* adj, long long n, int R, uint32_t* deg, hipStream_t st);

}  // namespace jx

// ---- the index object --------------------------------------------------------
struct jx_index {
    jx_params p;
    int64_t n;        // points stored and linked
    uint32_t entry;
    int vec_bytes;    // dim * element size
    // arena sub-buffers
    uint8_t* d_arena;
    int64_t arena_bytes;
    uint8_t* d_vecs;     // [capacity][vec_bytes]
    uint32_t* d_adj;     // [capacity][R]
    uint8_t* d_codes;    // [capacity][code_stride] RaBitQ records
    float* d_P;          // [dim][dim]
    float* d_centroid;   // [dim]
    uint8_t* d_work;     // workspace shared by the phases
    int64_t work_bytes;
    unsigned long long* d_stats;  // [8] = vertices marked deleted so far, [10] scratch of jx_import_graph
    unsigned long long* d_stripes;  // [64][16] search counters (BeamArgs::stats)
    uint8_t* d_deleted;  // [capacity] 1 = logically deleted
    uint8_t* d_clean;    // [capacity] see InsertArgs::clean
    int any_delete;      // a delete call has been made since the graph was created / imported
    uint32_t flags;      // JX_FLAG_* switches (jx_params.flags, jx_set_flags)
    // RaBitQ state
    int quantized;    // 0 or bits
    int qbits, rule;
    int code_bytes;   // dim*bits/8
    int meta_chunk;   // chunks of code planes in front of the meta chunk
    int plane_chunks; // chunks per code plane
    int plane_shift;  // log2 weight of the high plane (2- and 8-bit codes), else 0
    int code_stride;  // (meta_chunk+1)*16
};
