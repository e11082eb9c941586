/*
 * lychee.h -- C ABI of the LycheeCluster decode hot path for AMD MI355X (gfx950).
 *
 * The library implements, as hand-written HIP kernels, the decode-time path of
 * the LycheeCluster method: a hierarchical index over variable-length KV chunks
 * (Section 4.1, 4.3), retrieval with the triangle-inequality score bound
 * (Eq. 2; Algorithm 1 steps 1-2), exact attention over the retrieved chunks
 * (Eq. 1; Algorithm 1 step 3) and the lazy index update for streamed tokens
 * (Section 4.4; Algorithm 1 step 4).
 *
 * Conventions
 *   - Plain C.  Every call returns an int: LC_OK (0) or a negative LC_ERR_*.
 *     Nothing throws.  Host-side argument errors are detected before any GPU
 *     work is enqueued and leave all buffers untouched.
 *   - Pointers are DEVICE pointers unless marked "host".  The library never
 *     allocates or frees device memory: the caller provides the index buffer
 *     and a workspace, sized by lc_index_bytes() / lc_workspace_bytes().
 *   - All GPU work is enqueued on the caller's stream (a hipStream_t passed as
 *     void*, NULL = the default stream) and is asynchronous.  Calls on the same
 *     index must be stream-ordered; two calls that overlap on one index race.
 *   - Shapes: B sequences, H_q query heads, H_kv KV heads, G = H_q / H_kv
 *     (1 <= G <= 8), head dimension d = 128.  Query head hq uses KV head hq / G.
 *   - q, k, v are bfloat16; K and V caches are bfloat16 [B][H_kv][tokens][d]
 *     addressed through element strides {sequence, head, token} with d
 *     contiguous; outputs are float32.
 *   - Levels: level 0 = chunks, level L-1 = top.  `fanout` F is the average
 *     number of children: level l+1 has ceil(N_l / F) nodes.
 *   - A chunk id is the chunk's position in its sequence's boundary list.
 */
#ifndef LYCHEE_H
#define LYCHEE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LC_MAX_LEVELS 6
#define LC_MAX_GROUP 8
#define LC_HEAD_DIM 128

enum {
    LC_OK = 0,
    LC_ERR_INVALID_ARG = -1,          /* null pointer, negative size, unknown enum value   */
    LC_ERR_BAD_SHAPE = -2,            /* d != 128, H_q not a multiple of H_kv, G > 8, ...  */
    LC_ERR_WORKSPACE_TOO_SMALL = -3,  /* index buffer or workspace smaller than required   */
    LC_ERR_CAPACITY = -4,             /* max_chunks / max_tokens / id capacity exceeded    */
    LC_ERR_HIP = -5,                  /* a HIP runtime call failed (see lc_last_hip_error) */
    LC_ERR_BAD_BLOB = -6              /* lc_index_import: malformed or mismatching blob    */
};

/* How a node's (center, radius) is stored.
 * TOKEN_BALL: a chunk's center is its mean key and its radius covers the chunk's
 *   token keys, so Eq. 2 bounds every token logit beneath a node.
 * PAPER_UNIT: the literal representative of Section 4.1: the mean key projected
 *   onto the unit sphere, radius 0; internal centers are spherical centroids. */
enum { LC_GEOMETRY_TOKEN_BALL = 0, LC_GEOMETRY_PAPER_UNIT = 1 };

/* EXACT: the selection equals a flat scan over all chunks; subtrees are pruned
 *   only when Eq. 2 proves they cannot reach the cutoff.
 * BEAM: Algorithm 1's top-k per level (beam[l] nodes kept at level l). */
enum { LC_POLICY_EXACT = 0, LC_POLICY_BEAM = 1 };

/* EXACT only: whether the level-by-level pruning pass runs before the chunks are
 * scored.  The selection is the same either way (it is defined as the flat scan);
 * the pass costs a chain of dependent memory round trips in one workgroup per
 * (sequence, head) and pays off only when it removes most of a very large chunk
 * level -- with an 8 TB/s memory the flat scan was faster in every case measured,
 * up to 300 MB of chunk centers.  AUTO runs the pass when the chunk-level index
 * of the whole batch exceeds LC_PRUNE_AUTO_BYTES.  BEAM always walks the levels. */
enum { LC_PRUNE_AUTO = 0, LC_PRUNE_ALWAYS = 1, LC_PRUNE_NEVER = 2 };
#define LC_PRUNE_AUTO_BYTES (1u << 30)

/* How the centers of the chunk level (level 0) are stored.  The chunk level is almost the whole
 * index (N_0 nodes against N_0 / F above it) and every decode step reads all of it.
 * F32: float32 values.
 * BF16: rounded to the nearest bfloat16 (ties to even) when the chunk is pooled; its radius, the
 *   direction used for clustering and everything above it are then computed from the rounded
 *   center, so the covering property of the radii (and with it Eq. 2) holds for the stored
 *   values.  Halves the bytes of the chunk level.  The levels above keep float32: their centers
 *   are running means that the lazy update (Section 4.4) moves by small steps. */
enum { LC_CENTER_F32 = 0, LC_CENTER_BF16 = 1 };

typedef struct lc_config {
    int32_t levels;                 /* L >= 1, counts the chunk level (paper: 3)            */
    int32_t fanout;                 /* F >= 1                                               */
    int32_t kmeans_iters;           /* spherical k-means iterations (Appendix A: 10)        */
    int32_t geometry;               /* LC_GEOMETRY_*                                        */
    int32_t policy;                 /* LC_POLICY_*                                          */
    int32_t beam[LC_MAX_LEVELS];    /* BEAM: nodes kept per level; <= 0 means no limit.
                                       beam[0] limits the number of chunks returned.        */
    int32_t sink_tokens;            /* leading chunks covering this many tokens are always
                                       attended, never scored, not charged to the budget    */
    int32_t max_chunks;             /* capacity: closed chunks per sequence                 */
    int32_t max_tokens;             /* capacity: tokens per sequence (rows of K and V)      */
    int32_t decode_splits;          /* split-K factor of the attention kernel; 0 = auto     */
    int32_t prune;                  /* LC_PRUNE_*                                           */
    int32_t center_dtype;           /* LC_CENTER_*: storage of the chunk-level centers      */
    int32_t fanouts[LC_MAX_LEVELS]; /* fanouts[l], l >= 1: average children of a level-l node,
                                       i.e. level l has ceil(N_{l-1} / fanouts[l]) nodes;
                                       0 = use `fanout`.  The paper's three tiers are e.g.
                                       {0, 2, 22}: 2 chunks per fine cluster, 22 fine
                                       clusters per coarse unit (Appendix A)                */
} lc_config;

typedef struct lc_index lc_index;   /* opaque host-side handle */

/* Fill *cfg with defaults: levels 3, fanout 16, kmeans_iters 10, TOKEN_BALL,
 * EXACT, no beam limits, sink 0, prune AUTO, float32 centers, capacities 0 (the caller must
 * set them). */
void lc_config_default(lc_config* cfg /* host */);

/* Text for an error code (static storage). */
const char* lc_strerror(int code);

/* The last hipError_t seen by a failing call on this thread, as text. */
const char* lc_last_hip_error(void);

/* Bytes of device memory an index needs for B sequences (pure host function;
 * 0 on invalid arguments). */
size_t lc_index_bytes(const lc_config* cfg /* host */, int B, int H_kv, int d);

/* Bytes of workspace sufficient for lc_build_index, lc_retrieve,
 * lc_sparse_decode and lc_append on such an index (pure host function; 0 on
 * invalid arguments).  The workspace holds no state between calls. */
size_t lc_workspace_bytes(const lc_config* cfg /* host */, int B, int H_q, int H_kv, int d);

/*
 * lc_build_index -- index construction at prefill (Section 4.3).
 * Per (sequence, KV head): mean-pools the keys of every chunk (representative
 * key, Section 4.1), then builds levels-1 rounds of spherical k-means
 * (inner-product similarity, cfg->kmeans_iters iterations, k = ceil(N/F),
 * centroid c starts at point floor(c*N/k), ties to the lower id, an empty
 * cluster keeps its centroid) over the unit directions of the level below; each
 * node stores a center and a radius covering all descendant chunks' balls.
 *
 *   out           host: receives the new handle (destroy with lc_index_destroy)
 *   K             bf16 key cache, k_strides = {sequence, head, token} in elements
 *   seq_lens      host int32[B]: tokens written per sequence (<= cfg->max_tokens)
 *   chunk_bounds  host int32: per sequence, chunk_counts[b]+1 ascending boundaries
 *                 starting at 0 and ending <= seq_lens[b], concatenated over b;
 *                 tokens after the last boundary form the open tail (attended,
 *                 not indexed).  Boundaries are shared by all heads.
 *   chunk_counts  host int32[B]: closed chunks per sequence (<= cfg->max_chunks)
 *   index_buf     device buffer of >= lc_index_bytes() bytes, 256-byte aligned,
 *                 owned by the caller, must outlive the handle
 *   ws            device workspace of >= lc_workspace_bytes() bytes
 *
 * Asynchronous: the host arrays are copied (into pinned staging memory the library keeps per
 * device for the life of the process) before the call returns, the stream is not waited for.
 * Not meant for stream capture: the host arrays are read when the call is made, not when a
 * captured graph is replayed.
 */
int lc_build_index(lc_index** out, const lc_config* cfg,
                   const void* K, const int64_t k_strides[3],
                   const int32_t* seq_lens, const int32_t* chunk_bounds, const int32_t* chunk_counts,
                   int B, int H_kv, int d,
                   void* index_buf, size_t index_bytes, void* ws, size_t ws_bytes, void* stream);

/*
 * lc_recluster -- global re-clustering against drift (the remedy the paper's limitations
 * section proposes for long generations: the lazy update only ever attaches chunks to existing
 * nodes and lets radii grow).  Keeps the chunk nodes (level 0) as they are and rebuilds every
 * level above them exactly as lc_build_index does -- ceil(N/F) clusters per level for the
 * current chunk counts, the same k-means -- so the result equals lc_build_index on the whole
 * sequence as it now stands.  K and V are not read.  Asynchronous like lc_build_index.  Same
 * workspace size as lc_build_index.
 */
int lc_recluster(lc_index* idx, void* ws, size_t ws_bytes, void* stream);

/*
 * lc_index_drift -- how far the lazy update has inflated the radii of one internal level since the
 * index was built, imported or last re-clustered (the paper's limitations section: re-cluster
 * "when radii inflate").  Per (sequence, head), over the nodes that held chunks at that time:
 *   drift[(b * H_kv + h) * 4 + 0]   sum of those nodes' radii then
 *   drift[... + 1]                  sum of their radii now (never smaller: radii only grow)
 *   drift[... + 2]                  largest growth of a single node
 *   drift[... + 3]                  number of nodes counted
 * A caller triggers lc_recluster when sum now > (1 + tau) * sum then (tau 0.25 is a reasonable
 * start: the Eq. 2 bounds of that level have then loosened by a quarter on average).
 *   level   1 <= level < cfg.levels
 *   drift   host float[B * H_kv * 4]
 *   ws      device workspace of at least B * H_kv * 16 bytes (any lc_workspace_bytes() buffer does)
 * Synchronises the stream (the result is copied to the host).
 */
int lc_index_drift(const lc_index* idx, int level, float* drift /* host */, void* ws, size_t ws_bytes, void* stream);

/* Change the retrieval policy of an existing index (host state only). */
int lc_set_policy(lc_index* idx, int policy, const int32_t* beam /* host, LC_MAX_LEVELS, may be NULL */,
                  int sink_tokens);
/* Change the pruning mode (LC_PRUNE_*) of an existing index (host state only). */
int lc_set_prune(lc_index* idx, int prune);

/*
 * lc_retrieve -- hierarchical retrieval for one decode step (Eq. 2, Algorithm 1
 * steps 1-2).  Per (sequence, KV head) every node u gets the group score
 *   s(u) = max over the G query heads of (q_g . mu_u + |q_g| r_u) / sqrt(d);
 * chunks are ordered by (score descending, id ascending) and the longest prefix
 * whose token total is <= budget is returned, ids ascending.  EXACT prunes a
 * subtree only if its bound is below a proven lower bound of the cutoff, so the
 * result equals the flat scan; BEAM keeps beam[l] nodes per level.
 *
 *   q          bf16 [B][H_q][d]
 *   chunk_ids  int32 [B][H_kv][cap]  (entries past counts[] are unspecified)
 *   counts     int32 [B][H_kv]
 *   scores     optional float32 [B][H_kv][cfg.max_chunks]: chunk scores; -inf for
 *              chunks that were pruned or pinned.  May be NULL.
 *   cap        ids capacity per (sequence, head); must be >= min(chunks, budget +
 *              sink chunks) for every sequence, else LC_ERR_CAPACITY
 */
int lc_retrieve(const lc_index* idx, const void* q, int H_q, int budget,
                int32_t* chunk_ids, int32_t* counts, float* scores, int cap,
                void* ws, size_t ws_bytes, void* stream);

/*
 * lc_sparse_decode -- exact attention over the retrieved chunks (Eq. 1 restricted
 * to the active set; Algorithm 1 step 3), as a split-K flash-decode followed by a
 * log-sum-exp merge.  The active set of (b, h) is the listed chunks plus the open
 * tail.  Logits q.k/sqrt(d), bf16 inputs, float32 accumulation.
 *
 *   chunk_ids, counts, cap   as produced by lc_retrieve (ids ascending, distinct)
 *   out        float32 [B][H_q][d]; an empty active set gives 0
 *   lse        optional float32 [B][H_q]: ln sum exp(logit); -inf if empty
 * One (sequence, head) slab of the cache must span less than 2 GiB
 * (cfg.max_tokens * kv_strides[2] * 2 bytes), else LC_ERR_BAD_SHAPE.
 */
int lc_sparse_decode(const lc_index* idx, const void* q, const void* K, const void* V,
                     const int64_t kv_strides[3],
                     const int32_t* chunk_ids, const int32_t* counts, int cap, int H_q,
                     float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/*
 * lc_decode_step -- lc_retrieve followed by lc_sparse_decode in one call (Algorithm 1
 * steps 1-3; Eq. 2 scoring, budgeted selection, Eq. 1 over the active set), for
 * callers that do not need the chunk list between the two.  Same selection (bit
 * for bit) and same attention result as the two calls.  The chunk score keys go
 * from the scoring kernel to the attention kernel through the workspace; every
 * workgroup of the attention kernel repeats the selection of its (sequence,
 * head) from them, so no chunk list travels through memory on the critical path.
 * When a sequence has more than 4096 chunks, the chunks no longer fit the registers of
 * the selecting workgroups and the call runs the kernels of the two separate entry
 * points instead (through a chunk list in the workspace); so it does under the BEAM
 * policy, whose selection needs the kept set of every level.  The results are the same.
 *
 *   chunk_ids, counts  optional outputs as in lc_retrieve (both or neither); cap
 *                      is checked only when they are given
 *   everything else    as in lc_retrieve / lc_sparse_decode
 */
int lc_decode_step(const lc_index* idx, const void* q, const void* K, const void* V,
                   const int64_t kv_strides[3], int H_q, int budget,
                   float* out, float* lse, int32_t* chunk_ids, int32_t* counts, int cap,
                   void* ws, size_t ws_bytes, void* stream);

/*
 * lc_decode_step_static -- lc_decode_step for callers that cannot allocate device memory or
 * pass a workspace: code that runs under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, checks, kernels and results as lc_decode_step, except that
 * the step's workspace (chunk score keys, kept flags, select staging, chunk list, split-K
 * partials) lives in a device array of LC_STATIC_SCRATCH_BYTES that is part of the library image:
 * every GPU the library runs on holds one copy until the process ends.  The call allocates and
 * frees nothing.  LC_ERR_CAPACITY (nothing enqueued) if the step needs more than that, i.e. if
 * lc_decode_workspace_bytes(cfg, B, H_q, H_kv, d) > LC_STATIC_SCRATCH_BYTES.
 * All calls on one GPU share that GPU's array: two calls that overlap on one GPU (different
 * streams, or different indices) race; stream-ordered calls are fine, nothing in the array has to
 * survive from one call to the next and nothing in it has to be cleared by the caller.
 */
#define LC_STATIC_SCRATCH_BYTES (16u << 20)
int lc_decode_step_static(const lc_index* idx, const void* q, const void* K, const void* V,
                          const int64_t kv_strides[3], int H_q, int budget,
                          float* out, float* lse, int32_t* chunk_ids, int32_t* counts, int cap,
                          void* stream);
/* Bytes of workspace one decode step (lc_retrieve, lc_sparse_decode, lc_decode_step) uses: the
 * part of lc_workspace_bytes() without the scratch of lc_build_index / lc_recluster (pure host
 * function; 0 on invalid arguments). */
size_t lc_decode_workspace_bytes(const lc_config* cfg /* host */, int B, int H_q, int H_kv, int d);
/* LC_STATIC_SCRATCH_BYTES as the loaded library was built with. */
size_t lc_static_workspace_bytes(void);

/*
 * lc_append -- lazy update for one streamed token per sequence (Section 4.4,
 * Algorithm 1 step 4).  Writes k_new/v_new at row T_b of K and V and advances
 * T_b.  Where close_chunk[b] != 0 the open tail (including the new token) becomes
 * chunk M_b: it is attached to the level-1 node of nearest direction (largest
 * inner product of unit directions, ties to the lower id); that node and its
 * ancestors take the count-weighted moving average of the new center, and their
 * radii grow monotonically (by the centroid shift, and to cover the new chunk).
 *
 *   k_new, v_new   bf16 [B][H_kv][d]
 *   close_chunk    host uint8[B] (the caller's boundary decision); NULL = none
 * Returns LC_ERR_CAPACITY (nothing enqueued) if a sequence is at max_tokens, or
 * would exceed max_chunks.
 * The handle keeps host-side counts of tokens and chunks that every call updates: a captured
 * graph that replays lc_append leaves them behind (the kernel itself never writes past the
 * capacities), so append outside graphs or rebuild the handle's view with lc_index_export/import.
 */
int lc_append(lc_index* idx, void* K, void* V, const int64_t kv_strides[3],
              const void* k_new, const void* v_new, const uint8_t* close_chunk,
              void* ws /* unused, may be NULL */, size_t ws_bytes, void* stream);

/* Sizes the two level walks are limited to (pure host function; either pointer may be NULL).
 *   exact_walk_internal_nodes   EXACT with the level walk on: internal nodes (all levels above the
 *                               chunks together) of one (sequence, head); the walk keeps them in LDS.
 *                               Beyond it LC_PRUNE_ALWAYS gives LC_ERR_CAPACITY and LC_PRUNE_AUTO
 *                               scans flat (same selection).  A flat scan has no such limit.
 *   beam_level_nodes            BEAM: nodes of one internal level of one (sequence, head); beyond it
 *                               lc_retrieve / lc_decode_step give LC_ERR_CAPACITY. */
void lc_walk_limits(int32_t* exact_walk_internal_nodes, int32_t* beam_level_nodes);

/* Host-side view of the index state: tokens, closed chunks and level sizes of
 * sequence b (n_per_level: host int32[LC_MAX_LEVELS], may be NULL). */
int lc_index_info(const lc_index* idx, int b, int32_t* T, int32_t* M, int32_t* n_per_level);

/*
 * Export / import of the stored index as a flat little-endian host blob, so that
 * a CPU reference and the GPU can run on the identical stored values.
 *   int32 header[16] = {magic 'LCIX', version 1, B, H_kv, d, L, F, geometry, center_dtype,
 *                       fanouts[1..5] (0 = F), 0...}
 *   per sequence b:    int32 T_b, M_b, N_1..N_{L-1};  int32 bounds[M_b+1]
 *   per (b, h, level): float32 center[N_l][d], float32 radius[N_l],
 *                      int32 parent[N_l], int32 ntok[N_l], int32 nchunk[N_l]
 * Centers are float32 in the blob whatever center_dtype says (bfloat16 values widened); import
 * requires the blob's L, fan-outs, geometry and center_dtype to equal the configuration's.
 * lc_index_export and lc_index_import synchronise the stream (import copies with blocking
 * copies; it is a test and checkpoint path, not a hot one).  With blob == NULL export only
 * stores the required size in *bytes.
 */
int lc_index_export(const lc_index* idx, void* blob /* host */, size_t* bytes /* host, in/out */, void* stream);
int lc_index_import(lc_index** out, const lc_config* cfg, const void* blob /* host */, size_t blob_bytes,
                    void* index_buf, size_t index_bytes, void* stream);

void lc_index_destroy(lc_index* idx);

/*
 * lc_chunk_tokens -- structure-aware chunk boundaries for a token stream
 * (Section 4.3 "Structure-Aware Chunking", Appendix B separator table).  Host
 * routine, no GPU work: its output is the chunk_bounds argument of
 * lc_build_index and decides the close_chunk bits of lc_append.
 * Tokens are accumulated greedily; once a chunk holds min_len tokens the
 * delimiter of strongest level among its tokens min_len..max_len ends the chunk
 * (the earliest one of that level); with no delimiter the chunk ends at max_len
 * tokens.  The last chunk of the text may be shorter than min_len.
 * A token's level comes from the end of its text, trailing blanks and tabs
 * ignored for levels 1-3:
 *   1  contains a blank line, "---", "***" or a code fence, or ends in } ] >
 *   2  contains a newline, or ends in . ? ! or their full-width forms
 *   3  ends in , ; : or their full-width forms or the ideographic comma
 *   4  ends in a blank or tab
 *
 *   text     host: the tokens' UTF-8 bytes, concatenated
 *   offsets  host int64[n+1]: token i is text[offsets[i] .. offsets[i+1])
 *   n        number of tokens (0 allowed)
 *   bounds   host int32[capacity] out: b_0 = 0 < ... < b_M = n
 *   n_chunks host out: M
 * Returns LC_ERR_INVALID_ARG for NULL pointers, min_len < 1, max_len < min_len or
 * decreasing offsets; LC_ERR_CAPACITY if capacity < M + 1 (nothing useful is
 * left in bounds then; capacity n + 1 always suffices).
 */
int lc_chunk_tokens(const char* text, const int64_t* offsets, int n, int min_len, int max_len,
                    int32_t* bounds, int capacity, int* n_chunks);

#ifdef __cplusplus
}
#endif
#endif /* LYCHEE_H */
