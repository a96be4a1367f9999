/*
 * rc.h -- C ABI of the reusable-KV-block search (ReasonCache, Sec. IV-A Stage 2
 * "Block-Level Distance Filtering" and Sec. IV-B "Zero-Copy KV Sharing").
 *
 * Newly written, sealed paged-KV blocks ("query blocks", the blocks B_c of the
 * current step) are scored layer by layer against the resident blocks of the
 * cache ("pool blocks", the candidates B_k).  A query block whose best pool
 * partner clears the reuse threshold is redirected to that partner in the
 * PagedAttention block table; no KV data is copied.
 *
 * Conventions shared by every entry point
 *   - "DEVICE" pointers are HIP device memory on the current device; "HOST"
 *     pointers are ordinary host memory.  The caller owns every buffer.  The
 *     library allocates nothing, frees nothing and never synchronises: all
 *     work is enqueued on the caller's stream (`hip_stream` is a hipStream_t,
 *     NULL = the default stream).
 *   - Arguments are validated on the host before anything is launched; on an
 *     error the outputs are untouched, the return code says what kind of
 *     error it was and rc_last_error() returns a description.
 *   - [L] is a pure batch dimension: every layer is an independent problem
 *     with its own pool, queries, decisions, block tables and refcounts.
 *   - KV layout: element (layer l, block b, token t, head h, dim d) of a K (or
 *     V) tensor sits at  l*layer_stride + ((b*T + t)*H + h)*Dh + d  elements
 *     from the base pointer.  K and V are separate tensors.  Base pointers and
 *     layer strides must keep every block 16-byte aligned.
 *   - Supported shapes: head_dim == 128, block_tokens in {16, 32},
 *     1 <= n_kv_heads <= 16, dtype fp16 or bf16.
 */
#ifndef RC_H_
#define RC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  RC_OK = 0,
  RC_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned pointer, mismatching descriptors */
  RC_ERR_UNSUPPORTED = 2, /* shape, dtype or mode outside the supported set                           */
  RC_ERR_WORKSPACE = 3,   /* workspace missing or smaller than rc_*_workspace_size() asks             */
  RC_ERR_DEVICE = 4       /* the HIP runtime refused a launch                                         */
} rc_status;

typedef enum { RC_F16 = 0, RC_BF16 = 1 } rc_dtype;

typedef enum {
  RC_SCORE_BLOCK = 0,       /* one score per block pair over the flattened [T][H][Dh] tensor   */
  RC_SCORE_PER_HEAD_ALL = 1 /* score per KV head on its [T][Dh] slice, block score = min over  */
                            /* heads: a block is shared only if every head clears the threshold */
} rc_mode;

/* Shape of one K (or V) tensor.  HOST struct, read during the call only. */
typedef struct {
  int32_t n_layers;     /* L  */
  int32_t block_tokens; /* T, the paper's block size d                  */
  int32_t n_kv_heads;   /* H, the paper's h                             */
  int32_t head_dim;     /* Dh                                           */
  int32_t dtype;        /* rc_dtype                                     */
  int64_t layer_stride; /* elements between layer l and l+1 of a tensor */
} rc_kv_desc;

/*
 * Squared L2 norm of every K block and every V block (Sec. IV-A Stage 2, the
 * norm terms of the squared-distance expansion ||x_c||^2 + ||x_k||^2 - 2 x_c.x_k;
 * the paper computes them once per block by a single reduction and caches them).
 *
 *   k, v            DEVICE, n_blocks blocks per layer in the KV layout above
 *   k_sqnorm,       DEVICE float, [L][n_blocks] in RC_SCORE_BLOCK mode,
 *   v_sqnorm        [L][n_blocks][H] in RC_SCORE_PER_HEAD_ALL mode (norm of the head's
 *                   [T][Dh] slice).  Products are exact in fp32; the sum is an fp32 tree.
 * n_blocks == 0 is legal and launches nothing.
 */
rc_status rc_block_norms(const rc_kv_desc* desc, int32_t mode,
                         const void* k, const void* v, int64_t n_blocks,
                         float* k_sqnorm, float* v_sqnorm, void* hip_stream);

/* Bytes of DEVICE workspace rc_match_blocks needs for this problem (0 on bad arguments).
 * 16 bytes per (layer, pool tile of 256 blocks, query block).  A problem of at most 256 tiles of
 * 256 x 256 blocks (one layer at a time, a small pool) may instead be computed as several shares
 * per tile (parts of the reduction, or heads in per-head mode) and then needs up to 512 MB: 256 KB
 * per share plus the 16-byte partials.  The size depends on the arguments only, not on the
 * current device. */
size_t rc_match_workspace_size(const rc_kv_desc* qdesc, int32_t mode, int64_t Q, int64_t P);

/*
 * Score every query block against every live pool block of its layer and pick
 * the best partner (Sec. IV-A Stage 2: the dot-product term of the expansion
 * with the cached norms; the sharing decision against a threshold).
 *
 * Score of a pair, RC_SCORE_BLOCK:  s = (cos(Kq,Kp) + cos(Vq,Vp)) / 2  on the
 * flattened tensors, cos = <x,y>/sqrt(|x|^2 |y|^2), defined 0 when a norm is 0.
 * K and V are normalised separately and averaged, as the paper sums the K and V
 * distances.  For unit vectors |x-y|^2 = 2 - 2cos, so a cosine threshold tau is
 * the threshold sqrt(2 - 2 tau) on the normalised Euclidean distance.
 * RC_SCORE_PER_HEAD_ALL: the same on each head's [T][Dh] slice, then the minimum
 * over heads.
 *
 *   qdesc, pdesc    HOST; must agree in everything but layer_stride
 *   kq, vq          DEVICE, Q query blocks per layer;  kp, vp: P pool blocks per layer
 *   q_ksq .. p_vsq  DEVICE float, squared norms as rc_block_norms writes them for `mode`
 *   pool_live       DEVICE uint8 [L][P], 1 = sealed and referenced (eligible target);
 *                   dead blocks are skipped by the argmax.  NULL = all live.
 *   tau             reuse threshold on the score; a query matches iff best_score >= tau
 *   best_idx        DEVICE int32 [L][Q]: argmax over live pool blocks, lowest index on
 *                   exact ties; -1 if the layer has no live pool block
 *   best_score      DEVICE float [L][Q]: its score (-inf if none)
 *   match_idx       DEVICE int32 [L][Q]: best_idx if best_score >= tau, else -1
 *   second_score    DEVICE float [L][Q] or NULL: second-largest score over live pool
 *                   blocks, counted with multiplicity (-inf if fewer than two)
 *   workspace       DEVICE, >= rc_match_workspace_size() bytes, 16-byte aligned; contents
 *                   are scratch.  Calls that share a workspace must not overlap.
 * Accumulation is fp32 on the matrix cores, the epilogue is fp32.  In RC_SCORE_PER_HEAD_ALL
 * mode every head's score is rounded to the nearest multiple of 1/32767 before the minimum over
 * heads is taken (the running minimum is held as 16-bit fixed point next to the accumulators), so
 * reported scores of that mode are multiples of 1/32767 (error <= 1.6e-5; an exact duplicate still
 * scores exactly 1; pairs closer than that tie and go to the lower index).  The same pair reports
 * the same bits whatever the number of layers or tiles of the call.
 * Q == 0 launches nothing; P == 0 writes -1 / -inf.
 */
rc_status rc_match_blocks(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode,
                          const void* kq, const void* vq, int64_t Q,
                          const float* q_ksq, const float* q_vsq,
                          const void* kp, const void* vp, int64_t P,
                          const float* p_ksq, const float* p_vsq,
                          const uint8_t* pool_live, float tau,
                          int32_t* best_idx, float* best_score, int32_t* match_idx,
                          float* second_score,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of DEVICE workspace rc_remap_block_table needs (0 on bad arguments). */
size_t rc_remap_workspace_size(int32_t n_layers, int64_t R, int64_t E, int64_t Q, int64_t NB);

/*
 * Apply the sharing decisions to the block tables without copying KV data
 * (Sec. IV-B: sharing raises the kept block's reference count and rewrites the
 * block-table entry; a block returns to the free pool only at reference count 0).
 * The resident pool block survives, the new query block is released; pool blocks
 * are never redirected, so there are no redirect chains.
 *
 * Per layer l:  every table entry equal to query_ids[q] with match_idx[l][q] = m >= 0
 * becomes target(m) = pool_ids ? pool_ids[m] : m.  With cnt[q] the number of such
 * entries:  refcount[target(m)] += cnt[q],  refcount[query_ids[q]] -= cnt[q],
 * freed[l][q] = 1 iff q matched and its refcount reached 0.  All other entries and
 * refcounts are copied unchanged.  n_remapped[l] = number of entries rewritten.
 *
 *   tables_in/out   DEVICE int32 [L][R][E]; tables_out may be tables_in (in place).
 *                   Entries outside [0, NB) (e.g. -1 padding) pass through unchanged.
 *   query_ids       DEVICE int32 [Q], distinct physical block ids in [0, NB), same for all layers
 *   pool_ids        DEVICE int32 [P] physical ids in [0, NB), disjoint from query_ids; NULL = identity (then P <= NB)
 *   match_idx       DEVICE int32 [L][Q], values in [-1, P) (others are treated as -1)
 *   refcount_in/out DEVICE int32 [L][NB]; refcount_out may be refcount_in
 *   freed           DEVICE uint8 [L][Q];  n_remapped: DEVICE int32 [L]
 *   workspace       DEVICE, >= rc_remap_workspace_size() bytes, 16-byte aligned
 * No atomics are used: the result is the same on every run.  Q is limited to 8192.
 */
rc_status rc_remap_block_table(int32_t n_layers,
                               const int32_t* tables_in, int32_t* tables_out,
                               int64_t R, int64_t E,
                               const int32_t* query_ids, const int32_t* pool_ids,
                               const int32_t* match_idx, int64_t Q, int64_t P, int64_t NB,
                               const int32_t* refcount_in, int32_t* refcount_out,
                               uint8_t* freed, int32_t* n_remapped,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of the library's built-in scratch buffer behind rc_remap_block_table_static. */
#define RC_REMAP_STATIC_SCRATCH_BYTES (4u << 20)
size_t rc_remap_static_scratch_size(void);

/*
 * rc_remap_block_table for callers that cannot allocate or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results; the scratch memory is a buffer of
 * RC_REMAP_STATIC_SCRATCH_BYTES (4 MiB) that is part of the library's device code, one copy per
 * GPU, held until the process ends.  The call allocates and frees nothing and does not synchronise.
 * A problem whose rc_remap_workspace_size() exceeds the buffer is refused with RC_ERR_WORKSPACE
 * before anything is launched (the five benchmark workloads need at most 3.3 MB).  Every call on
 * one GPU uses that GPU's buffer: calls on the same GPU must not overlap in time (on different
 * streams, or from different threads), or they race on it.  No part of the buffer has to be
 * cleared between calls: the kernels validate or overwrite everything they read from it.
 */
rc_status rc_remap_block_table_static(int32_t n_layers,
                                      const int32_t* tables_in, int32_t* tables_out,
                                      int64_t R, int64_t E,
                                      const int32_t* query_ids, const int32_t* pool_ids,
                                      const int32_t* match_idx, int64_t Q, int64_t P, int64_t NB,
                                      const int32_t* refcount_in, int32_t* refcount_out,
                                      uint8_t* freed, int32_t* n_remapped, void* hip_stream);

/*
 * Candidate-restricted scoring: Stage 2 in the shape the paper runs it (Sec. IV-A:
 * only the blocks of the steps that Stage 1 flagged are compared; k candidates per
 * step with k << m in the complexity analysis).  Every listed pair gets the same
 * score as in rc_match_blocks; nothing else is read.  HBM bound: one pool block
 * (2*T*H*Dh*2 bytes) per listed pair.
 *
 *   cand            DEVICE int32 [L][Q][C]: pool index, or -1 for an empty slot.  Entries
 *                   outside [0, P) and dead blocks score -inf.
 *   scores          DEVICE float [L][Q][C]
 *   best_idx        DEVICE int32 [L][Q]: candidate with the highest score, equal scores to
 *                   the lowest pool index; -1 if the list has no valid entry
 *   best_score      DEVICE float [L][Q] (-inf if none);  match_idx: best_idx if >= tau else -1
 * Everything else as in rc_match_blocks.  C == 0 writes -1 / -inf.
 */
rc_status rc_score_candidates(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode,
                              const void* kq, const void* vq, int64_t Q,
                              const float* q_ksq, const float* q_vsq,
                              const void* kp, const void* vp, int64_t P,
                              const float* p_ksq, const float* p_vsq,
                              const uint8_t* pool_live, const int32_t* cand, int64_t C, float tau,
                              float* scores, int32_t* best_idx, float* best_score, int32_t* match_idx,
                              void* hip_stream);

/* Bytes of DEVICE workspace rc_match_blocks_layer_mean needs (0 on bad arguments). */
size_t rc_layer_mean_workspace_size(const rc_kv_desc* qdesc, int64_t Q, int64_t P);

/*
 * The paper's own Stage 2 measure and decision (Sec. IV-A, the per-layer K and V distance
 * equations and the block-distance equation): per layer i the Euclidean distances
 * dK_i = |K_i[q] - K_i[p]| and dV_i = |V_i[q] - V_i[p]| of the flattened tensors, through the
 * expansion |x-y|^2 = |x|^2 + |y|^2 - 2 x.y with the cached squared norms, and
 *
 *     dist(q, p) = (1/L) * sum_i (dK_i + dV_i) / (2 * T * H).
 *
 * One decision per query block, shared by all layers (a layer-shared block table, as
 * PagedAttention keeps it): the nearest live pool block, match iff dist <= threshold.
 * Apply it with rc_remap_block_table(n_layers = 1, ...).
 *
 *   q_ksq .. p_vsq  DEVICE float [L][Q] / [L][P], squared norms of rc_block_norms in RC_SCORE_BLOCK mode
 *   pool_live       DEVICE uint8 [P] (one flag per block, all layers), NULL = all live
 *   threshold       on dist, e.g. the percentile rc_pat_threshold returns
 *   best_idx        DEVICE int32 [Q]: argmin over live pool blocks, lowest index on exact ties, -1 if none
 *   best_dist       DEVICE float [Q] (+inf if none);  match_idx: best_idx if best_dist <= threshold else -1
 *   second_dist     DEVICE float [Q] or NULL: second-smallest distance, with multiplicity (+inf if fewer than two)
 *   workspace       DEVICE, >= rc_layer_mean_workspace_size() bytes, 16-byte aligned, scratch
 * fp32 throughout; a radicand that rounding pushes below 0 is clamped to 0.  n_layers must be
 * >= 1 (RC_ERR_INVALID_ARG otherwise); Q == 0 launches nothing; P == 0 writes -1 / +inf.
 */
rc_status rc_match_blocks_layer_mean(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc,
                                     const void* kq, const void* vq, int64_t Q,
                                     const float* q_ksq, const float* q_vsq,
                                     const void* kp, const void* vp, int64_t P,
                                     const float* p_ksq, const float* p_vsq,
                                     const uint8_t* pool_live, float threshold,
                                     int32_t* best_idx, float* best_dist, int32_t* match_idx,
                                     float* second_dist,
                                     void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of DEVICE workspace rc_candidate_distances needs (0 on bad arguments). */
size_t rc_candidate_distances_workspace_size(const rc_kv_desc* qdesc, int64_t Q, int64_t C);

/*
 * Stage 2 exactly as the paper runs it (Sec. IV-A): the layer-mean block distance
 * dist(q, p) = (1/L) sum_i (|K_i[q] - K_i[p]| + |V_i[q] - V_i[p]|) / (2 T H)  of the listed
 * candidate pairs only (the blocks of the steps that Stage 1 flagged), one decision per query
 * block shared by all layers.  HBM bound: every listed pool block is streamed once per layer
 * against the query block; since both are in registers anyway the differences are formed
 * directly (exact in fp32) instead of through the expansion with cached norms, so no norms
 * are taken and near-duplicate pairs lose no digits.
 *
 *   cand            DEVICE int32 [Q][C]: pool index, or -1 for an empty slot; the same list for
 *                   every layer.  Entries outside [0, P) and dead blocks get +inf.
 *   pool_live       DEVICE uint8 [P], NULL = all live
 *   dist            DEVICE float [Q][C]
 *   best_idx        DEVICE int32 [Q]: nearest listed block, equal distances to the lowest pool
 *                   index; -1 if the list has no valid entry.  best_dist: +inf if none.
 *   match_idx       DEVICE int32 [Q]: best_idx if best_dist <= threshold, else -1
 *   workspace       DEVICE, >= rc_candidate_distances_workspace_size() bytes, 16-byte aligned, scratch
 * n_layers must be >= 1.  Q == 0 launches nothing; C == 0 or P == 0 writes -1 / +inf.
 */
rc_status rc_candidate_distances(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc,
                                 const void* kq, const void* vq, int64_t Q,
                                 const void* kp, const void* vp, int64_t P,
                                 const uint8_t* pool_live, const int32_t* cand, int64_t C, float threshold,
                                 float* dist, int32_t* best_idx, float* best_dist, int32_t* match_idx,
                                 void* workspace, size_t workspace_bytes, void* hip_stream);

/* Bytes of DEVICE workspace rc_pat_threshold needs (a constant, about 4 KB). */
size_t rc_pat_workspace_size(void);

/*
 * Percentile-based adaptive threshold (Sec. IV-A, "Percentile-based Adaptive Thresholding";
 * p = 80 in the evaluation's parameter paragraph: the p % of the candidates with the lowest
 * distances are kept).  During warm-up the caller runs the search with sharing disabled
 * (threshold -inf) and collects the distances; this call turns them into the threshold:
 * the nearest-rank p-th percentile, i.e. with n_f finite samples the k-th smallest of them,
 * k = ceil(p/100 * n_f) clamped to [1, n_f] (evaluated in double).  The result is a member of
 * the sample and is exact (a radix select on the bit patterns, no interpolation); p = 100
 * returns the largest collected distance.  Non-finite samples (queries that had no candidate)
 * are left out; with no finite sample the threshold is -inf, which shares nothing.
 *
 *   samples         DEVICE float [n], n < 2^31, any order
 *   p               percentile in [0, 100], a double: the rank is formed from exactly the value the caller
 *                   passes (p = 0.1 with n_f = 1000 is rank 1; rounded to float it would be rank 2)
 *   threshold       DEVICE float [1], written on the stream (no host synchronisation)
 *   n_finite        DEVICE int64 [1] or NULL: number of samples that took part
 *   workspace       DEVICE, >= rc_pat_workspace_size() bytes, 16-byte aligned, scratch
 */
rc_status rc_pat_threshold(const float* samples, int64_t n, double p,
                           float* threshold, int64_t* n_finite,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The sharing decision against a threshold that lives in device memory (the output of
 * rc_pat_threshold): match_idx[i] = best_idx[i] if best_idx[i] >= 0 and best_dist[i] <= *threshold,
 * else -1 (Sec. IV-A: the percentile is the threshold "for all sharing decisions").
 * All pointers DEVICE; n == 0 launches nothing.
 */
rc_status rc_apply_threshold(const int32_t* best_idx, const float* best_dist, int64_t n,
                             const float* threshold, int32_t* match_idx, void* hip_stream);

/* Bytes of DEVICE workspace rc_pool_admit needs (0 on bad arguments). */
size_t rc_pool_admit_workspace_size(int64_t Q, int64_t P);

/*
 * Streaming pool maintenance (Sec. IV-B: the search is part of every decoding step, so a new
 * block that found no partner stays resident and is itself a candidate from the next step on;
 * Sec. IV-A: a block's squared norms are computed once and kept with the block).  Every
 * unmatched query block (match_idx[q] < 0), in ascending q, takes the lowest-numbered pool slot
 * that is not live: its K and V tensors of every layer and its squared norms are stored there
 * and the slot becomes live.  When the free slots run out the remaining queries are left out.
 * Matched queries need no slot.  The norm cache is dense (8 bytes per block and layer next to
 * 64 KiB of KV), so no cached norm is ever evicted while its block is resident.
 *
 *   kq, vq, q_ksq, q_vsq   DEVICE, the step's query blocks and their norms (as for rc_match_blocks, `mode` gives
 *                          the norm shape: [L][Q] or [L][Q][H])
 *   kp, vp, p_ksq, p_vsq   DEVICE, the pool and its norm cache, updated in place; must not overlap the query buffers
 *   pool_live              DEVICE uint8 [P], one flag per slot for all layers, updated in place
 *   match_idx              DEVICE int32 [Q], the step's decisions (layer-shared, e.g. from rc_match_blocks_layer_mean)
 *   slot_of_query          DEVICE int32 [Q]: the slot a query was admitted to, -1 if it matched or found no room
 *   n_admitted             DEVICE int32 [1]
 *   workspace              DEVICE, >= rc_pool_admit_workspace_size() bytes, 16-byte aligned, scratch
 * No atomics: the same slots on every run.  Q == 0 or P == 0 admits nothing.
 */
rc_status rc_pool_admit(const rc_kv_desc* qdesc, const rc_kv_desc* pdesc, int32_t mode,
                        const void* kq, const void* vq, int64_t Q,
                        const float* q_ksq, const float* q_vsq,
                        void* kp, void* vp, int64_t P, float* p_ksq, float* p_vsq,
                        uint8_t* pool_live, const int32_t* match_idx,
                        int32_t* slot_of_query, int32_t* n_admitted,
                        void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Block metadata update (Sec. IV-A: per-block metadata is kept in LRU order, i.e. with a record of when
 * the block was last used): array[slots[i]] = value for every listed slot inside [0, P); entries outside
 * (-1 = "no slot", as rc_pool_admit and the search write them) are skipped.  Used with the step number as
 * value on the last-use stamps of the matched and of the admitted slots, and with 1 on the reference
 * counts of the admitted slots.  All pointers DEVICE; n == 0 launches nothing.
 */
rc_status rc_pool_touch(const int32_t* slots, int64_t n, int32_t value, int32_t* array, int64_t P, void* hip_stream);

/*
 * References that the engine drops, e.g. the table entries of a request that has ended (Sec. IV-B: a
 * block returns to the free pool only when its reference count reaches 0): refcount[ids[i]] -= 1 for
 * every listed id inside [0, NB), once per time it is listed (integer atomics: the same counts whatever
 * the order).  All pointers DEVICE; n == 0 launches nothing.
 */
rc_status rc_refcount_release(const int32_t* ids, int64_t n, int32_t* refcount, int64_t NB, void* hip_stream);

/*
 * Room for the admissions of a step (Sec. IV-B: the evictor returns a block to the free pool only at
 * reference count 0; Sec. IV-A: block metadata in LRU order).  wanted = number of unmatched queries
 * (match_idx[q] < 0) + extra_wanted; free = number of slots that are not live.  If free < wanted, live
 * slots that nobody references (refcount[p] == 0; every live slot when refcount is NULL) leave the pool
 * (pool_live = 0), least recently used first (smallest last_used, equal values by lowest slot number),
 * until free == wanted or none is left.  Referenced slots never leave: a pool of referenced blocks only
 * stays full, and rc_pool_admit then leaves the surplus queries out.  Call it before rc_pool_admit.
 *
 *   pool_live       DEVICE uint8 [P], updated in place
 *   refcount        DEVICE int32 [P] or NULL (references held on each slot, e.g. the first P entries of a
 *                   layer-shared refcount array of rc_remap_block_table with identity pool ids)
 *   last_used       DEVICE int32 [P], any monotone stamp (e.g. the step number), see rc_pool_touch
 *   match_idx       DEVICE int32 [Q], the step's decisions
 *   n_free          DEVICE int32 [1]: free slots afterwards;  n_evicted: DEVICE int32 [1]
 * One workgroup walks the metadata (9 bytes per slot) seven times; no workspace.  The same slots on every run.
 */
rc_status rc_pool_evict(int64_t P, uint8_t* pool_live, const int32_t* refcount, const int32_t* last_used,
                        const int32_t* match_idx, int64_t Q, int64_t extra_wanted,
                        int32_t* n_free, int32_t* n_evicted, void* hip_stream);

/* HOST string describing the calling thread's last error ("" if none). Never NULL. */
const char* rc_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int32_t rc_version(void);

#ifdef __cplusplus
}
#endif
#endif /* RC_H_ */
