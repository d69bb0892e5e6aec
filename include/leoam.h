/*
 * leoam.h - C ABI of the MI355X (gfx950) chunked sparse-attention decode path.
 *
 * One decode step of one transformer layer, following arXiv 2506.20187
 * (LeoAM), with every KV tier held in one GPU's HBM:
 *
 *   kv_chunk_abstract_build        Sec. 4.3: per chunk, the element-wise maximum
 *                                  and minimum key vectors (the "KV abstract").
 *   kv_chunk_abstract_append       the same, updated for one new token per step.
 *   chunk_score                    Sec. 4.1 / 4.3: chunk importance = upper bound
 *                                  of q.k over the chunk, from abstract + query.
 *   chunk_topk_select              Sec. 4.2 / 6.1: order chunks by upper bound,
 *                                  keep the front of the list under a budget.
 *   sparse_chunk_attention_decode  Sec. 2.1 Eq. (1) over the kept chunks only.
 *   chunk_select_attention_decode  the last two steps in one launch.
 *   chunk_tree_refine              Sec. 4.2: tree-structured split / merge of chunks
 *                                  around the k most important tokens.
 *
 * Conventions (all entry points)
 *   - Every pointer except `const leoam_shape*` is a DEVICE pointer owned by the
 *     caller.  The library allocates nothing and keeps no state between calls.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls
 *     enqueue kernels and return; nothing synchronises.  Outputs are valid once
 *     the stream reaches that point.
 *   - Return value: LEOAM_OK or a negative leoam_status.  Faults that the host
 *     can see (null pointer, unsupported shape or dtype, workspace too small)
 *     are reported before anything is enqueued.  Faults in device-resident data
 *     (boundaries that do not tile the context, chunk ids out of range) cannot be
 *     seen without a sync: kernels clamp such values so that no access leaves
 *     the buffers, and leoam_validate_boundaries() is there for checking.
 *   - Layouts are row-major and contiguous:
 *       K, V       [batch, n_kv_heads, n_ctx, head_dim]   kv_dtype
 *       q          [batch, n_q_heads, head_dim]            kv_dtype
 *       abstract   [batch, n_kv_heads, c_max, 2, head_dim] abstract_dtype
 *                  ([..,0,:] = kmax, [..,1,:] = kmin)
 *       chunk_off  [batch, c_max + 1] int32, row b = 0 = off[0] < off[1] < ... <
 *                  off[n_chunks[b]] = n_ctx; entries past that are ignored
 *       n_chunks   [batch] int32, 0 <= n_chunks[b] <= c_max
 *       score      [batch, n_kv_heads, c_max] float
 *       sel_idx    [batch, n_kv_heads, k_max] int32
 *       out        [batch, n_q_heads, head_dim] float
 *     K, V, q, abstract (and the blobs and chunk records of the compressed
 *     store) are read with 16-byte loads: their addresses must be multiples of
 *     16 (LEOAM_E_INVALID_ARG otherwise).  The other arrays need the natural
 *     alignment of their element type.
 *     Chunk boundaries belong to a (sequence, layer) and are shared by its
 *     heads; abstracts, scores and selections are per (sequence, kv head).
 *     Query head j belongs to kv head j / (n_q_heads / n_kv_heads).
 *   - Same inputs give bit-identical outputs (no floating-point atomics).
 */
#ifndef LEOAM_H
#define LEOAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LEOAM_OK = 0,
    LEOAM_E_INVALID_ARG = -1,    /* null pointer, misaligned pointer, non-positive size, Hq % Hkv != 0 */
    LEOAM_E_BAD_BOUNDARIES = -2, /* only from leoam_validate_boundaries */
    LEOAM_E_UNSUPPORTED = -3,    /* head_dim != 128, group size not in {1,2,4,8}, dtype combination, c_max > 16384 */
    LEOAM_E_WORKSPACE = -4,      /* workspace missing or too small */
    LEOAM_E_HIP = -6             /* a HIP call or launch failed */
} leoam_status;

typedef enum { LEOAM_F32 = 0, LEOAM_F16 = 1, LEOAM_BF16 = 2, LEOAM_Q8Q4 = 3 } leoam_dtype;

/*
 * Compressed KV store (kv_dtype == LEOAM_Q8Q4; paper Sec. 4.4 "Dynamic KV
 * compression", Sec. 6.1: compressed KV is INT4).  Every chunk of a (b,h) is
 * stored either as 8-bit codes 0..255 (one byte per element, a token row is 128
 * bytes) or as 4-bit codes 0..15 (two per byte, channel 2i in the low nibble of
 * byte i, a row is 64 bytes), K and V in separate byte blobs that use the same
 * per-chunk offsets.  A stored value is  scale * code + zero  with one
 * (scale, zero) pair per (b, h, chunk, tensor), scale >= 0.  Which chunks are
 * 4-bit is the caller's decision (the paper picks a share theta from a latency
 * model; the tag is an input here).  q and the abstract are fp16.
 * qmeta: [batch, n_kv_heads, c_max] records of 32 bytes.
 */
typedef struct {
    int64_t byte_off; /* offset of the chunk's first row in the K blob and in the V blob; multiple of 16 */
    int32_t bits;     /* 8 or 4 */
    float scale_k, zero_k, scale_v, zero_v;
    int32_t reserved;
} leoam_qchunk;

typedef struct {
    int32_t batch;          /* B  >= 1 */
    int32_t n_q_heads;      /* Hq, multiple of n_kv_heads, Hq/Hkv in {1,2,4,8} */
    int32_t n_kv_heads;     /* Hkv >= 1 */
    int32_t head_dim;       /* D, must be 128 */
    int32_t n_ctx;          /* N, tokens per sequence (same for the whole batch) */
    int32_t c_max;          /* row stride of per-chunk arrays, 1..16384 (any value is correct; a multiple of 32
                             * lets every (b,h)'s abstract start at the same offset inside 16 KiB, which is
                             * what chunk_score streams fastest) */
    int32_t k_max;          /* row stride of sel_idx, 1..c_max; also caps the kept count */
    int32_t kv_dtype;       /* leoam_dtype of K and V */
    int32_t abstract_dtype; /* dtype of the abstract and of q: == kv_dtype, or LEOAM_F16 when kv_dtype == LEOAM_Q8Q4 */
} leoam_shape;

/*
 * Sec. 4.3 "KV abstract extraction".  For every (b, h, c < n_chunks[b]):
 *   abstract[b,h,c,0,d] = max over off[c] <= t < off[c+1] of K[b,h,t,d]
 *   abstract[b,h,c,1,d] = min over the same tokens.
 * Exact (a maximum of stored values); the sign of a zero result is unspecified.
 * Rows of chunks >= n_chunks[b] are not written.  Token indices are clamped to
 * [0, n_ctx]; an empty chunk gives (-inf, +inf).
 * LEOAM_Q8Q4: K is the K blob, qmeta the chunk records (NULL otherwise).  The
 * maximum / minimum is taken over the stored values  scale_k*code + zero_k
 * (evaluated in double) and rounded OUTWARD to fp16 (kmax up, kmin down), so the
 * bounds of chunk_score still enclose every stored key.
 */
int kv_chunk_abstract_build(const leoam_shape* shape, const void* K, const void* qmeta, const int32_t* chunk_off,
                            const int32_t* n_chunks, void* abstract, void* stream);

/*
 * The abstract of Sec. 4.3 kept up to date while decoding adds one token per
 * sequence and step (Sec. 2.1: output tokens are generated one by one and join
 * the context).  For every sequence b the new token is t = chunk_off[b][n_chunks[b]]
 * (the current length; rows need not reach n_ctx, which is the capacity of the
 * K rows), and the caller has already stored its key in K[b,:,t,:].  If the last
 * chunk holds fewer than chunk_size tokens it grows by one and its abstract rows
 * become max(kmax, k_t) / min(kmin, k_t); otherwise a new one-token chunk with
 * kmax = kmin = k_t is opened (chunk_size is the layer's initial chunk size;
 * Sec. 6.1 uses 64, and 8 in the first two layers).  The result equals
 * kv_chunk_abstract_build on the new boundaries.  chunk_off, n_chunks and
 * abstract are updated in place; status[b] (nullable) = 0 done, 1 cache full
 * (t == n_ctx), 2 no room for another chunk (n_chunks == c_max); sequences with a
 * non-zero status are left untouched.  fp32 / fp16 / bf16 stores only.
 */
int kv_chunk_abstract_append(const leoam_shape* shape, const void* K, int32_t* chunk_off, int32_t* n_chunks,
                             int32_t chunk_size, void* abstract, int32_t* status, void* stream);

/*
 * Sec. 4.2 "Tree-structured KV chunk management" (Fig. 9).  Per (b, kv head) the
 * context starts as chunks of chunk_size tokens (the last one may be shorter)
 * whose abstract rows `abstract[b,h,c]`, c < ceil(n_ctx / chunk_size) <= c_max,
 * were built by kv_chunk_abstract_build.  Every chunk gets an upper bound U and a
 * lower bound L of the importance of its tokens (importance of token t = max over
 * the group's query heads of q_j.k_t; U = max_j U_j, L = max_j L_j with U_j, L_j
 * as in chunk_score, each the double sum rounded once to float).  With order
 * statistics taken over tokens (a chunk counts `size` times),
 *   v = k-th largest U,  mu = (k+1)-th largest U (-inf if k == n_ctx),  lambda = k-th largest L,
 * a chunk with L > mu holds only tokens of the k most important ones (confirmed),
 * a chunk with U < lambda holds none (unimportant), and every chunk with U >= v
 * (the front of the queue ordered by U, read until it covers k tokens) that is
 * neither confirmed nor a single token is split in two (ceil(size/2) tokens to
 * the left) and its halves are evaluated from their keys.  This is repeated until
 * nothing is split, max_rounds rounds were made, or a round would need more than
 * node_cap nodes (then ref_status = 1 and that round is not made).  Finally runs
 * of confirmed chunks and runs of unimportant chunks are merged.
 *   ref_off   [batch, n_kv_heads, node_cap + 1]  boundaries of the final partition
 *   ref_score [batch, n_kv_heads, node_cap]      FLT_MAX for a confirmed chunk, else its U
 *                                               (a merged unimportant run: the largest U in it)
 *   ref_count, ref_evals, ref_status [batch, n_kv_heads]   chunks; evaluations made
 *                                               (initial chunks + 2 per split); 0 or 1
 * Reading ref_off / ref_score / ref_count as the boundaries, scores and counts of
 * batch * n_kv_heads sequences with one kv head each, chunk_topk_select with
 * token_budget = k keeps the k most important tokens (exactly, once nothing is
 * left to split), and sparse_chunk_attention_decode attends to them.
 * fp32 / fp16 / bf16 stores.  Workspace: leoam_tree_workspace_bytes(), 16-byte
 * aligned, contents irrelevant.
 */
int chunk_tree_refine(const leoam_shape* shape, const void* q, const void* K, const void* abstract, int32_t chunk_size,
                      int32_t k_tokens, int32_t max_rounds, int32_t node_cap, int32_t* ref_off, float* ref_score,
                      int32_t* ref_count, int32_t* ref_evals, int32_t* ref_status, void* workspace,
                      size_t workspace_bytes, void* stream);

size_t leoam_tree_workspace_bytes(const leoam_shape* shape, int32_t node_cap);

/*
 * Sec. 4.2 "Dynamic chunk resizing": the expected number of importance
 * evaluations when n_tokens start as n_chunks equal chunks, a split costs two
 * evaluations and happens with probability rho at every tree level (rho = share
 * of important tokens of the layer), and a chunk of size n/m is split at most
 * log2(n/m) - 1 times:
 *   f(m) = m * sum_{i=0}^{log2(n/m)-1} (2 rho)^i.
 * Host arithmetic only.  -1 unless n_chunks divides n_tokens into a power-of-two
 * chunk size and 0 <= rho <= 1.
 */
double leoam_tree_evaluations(int64_t n_tokens, int64_t n_chunks, double rho);

/*
 * Sec. 4.1 (chunk importance is the upper bound of the token importance in the
 * chunk) and Sec. 4.3 (bounds from the abstract and the current query).  For
 * every query head j of kv head h and every chunk c < n_chunks[b]:
 *   U_j[c] = sum_d max(q_j[d]*kmax[d], q_j[d]*kmin[d])
 *   L_j[c] = sum_d min(q_j[d]*kmax[d], q_j[d]*kmin[d])
 *   score_ub[b,h,c] = max_j U_j[c],   score_lb[b,h,c] = min_j L_j[c]
 * so score_lb <= q_j.k_t <= score_ub for every token t of the chunk and every
 * head j of the group.  The sums are accumulated in double over exact products
 * and rounded once to float; -0 is stored as +0.  Entries c >= n_chunks[b] are
 * set to -inf (ub) and +inf (lb).  score_lb may be NULL.
 */
int chunk_score(const leoam_shape* shape, const void* q, const void* abstract, const int32_t* n_chunks,
                float* score_ub, float* score_lb, void* stream);

/*
 * Always-kept chunks.  The paper forces no tokens into the selection; a caller
 * that wants the first chunks of a sequence (attention sink) or its last chunks
 * (the most recent tokens, among them the tail chunk that decoding appends to,
 * Sec. 2.1) kept whatever the query says marks them here: for every kv head the
 * scores of chunks [0, sink_chunks) and [n_chunks[b] - tail_chunks, n_chunks[b])
 * become FLT_MAX, which puts them at the front of the Sec. 4.2 order (ties by
 * index), so the selection keeps them first - as far as they fit the budget.
 * Counts beyond n_chunks[b] mark every chunk; negative counts are invalid.
 */
int chunk_score_pin(const leoam_shape* shape, const int32_t* n_chunks, int32_t sink_chunks, int32_t tail_chunks,
                    float* score_ub, void* stream);

/*
 * Sec. 4.2 (priority queue ordered by upper bound, read from the front) and
 * Sec. 6.1 (only the most important share of the cache is loaded).  Per (b,h):
 * order chunks by (score descending, chunk index ascending); keep the longest
 * front of that list whose length is <= max_chunks and <= k_max and whose token
 * total is <= token_budget; the walk stops at the first chunk that does not fit.
 * max_chunks <= 0 and token_budget <= 0 mean "no limit".  Scores must be finite
 * for c < n_chunks[b] (+0 and -0 compare equal).
 *   sel_idx[b,h,0..count)  kept chunk ids in ascending order, rest of row = -1
 *   sel_count[b,h]         number kept
 *   sel_tokens[b,h]        their token total (nullable)
 * workspace is not used by this call (pass NULL, 0).
 */
int chunk_topk_select(const leoam_shape* shape, const float* score_ub, const int32_t* chunk_off,
                      const int32_t* n_chunks, int32_t max_chunks, int32_t token_budget, int32_t* sel_idx,
                      int32_t* sel_count, int32_t* sel_tokens, void* workspace, size_t workspace_bytes,
                      void* stream);

/*
 * Sec. 2.1 Eq. (1) restricted to the tokens T of the kept chunks.  For query
 * head j of kv head h:  z_t = softmax_scale * (q_j . K[b,h,t]),
 *   out[b,j,:] = sum_T softmax_T(z)_t * V[b,h,t,:],  lse[b,j] = log sum_T exp(z_t).
 * Nothing kept: out = 0, lse = -inf.  lse may be NULL.  Ids in sel_idx outside
 * [0, n_chunks) contribute no tokens.  k_max must be <= 8192 here (<= 1024 for
 * LEOAM_Q8Q4).  LEOAM_Q8Q4: K, V are the byte blobs, qmeta the chunk records
 * (NULL otherwise); codes are expanded inside the kernel (Sec. 4.4: the cost of
 * compression is decompression on the GPU), K[t] and V[t] above being the
 * stored values scale*code + zero.
 * The kept tokens are split across workgroups; every split leaves a partial
 * (m, l, acc[D]) in the workspace and a second small kernel combines them in
 * split order, so results do not depend on scheduling.  Workspace: 16-byte
 * aligned, contents irrelevant on entry.  The number of splits is the largest
 * the workspace allows, up to what leoam_workspace_bytes() asks for, so a
 * workspace of that size gives the intended launch.  Calls that share a
 * workspace must not overlap.
 */
int sparse_chunk_attention_decode(const leoam_shape* shape, const void* q, const void* K, const void* V,
                                  const void* qmeta, const int32_t* chunk_off, const int32_t* n_chunks, const int32_t* sel_idx,
                                  const int32_t* sel_count, float softmax_scale, float* out, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * chunk_topk_select followed by sparse_chunk_attention_decode (Sec. 4.2 / 6.1,
 * then Sec. 2.1 Eq. (1) over the kept chunks; Sec. 4.1: the evaluation result
 * selects the KV the decoding computation uses), with the same arguments,
 * outputs and preconditions as those two calls.  For fp16 / bf16 K and V with
 * group size <= 4, k_max <= 2048 and c_max <= 8192 both steps run in a single
 * kernel: every workgroup selects for its (b,h), keeps the kept chunks' token
 * ranges on chip and streams its share of the kept tokens; workgroups that share
 * a (b,h) combine their partials in the same launch, in split order, so results
 * do not depend on scheduling.  Other shapes run the two kernels of the separate
 * calls back to back.  sel_idx / sel_count / sel_tokens are written as by
 * chunk_topk_select.
 * With LEOAM_STREAM_ORDERED_MERGE=1 in the environment (read once per process)
 * every shape runs the kernels of the separate calls, merge kernel included:
 * the in-launch combination of the splits orders its hand-over by waiting for
 * store acknowledgements rather than by fences, which the memory system of the
 * part guarantees and the programming model does not; the switch trades a few
 * microseconds per call for a path that is ordered by the stream alone.
 * score_ub == NULL: the selection was made earlier (for instance by one
 * chunk_topk_select call over all layers of a step, Sec. 4.4: the evaluation runs
 * ahead of the computation); sel_idx / sel_count are then INPUTS, as for
 * sparse_chunk_attention_decode (ids outside [0, n_chunks) contribute no tokens,
 * counts are clamped to [0, k_max]), max_chunks / token_budget / sel_tokens are
 * not used, and the call only attends - in the same single kernel, with the
 * in-launch merge, where the separate call needs a second kernel.
 * Workspace: leoam_fused_workspace_bytes() bytes, 16-byte aligned.  Its first
 * leoam_fused_control_bytes() bytes are control words (arrival counters of the
 * (b,h) pairs and, for batch sizes that give two splits per (b,h), one 64-bit
 * exchange word per (b, q head, channel)): they must be ZERO when the call is
 * issued and are zero again when it completes, so a workspace is cleared once
 * (leoam_workspace_init) and then reused; the rest needs no initialisation.  A
 * smaller workspace gives fewer splits.  Calls that share a workspace must not
 * overlap.
 */
int chunk_select_attention_decode(const leoam_shape* shape, const float* score_ub, const void* q, const void* K,
                                  const void* V, const void* qmeta, const int32_t* chunk_off, const int32_t* n_chunks,
                                  int32_t max_chunks, int32_t token_budget, float softmax_scale, int32_t* sel_idx,
                                  int32_t* sel_count, int32_t* sel_tokens, float* out, float* lse, void* workspace,
                                  size_t workspace_bytes, void* stream);

/*
 * chunk_select_attention_decode for callers that cannot allocate device memory or
 * bring a workspace: code inside a HIP graph capture, tight serving loops,
 * harnesses that forbid allocation.  Same arguments, outputs and preconditions,
 * without the workspace: arrival counters and split partials live in a buffer of
 * LEOAM_STATIC_SCRATCH_BYTES that is part of the library image (every GPU the
 * library runs on holds its own copy until the process ends).  The call allocates
 * nothing and frees nothing; it enqueues one small fill kernel (the counters) and
 * the kernels of chunk_select_attention_decode.  The number of splits is what
 * leoam_fused_workspace_bytes(shape, token_budget) would give, or fewer if that
 * exceeds the buffer; a shape whose smallest workspace does not fit (a two-launch
 * shape with batch * n_q_heads * 520 bytes above the limit, or more than 64 Ki
 * (sequence, kv head) pairs' counters) returns LEOAM_E_WORKSPACE and enqueues
 * nothing.  All calls on one GPU share the buffer: calls that may overlap on a
 * GPU (two streams, two threads) race and must be serialised by the caller.  The
 * buffer's address is looked up on the first call on each device (not inside a
 * graph capture: issue one call before capturing).
 */
#define LEOAM_STATIC_SCRATCH_BYTES (4u << 20)
int chunk_select_attention_decode_static(const leoam_shape* shape, const float* score_ub, const void* q, const void* K,
                                         const void* V, const void* qmeta, const int32_t* chunk_off,
                                         const int32_t* n_chunks, int32_t max_chunks, int32_t token_budget,
                                         float softmax_scale, int32_t* sel_idx, int32_t* sel_count, int32_t* sel_tokens,
                                         float* out, float* lse, void* stream);

/* Bytes of workspace chunk_select_attention_decode wants when at most
 * `max_tokens` tokens are kept per (b,h) (<= 0: n_ctx).  0 on a bad shape. */
size_t leoam_fused_workspace_bytes(const leoam_shape* shape, int32_t max_tokens);

/* Leading bytes of that workspace that must be zero when chunk_select_attention_decode
 * is issued (and are zero again when it completes).  0 on a bad shape. */
size_t leoam_fused_control_bytes(const leoam_shape* shape);

/* Zero-fills a workspace (size a multiple of 16, 16-byte aligned) on `stream`. */
int leoam_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of workspace sparse_chunk_attention_decode wants when at most
 * `max_tokens` tokens are kept per (b,h) (<= 0: n_ctx).  0 on a bad shape. */
size_t leoam_workspace_bytes(const leoam_shape* shape, int32_t max_tokens);

/* Debug helper: copies the boundary lists to the host (synchronises `stream`)
 * and returns LEOAM_E_BAD_BOUNDARIES unless every row tiles [0, n_ctx). */
int leoam_validate_boundaries(const leoam_shape* shape, const int32_t* chunk_off, const int32_t* n_chunks,
                              void* stream);

/*
 * Sec. 4.4 "Dynamic KV compression", Sec. 6.1 (KV held in FP16, compressed to
 * INT4): builds the compressed store described at leoam_qchunk from an fp16 or
 * bf16 cache.  Per (b, h, chunk c < n_chunks[b], tensor):
 *   zero = min over the chunk's elements, scale = (max - min) / levels,
 *   code = round-half-even((x - zero) / scale) kept inside 0..levels,
 * levels = 15 where four_bit[b, c] != 0, else 255; max - min, the two divisions
 * and x - zero are single correctly rounded float operations; scale == 0 (all
 * elements equal) stores code 0.  Layout: the chunks of a (b,h) follow each
 * other, then the next (b,h); K and V blobs use the same offsets.
 *   shape->kv_dtype   dtype of K and V: LEOAM_F16 or LEOAM_BF16 (others: LEOAM_E_UNSUPPORTED)
 *   K, V      [batch, n_kv_heads, n_ctx, 128]       in
 *   four_bit  [batch, c_max] bytes                  in   which chunks are 4-bit
 *   kblob, vblob  blob_bytes bytes each, 16-byte aligned   out
 *   qmeta     [batch, n_kv_heads, c_max] leoam_qchunk      out  (records of chunks >= n_chunks[b]: all zero)
 *   total_bytes  device int64, nullable                    out  bytes used of each blob
 * blob_bytes must be at least leoam_compressed_bytes_bound() (the size with
 * every chunk 8-bit), else LEOAM_E_WORKSPACE; the bytes past *total_bytes are
 * not written.  Boundaries must tile the context: a chunk whose boundaries do not
 * lie in [0, n_ctx] in ascending order takes no room and is skipped, and no chunk
 * is written past blob_bytes whatever the boundaries hold.
 */
int kv_chunk_compress(const leoam_shape* shape, const void* K, const void* V, const int32_t* chunk_off,
                      const int32_t* n_chunks, const uint8_t* four_bit, void* kblob, void* vblob, size_t blob_bytes,
                      void* qmeta, int64_t* total_bytes, void* stream);

size_t leoam_compressed_bytes_bound(const leoam_shape* shape);

/*
 * Sec. 4.4: the compressed share is chosen dynamically (theta follows the measured
 * times, and which chunks are unimportant follows the scores), so the tags of a
 * store change while it is in use.  Brings a store that was written under the
 * tags four_bit_old (by kv_chunk_compress or by earlier calls of this function)
 * to the tags four_bit_new by encoding again, from the uncompressed cache and as
 * kv_chunk_compress does, ONLY the chunks whose tag changed:
 *   8-bit -> 4-bit   the chunk is encoded where it lies (half of its old room);
 *   4-bit -> 8-bit   the chunk moves to fresh room behind the used part of the
 *                    blobs; moved chunks are placed in (b, h, chunk) order from
 *                    *used_bytes on, which grows by the room they take.
 * Every other byte of the blobs and every other record stays as it is (records
 * carry each chunk's own offset, so the kernels that read the store need no
 * particular order; the room a moved chunk leaves stays unused until the next
 * kv_chunk_compress).  Afterwards every chunk decodes to exactly what
 * kv_chunk_compress under four_bit_new would store.
 *   used_bytes  device int64, in / out: bytes in use of each blob (kv_chunk_compress's total_bytes)
 *   info        device int64[3], out: {1 if the fresh room did not fit blob_bytes - then nothing
 *               was changed -, chunks encoded again counted per (b, h, chunk), bytes of fresh room}
 * shape->kv_dtype is the dtype of K and V (LEOAM_F16 or LEOAM_BF16), as for kv_chunk_compress.
 */
int kv_chunk_recompress(const leoam_shape* shape, const void* K, const void* V, const int32_t* chunk_off,
                        const int32_t* n_chunks, const uint8_t* four_bit_old, const uint8_t* four_bit_new, void* kblob,
                        void* vblob, size_t blob_bytes, void* qmeta, int64_t* used_bytes, int64_t* info, void* stream);

/*
 * Sec. 4.4 (the compressed share) with Sec. 4.2 (chunks ordered by importance): the
 * paper fixes the size of the share, not which data it holds.  Here a chunk is
 * tagged 4-bit unless some kv head of its sequence keeps it in the selection
 * (sel_idx / sel_count as written by chunk_topk_select, e.g. with a token budget of
 * (1 - theta) * n_ctx):
 *   four_bit [batch, c_max] bytes   out   1 = 4-bit, 0 = kept chunk or slot >= n_chunks[b]
 * Ids outside [0, n_chunks[b]) and entries past sel_count are ignored.
 */
int chunk_compression_tags(const leoam_shape* shape, const int32_t* n_chunks, const int32_t* sel_idx,
                           const int32_t* sel_count, uint8_t* four_bit, void* stream);

/*
 * Sec. 4.4: the share theta of a layer's n_bytes transmitted KV bytes that is
 * sent compressed.  Sent at `bandwidth` bytes/s with a share theta compressed
 * to `ratio` (compressed / uncompressed size), the data arrives after
 *   t_other + n_bytes * (1 - theta + theta * ratio) / bandwidth
 * (t_other: the other evaluation and transmission time); it is hidden while
 * that does not exceed  t_compute + n_bytes * theta / decompress_rate  (the
 * computation plus the decompression of the compressed share).  Returns the
 * theta at which the two are equal, kept inside [0, 1]: 0 if the transfer is
 * hidden without compression, 1 if it is not hidden even when everything is
 * compressed.  Host arithmetic only; a negative value reports an invalid
 * argument (sizes, rates not positive, ratio outside (0, 1]).
 */
double leoam_compression_share(double n_bytes, double ratio, double bandwidth, double t_other, double t_compute,
                               double decompress_rate);

const char* leoam_status_string(int status);
int leoam_version(void);

/* ------------------------------------------------------------------------
 * Measuring aids.  Not part of the decode path: two plain streaming kernels of
 * known size that the benchmark and the profiles compare the path's kernels
 * with on the same GPU.
 * ------------------------------------------------------------------------ */

/* Plain device copy of `bytes` bytes (multiple of 16, 16-byte aligned): the
 * known-size kernel that hardware byte counters are scaled against. */
int leoam_copy_probe(void* dst, const void* src, size_t bytes, void* stream);

/* Reads `bytes` bytes (multiple of 16, 16-byte aligned) and keeps nothing: the
 * read-only stream whose rate is the measured ceiling the path's HBM-bound
 * kernels are reported against.  `sink`: 4 writable bytes (device), written
 * only for one data pattern in 2^64. */
int leoam_read_probe(const void* src, size_t bytes, void* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LEOAM_H */
