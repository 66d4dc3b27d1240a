/*
 * specvlm.h -- C ABI of libspecvlm: the target model's verification step over a
 * draft token tree (SpecVLM Sec. 3.1: in every speculative round the target
 * verifies the drafted tokens in ONE forward pass and the incorrect ones are
 * discarded; Sec. 4.1: the draft is an EAGLE-2 style token tree with Top-K 10,
 * 60 tokens, depth 7; evaluation at temperature 0, batch 1).
 *
 * Conventions
 *  - Every pointer named *_dev is DEVICE memory owned by the caller; the library
 *    allocates nothing, keeps no pointer after return and is re-entrant.
 *  - All work is enqueued on `stream` (a hipStream_t passed as void*; NULL is the
 *    default stream).  Calls are asynchronous; outputs are valid once the stream
 *    has reached them.
 *  - Every function returns a specvlm_status.  Scalar arguments are validated on
 *    the host without synchronising.  Data-dependent violations (malformed parent
 *    array, node counts or tokens out of range) are reported by OR-ing
 *    SPECVLM_ERR_* bits into the optional device word `err_flag_dev`; the kernels
 *    then leave that request's outputs defined but unspecified and never touch
 *    memory outside the given buffers.
 *  - Tree convention: node 0 is the root (the token the target committed last,
 *    Fig. 3a), parent[0] = -1, 0 <= parent[i] < i for i >= 1.  At most 64 nodes.
 *  - Strides are in ELEMENTS of the tensor's type.  The innermost (head_dim or
 *    vocab) dimension is always contiguous.
 */
#ifndef SPECVLM_H
#define SPECVLM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum specvlm_status {
    SPECVLM_OK = 0,
    SPECVLM_INVALID_ARG = 1,         /* null pointer, bad dimension, misaligned pointer/stride */
    SPECVLM_UNSUPPORTED = 2,         /* legal but not implemented dtype/layout combination   */
    SPECVLM_WORKSPACE_TOO_SMALL = 3,
    SPECVLM_HIP_ERROR = 4            /* launch failed; see specvlm_last_hip_error()           */
} specvlm_status;

typedef enum specvlm_dtype {
    SPECVLM_BF16 = 0,                /* bfloat16 in, fp32 accumulate/softmax, bfloat16 out */
    SPECVLM_F32 = 1                  /* IEEE fp32 throughout                                */
} specvlm_dtype;

/* bits of *err_flag_dev */
#define SPECVLM_ERR_BAD_PARENT   1   /* parent[0] != -1 or parent[i] not in [0,i)            */
#define SPECVLM_ERR_BAD_NUM_NODES 2  /* num_nodes[b] not in [1, N_max]                       */
#define SPECVLM_ERR_BAD_LENGTH   4   /* prefix_len[b] < 0 or prefix_len+num_nodes > capacity */
#define SPECVLM_ERR_PATH_TOO_LONG 8  /* an accepted path would not fit in path_cap           */
#define SPECVLM_ERR_BAD_BLOCK    16  /* block_table entry outside [0, num_blocks)            */
#define SPECVLM_ERR_BAD_TOKEN    32  /* a drafted token outside [0, V)                       */
#define SPECVLM_ERR_TREE_NOT_CLOSED 64 /* draft growth: a chosen candidate whose parent was not chosen */

#define SPECVLM_MAX_NODES 64
#define SPECVLM_PAGE_SIZE 16
#define SPECVLM_MAX_SPLITS 64        /* key-range splits per (request, head) */
#define SPECVLM_COUNTER_STRIDE 32              /* int32 words between the arrival counters of two requests */
#define SPECVLM_MAX_CANDIDATES 8192  /* draft growth: scored candidates per request */

/*
 * Geometry of one attention layer's tensors.
 *
 *   q, o     : [B, N_max, H_q, D]      via (q|o)_stride_b / _n / _h
 *   K, V     : contiguous (paged == 0): [B, H_kv, kv_capacity, D] via kv_stride_b (request),
 *              kv_stride_h, kv_stride_t (token);
 *              paged (paged == 1): [num_blocks, H_kv, 16, D] via kv_stride_b (BLOCK),
 *              kv_stride_h, kv_stride_t, addressed through block_table[B, max_blocks_per_req]
 *              (logical slot s of request b lives in block block_table[b][s/16], row s%16).
 *   K and V share one geometry.  H_q must be a multiple of H_kv (query head h reads KV
 *   head h / (H_q/H_kv)).  D is 64 or 128.  N_max <= 64.
 *   All kv_capacity slots of every request of a contiguous cache, and every block of a paged pool
 *   that a block table names, must be readable memory: the attention call may FETCH slots past
 *   prefix_len + num_nodes (up to kv_capacity; paged: up to the end of the request's last block);
 *   it never USES what they hold, whatever bit patterns are there.
 */
typedef struct specvlm_attn_desc {
    int32_t dtype;                 /* specvlm_dtype */
    int32_t B, H_q, H_kv, D, N_max;
    float   softmax_scale;         /* 0 selects 1/sqrt(D) */
    int32_t paged;
    int32_t block_size;            /* must be 16 when paged */
    int32_t max_blocks_per_req;    /* second dimension of block_table (paged only) */
    int32_t num_blocks;            /* physical blocks in the pool (paged only)     */
    int32_t kv_capacity;           /* slots per request (contiguous); paged: max_blocks_per_req*16 */
    int32_t num_splits;            /* key-range splits per (request, head): 0 lets the library choose, 1 ..
                                      SPECVLM_MAX_SPLITS is taken as given (anything else: SPECVLM_INVALID_ARG);
                                      with more than 1024 (request, head) pairs a call always runs unsplit */
    int64_t q_stride_b, q_stride_n, q_stride_h;
    int64_t o_stride_b, o_stride_n, o_stride_h;
    int64_t kv_stride_b, kv_stride_h, kv_stride_t;
} specvlm_attn_desc;

/* Library version, major*10000 + minor*100 + patch. */
int32_t specvlm_version(void);

/* hipError_t of the most recent failed HIP call made by this thread's library calls (0 if none). */
int32_t specvlm_last_hip_error(void);

/*
 * Scratch bytes specvlm_tree_verify_attn needs for `desc` (arrival counters and split-key
 * partial results; 0 when the shape needs none).  Returns 0 when desc is invalid.  The
 * workspace is device memory, 256-byte aligned.  It must be ZERO-FILLED ONCE after
 * allocation; every call leaves its counter words zero again, and the counters occupy the
 * same fixed region at the start whatever the shape, so the same workspace can be reused by
 * later calls (of any shape it is large enough for) without clearing.  Two calls that may
 * run concurrently need separate workspaces.
 */
size_t specvlm_tree_verify_attn_workspace_bytes(const specvlm_attn_desc *desc);

/*
 * Number of key-range splits per (request, head) specvlm_tree_verify_attn will use for
 * `desc` (desc->num_splits when that is positive, otherwise the library's choice for the
 * shape).  Returns 0 when desc is invalid, 1 for SPECVLM_F32 (no split path).
 */
int32_t specvlm_tree_verify_attn_num_splits(const specvlm_attn_desc *desc);

/*
 * Tree-masked verification attention for ONE layer (Sec. 3.1: the target checks all drafted
 * tokens of a round in one forward pass; Sec. 4.1: the drafted tokens form a tree and the
 * pass uses tree attention; Sec. 3.2: the whole KV cache is streamed from HBM once per
 * step).  For request b, query head h and tree
 * node i < num_nodes[b]:
 *     J(i) = {0 .. prefix_len[b]-1}  U  {prefix_len[b] + j : j is i or an ancestor of i}
 *     o[b,i,h,:] = softmax_{j in J(i)}(scale * q[b,i,h,:] . K[b,kv(h),j,:]) . V[b,kv(h),j,:]
 *     lse[b,h,i] = natural-log-sum-exp of the scaled scores over J(i)   (optional)
 * Precondition: the caller has already written the tree tokens' K/V rows into
 * logical slots [prefix_len[b], prefix_len[b]+num_nodes[b]) of the cache, with
 * position encoding applied.  Rows i >= num_nodes[b] of o / lse are not written.
 * Slots at or beyond prefix_len[b]+num_nodes[b] may be fetched (see the geometry note
 * above) but never influence a result.  A block table entry outside [0, num_blocks)
 * sets SPECVLM_ERR_BAD_BLOCK (memory outside the pool is still never touched).
 *
 *   q_dev, o_dev         device, desc->dtype, geometry from desc; 16-byte aligned rows
 *   k_cache_dev, v_cache_dev  device, desc->dtype, read-only here
 *   block_table_dev      device int32 [B, max_blocks_per_req]; NULL iff !paged
 *   prefix_len_dev       device int32 [B]
 *   num_nodes_dev        device int32 [B], or NULL meaning N_max for every request
 *   parent_dev           device int32 [B, N_max]
 *   lse_dev              device fp32 [B, H_q, N_max] or NULL
 *   workspace_dev/bytes  see specvlm_tree_verify_attn_workspace_bytes
 *   err_flag_dev         device int32 or NULL
 */
int32_t specvlm_tree_verify_attn(const specvlm_attn_desc *desc,
                                 const void *q_dev, const void *k_cache_dev, const void *v_cache_dev,
                                 const int32_t *block_table_dev, const int32_t *prefix_len_dev,
                                 const int32_t *num_nodes_dev, const int32_t *parent_dev,
                                 void *o_dev, float *lse_dev,
                                 void *workspace_dev, size_t workspace_bytes,
                                 int32_t *err_flag_dev, void *stream);

/*
 * specvlm_tree_verify_attn for callers that cannot allocate device memory or carry a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and error reporting, without workspace_dev/workspace_bytes: the scratch is a
 * static device array inside the library, SPECVLM_STATIC_WORKSPACE_BYTES long, one per GPU, held
 * from the moment the library is loaded on that GPU until the process ends.  The call allocates
 * and frees nothing (the first call on a device asks the runtime once for the array's address).
 * A shape whose specvlm_tree_verify_attn_workspace_bytes exceeds the array returns
 * SPECVLM_WORKSPACE_TOO_SMALL and launches nothing.  Every call on a GPU uses that GPU's one
 * array: calls that may overlap on one GPU (two streams) race on it and must use
 * specvlm_tree_verify_attn with workspaces of their own instead; calls ordered by a stream, or
 * replays of a captured graph, are fine.  The device must be the current one at the call.
 */
#define SPECVLM_STATIC_WORKSPACE_BYTES (16u << 20)
int32_t specvlm_tree_verify_attn_static(const specvlm_attn_desc *desc,
                                        const void *q_dev, const void *k_cache_dev, const void *v_cache_dev,
                                        const int32_t *block_table_dev, const int32_t *prefix_len_dev,
                                        const int32_t *num_nodes_dev, const int32_t *parent_dev,
                                        void *o_dev, float *lse_dev,
                                        int32_t *err_flag_dev, void *stream);

/*
 * Measurement aid, not part of the verification path: the same operation and arguments as
 * specvlm_tree_verify_attn_static, computed by the vector-ALU kernel that serves SPECVLM_F32
 * (one workgroup per (request, head, node), no matrix cores, no key-range splits, no scratch)
 * also when desc->dtype is SPECVLM_BF16.  It exists so that the choice of the matrix-core kernel
 * for bf16 can be re-measured on the same inputs (bench.py --vector-alu-evidence); results
 * agree with specvlm_tree_verify_attn within the bf16 tolerance.
 */
int32_t specvlm_tree_verify_attn_vector_alu(const specvlm_attn_desc *desc,
                                            const void *q_dev, const void *k_cache_dev, const void *v_cache_dev,
                                            const int32_t *block_table_dev, const int32_t *prefix_len_dev,
                                            const int32_t *num_nodes_dev, const int32_t *parent_dev,
                                            void *o_dev, float *lse_dev,
                                            int32_t *err_flag_dev, void *stream);

/*
 * Greedy target token per tree node (temperature 0, Sec. 4.1):
 *     amax[b,i] = the LOWEST v with logits[b,i,v] == max_v' logits[b,i,v']
 * (values compare as real numbers, -0 == +0; precondition: no NaN; an all -inf
 * row gives 0).  Rows i >= num_nodes[b] get -1.
 *   logits_dev  device, dtype, element (b,i,v) at b*stride_b + i*stride_n + v
 *   amax_dev    device int32 [B, N_max]
 */
int32_t specvlm_node_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t V,
                            const void *logits_dev, int64_t stride_b, int64_t stride_n,
                            const int32_t *num_nodes_dev, int32_t *amax_dev, void *stream);

/*
 * Greedy acceptance walk (Sec. 3.1: incorrect drafted tokens are discarded;
 * decoding stays lossless).  For i >= 1, node i matches when
 * draft_tok[b,i] == amax[b,parent[b,i]]; a node is accepted when it and all its
 * ancestors below the root match.  best = the accepted node of greatest depth
 * (lowest node index on ties); path = root..best = a_0..a_m.
 *   accept_len_dev    int32 [B]            m, the number of accepted DRAFT nodes
 *   path_dev          int32 [B, path_cap]  a_0..a_m, then -1
 *   bonus_tok_dev     int32 [B]            amax[b, best]: the next round's root token
 *   committed_tok_dev int32 [B, path_cap]  draft_tok[a_1..a_m], bonus_tok, then -1
 *                                          (the m+1 tokens this round emits: sigma counts these)
 * draft_tok[b,0] is ignored.  1 <= path_cap <= 64; a path that does not fit sets
 * SPECVLM_ERR_PATH_TOO_LONG and nodes deeper than path_cap-1 are not accepted.
 */
int32_t specvlm_tree_accept(int32_t B, int32_t N_max, int32_t path_cap,
                            const int32_t *parent_dev, const int32_t *draft_tok_dev,
                            const int32_t *amax_dev, const int32_t *num_nodes_dev,
                            int32_t *accept_len_dev, int32_t *path_dev, int32_t *bonus_tok_dev,
                            int32_t *committed_tok_dev, int32_t *err_flag_dev, void *stream);

/*
 * specvlm_node_argmax and specvlm_tree_accept as ONE launch (both are launch-bound): every
 * (request, node) row is reduced as in specvlm_node_argmax, and the workgroup that finishes the
 * last row of a request also walks that request's tree as in specvlm_tree_accept.  Arguments and
 * outputs are those of the two calls (amax_dev is written as well), plus
 *   counters_dev  device int32 [B * SPECVLM_COUNTER_STRIDE]: arrival counters, one per request, each on a
 *                 128-byte line of its own (the rows of a request all add to its counter; counters of
 *                 several requests on one line would queue up behind each other).  ZERO-FILLED ONCE
 *                 after allocation (every call leaves them zero); calls that may run concurrently
 *                 need separate counters.
 */
int32_t specvlm_node_argmax_accept(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                   const void *logits_dev, int64_t stride_b, int64_t stride_n,
                                   const int32_t *num_nodes_dev, const int32_t *parent_dev,
                                   const int32_t *draft_tok_dev, int32_t *amax_dev,
                                   int32_t *accept_len_dev, int32_t *path_dev, int32_t *bonus_tok_dev,
                                   int32_t *committed_tok_dev, int32_t *counters_dev,
                                   int32_t *err_flag_dev, void *stream);

/*
 * Sampling-based acceptance walk, temperature > 0 (Sec. 3.1: speculative sampling discards
 * the incorrect drafted tokens; Sec. 4.1: temperature 1 is evaluated with the same Top-K tree,
 * decoding stays lossless).  The children of a node are fixed candidates, i.e. point-mass
 * proposals.  With p = softmax(logits[b,cur,:] / temperature) at the current node (cur starts
 * at the root), the children c of cur are tried in increasing node index:
 *     x = draft_tok[b,c];  accept c when  u_accept[b,c] < p(x) / (1 - mass rejected at cur so far),
 *     cur <- c and continue with c's own distribution; otherwise x joins cur's rejected tokens
 *     (a token already rejected there, or outside [0,V), is rejected outright).
 * When no child is accepted (or the path holds path_cap nodes) the bonus token is drawn from
 * the residual distribution at cur -- p with cur's rejected tokens removed, renormalised -- by
 * inverse CDF in vocabulary order with u_bonus[b].  Every emitted token is distributed as the
 * target's own sample would be.
 *   logits_dev    device, dtype, element (b,i,v) at b*stride_b + i*stride_n + v; every visited row
 *                 needs a finite maximum (no NaN, no +inf); -inf entries have probability 0
 *   u_accept_dev  device fp32 [B, N_max], u_bonus_dev device fp32 [B]: uniform numbers in [0,1)
 *                 drawn by the caller (entry c is read only if child c is tried)
 *   outputs       as specvlm_tree_accept: accept_len, path, bonus_tok, committed_tok
 * Arithmetic is fp32; a comparison whose two sides differ by less than fp32 rounding of the
 * row sums may fall either way.  Stopping at path_cap with children left sets
 * SPECVLM_ERR_PATH_TOO_LONG; a malformed parent array commits the root only and sets
 * SPECVLM_ERR_BAD_PARENT.
 */
int32_t specvlm_tree_accept_sample(int32_t dtype, int32_t B, int32_t N_max, int32_t V, int32_t path_cap,
                                   const int32_t *parent_dev, const int32_t *draft_tok_dev,
                                   const void *logits_dev, int64_t stride_b, int64_t stride_n,
                                   const int32_t *num_nodes_dev, float temperature,
                                   const float *u_accept_dev, const float *u_bonus_dev,
                                   int32_t *accept_len_dev, int32_t *path_dev, int32_t *bonus_tok_dev,
                                   int32_t *committed_tok_dev, int32_t *err_flag_dev, void *stream);

/*
 * Compaction of the accepted path's K/V rows, all layers in one call (not spelled
 * out by the paper; it is what keeps the cache holding committed tokens only, so
 * that the next round's prefix is contiguous).  For every layer, KV head, and for
 * K and V:
 *     cache[prefix_len[b] + j] <- OLD cache[prefix_len[b] + path[b,j]],  j = 0..accept_len[b]
 * (gather semantics: all sources are read before any destination is written), then
 *     new_prefix_len[b] = prefix_len[b] + accept_len[b] + 1.
 * Layer l's cache is k_base_dev + l*layer_stride elements (same for V), or, when
 * k_layer_ptrs_dev / v_layer_ptrs_dev are non-NULL, the l-th pointer of those DEVICE
 * arrays of L device pointers (then k_base_dev/v_base_dev/layer_stride are ignored).
 * Only desc's dtype, B, H_kv, D, paged, block_size, max_blocks_per_req, kv_capacity
 * and kv_stride_* are used.  new_prefix_len_dev may alias prefix_len_dev (that costs a second,
 * tiny launch: the old lengths may only be overwritten after every workgroup has read them).
 *   moved_idx_dev  optional int32 [B, path_cap, 2]: (src_slot, dst_slot) per j, -1 padded.
 *   err_flag_dev   device int32 or NULL.  A move whose source or destination block id (paged) is
 *                  outside [0, num_blocks) is NOT made -- nothing is ever written into a block the
 *                  table does not validly name -- and sets SPECVLM_ERR_BAD_BLOCK.
 */
int32_t specvlm_kv_compact(const specvlm_attn_desc *desc, int32_t L,
                           void *k_base_dev, void *v_base_dev, int64_t layer_stride,
                           void *const *k_layer_ptrs_dev, void *const *v_layer_ptrs_dev,
                           const int32_t *block_table_dev, const int32_t *prefix_len_dev,
                           const int32_t *path_dev, int32_t path_cap, const int32_t *accept_len_dev,
                           int32_t *new_prefix_len_dev, int32_t *moved_idx_dev, int32_t *err_flag_dev,
                           void *stream);

/*
 * Parameter-free visual token compressors (Sec. 3.4, the elastic vision compressor's two
 * parameter-free experts: the pruning expert discards a random subset of the visual tokens, the
 * pooling expert is a plain pooling operator; Table 4: ratios 2x .. 30x).  They shorten the visual prefix the DRAFT reads;
 * the target keeps the full sequence (that is what keeps decoding lossless).  The paper fixes
 * neither the pooling window nor the treatment of a ragged tail; here: average pooling along the
 * token sequence, window = stride = ratio, the last window shorter when the length is not a multiple:
 *     y[b,j,:] = mean_{t = j*ratio .. min((j+1)*ratio, T_b) - 1} x[b,t,:]   for j < ceil(T_b / ratio)
 * (fp32 sum in token order, one multiplication by 1/count, rounded to dtype), T_b = num_tokens[b]
 * (NULL: T); rows j >= ceil(T_b / ratio) of y are left untouched; out_tokens[b] = ceil(T_b / ratio).
 * num_tokens[b] outside [0, T] is clamped and sets SPECVLM_ERR_BAD_LENGTH.
 *   x_dev  device, dtype, element (b,t,e) at b*x_stride_b + t*x_stride_t + e; E*sizeof(dtype) a
 *          multiple of 16, rows 16-byte aligned
 *   y_dev  device, dtype, [B, ceil(T/ratio), E] via y_stride_b / y_stride_t, same alignment
 */
int32_t specvlm_visual_pool(int32_t dtype, int32_t B, int32_t T, int32_t E, int32_t ratio,
                            const void *x_dev, int64_t x_stride_b, int64_t x_stride_t,
                            const int32_t *num_tokens_dev, void *y_dev, int64_t y_stride_b,
                            int64_t y_stride_t, int32_t *out_tokens_dev, int32_t *err_flag_dev,
                            void *stream);

/*
 * Pruning: y[b,j,:] = x[b, keep[b,j], :] (bit copy) for the T_keep token indices the caller drew
 * (any order, repeats allowed; keep[b,j] == -1 marks padding and leaves row j untouched; an index
 * outside [0, T) leaves the row untouched and sets SPECVLM_ERR_BAD_LENGTH).  Layout rules as above.
 */
int32_t specvlm_visual_prune(int32_t dtype, int32_t B, int32_t T, int32_t T_keep, int32_t E,
                             const void *x_dev, int64_t x_stride_b, int64_t x_stride_t,
                             const int32_t *keep_dev, void *y_dev, int64_t y_stride_b,
                             int64_t y_stride_t, int32_t *err_flag_dev, void *stream);

/*
 * Output head fused with the greedy choice (Fig. 3: target and draft share one output head;
 * Sec. 4.1: temperature 0).  Replaces "project to logits, store them, specvlm_node_argmax":
 *     logit[b,i,v] = sum_e hidden[b,i,e] * W[v,e]          (bf16 products, fp32 accumulation)
 *     amax[b,i]    = the LOWEST v whose logit is the row's greatest (-0 == +0; inputs finite)
 * The [nodes, vocabulary] logits are never stored and W is streamed from HBM once per block of 64
 * node rows.  The choice is taken on the fp32 sums, so against exact arithmetic it can differ
 * only where the two greatest logits of a row are closer than the fp32 accumulation error.
 * Rows i >= num_nodes[b] get amax -1 (their hidden rows are still read and must be finite memory).
 *   dtype          SPECVLM_BF16 only (SPECVLM_F32 returns SPECVLM_UNSUPPORTED)
 *   hidden_dev     device bf16, element (b,i,e) at b*h_stride_b + i*h_stride_n + e, with
 *                  h_stride_b == N_max*h_stride_n; rows 16-byte aligned; E a multiple of 128
 *   w_dev          device bf16 [V, E], row v at v*w_stride_v (the layout of a linear layer's weight)
 *   amax_dev       device int32 [B, N_max]
 *   max_logit_dev  device fp32 [B, N_max] or NULL: the greatest logit (0 for rows past num_nodes)
 *   workspace_dev  specvlm_head_argmax_workspace_bytes(B, N_max, V) bytes, 256-byte aligned,
 *                  ZERO-FILLED ONCE after allocation (every call leaves its counters zero);
 *                  calls that may run concurrently need separate workspaces
 */
size_t specvlm_head_argmax_workspace_bytes(int32_t B, int32_t N_max, int32_t V);
int32_t specvlm_head_argmax(int32_t dtype, int32_t B, int32_t N_max, int32_t E, int32_t V,
                            const void *hidden_dev, int64_t h_stride_b, int64_t h_stride_n,
                            const void *w_dev, int64_t w_stride_v, const int32_t *num_nodes_dev,
                            int32_t *amax_dev, float *max_logit_dev,
                            void *workspace_dev, size_t workspace_bytes, void *stream);

/*
 * ---- Draft side: growth of the token tree that the calls above verify ----------------------
 * Sec. 4.1: following EAGLE-2 the draft grows a tree with Top-K = 10, 60 tokens in total and
 * depth 7 (Fig. 3: its root is the token the target produced last).  The paper gives the three
 * numbers; the growth rule is that method's: the value of a candidate node is the sum of the
 * draft's log-probabilities along its root path; every level expands the most valuable nodes of
 * the previous level by their Top-K tokens; at the end the most valuable candidates of all
 * levels form the tree.  One level is specvlm_draft_select (not needed for the root level)
 * followed by specvlm_draft_topk; specvlm_draft_finalize ends the growth.  The draft model's own
 * attention over the growing tree is specvlm_tree_verify_attn.
 *
 * specvlm_draft_topk: for request b and expanded node w (W per request), over its logits row l:
 *     lse = ln sum_v exp(l_v)
 *     token[k] = the K tokens of greatest logit, greater first, the LOWER token first among
 *                equal logits (values compare as real numbers, -0 == +0; no NaN; finite maximum)
 *     score[k] = cum[b,w] + (l_token[k] - lse)            (fp32; cum NULL means 0)
 *     parent[k] = parent_idx[b,w]                          (copied; -1 when parent_idx is NULL)
 * written to out[b*out_stride_b + w*K + k], so a level can write straight into a request's
 * candidate arrays.  1 <= K <= min(V, 64).
 *   logits_dev      device, dtype, element (b,w,v) at b*stride_b + w*stride_w + v
 *   cum_dev         device fp32, element (b,w) at b*cum_stride_b + w, or NULL
 *   parent_idx_dev  device int32, element (b,w) at b*parent_stride_b + w, or NULL
 *   score_out_dev, token_out_dev, parent_out_dev (optional)   device, indexed as above
 *   lse_out_dev     device fp32 [B, W] or NULL
 */
int32_t specvlm_draft_topk(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K,
                           const void *logits_dev, int64_t stride_b, int64_t stride_w,
                           const float *cum_dev, int64_t cum_stride_b,
                           const int32_t *parent_idx_dev, int64_t parent_stride_b,
                           float *score_out_dev, int32_t *token_out_dev, int32_t *parent_out_dev,
                           int64_t out_stride_b, float *lse_out_dev, void *stream);

/*
 * specvlm_draft_topk followed by specvlm_draft_select over the level's W*K new candidates
 * (score = score_out[b, 0 .. W*K), same M / index_base / sel_* / count_out meaning), as one
 * launch: the workgroup that finishes a request's last row makes the selection.  W*K <= 1024.
 *   counters_dev   device int32 [B * SPECVLM_COUNTER_STRIDE] (request b's counter is word
 *                  b * SPECVLM_COUNTER_STRIDE), ZERO-FILLED ONCE after allocation (every call leaves
 *                  it zero); calls that may run concurrently need separate counters
 */
int32_t specvlm_draft_topk_select(int32_t dtype, int32_t B, int32_t W, int32_t V, int32_t K,
                                  const void *logits_dev, int64_t stride_b, int64_t stride_w,
                                  const float *cum_dev, int64_t cum_stride_b,
                                  const int32_t *parent_idx_dev, int64_t parent_stride_b,
                                  float *score_out_dev, int32_t *token_out_dev, int32_t *parent_out_dev,
                                  int64_t out_stride_b, float *lse_out_dev,
                                  int32_t M, int32_t index_base, int32_t *sel_out_dev,
                                  float *sel_score_out_dev, int32_t *count_out_dev,
                                  int32_t *counters_dev, void *stream);

/*
 * The M most valuable of a request's scored candidates: candidate i beats j when
 * score[i] > score[j], or the scores are equal and i < j (scores are compared as the stored fp32
 * numbers).  Winners are listed in increasing candidate index.
 *   score_dev          device fp32, element (b,i) at b*score_stride_b + i, i < C <= SPECVLM_MAX_CANDIDATES
 *   num_cand_dev       device int32 [B] (clamped to [0, C]) or NULL meaning C
 *   index_base         added to every listed index (position of the scored range in a larger array)
 *   sel_out_dev        device int32 [B, M]: winners, then -1
 *   sel_score_out_dev  device fp32 [B, M] or NULL: their scores, then -inf
 *   count_out_dev      device int32 [B] or NULL: min(M, num_cand[b])
 */
int32_t specvlm_draft_select(int32_t B, int32_t C, int32_t M, const float *score_dev, int64_t score_stride_b,
                             const int32_t *num_cand_dev, int32_t index_base, int32_t *sel_out_dev,
                             float *sel_score_out_dev, int32_t *count_out_dev, void *stream);

/*
 * End of the growth: the N_max - 1 most valuable candidates (rule of specvlm_draft_select) become
 * tree nodes 1.., in increasing candidate index -- a topological order, because a candidate's
 * parent cand_parent[i] (< i, or -1 for a child of the root) was created before it -- and node 0
 * is the root carrying root_token[b]:
 *     node_cand[b,j]  candidate behind node j (-1 for the root and for padding)
 *     parent[b,j]     node index of its parent (-1 for the root and for padding)
 *     draft_tok[b,j]  its token (-1 for padding)
 *     num_nodes[b]    1 + number of chosen candidates
 * These are the parent / draft_tok / num_nodes arrays the verification calls take.  Scores that
 * are sums of log-probabilities never rise from parent to child, so the choice is closed under
 * "parent of"; if it is not, SPECVLM_ERR_TREE_NOT_CLOSED is set (SPECVLM_ERR_BAD_PARENT for a
 * cand_parent entry outside [-1, i), SPECVLM_ERR_BAD_NUM_NODES for num_cand outside [0, C]).
 *   cand_*_dev   device, element (b,i) at b*cand_stride_b + i; C <= SPECVLM_MAX_CANDIDATES
 *   node_cand_out_dev may be NULL; 1 <= N_max <= 64
 */
int32_t specvlm_draft_finalize(int32_t B, int32_t C, int32_t N_max, const float *cand_score_dev,
                               const int32_t *cand_parent_dev, const int32_t *cand_token_dev,
                               int64_t cand_stride_b, const int32_t *num_cand_dev,
                               const int32_t *root_token_dev, int32_t *parent_out_dev,
                               int32_t *draft_tok_out_dev, int32_t *node_cand_out_dev,
                               int32_t *num_nodes_out_dev, int32_t *err_flag_dev, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVLM_H */
