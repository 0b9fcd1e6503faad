/*
 * spex_tree.h -- C ABI of the tree decode-attention library for MI355X (gfx950).
 *
 * Problem served.  Tree-of-Thought search frames reasoning as a tree whose node is
 * the state reached by one step, a coherent run of tokens (paper Sec. 2.1).  The
 * consumer loop of Alg. 2 (Sec. 4.5) adds a child for every finished primary or
 * speculative expansion, BFS mis-speculation terminates a branch at once
 * (Sec. 4.2, "Mis-speculation Handling"), early termination ends a whole query
 * (Sec. 4.4), and sibling branches reuse the KV cache of their shared prefix
 * (Sec. 3.2; Sec. 4.1, insight 2; S_KV(q) of Eq. 1 in Sec. 4.3).  This library keeps
 * that tree as a paged KV cache in which a node owns the pages of its own step and
 * reaches its prefix through parent links, and computes, for many branches in one
 * launch, decode attention over each branch's root-to-node KV while reading every
 * shared page only once.
 *
 * All functions return a spex_status_t, never throw and never abort.  On error the
 * out-parameters are untouched and the tree is unchanged.  A handle is not thread
 * safe: one consumer loop owns it.  Device work is enqueued on the HIP stream given
 * to the call and is asynchronous; the library synchronises only where stated.
 * "HOST" / "DEVICE" below say where a pointer must point.
 */
#ifndef SPEX_TREE_H
#define SPEX_TREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spex_tree spex_tree_t; /* opaque: one forest over one page pool */
typedef int32_t spex_node_t;          /* dense id in creation order, never reused */
#define SPEX_NO_NODE (-1)

typedef enum {
  SPEX_OK = 0,
  SPEX_ERR_INVALID_ARG = 1, /* NULL where data is needed, negative count, bad config */
  SPEX_ERR_BAD_NODE = 2,    /* id unknown or pruned */
  SPEX_ERR_NOT_LEAF = 3,    /* append to a node that has live children */
  SPEX_ERR_OOM_PAGES = 4,   /* the pool has too few free pages; nothing was allocated */
  SPEX_ERR_EMPTY_PATH = 5,  /* a requested node has fewer path tokens than queries (or none) */
  SPEX_ERR_UNSUPPORTED = 6, /* dtype / shape combination without a kernel */
  SPEX_ERR_DEVICE = 7,      /* a HIP call failed; see spex_last_device_error() */
  SPEX_ERR_CAPACITY = 8     /* caller-provided output array too small */
} spex_status_t;

typedef enum { SPEX_F32 = 0, SPEX_BF16 = 1, SPEX_FP8_E4M3 = 2 } spex_dtype_t;

/*
 * Pool layout.  k_pool and v_pool are caller-owned DEVICE buffers of (page, kv head) tiles of
 * page_size * head_dim elements of kv_dtype; with the dense stride each holds
 * num_pages * num_kv_heads tiles (see spex_pool_bytes and page_stride_tiles).  The tile at element
 * offset (page * page_stride_tiles + head) * page_size * head_dim holds page_size tokens; only
 * the library reads and writes inside a tile, in one of two arrangements:
 *
 *  ROW-MAJOR  (kv_dtype F32, or page_size != 16, or head_dim not 64 / 128):
 *     K and V element (token t, dim d) at t * head_dim + d.
 *
 *  MFMA-TILED (kv_dtype BF16 / FP8_E4M3 with page_size 16 and head_dim 64 or 128):
 *     the order in which a 64-lane wavefront consumes MFMA 16x16x32 operands, so that
 *     every 128-bit load instruction of the attention kernels reads contiguous memory
 *     and lands directly in operand registers.
 *     K, bf16:  ((t>>2)&1) * 8*head_dim + (d/32)*256 + ((d%32)/8)*64 + (4*(t>>3) + (t&3))*8 + d%8
 *     V, bf16:  (d/16)*256 + (t/8)*128 + (d%16)*8 + t%8              (token-minor: V transposed;
 *               the 16-bit element is the IEEE half-precision image of the bf16 value, written by
 *               the append calls and turned back into bf16 by spex_tree_gather_kv -- see Value range)
 *     K, fp8 :  ((t>>2)&1) * 8*head_dim + (d/64)*512 + ((d%32)/8)*128 + (4*(t>>3) + (t&3))*16 + ((d/32)&1)*8 + d%8
 *     V, fp8 :  (d/32)*512 + (t/8)*256 + (d%16)*16 + ((d/16)&1)*8 + t%8
 *  Use spex_tree_gather_kv to read tokens back in logical order.
 *
 * fp8 (OCP e4m3fn): value = code * scale, one fp32 scale per (page, kv head), separately
 * for K and V, in the caller-owned DEVICE arrays k_scale / v_scale [num_pages][num_kv_heads].
 * Scales must be finite and >= 0 (0: a page of zeros).
 *
 * Value range.  K, V and q must be finite.  On MFMA-tiled pools the product of the softmax weights
 * with V runs in IEEE half precision.  For a bf16 pool the append calls store V in that format
 * (rounding toward zero), which is exact for zero and every bf16 magnitude in [2^-17, 65504]:
 *   - a bf16 V magnitude above 65504 is stored as 65504 (saturation, never infinity;
 *     spex_tree_gather_kv returns 65280, the bf16 below it);
 *   - a bf16 V magnitude below 2^-17 is stored as the multiple of 2^-24 below it (absolute error
 *     below 2^-24);
 * every kernel on such a pool, the generic one included, sees the stored values.  For an fp8 pool
 * the codes are stored as given and widened when read by the tree-walk and cooperative kernels
 * (kernel_mode 0 / 3, and 2 for nodes shared by more than 16 query rows):
 *   - an fp8 v_scale above 146 (448 * 146 = 65408) is read as 146;
 *   - code * v_scale is formed in half precision in two steps (the power of two of the scale,
 *     then its mantissa rounded to 11 bits): relative error at most 2^-10, and for a magnitude
 *     below 2^-14 an absolute error below 2^-23;
 * the other kernels of an fp8 pool reproduce code * v_scale exactly.  Row-major pools (fp32, other
 * page sizes and head dims) hold and return V as given.  Inside the range every kernel meets the
 * same error bound.
 */
typedef struct {
  int32_t num_q_heads;  /* multiple of num_kv_heads; query head h uses kv head h / (Hq/Hkv) */
  int32_t num_kv_heads;
  int32_t head_dim;     /* 1..256 */
  int32_t page_size;    /* power of two, 1..64 */
  int32_t q_dtype;      /* spex_dtype_t: (F32,F32) | (BF16,BF16) | (BF16,FP8_E4M3) as (q, kv) */
  int32_t kv_dtype;
  int64_t num_pages;
  void *k_pool;         /* DEVICE; may be NULL for a host-only handle (no append data, no attention) */
  void *v_pool;         /* DEVICE */
  float *k_scale;       /* DEVICE, fp8 only, else NULL */
  float *v_scale;       /* DEVICE, fp8 only, else NULL */
  const int32_t *free_order; /* HOST, optional: permutation of 0..num_pages-1, the order in which
                                pages are first handed out; NULL = ascending.  Copied by create. */
  int32_t prefix_chunk_pages; /* split granularity of shared-prefix segments; 0 = automatic */
  int32_t suffix_chunk_pages; /* split granularity of private suffixes;       0 = automatic */
  int32_t kernel_mode;  /* 0 = automatic; 1 = generic (non-MFMA) kernels; 2 = shared-prefix + suffix +
                           merge kernels; 3 = tree-walk kernel (decode_attention fails with
                           SPEX_ERR_UNSUPPORTED where it does not apply) */
  int32_t page_stride_tiles; /* distance between consecutive pages of a pool, in (page, head) tiles;
                                0 = num_kv_heads (dense).  2 * num_kv_heads with
                                v_pool = k_pool + num_kv_heads tiles interleaves K and V of a page
                                in one buffer, so that a page's K and V share a 64 KiB region. */
  int32_t walk_row_tiles; /* tree-walk kernel: 16-row tiles per wavefront, 1 / 2 / 4; 0 = automatic */
  int32_t walk_waves;     /* tree-walk kernel: wavefronts of query rows per workgroup, 2 / 4 / 8; 0 = 4.
                             2: four wavefronts run, two on each set of rows, and split the rows' path
                             between them (walk_row_tiles 1 or 2, no draft masks) */
} spex_config_t;

/* Bytes each of k_pool and v_pool must hold for this config. */
spex_status_t spex_pool_bytes(const spex_config_t *cfg, size_t *bytes_per_pool);

const char *spex_status_string(spex_status_t s);
/* Text of the last HIP error seen by this thread's calls ("" if none). */
const char *spex_last_device_error(void);

/* Create an empty forest over the caller's pool.  The config is copied. */
spex_status_t spex_tree_create(const spex_config_t *cfg, spex_tree_t **out);
/* Frees host state and the library's own device workspace (plan, partial results).
 * Synchronises the device.  The pools stay the caller's. */
void spex_tree_destroy(spex_tree_t *tree);

/*
 * Alg. 2 "add_node / add_spec_node": create n_children empty nodes under parent
 * (SPEX_NO_NODE: new roots, i.e. new user queries).  Ids written to out_children[n_children]
 * (HOST) are consecutive.  Children share the parent's pages through the parent link; nothing
 * is copied, and a child's first token always starts a fresh page.  Primary and speculative
 * children are the same kind of node.
 */
spex_status_t spex_tree_fork(spex_tree_t *tree, spex_node_t parent, int32_t n_children,
                             spex_node_t *out_children);

/*
 * Append the K/V of n_tokens generated tokens (a step, or one decode token of it) to a node
 * without live children.  k, v: DEVICE, [n_tokens][num_kv_heads][head_dim] in kv_dtype.
 * fp8: k_scales / v_scales are DEVICE arrays [n_new_pages][num_kv_heads] with the scale of
 * every page this append newly starts (see spex_tree_append_new_pages); tokens that continue a
 * partially filled page use the scale that page already has.  Pages are taken from the
 * allocator one at a time in token order; if too few are free the call fails with
 * SPEX_ERR_OOM_PAGES and changes nothing.  Unused slots of a newly started page are zeroed.
 * The scatter into the pool is enqueued on hip_stream (a hipStream_t, NULL = default stream);
 * the source buffers must stay valid until that work has run.
 * k == NULL and v == NULL: only the page table is updated (host-only handles, or callers that
 * never read these tokens back).
 */
spex_status_t spex_tree_append_step(spex_tree_t *tree, spex_node_t node, int32_t n_tokens,
                                    const void *k, const void *v, const float *k_scales,
                                    const float *v_scales, void *hip_stream);
/*
 * The same append with the cache quantised on the fly (fp8 pools only, else SPEX_ERR_UNSUPPORTED):
 * k, v are DEVICE [n_tokens][num_kv_heads][head_dim] in bf16 with finite values.  For every page
 * the append starts, the scatter kernel first takes amax = the largest magnitude among the tokens
 * this append puts into that page, per kv head and separately for K and V, and sets the page's
 * scale = max(amax / 448, 2^-40); tokens that continue a partially filled page use the scale the
 * page already has (never requantised; they saturate).  code = e4m3fn(x * (1 / scale)), division,
 * reciprocal and product in fp32, round to nearest even, saturating at +-448.
 */
spex_status_t spex_tree_append_step_quantize(spex_tree_t *tree, spex_node_t node, int32_t n_tokens,
                                             const void *k, const void *v, void *hip_stream);
/*
 * The decode iteration between two steps (Sec. 3.1: a step is tens to hundreds of tokens, generated
 * one at a time; Alg. 2: all live branches are generated concurrently): append ONE token to each
 * of n_nodes distinct nodes without live children, with one kernel launch.
 *   nodes : HOST [n_nodes]
 *   k, v  : DEVICE [n_nodes][num_kv_heads][head_dim] in kv_dtype (both NULL: page table only)
 *   k_scales, v_scales : DEVICE fp32 [n_nodes][num_kv_heads], fp8 only: row i is used if node i's
 *           token starts a new page and ignored otherwise
 * All or nothing: if a node is unknown, repeated (SPEX_ERR_INVALID_ARG), has live children, or
 * the pool has too few free pages for all of them, nothing is changed.  Pages are taken in the
 * order of `nodes`.  If the handle holds launch lists on the device that the appends can be
 * patched into (see spex_tree_decode_attention), the same launch that scatters the tokens also
 * writes the new page lengths, query limits and started pages into them, and a decode_attention
 * call that repeats the previous request then runs without planning, upload or patch launch (it
 * reports plan state 2).  Both calls must be on the same stream, or ordered by the caller.
 */
spex_status_t spex_tree_append_tokens(spex_tree_t *tree, const spex_node_t *nodes, int32_t n_nodes,
                                      const void *k, const void *v, const float *k_scales,
                                      const float *v_scales, void *hip_stream);
/*
 * The same step with the cache quantised on the fly (fp8 pools only, else SPEX_ERR_UNSUPPORTED):
 * k, v are DEVICE [n_nodes][num_kv_heads][head_dim] in bf16, as the model produces them, and the
 * kernel that scatters them also encodes them: code = e4m3fn(x * (1 / scale)), product and
 * reciprocal in fp32, round to nearest even, saturating at +-448, NaN kept.  scale is row i of
 * k_scales / v_scales if node i's token starts a page (the row becomes that page's scale) and the
 * scale the page already has otherwise -- a page is never requantised, later tokens saturate.
 * Everything else (argument checks, all or nothing, page order, structure version) as
 * spex_tree_append_tokens.
 */
spex_status_t spex_tree_append_tokens_quantize(spex_tree_t *tree, const spex_node_t *nodes,
                                               int32_t n_nodes, const void *k, const void *v,
                                               const float *k_scales, const float *v_scales,
                                               void *hip_stream);
/* Number of pages an append of n_tokens to node would newly start. */
spex_status_t spex_tree_append_new_pages(const spex_tree_t *tree, spex_node_t node,
                                         int32_t n_tokens, int32_t *n_new_pages);

/*
 * Sec. 4.2 mis-speculation / Sec. 4.4 early termination: remove node and its whole subtree and
 * return their pages to the allocator (pre-order over the subtree, children in creation order,
 * each node's pages in order; the page returned last is handed out first).  Pruning a root ends
 * that query.  A parent left without children may be appended to again.
 */
spex_status_t spex_tree_prune(spex_tree_t *tree, spex_node_t node);

/*
 * Decode attention for n_leaves requested nodes (usually the live leaves; any live node is
 * accepted, also twice).  q_lens[i] >= 1 queries belong to leaves[i] (NULL: all 1): the last
 * q_lens[i] tokens of its path are the query tokens (already appended), and query j sees path
 * positions 0 .. T_i - q_lens[i] + j, T_i being the number of tokens on the root-to-node path.
 *   leaves, q_lens : HOST
 *   q   : DEVICE [sum(q_lens)][num_q_heads][head_dim] in q_dtype, requested-node major
 *   out : DEVICE fp32, same shape:  sum_t softmax_t(sm_scale * <q, K_t>) V_t  over visible t
 *   lse : DEVICE fp32 [sum(q_lens)][num_q_heads] or NULL:  ln sum_t exp(sm_scale * <q, K_t>)
 *   sm_scale must be positive and finite.
 * The call flattens parent links into per-launch work lists, uploads them when the request or
 * the tree changed since the previous call, and enqueues the kernels on hip_stream without
 * waiting for them.  If the only change is that tokens were appended to requested nodes (the
 * usual decode iteration), the cached lists are patched instead, on the host and -- with one
 * small kernel, or inside the spex_tree_append_tokens launch -- in the device copy: the valid
 * count of each grown page and the limits of its queries; and, if the tree-walk lists are the
 * only lists the cached plan holds, the pages the appends started: such a page becomes page b of
 * its node's last block or a new block in the room kept behind the private blocks of the node's
 * wavefront (two blocks per requested childless node when the plan is made; when a wavefront's
 * room is used up, or a started page belongs to a node that several wavefronts or requests
 * share, the call plans afresh).  Two kernel sets compute the same result:
 *   tree-walk: one workgroup carries a block of up to 16 * walk_row_tiles * walk_waves query rows (requested
 *     nodes that are neighbours in the tree) from the root to the requested nodes; pages shared
 *     by rows of several wavefronts are fetched once per workgroup, the softmax state stays in
 *     registers, only the output is written.  Needs MFMA-tiled pools and Hq / Hkv <= 64 (one
 *     query token's rows fit a wavefront; a requested node with more rows than a wavefront takes
 *     is cut into pieces of whole query tokens).  Chosen automatically when it yields >= 128
 *     workgroups, or when no wavefront has more two-page blocks to walk than 20 (up to 32
 *     workgroups) rising to 87 (127 workgroups): 20 + (workgroups - 32) * 7 / 10;
 *   shared-prefix + suffix + merge: every shared node is read once for all rows below it, private
 *     suffixes are split for parallelism, partial softmax states go through memory.  Any shape.
 * Consecutive calls on one handle must use one stream or be separated by a synchronisation,
 * because they share the handle's workspace.  A call that repeats the previous request on an
 * unchanged tree (plan state 0, profiling off) only launches kernels -- no planning, allocation,
 * copy or event -- and may therefore be recorded in a HIP graph; the recorded launches read the
 * handle's device lists, so the graph is valid until a call plans afresh or the handle goes.
 */
spex_status_t spex_tree_decode_attention(spex_tree_t *tree, const spex_node_t *leaves,
                                         const int32_t *q_lens, int32_t n_leaves, const void *q,
                                         float *out, float *lse, float sm_scale, void *hip_stream);

/*
 * For callers that cannot allocate device memory (code under HIP graph capture set-up, tight
 * serving loops, harnesses that forbid hipMalloc): spex_tree_decode_attention with the same
 * arguments, result and kernels, except that the call allocates nothing -- no hipMalloc, hipFree,
 * pinned host memory or event.  The launch lists and the partial softmax states of the
 * shared-prefix / suffix kernels go into a 64 MiB array that the library holds statically on every
 * GPU it runs on, from the load of its code object until the process ends (16 MiB for the lists,
 * 48 MiB for partial states), instead of the handle's grow-only workspace; the lists are copied
 * there from pageable host memory on every call, so nothing stays cached on the device between
 * calls and no plan state is shared with spex_tree_decode_attention's device copy (the host side
 * of the plan -- planning afresh, patching after appends -- is shared).  A request whose lists or
 * partial states exceed the array fails with SPEX_ERR_CAPACITY before anything is launched.
 * Per-kernel profiling is not recorded for these calls.  All calls on one GPU share the array,
 * whichever handle they use: calls that overlap in time on one GPU (different streams, threads or
 * handles) race; calls in stream order do not, each call rewrites what it reads.
 */
spex_status_t spex_tree_decode_attention_static(spex_tree_t *tree, const spex_node_t *leaves,
                                                const int32_t *q_lens, int32_t n_leaves, const void *q,
                                                float *out, float *lse, float sm_scale, void *hip_stream);

/*
 * Sec. 6.5 (composition with token-level speculative decoding): the draft tokens a branch
 * verifies in one step form a small token TREE rather than a chain.  Same as decode_attention,
 * except that the last q_lens[i] tokens of leaves[i]'s path are drafts whose mutual visibility
 * the caller states:
 *   draft_masks : HOST [sum(q_lens)], requested-node major like q.  With B_i = T_i - q_lens[i],
 *     query j of request i sees path positions 0 .. B_i - 1 (everything before the drafts) and
 *     position B_i + k iff bit k of its mask is set.  For a draft tree the mask holds the bits of
 *     the draft's ancestors and of itself; the chain is mask_j = 2^(j+1) - 1, which gives
 *     decode_attention's result.  NULL = that chain.
 * With masks, q_lens must be given and q_lens[i] <= 32; bits at or above q_lens[i] must be clear
 * (SPEX_ERR_INVALID_ARG); a query that sees no position at all is SPEX_ERR_EMPTY_PATH.  Nothing is
 * launched when an error is returned.  Every kernel set evaluates masks (the automatic choice
 * between them is the one of decode_attention), except the tree-walk kernel that splits the path:
 * kernel_mode 3 where the tree-walk kernel cannot take the request, or with walk_waves 2, is
 * SPEX_ERR_UNSUPPORTED.
 * Length patches work as for decode_attention: the masks are part of the cached request.
 */
spex_status_t spex_tree_decode_attention_masked(spex_tree_t *tree, const spex_node_t *leaves,
                                                const int32_t *q_lens, const uint32_t *draft_masks,
                                                int32_t n_leaves, const void *q, float *out,
                                                float *lse, float sm_scale, void *hip_stream);

/* ---- introspection (host only unless stated) -------------------------------------------- */

typedef struct {
  spex_node_t parent;
  int32_t n_tokens;
  int32_t n_pages;
  int32_t n_live_children;
} spex_node_info_t;
spex_status_t spex_tree_node_info(const spex_tree_t *tree, spex_node_t node, spex_node_info_t *out);

/* Pages of the root-to-node path in order and the number of valid tokens in each.  At most cap
 * entries are written (SPEX_ERR_CAPACITY if more are needed; *n is set to the needed count). */
spex_status_t spex_tree_path_pages(const spex_tree_t *tree, spex_node_t node, int32_t *pages,
                                   int32_t *valid, int32_t cap, int32_t *n);
/* Free pages, the one handed out next first. */
spex_status_t spex_tree_free_pages(const spex_tree_t *tree, int32_t *pages, int32_t cap, int32_t *n);
spex_status_t spex_tree_stats(const spex_tree_t *tree, int64_t *live_nodes, int64_t *used_pages,
                              int64_t *free_pages);

/*
 * The work lists a decode_attention call with the same arguments would use.  All pointers are
 * HOST arrays owned by the tree, valid until the next call that plans or mutates the tree.
 *   leaf_indptr[n_leaves+1], leaf_pages[], leaf_valid[]: root-to-node page lists (CSR).
 *   qt_limit[n_qtok]: visible path length of every query token.
 *   group_node[n_groups]: nodes with >= 2 requested nodes below them and >= 1 token, ascending.
 *   Tasks (one per chunk of a segment; the n_prefix_tasks group chunks first, then the suffix
 *   chunks in request order): pages pg_id/pg_valid/pg_pos[task_pg_begin .. + task_pg_count)
 *   (page id, valid tokens, path position of the page's first token), rows
 *   qt_list[task_qt_begin .. + task_qt_count) (query-token indices), first partial slot
 *   task_pbase, task_flags bit 0 = some page partial or some row's limit inside the chunk,
 *   bit 1 = suffix task that is the only chunk of its suffix (the suffix kernel then folds the
 *   rows' other pieces in and writes the output rows itself).
 *   Merge lists: query token t combines entries part_indptr[t] .. part_indptr[t+1]; the slot of
 *   (kv head g, head-in-group hh) in entry e is part_base[e] + g * part_hstride[e] + hh.
 *   merge_qt[n_merge_qt]: the query tokens that still need the separate merge kernel.
 */
typedef struct {
  int32_t n_leaves, n_qtok, n_groups, n_tasks, n_prefix_tasks, n_pg, n_qt_list, n_parts, n_merge_qt;
  int64_t n_partial_rows;
  int32_t prefix_chunk_pages, suffix_chunk_pages; /* the values actually used */
  const int32_t *leaf_indptr, *leaf_pages, *leaf_valid;
  const int32_t *qt_limit;
  const int32_t *group_node;
  const int32_t *task_pg_begin, *task_pg_count, *task_qt_begin, *task_qt_count, *task_pbase,
      *task_flags;
  const int32_t *pg_id, *pg_valid, *pg_pos;
  const int32_t *qt_list;
  const int32_t *part_indptr, *part_base, *part_hstride;
  const int32_t *merge_qt;
} spex_plan_view_t;
spex_status_t spex_tree_plan_dump(spex_tree_t *tree, const spex_node_t *leaves,
                                  const int32_t *q_lens, int32_t n_leaves, spex_plan_view_t *out);

/* Copy a node's own tokens [first, first + n) out of the pool in logical order:
 * k_out, v_out DEVICE [n][num_kv_heads][head_dim] in kv_dtype; fp8 codes are copied as stored and
 * k_scale_out / v_scale_out (DEVICE [n][num_kv_heads] fp32, may be NULL) receive each token's
 * page scale.  Enqueued on hip_stream. */
spex_status_t spex_tree_gather_kv(spex_tree_t *tree, spex_node_t node, int32_t first, int32_t n,
                                  void *k_out, void *v_out, float *k_scale_out, float *v_scale_out,
                                  void *hip_stream);

/* Change the split granularities (0 = automatic), kernel_mode, walk_row_tiles and walk_waves
 * after creation. */
spex_status_t spex_tree_set_tuning(spex_tree_t *tree, int32_t prefix_chunk_pages,
                                   int32_t suffix_chunk_pages, int32_t kernel_mode,
                                   int32_t walk_row_tiles, int32_t walk_waves);

/*
 * The tree-walk kernel's lists for a request (HOST arrays owned by the tree, valid until the next
 * call that plans or mutates it).  available = 0: one query token has more rows (Hq / Hkv) than
 * one wavefront takes; the arrays are then empty.  With G = Hq / Hkv, C = 16 * row_tiles rows per
 * wavefront and NW = waves wavefronts per row block (a requested node with more than C / G
 * queries counts as ceil(q_len / (C / G)) requests of consecutive queries, sizes differing by
 * at most one, the longer ones first):
 *   qt[2 * n_qt]: {query token, visible path length} of the requested nodes, grouped by root
 *     (roots in order of first appearance) and sorted by path below a root, so that the requests
 *     below any node are consecutive.
 *   row_blocks[(3 + 3 * NW) * n_row_blocks]: {root node, first block, shared blocks, private
 *     blocks of wavefronts 0..NW-1 as count | room << 16, first qt entry of each wavefront, qt
 *     entries of each wavefront}.  room >= count records belong to the wavefront; those beyond
 *     count are zero until an append starts a block there (a fresh plan leaves two per requested
 *     node without live children that is private to the wavefront).  Requests fill a wavefront while their q_len * G rows fit into C; wavefront NW
 *     or a new root starts a new row block.  Row of a request: wavefront * C + rows before it in the wavefront.
 *   blocks[8 * n_blocks]: {page a, pos_a << 7 | valid_a, page b, pos_b << 7 | valid_b (0 = no page
 *     b), first row | (last row + 1) << 16, flags, 0, 0}: two consecutive pages of one node on the
 *     row block's paths, the path position and valid tokens of each, and the rows whose path
 *     holds the node.  A row block's blocks: first the nodes whose rows touch several
 *     wavefronts, then those of wavefront 0, 1, .. alone, each followed by its unused room; every
 *     page of every row's path appears exactly once per row block.  Flag bit 0: a page is partial or missing, or some
 *     row in the range may not see every position the block holds (the block ends beyond the
 *     first position that some query of a request in the range does not see: T - q_len + 1 for
 *     the chain, T - q_len + the number of leading drafts all its queries see with draft_masks,
 *     which may be NULL as in decode_attention_masked).  Flag bit 1: the node is also on the
 *     paths of another row block.
 *   items[S * n_items], S = 16 for NW = 4 and 32 for NW = 8: launch order, one workgroup each:
 *     {kv head, copy of row block fields 1.., zeros, row block index in the last int}; index -1 =
 *     padding that keeps the row blocks of one root on one XCD when fewer than 8 kv heads exist.
 */
typedef struct {
  int32_t available, row_tiles, waves, n_row_blocks, n_blocks, n_qt, n_items;
  int32_t plan_state; /* how this call got its plan: 0 cached, 1 planned afresh, 2 cached plan patched */
  const int32_t *row_blocks, *blocks, *qt, *items;
} spex_walk_view_t;
spex_status_t spex_tree_walk_dump(spex_tree_t *tree, const spex_node_t *leaves,
                                  const int32_t *q_lens, const uint32_t *draft_masks,
                                  int32_t n_leaves, spex_walk_view_t *out);

/*
 * Per-kernel timing.  While profiling is enabled, every decode_attention call brackets each of
 * its kernels with HIP events on the call's stream (the last 256 calls are kept).
 * spex_tree_read_profile waits for those events and writes, for each recorded call in order,
 * milliseconds for ms[4*c+0] = shared-prefix kernel, ms[4*c+1] = suffix kernel, ms[4*c+2] = merge
 * kernel, ms[4*c+3] = tree-walk kernel (0 for a kernel that was not launched; cap counts calls,
 * ms holds 4 * cap floats); *n = number of calls; the record is then
 * cleared.  SPEX_ERR_CAPACITY (with *n set) if cap calls are too few.  Enabling or disabling
 * profiling also clears the record.
 */
spex_status_t spex_tree_set_profiling(spex_tree_t *tree, int32_t enabled);
spex_status_t spex_tree_read_profile(spex_tree_t *tree, float *ms, int32_t cap, int32_t *n);

/* Counts of the last decode_attention call, for the throughput metric:
 * info[0] distinct KV tokens on the requested paths, [6] 0 = the cached plan was used, 1 = planned
 * afresh, 2 = the cached plan was patched (tokens had been appended to requested nodes),
 * [7] 0 = shared-prefix + suffix + merge kernels ran ([1] tokens in shared-prefix tasks, [2] tokens in
 * suffix tasks, [3] prefix work items, [4] suffix work items, [5] partial rows), else the tree-walk
 * kernel ran with [7] = row tiles per wavefront + 256 * wavefronts per workgroup ([3] workgroups
 * with work, [4] two-page blocks summed over workgroups of one kv head, [5] 0). */
spex_status_t spex_tree_last_launch_info(const spex_tree_t *tree, int64_t info[8]);

#ifdef __cplusplus
}
#endif
#endif /* SPEX_TREE_H */
