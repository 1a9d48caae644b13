/*
 * eagletv - teacher verification step of tree speculative decoding on AMD MI355X (gfx950).
 *
 * C ABI of the HIP library (libeagletv.so).  The five operations follow the
 * problem statement of "EAGLE-Pangu" (arXiv 2603.08088): Section 2.4 / 3.3 (tree
 * attention mask), Section 3.3 (tree-masked teacher attention over the committed
 * prefix cache plus the speculative tokens), Section 3.2 (sentinel-free gathers
 * through a valid dummy index), Section 2.3 / 5.1 (greedy posterior acceptance)
 * and Section 3.1 (commit of the accepted path into the prefix cache).
 *
 * Conventions
 *  - Every pointer is a DEVICE pointer unless its name starts with h_ (the
 *    descriptor structs are host memory).  The caller owns every buffer,
 *    including workspaces; the library never allocates, frees or keeps a pointer.
 *  - Every launch call is asynchronous on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and never synchronises the device.
 *  - Return value: ETV_OK or a negative ETV_ERR_* for errors detectable on the
 *    host (bad shapes, unsupported dtype, workspace too small, launch failure).
 *    Data-dependent conditions (malformed tree, cache capacity) are reported in
 *    a per-sequence device `status` array that the caller reads with the results.
 *  - Node rows: sequence b has n_nodes[b] valid rows 0..n_nodes[b]-1 out of
 *    T_max; row 0 is the root (the last accepted token; it plays the role of the
 *    paper's dummy-root row 0), rows >= n_nodes[b] are padding.
 *  - Query head h reads KV head h / (Hq / Hkv).
 *  - bf16 tensors are IEEE bfloat16 (upper half of fp32).
 */
#ifndef EAGLETV_H
#define EAGLETV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* The library is built with hidden visibility; only the entry points below are exported. */
#if defined(ETV_BUILDING)
#define ETV_API __attribute__((visibility("default")))
#else
#define ETV_API
#endif

#define ETV_OK 0
#define ETV_ERR_INVALID_ARG (-1)        /* null pointer, non-positive size, dummy out of range ...      */
#define ETV_ERR_UNSUPPORTED (-2)        /* dtype / head_dim / T_max / grouping outside the built kernels */
#define ETV_ERR_WORKSPACE_TOO_SMALL (-3)
#define ETV_ERR_HIP (-4)                /* a kernel launch failed; see etv_last_hip_error()             */
#define ETV_ERR_UNIMPLEMENTED (-5)      /* a defined operation this library does not build (a replica of a contiguous cache) */

#define ETV_F32 0
#define ETV_BF16 1

/* status bits written by etv_build_tree_mask (Section 3.2, "Structural invariants") */
#define ETV_TREE_RANGE 1   /* parent[k] outside [0, T_max), or parent[0] != 0                   */
#define ETV_TREE_CYCLE 2   /* repeated parent application from k does not reach row 0           */
#define ETV_TREE_CLOSURE 4 /* valid node whose parent slot is padding (>= n_nodes)              */
#define ETV_TREE_PATHS 8   /* etv_tensorize_tree: more leaves than rows in the path table        */
#define ETV_TREE_DEPTH 16  /* etv_tensorize_tree: a root-to-leaf path has more than W nodes      */

/* status bits written by etv_commit_accepted_kv */
#define ETV_COMMIT_CAPACITY 1  /* prefix_len + accept_len + 1 exceeds capacity[b] (or the block table) */
#define ETV_COMMIT_BAD_NODE 2  /* an accepted node index is not a valid node row (in place: or not increasing) */
#define ETV_COMMIT_BAD_LEN 4   /* accept_len outside [0, W-1]                                          */
#define ETV_COMMIT_BAD_BLOCK 8 /* a needed block-table entry is outside [0, num_blocks)                */
/* additional status bits of etv_replicate_branches */
#define ETV_BRANCH_NO_BLOCKS 16 /* the free list is shorter than what the call needs: nothing was taken   */
#define ETV_BRANCH_BAD_FREE 32  /* a free-list entry this sequence would use is outside [0, num_blocks)   */

#define ETV_MAX_TREE 256       /* largest T_max of the mask builder, gather and posterior              */
#define ETV_ATTN_MAX_TREE 256  /* largest T_max of tree_verify_attention                               */

ETV_API const char *etv_status_string(int32_t status);
ETV_API const char *etv_version(void);
/* hipError_t code of the most recent failed launch in this thread (0 if none). */
ETV_API int32_t etv_last_hip_error(void);

/* ---------------------------------------------------------------------------
 * build_tree_mask - Section 3.2 "Ancestor tables", Section 3.3 "Tree attention
 * mask" and "Implementation note" (compact ancestor encoding generated on device).
 *
 * For every valid node k the set of its ancestors-or-self is found by bounded
 * parent walking and emitted (a) as a per-row bitmask, the form the attention
 * kernel consumes, and (b) optionally as the dense 4D mask [B,1,T_max,T_max]
 * (1 = may attend; the additive form is dense ? 0 : -inf).  The structural
 * invariants are checked on the way.  A node that violates one is treated as a
 * child of the root, so every output is defined for every input.
 *
 *  parent   in  int32 [B, T_max]   parent row of each node; parent[b][0] must be 0
 *  n_nodes  in  int32 [B]          valid rows per sequence (clamped to [0, T_max])
 *  bitmask  out uint64 [B, T_max, ceil(T_max/64)]  bit (j%64) of word j/64 of row k: k attends j
 *  dense    out uint8 [B, 1, T_max, T_max]  nullable
 *  depth    out int32 [B, T_max]   parent steps to the root (0 for padding)     nullable
 *  status   out int32 [B]          OR of ETV_TREE_* bits (0 = all invariants hold)
 * Requires 1 <= T_max <= ETV_MAX_TREE.
 * ------------------------------------------------------------------------- */
ETV_API int32_t etv_build_tree_mask(const int32_t *parent, const int32_t *n_nodes, int32_t B, int32_t T_max,
                            uint64_t *bitmask, uint8_t *dense, int32_t *depth, int32_t *status, void *stream);

/* ---------------------------------------------------------------------------
 * tensorize_tree -- Section 3.2 ("Node linearization and base arrays", "Dummy-root
 * indexing", "Ancestor tables", "Padding and batch semantics", "Structural
 * invariants") and Section 3.3 ("Execution view": node k sits at position
 * prefix length + depth[k]).
 *
 * Everything the verification step needs to know about the tree, from the parent
 * array alone and in one launch: the outputs of etv_build_tree_mask plus position
 * ids and the table of root-to-leaf paths (the retrieve indices that
 * etv_safe_gather_paths and etv_evaluate_posterior consume).  One row per leaf,
 * leaves in ascending row order; entry i of a row is the path's node at depth i;
 * -1 behind the leaf and in the rows behind the last leaf.  A leaf is a valid node
 * that no valid node names as its parent.  Nodes that break an invariant hang off
 * the root, as in etv_build_tree_mask.
 *
 *  parent, n_nodes, bitmask, dense, depth, status   as for etv_build_tree_mask;
 *                status may also carry ETV_TREE_PATHS (more than L_max leaves: the
 *                first L_max are kept) and ETV_TREE_DEPTH (a path of more than W
 *                nodes: its first W are kept)
 *  prefix_len    in  int32 [B]              needed if position_ids is given; negative counts as 0
 *  position_ids  out int32 [B, T_max]       prefix_len[b] + depth (prefix_len[b] for padding)  nullable
 *  retrieve      out int32 [B, L_max, W]
 *  n_paths       out int32 [B]              rows written per sequence                           nullable
 * Requires 1 <= T_max <= ETV_MAX_TREE, L_max >= 1, W >= 1, L_max * W <= 2^24.
 * ------------------------------------------------------------------------- */
ETV_API int32_t etv_tensorize_tree(const int32_t *parent, const int32_t *n_nodes, const int32_t *prefix_len, int32_t B,
                           int32_t T_max, int32_t L_max, int32_t W, uint64_t *bitmask, uint8_t *dense, int32_t *depth,
                           int32_t *position_ids, int32_t *retrieve, int32_t *n_paths, int32_t *status, void *stream);

/* ---------------------------------------------------------------------------
 * tree_verify_attention - Section 3.3 "Execution view" and "Tree attention mask".
 *
 * out[b,k,h,:] = sum_j softmax_j(q[b,k,h,:] . K_j * scale) V_j over the keys
 * visible to node k: every committed prefix key 0..prefix_len[b]-1 and the tree
 * keys j whose bit is set in bitmask[b,k].  Padded rows (k >= n_nodes[b]) give
 * zeros and lse = -inf.  The prefix cache is only read.
 *
 * Layouts (row-major, innermost last; element type per h_desc->dtype):
 *  q, out        [B, T_max, Hq, d]
 *  kt, vt        [B, T_max, Hkv, d]                    K/V of the tree tokens of this step; both NULL: an
 *                in-place branch cache (Section 3.3 "KV-cache writes and commit") -- the verification pass has
 *                written the K/V of node j of sequence b into the cache itself at position prefix_len[b] + j
 *                (so P_max + T_max positions must exist: P_cap, or max_blocks * block_size when paged)
 *  k_cache/v_cache  contiguous (block_size == 0): [B, P_cap, Hkv, d]
 *                   paged (block_size == 16):     [num_blocks, Hkv, block_size, d], logical position p of
 *                   sequence b lives in block block_table[b][p / block_size] at offset p % block_size
 *  block_table   int32 [B, max_blocks]  (paged only, else NULL)
 *  prefix_len    int32 [B]              0 <= prefix_len[b] <= P_max
 *  bitmask       as written by etv_build_tree_mask with the same T_max
 *  lse           float [B, Hq, T_max]   natural-log sum of exp of the scaled scores, nullable
 *  workspace     etv_tree_verify_attention_workspace_bytes(h_desc) bytes, 256-byte aligned
 * Supported: dtype F32 or BF16 (fp32 accumulation), d in {64, 128}, Hq % Hkv == 0,
 * 1 <= T_max <= ETV_ATTN_MAX_TREE.  bf16 with d = 128 runs on the MFMA kernel.
 * ------------------------------------------------------------------------- */
typedef struct etv_attn_desc {
    int32_t B, T_max, Hq, Hkv, d;
    int32_t dtype;      /* ETV_F32 | ETV_BF16 */
    int32_t block_size; /* 0: contiguous cache; 16: paged cache */
    int32_t max_blocks; /* paged: row length of block_table */
    int32_t num_blocks; /* paged: blocks in the pool (not read by attention) */
    int32_t P_cap;      /* contiguous: rows allocated per sequence */
    int32_t P_max;      /* host-known upper bound of prefix_len[b]; sizes the launch */
    float scale;        /* 0 => 1/sqrt(d) */
    int32_t kv_split;   /* keys per work unit (multiple of 64); 0 => chosen by the library */
    int32_t flags;      /* ETV_ATTN_FLAG_* */
} etv_attn_desc;

#define ETV_ATTN_FLAG_GENERIC 1 /* run the fp32-VALU kernel even where the MFMA kernel applies (diagnostics) */
#define ETV_ATTN_FLAG_SMALL_WG 2 /* always use 4-wavefront workgroups (tuning) */
#define ETV_ATTN_FLAG_WHOLE_TILE 4 /* every wavefront takes whole 64-key tiles, never key halves (tuning) */
#define ETV_ATTN_FLAG_KEY_HALVES 8 /* two wavefronts per 32-row chunk wherever the tree is small enough (tuning) */

#define ETV_ATTN_FLAG_LARGE_WG 16 /* 8-wavefront workgroups wherever the tree has enough rows for them (tuning) */
#define ETV_ATTN_FLAG_UNIFORM_SPLITS 32 /* one split size for the whole batch, also where the splits could follow the
                                           sequences' lengths (tuning) */

ETV_API size_t etv_tree_verify_attention_workspace_bytes(const etv_attn_desc *h_desc);

/* The launch shape the library picks for h_desc (host only, launches nothing): which kernel, how many wavefronts
 * per workgroup, whether two wavefronts share a 32-row chunk (key halves), the depth of the K/V tile ring, the row
 * groups per (split, KV head), the keys per split and the number of splits.  The pick comes from a small cost
 * model fitted on one machine; kv_split and the ETV_ATTN_FLAG_* tuning flags of h_desc override every part of it,
 * and this call shows the outcome, so that a poor pick on another shape or machine can be seen and corrected. */
typedef struct etv_attn_plan {
    int32_t mfma;        /* 1: attn_mfma_kernel (bf16, d = 128); 0: the fp32-VALU kernel */
    int32_t wavefronts;  /* per workgroup: 4 or 8 (1 for the VALU kernel) */
    int32_t key_halves;  /* 1: two wavefronts per 32-row chunk, each with 32 of a tile's 64 keys */
    int32_t ring_stages; /* K/V tiles of LDS ring */
    int32_t row_groups;  /* workgroups per (split, KV head, sequence) */
    int32_t kv_split;    /* prefix keys per split (multiple of 64) */
    int32_t n_splits;    /* splits the launch provides; more than 1 means partials + the combine launch */
    int32_t balanced_splits; /* 1: the launch's B * n_splits split slots are shared out among the sequences by their
                                lengths (on the device): sequence b cuts its prefix into as many equal parts as its
                                share; kv_split is then the size for a sequence of P_max keys */
    int64_t workgroups;  /* grid size of the partial kernel */
} etv_attn_plan;

ETV_API int32_t etv_tree_verify_attention_plan(const etv_attn_desc *h_desc, etv_attn_plan *out);

ETV_API int32_t etv_tree_verify_attention(const etv_attn_desc *h_desc, const void *q, const void *k_cache,
                                  const void *v_cache, const int32_t *block_table, const int32_t *prefix_len,
                                  const void *kt, const void *vt, const uint64_t *bitmask, const int32_t *n_nodes,
                                  void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/* etv_tree_verify_attention for callers that cannot allocate device memory or carry a workspace around: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * errors, without workspace / workspace_bytes: the partial results of the key splits go to a fixed array of
 * ETV_ATTN_STATIC_WORKSPACE_BYTES bytes of device memory inside the library (every GPU the library runs on holds
 * its own copy until the process ends).  The call allocates and frees nothing.
 *  - A shape whose etv_tree_verify_attention_workspace_bytes() exceeds the array returns
 *    ETV_ERR_WORKSPACE_TOO_SMALL and launches nothing (use the call above with a workspace of your own, or a
 *    larger h_desc->kv_split, which means fewer splits).
 *  - All calls on one GPU share that GPU's array: two of them must not overlap in time (different streams without
 *    an ordering between them, or different host threads, race); calls on one stream are ordered and safe.
 *  - The device that is current when the call is made must be the one `stream` and the buffers belong to. */
#define ETV_ATTN_STATIC_WORKSPACE_BYTES (64u << 20)

ETV_API int32_t etv_tree_verify_attention_static(const etv_attn_desc *h_desc, const void *q, const void *k_cache,
                                         const void *v_cache, const int32_t *block_table, const int32_t *prefix_len,
                                         const void *kt, const void *vt, const uint64_t *bitmask,
                                         const int32_t *n_nodes, void *out, float *lse, void *stream);

/* ---------------------------------------------------------------------------
 * safe_gather_paths - contribution 2, Section 3.2 "Dummy-root indexing" and
 * "Padding and batch semantics", Section 2.5 (device-defined for every index value).
 *
 *   safe[b,p,i]   = idx if 0 <= idx < T_max else dummy          (idx = retrieve[b,p,i])
 *   pvalid[b,p,i] = 1 iff 0 <= idx < n_nodes[b]
 *   gathered[b,p,i,:] = src[b, safe[b,p,i], :]                   (row of row_bytes bytes)
 *
 *  retrieve in  int32 [B, L_max, W]   node indices root->leaf of each path, padding = any negative value
 *  n_nodes  in  int32 [B]             nullable (=> T_max)
 *  src      in  bytes [B, T_max, row_bytes]          nullable together with gathered
 *  safe     out int32 [B, L_max, W]   nullable;  pvalid out uint8 [B, L_max, W] nullable
 *  gathered out bytes [B, L_max, W, row_bytes]
 * dummy must lie in [0, T_max) (ETV_ERR_INVALID_ARG otherwise).
 * ------------------------------------------------------------------------- */
ETV_API int32_t etv_safe_gather_paths(const int32_t *retrieve, const int32_t *n_nodes, int32_t B, int32_t L_max,
                              int32_t W, int32_t T_max, int32_t dummy, const void *src, size_t row_bytes,
                              int32_t *safe, uint8_t *pvalid, void *gathered, void *stream);

/* ---------------------------------------------------------------------------
 * evaluate_posterior - greedy posterior acceptance (Section 2.3; temperature 0,
 * Section 5.1) with the score extraction of Section 3.3 "Mapping teacher outputs
 * to node verification scores" guarded by validity.
 *
 *   argmax[b,n]  = lowest index of the maximum of logits[b,n,:]  (n < n_nodes[b]; -1 for padding)
 *   len[b,p]     = number of leading positions i with both path entries valid and
 *                  tokens[safe[b,p,i+1]] == argmax[safe[b,p,i]]
 *   best[b]      = lowest p of maximal len;  accept_len[b] = len[b,best[b]]
 *   acc_nodes[b,0..accept_len] = safe node indices of the accepted prefix (root first), tail = dummy
 *   bonus[b]     = argmax at the last accepted node
 *
 *  logits float [B, T_max, V] (no NaN); tokens int32 [B, T_max]; retrieve int32 [B, L_max, W];
 *  argmax int32 [B,T_max]; len int32 [B,L_max]; best, accept_len, bonus int32 [B]; acc_nodes int32 [B,W].
 *  workspace: etv_evaluate_posterior_workspace_bytes(B, T_max, V) bytes.
 *  logits may be NULL.  With V == 0, argmax[B,T_max] is then an input (the teacher's choice per node) and no
 *  workspace is needed.  With V > 0, the workspace is the one etv_lm_head_argmax has just filled for the same
 *  B, T_max and V when called with argmax == NULL: the choice per node is finished from it here (and written
 *  to argmax), which saves that call's finishing launch.
 * Requires 1 <= T_max <= ETV_MAX_TREE, W >= 1, L_max >= 1, 0 <= dummy < T_max.
 * ------------------------------------------------------------------------- */
ETV_API size_t etv_evaluate_posterior_workspace_bytes(int32_t B, int32_t T_max, int32_t V);

ETV_API int32_t etv_evaluate_posterior(const float *logits, const int32_t *tokens, const int32_t *retrieve,
                               const int32_t *n_nodes, int32_t B, int32_t T_max, int32_t V, int32_t L_max,
                               int32_t W, int32_t dummy, int32_t *argmax, int32_t *len, int32_t *best,
                               int32_t *accept_len, int32_t *acc_nodes, int32_t *bonus, void *workspace,
                               size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * commit_accepted_kv - Section 3.1 "Path-index-based commit" in its
 * prefix-sharing fast form: the committed prefix stays where it is and only the
 * accepted rows are gathered from the tree buffer and appended, for all layers
 * in one launch.  Row acc_nodes[b,i] of the tree K/V goes to logical position
 * prefix_len[b] + i for i = 0..accept_len[b] (the root and the accepted draft
 * tokens); prefix_len_out[b] = prefix_len[b] + accept_len[b] + 1.
 *   slot_map[b,i] = physical slot of that position (block*block_size + offset when paged,
 *                   the position itself when contiguous), -1 for i > accept_len[b].
 * A sequence that fails a check is left untouched (status bit set, prefix_len_out
 * = prefix_len, slot_map = -1).
 *
 *  kt, vt       [n_layers, B, T_max, Hkv, d]; both NULL: in-place branch cache -- the tree rows are in the cache
 *               at positions prefix_len[b] + node, and the accepted ones are compacted to prefix_len[b] + i
 *               (path-index commit over the cache alone; needs prefix_len[b] + n_nodes[b] <= capacity[b], else
 *               ETV_COMMIT_CAPACITY, and an accepted path whose node indices increase strictly -- the tail was
 *               written in node order and every root-to-leaf path of a tree numbered parents-first reads it front
 *               to back -- else ETV_COMMIT_BAD_NODE; prefix_len_out must not alias prefix_len)
 *  k_cache/v_cache: layer l starts cache_layer_stride elements after layer l-1; per-layer layout as in attention
 *  prefix_len, capacity, n_nodes, accept_len int32 [B]; acc_nodes int32 [B, W]
 *  prefix_len_out int32 [B] (may alias prefix_len); slot_map int32 [B, W]; status int32 [B]
 * ------------------------------------------------------------------------- */
typedef struct etv_commit_desc {
    int32_t B, T_max, Hkv, d;
    int32_t elem_bytes; /* 2 (bf16) or 4 (fp32) */
    int32_t n_layers;
    int32_t W;          /* row length of acc_nodes and slot_map */
    int32_t block_size; /* 0: contiguous; > 0: paged */
    int32_t max_blocks;
    int32_t num_blocks;
    int32_t P_cap;
    int32_t reserved;
    int64_t cache_layer_stride; /* elements between consecutive layers of k_cache (and v_cache) */
} etv_commit_desc;

ETV_API int32_t etv_commit_accepted_kv(const etv_commit_desc *h_desc, const void *kt, const void *vt, void *k_cache,
                               void *v_cache, const int32_t *block_table, const int32_t *prefix_len,
                               const int32_t *capacity, const int32_t *n_nodes, const int32_t *acc_nodes,
                               const int32_t *accept_len, int32_t *prefix_len_out, int32_t *slot_map,
                               int32_t *status, void *stream);

/* ---------------------------------------------------------------------------
 * lm_head_argmax -- Section 3.3 ("Execution view", "Mapping teacher outputs to
 * node verification scores") and Section 5.1 (greedy decoding): the teacher's
 * head turns the hidden state of every tree node into logits over the
 * vocabulary, and greedy acceptance needs only their argmax.  One pass over the
 * head weights; the logits are never written to memory.
 *   logits[b,k,v] = sum_c hidden[b,k,c] * weight[v,c]   (bf16 inputs, fp32 accumulation)
 *   argmax[b,k]   = lowest v among the maxima; -1 for padded rows (k >= n_nodes[b])
 *
 *  hidden   in  bf16 [B, T_max, D]     16-byte aligned
 *  weight   in  bf16 [V, D] row-major (weight_packed = 0), or the same weights packed once by
 *               etv_pack_lm_head (weight_packed = 1), which streams a quarter faster; 16-byte aligned
 *  n_nodes  in  int32 [B]
 *  argmax   out int32 [B, T_max]       can be handed to etv_evaluate_posterior / etv_verify_epilogue
 *                                      in place of logits (see there).  NULL: stop after the weight pass
 *                                      and leave the per-tile maxima in the workspace for those calls
 *  maxval   out float [B, T_max]       the maximal logit, -inf for padded rows     nullable
 *  workspace: etv_lm_head_argmax_workspace_bytes(B, T_max, V) bytes.
 * Requires D % 128 == 0.  Up to 64 rows, and every group of 128 rows beyond that, stream the weights once
 * (repeats come from L2): the shape of a verify step, bound by the weight stream.  Beyond 256 rows (a batch of
 * trees) the product is bound by the matrix cores and runs as a GEMM tiling of 256 vocabulary rows x 256 node rows
 * per workgroup.  The result does not depend on which of the three kernels ran beyond the order of the fp32
 * accumulation.
 * ------------------------------------------------------------------------- */
ETV_API size_t etv_lm_head_argmax_workspace_bytes(int32_t B, int32_t T_max, int32_t V);

ETV_API int32_t etv_lm_head_argmax(const void *hidden, const void *weight, int32_t weight_packed,
                           const int32_t *n_nodes, int32_t B, int32_t T_max, int32_t D, int32_t V, int32_t *argmax,
                           float *maxval, void *workspace, size_t workspace_bytes, void *stream);

/* Head weights in the order etv_lm_head_argmax reads them: tiles of 128 vocabulary rows x 128 elements, each
 * 32 KiB of consecutive memory ([ceil(V/128)][D/128][128][128], rows past V are zero).  Done once per set of
 * weights.  packed: etv_lm_head_packed_bytes(V, D) bytes, 16-byte aligned.  Requires D % 128 == 0. */
ETV_API size_t etv_lm_head_packed_bytes(int32_t V, int32_t D);

ETV_API int32_t etv_pack_lm_head(const void *weight, int32_t V, int32_t D, void *packed, void *stream);

/* ---------------------------------------------------------------------------
 * verify_epilogue -- everything after the teacher forward in one launch (two when
 * the logits have to be scanned first): the safe gather (Section 3.2 "Dummy-root
 * indexing"), greedy acceptance (Sections 2.3 and 5.1) and the commit of the
 * accepted rows for all layers (Section 3.1 "Commit by path indices and
 * prefix-sharing fast reorder"), with the accepted length and nodes never leaving
 * the device.  Arguments, layouts, outputs and status bits are those of
 * etv_safe_gather_paths, etv_evaluate_posterior and etv_commit_accepted_kv called
 * in that order with W = h_desc->W as the row length of retrieve, acc_nodes and
 * slot_map; the results are identical.  safe, pvalid and (src, gathered) are
 * nullable as there; logits may be NULL as there (argmax is then an input).
 * Unlike etv_commit_accepted_kv, prefix_len_out must not alias prefix_len
 * (ETV_ERR_INVALID_ARG): several workgroups of the launch still read the old length.
 * workspace: etv_evaluate_posterior_workspace_bytes(B, T_max, V) bytes.
 * Requires T_max <= ETV_MAX_TREE and W <= ETV_MAX_TREE.
 * ------------------------------------------------------------------------- */
ETV_API int32_t etv_verify_epilogue(const etv_commit_desc *h_desc, const float *logits, int32_t V, const int32_t *tokens,
                            const int32_t *retrieve, int32_t L_max, int32_t dummy, const void *src, size_t row_bytes,
                            int32_t *safe, uint8_t *pvalid, void *gathered, int32_t *argmax, int32_t *len,
                            int32_t *best, int32_t *accept_len, int32_t *acc_nodes, int32_t *bonus, const void *kt,
                            const void *vt, void *k_cache, void *v_cache, const int32_t *block_table,
                            const int32_t *prefix_len, const int32_t *capacity, const int32_t *n_nodes,
                            int32_t *prefix_len_out, int32_t *slot_map, int32_t *status, void *workspace,
                            size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * Branch caches over a paged cache pool -- Section 3.1 "Branchable KV-cache
 * abstraction".  The two calls below work on block tables over ONE pool
 * (k_cache / v_cache, per-layer layout [num_blocks, Hkv, block_size, d] as in
 * attention; layer l starts cache_layer_stride elements after layer l-1).
 * ------------------------------------------------------------------------- */
typedef struct etv_cache_desc {
    int32_t B, Hkv, d;
    int32_t elem_bytes; /* 2 (bf16) or 4 (fp32) */
    int32_t n_layers;
    int32_t block_size; /* > 0: paged; 0: contiguous (etv_commit_path_indices only) */
    int32_t max_blocks; /* row length of every block table */
    int32_t num_blocks;
    int32_t P_cap;      /* contiguous: rows per sequence */
    int32_t reserved;
    int64_t cache_layer_stride;
} etv_cache_desc;

/* replicate_branches -- B_i <- Replicate(C*) for N branches per sequence (Section 3.1), as copy-on-write block
 * tables instead of a deep copy: a branch shares every block that lies wholly inside the committed prefix (nothing
 * writes below prefix_len) and owns the blocks from position prefix_len[b] on -- the partly filled block that
 * holds position prefix_len[b], with its committed rows copied in, and the blocks its tail of tail_len[b] rows
 * will reach.  Extending a branch in place therefore touches neither the committed cache nor another branch, and
 * every branch reads the committed rows.  Branch tables are ordinary block tables: attention, commit and the
 * epilogue take branch_table viewed as [B*N, max_blocks] with the per-sequence arrays repeated N times.
 *
 *   first = prefix_len[b] / block_size, last = ceil((prefix_len[b] + tail_len[b]) / block_size),
 *   need_b = last - first (0 if the lengths are refused: ETV_COMMIT_BAD_LEN, ETV_COMMIT_CAPACITY),
 *   block_base[b] = N * sum of need over b' < b; branch i owns free_blocks[block_base[b] + i*need_b + k] as logical
 *   block first + k.  n_taken[0] = N * sum_b need_b: the caller's free list continues behind it.  The accounting
 *   follows the lengths alone: a sequence refused for what a table holds (ETV_COMMIT_BAD_BLOCK, ETV_BRANCH_BAD_FREE)
 *   keeps its share of the free list, unused.  If n_taken would exceed n_free, nothing is copied, n_taken[0] = 0
 *   and every sequence that needs blocks gets ETV_BRANCH_NO_BLOCKS.
 *   Status bits per sequence: ETV_COMMIT_BAD_LEN (negative length), ETV_COMMIT_CAPACITY (last > max_blocks),
 *   ETV_COMMIT_BAD_BLOCK (a committed block outside the pool), ETV_BRANCH_NO_BLOCKS, ETV_BRANCH_BAD_FREE.
 *   The table rows of a failed sequence are -1 throughout; entries from `last` on are -1.
 *
 *  block_table  in  int32 [B, max_blocks]     the committed cache's table
 *  prefix_len, tail_len in int32 [B]
 *  free_blocks  in  int32 [n_free]            distinct blocks that no table uses (the caller's allocator)
 *  branch_table out int32 [B, N, max_blocks]
 *  block_base   out int32 [B];  n_taken out int32 [1];  status out int32 [B]
 * All device pointers.  Requires d * elem_bytes % 16 == 0 and a paged cache: block_size == 0 (a contiguous
 * cache, whose replica would be the paper's deep copy) returns ETV_ERR_UNIMPLEMENTED. */
ETV_API int32_t etv_replicate_branches(const etv_cache_desc *h_desc, void *k_cache, void *v_cache,
                               const int32_t *block_table, const int32_t *prefix_len, const int32_t *tail_len,
                               int32_t N, const int32_t *free_blocks, int32_t n_free, int32_t *branch_table,
                               int32_t *block_base, int32_t *n_taken, int32_t *status, void *stream);

/* commit_path_indices -- Section 3.1 "Commit by path indices and prefix-sharing fast reorder": path_indices maps
 * the next step's prefix sequence to positions of the selected branch cache, and the committed cache is the branch
 * cache gathered along the sequence axis,
 *     new[b, j] = branch[b, path_indices[b, j]],   0 <= j < new_len[b],
 * for every layer, KV head, K and V (any order, repeats allowed: the general full reorder).  Source and
 * destination are separate storage: two contiguous buffers [B, P_cap, Hkv, d] (src != dst), or two block tables
 * over one pool whose written blocks are not blocks of the source (the caller's contract).
 * fast != 0 (paged only): the part of the prefix whose order the indices preserve is not moved --
 * kept_len[b] = the longest j <= new_len[b] with path_indices[b, k] = k for all k < j, rounded down to whole blocks;
 * dst_table takes the source's block ids for those blocks and only rows >= kept_len[b] are gathered into the
 * destination's own blocks.  The decision comes from the indices themselves, so an inconsistent prefix shortens
 * what is kept, down to the full reorder (kept_len = 0, also for fast = 0 and for contiguous caches; the
 * prefix-sharing commit of a contiguous cache is etv_commit_accepted_kv).
 *   Status bits: ETV_COMMIT_BAD_LEN (new_len outside [0, L_cap] or src_len outside the source's capacity),
 *   ETV_COMMIT_CAPACITY (new_len beyond the destination), ETV_COMMIT_BAD_NODE (an index outside [0, src_len)),
 *   ETV_COMMIT_BAD_BLOCK (a needed table entry outside the pool).  A failed sequence writes nothing and keeps
 *   its dst_table row.
 *
 *  src_k, src_v in; dst_k, dst_v out   (paged: dst_k == src_k and dst_v == src_v, the one pool; else ETV_ERR_INVALID_ARG)
 *  src_table in int32 [B, max_blocks]; dst_table in/out int32 [B, max_blocks] (NULL when contiguous)
 *  path_indices in int32 [B, L_cap]; src_len, new_len in int32 [B]; kept_len, status out int32 [B]
 * All device pointers.  Requires d * elem_bytes % 16 == 0. */
ETV_API int32_t etv_commit_path_indices(const etv_cache_desc *h_desc, const void *src_k, const void *src_v, void *dst_k,
                                void *dst_v, const int32_t *src_table, int32_t *dst_table,
                                const int32_t *path_indices, int32_t L_cap, const int32_t *src_len,
                                const int32_t *new_len, int32_t fast, int32_t *kept_len, int32_t *status,
                                void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EAGLETV_H */
