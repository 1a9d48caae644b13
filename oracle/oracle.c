/*
 * CPU oracle for the teacher verification step of tree speculative decoding.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, fp64 statement of what
 * the step computes, written from the paper's definitions.  It shares no code
 * with the HIP library and must never be reached from the product path: only
 * the tests, the smoke check and the benchmark's cpu_baseline leg load it.
 *
 * All pointers are host pointers.  Floating-point work is done in double;
 * bf16 inputs (dtype 1, carried as uint16 bit patterns) convert exactly.
 * Loops over independent output rows carry an OpenMP pragma and nothing else
 * is blocked, fused or reordered.
 *
 * Parity pins (tests/test_oracle_*.py): every function below is pinned against
 * something other than itself - brute-force ancestor walks, closed forms,
 * numpy/torch float64 library attention on the special cases that reduce to it
 * (one-node tree = decode attention, chain = causal attention, per-node
 * sequential equivalence), a hand-worked 7-node example, sequential-append
 * commit, and for the path table parent walks from every leaf plus the closed
 * forms of a chain, a star and a complete binary tree; branch replication
 * against the deep copy it encodes (content, isolation, block accounting) and
 * the path-index commit against numpy's gather of the logical rows and the
 * length-based commit.  No function here is "parity unpinned".
 *
 * Conventions (shared with the seeded generators):
 *   node rows 0..n_nodes[b]-1 of sequence b are valid, row 0 is the root (the
 *   last accepted token, the paper's dummy-root row 0 of Section 3.2);
 *   parent[b][0] = 0; padded rows are ignored.
 */
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_OK 0
#define ORC_ERR_ARG (-1)
#define ORC_ERR_NOMEM (-2)

/* status bits of the structural invariants, Section 3.2 "Structural invariants" */
#define ORC_TREE_RANGE 1   /* parent outside [0, T_max) (or parent[0] != 0)            */
#define ORC_TREE_CYCLE 2   /* repeated parent application does not reach the root       */
#define ORC_TREE_CLOSURE 4 /* a valid node whose parent slot is not valid               */

/* status bits of commit */
#define ORC_COMMIT_CAPACITY 1 /* prefix_len + A + 1 exceeds the sequence's capacity     */
#define ORC_COMMIT_BAD_NODE 2 /* an accepted node index is not a valid node row         */
#define ORC_COMMIT_BAD_LEN 4  /* accept length outside [0, W-1]                         */
#define ORC_COMMIT_BAD_BLOCK 8 /* a needed block-table entry is outside the block pool  */

static double load_val(const void *p, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float *)p)[i];
    uint32_t u = ((uint32_t)((const uint16_t *)p)[i]) << 16; /* bf16 -> fp32 is exact */
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* ------------------------------------------------------------------------
 * Tree mask.  Section 3.2 "Ancestor tables": A[0][k] = k, A[l+1][k] =
 * parent(A[l][k]); Section 3.3 "Tree attention mask": k may attend j iff some
 * level l has A[l][k] == j and both slots are valid.  The invariants of
 * Section 3.2 are checked first; a node that violates one is re-attached to
 * the root (row 0) so the table is always well defined:
 *   - parent outside [0, T_max): RANGE; inside [n_nodes, T_max): CLOSURE;
 *   - a node whose parent chain does not reach row 0 within n_nodes steps: CYCLE.
 * Outputs: dense[b][k][j] in {0,1}; bitmask[b][k][w] bit (j%64) of word j/64;
 * depth[b][k]; status[b] (OR of the bits above).  Padded rows are all zero.
 * ---------------------------------------------------------------------- */
int orc_build_tree_mask(const int32_t *parent, const int32_t *n_nodes, int B, int T_max, uint64_t *bitmask,
                        uint8_t *dense, int32_t *depth, int32_t *status) {
    if (B < 0 || T_max < 1) return ORC_ERR_ARG;
    int words = (T_max + 63) / 64;
    int32_t *ep = (int32_t *)malloc(sizeof(int32_t) * (size_t)T_max);
    int32_t *dep = (int32_t *)malloc(sizeof(int32_t) * (size_t)T_max);
    int32_t *A = (int32_t *)malloc(sizeof(int32_t) * (size_t)T_max * (size_t)T_max);
    if (!ep || !dep || !A) return ORC_ERR_NOMEM;
    for (int b = 0; b < B; b++) {
        int n = n_nodes[b];
        if (n < 0) n = 0;
        if (n > T_max) n = T_max;
        const int32_t *par = parent + (size_t)b * T_max;
        int32_t st = 0;
        /* effective parents after the range and closure checks */
        for (int k = 0; k < n; k++) {
            int32_t p = par[k];
            if (k == 0) {
                if (p != 0) st |= ORC_TREE_RANGE;
                ep[0] = 0;
            } else if (p < 0 || p >= T_max) {
                st |= ORC_TREE_RANGE;
                ep[k] = 0;
            } else if (p >= n) {
                st |= ORC_TREE_CLOSURE;
                ep[k] = 0;
            } else {
                ep[k] = p;
            }
        }
        /* depth = number of parent steps to reach row 0; none within n steps => cycle */
        for (int k = 0; k < n; k++) {
            int cur = k, steps = 0;
            while (cur != 0 && steps < n) {
                cur = ep[cur];
                steps++;
            }
            dep[k] = (cur == 0) ? steps : -1;
        }
        for (int k = 0; k < n; k++)
            if (dep[k] < 0) {
                st |= ORC_TREE_CYCLE;
                ep[k] = 0;
                dep[k] = 1;
            }
        int Dmax = 0;
        for (int k = 0; k < n; k++)
            if (dep[k] > Dmax) Dmax = dep[k];
        /* ancestor table, (Dmax+1) x n */
        for (int k = 0; k < n; k++) A[k] = k;
        for (int l = 0; l < Dmax; l++)
            for (int k = 0; k < n; k++) A[(size_t)(l + 1) * T_max + k] = ep[A[(size_t)l * T_max + k]];
        /* mask */
        for (int k = 0; k < T_max; k++) {
            for (int j = 0; j < T_max; j++) {
                int anc = 0;
                if (k < n && j < n)
                    for (int l = 0; l <= Dmax; l++)
                        if (A[(size_t)l * T_max + k] == j) anc = 1;
                if (dense) dense[((size_t)b * T_max + k) * T_max + j] = (uint8_t)anc;
                if (bitmask) {
                    uint64_t *wrd = bitmask + ((size_t)b * T_max + k) * words + j / 64;
                    if (j % 64 == 0) *wrd = 0;
                    if (anc) *wrd |= ((uint64_t)1) << (j % 64);
                }
            }
            if (depth) depth[(size_t)b * T_max + k] = (k < n) ? dep[k] : 0;
        }
        if (status) status[b] = st;
    }
    free(ep);
    free(dep);
    free(A);
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Tree tensorization.  Section 3.2: node linearization with the dummy-root row
 * 0, the ancestor table A[0][k] = k, A[l+1][k] = parent(A[l][k]), padding with
 * device-defined values guarded by `valid`, and the structural invariants;
 * Section 3.3 "Execution view": node k sits at position t + depth[k] behind an
 * accepted prefix of length t.
 *
 * From parent[b][:] alone this writes, per sequence,
 *   depth[k]         steps from k to row 0 (0 for padding),
 *   position_ids[k]  prefix_len[b] + depth[k] (prefix_len[b] for padding),
 *   retrieve[r][i]   one row per leaf, leaves in ascending row index; entry i is
 *                    the node at depth i of the root-to-leaf path, read off the
 *                    ancestor table as A[depth[leaf] - i][leaf]; -1 beyond the
 *                    leaf and in rows beyond the last leaf,
 *   n_paths          number of rows written.
 * A leaf is a valid node that no valid node names as its parent (the root of a
 * one-node tree is a leaf).  Nodes that break an invariant are first re-attached
 * to the root exactly as orc_build_tree_mask does, so the two agree on the tree.
 * More leaves than L_max: PATHS bit, the first L_max leaves are kept.  A path
 * longer than W nodes: DEPTH bit, its first W nodes are kept.
 * ---------------------------------------------------------------------- */
#define ORC_TREE_PATHS 8  /* more leaves than rows in retrieve                         */
#define ORC_TREE_DEPTH 16 /* a root-to-leaf path has more than W nodes                 */

int orc_tensorize_tree(const int32_t *parent, const int32_t *n_nodes, const int32_t *prefix_len, int B, int T_max,
                       int L_max, int W, int32_t *depth, int32_t *position_ids, int32_t *retrieve, int32_t *n_paths,
                       int32_t *status) {
    if (B < 0 || T_max < 1 || L_max < 1 || W < 1) return ORC_ERR_ARG;
    int32_t *ep = (int32_t *)malloc(sizeof(int32_t) * (size_t)T_max);
    int32_t *dep = (int32_t *)malloc(sizeof(int32_t) * (size_t)T_max);
    int32_t *A = (int32_t *)malloc(sizeof(int32_t) * (size_t)(T_max + 1) * (size_t)T_max);
    uint8_t *has_child = (uint8_t *)malloc((size_t)T_max);
    if (!ep || !dep || !A || !has_child) return ORC_ERR_NOMEM;
    for (int b = 0; b < B; b++) {
        int n = n_nodes[b];
        if (n < 0) n = 0;
        if (n > T_max) n = T_max;
        const int32_t *par = parent + (size_t)b * T_max;
        int32_t st = 0;
        for (int k = 0; k < n; k++) {
            int32_t p = par[k];
            if (k == 0) {
                if (p != 0) st |= ORC_TREE_RANGE;
                ep[0] = 0;
            } else if (p < 0 || p >= T_max) {
                st |= ORC_TREE_RANGE;
                ep[k] = 0;
            } else if (p >= n) {
                st |= ORC_TREE_CLOSURE;
                ep[k] = 0;
            } else {
                ep[k] = p;
            }
        }
        for (int k = 0; k < n; k++) {
            int cur = k, steps = 0;
            while (cur != 0 && steps < n) {
                cur = ep[cur];
                steps++;
            }
            dep[k] = (cur == 0) ? steps : -1;
        }
        for (int k = 0; k < n; k++)
            if (dep[k] < 0) {
                st |= ORC_TREE_CYCLE;
                ep[k] = 0;
                dep[k] = 1;
            }
        int Dmax = 0;
        for (int k = 0; k < n; k++)
            if (dep[k] > Dmax) Dmax = dep[k];
        for (int k = 0; k < n; k++) A[k] = k;
        for (int l = 0; l < Dmax; l++)
            for (int k = 0; k < n; k++) A[(size_t)(l + 1) * T_max + k] = ep[A[(size_t)l * T_max + k]];
        int P = prefix_len ? prefix_len[b] : 0;
        if (P < 0) P = 0;
        for (int k = 0; k < T_max; k++) {
            if (depth) depth[(size_t)b * T_max + k] = (k < n) ? dep[k] : 0;
            if (position_ids) position_ids[(size_t)b * T_max + k] = P + ((k < n) ? dep[k] : 0);
        }
        memset(has_child, 0, (size_t)T_max);
        for (int k = 1; k < n; k++) has_child[ep[k]] = 1;
        int32_t *rows = retrieve + (size_t)b * L_max * W;
        for (size_t e = 0; e < (size_t)L_max * W; e++) rows[e] = -1;
        int r = 0;
        for (int k = 0; k < n; k++) {
            if (has_child[k]) continue;
            if (r >= L_max) {
                st |= ORC_TREE_PATHS;
                break;
            }
            if (dep[k] + 1 > W) st |= ORC_TREE_DEPTH;
            for (int i = 0; i <= dep[k] && i < W; i++) rows[(size_t)r * W + i] = A[(size_t)(dep[k] - i) * T_max + k];
            r++;
        }
        if (n_paths) n_paths[b] = r;
        if (status) status[b] = st;
    }
    free(ep);
    free(dep);
    free(A);
    free(has_child);
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Tree-masked attention.  Section 3.3 "Execution view" and "Tree attention
 * mask": each valid node row k of sequence b attends to every committed prefix
 * key (positions 0..prefix_len[b]-1 of the cache) and to the tree keys j with
 * dense[b][k][j] = 1; the output is the softmax-weighted mean of the matching
 * value rows with scores q.k * scale.  Two passes over the explicit list of
 * visible keys, no running rescale.  Query head h reads KV head h / (Hq/Hkv).
 * Padded rows (k >= n_nodes[b]) give zeros and lse = -inf.
 *
 * Layouts: q [B,T_max,Hq,d]; kt, vt [B,T_max,Hkv,d]; prefix cache either
 * contiguous [B,P_cap,Hkv,d] (block_table NULL) or paged
 * [num_blocks,Hkv,block_size,d] addressed through block_table [B,max_blocks].
 * out [B,T_max,Hq,d] double; lse [B,Hq,T_max] double (natural log), nullable.
 * ---------------------------------------------------------------------- */
int orc_tree_verify_attention(int B, int T_max, int Hq, int Hkv, int d, int dtype, const void *q,
                              const void *k_cache, const void *v_cache, const int32_t *block_table, int block_size,
                              int max_blocks, int P_cap, const int32_t *prefix_len, const void *kt, const void *vt,
                              const uint8_t *dense, const int32_t *n_nodes, double scale, double *out, double *lse) {
    if (B < 0 || T_max < 1 || Hq < 1 || Hkv < 1 || Hq % Hkv || d < 1) return ORC_ERR_ARG;
    if (dtype != 0 && dtype != 1) return ORC_ERR_ARG;
    if (block_table && block_size < 1) return ORC_ERR_ARG;
    int G = Hq / Hkv;
    if (scale == 0.0) scale = 1.0 / sqrt((double)d);
    long rows = (long)B * Hq * T_max;
    int err = 0;
#pragma omp parallel for schedule(dynamic, 4)
    for (long r = 0; r < rows; r++) {
        int b = (int)(r / ((long)Hq * T_max));
        int h = (int)((r / T_max) % Hq);
        int k = (int)(r % T_max);
        int kvh = h / G;
        double *o = out + (((size_t)b * T_max + k) * Hq + h) * d;
        for (int c = 0; c < d; c++) o[c] = 0.0;
        int n = n_nodes[b];
        if (k >= n) {
            if (lse) lse[((size_t)b * Hq + h) * T_max + k] = -INFINITY;
            continue;
        }
        int P = prefix_len[b];
        size_t nvis_max = (size_t)P + (size_t)n;
        double *s = (double *)malloc(sizeof(double) * nvis_max);
        size_t *voff = (size_t *)malloc(sizeof(size_t) * nvis_max); /* element offset of each visible K/V row */
        uint8_t *vsrc = (uint8_t *)malloc(nvis_max);                /* 0: prefix cache, 1: tree buffer */
        if (!s || !voff || !vsrc) {
            err = 1;
            free(s);
            free(voff);
            free(vsrc);
            continue;
        }
        size_t nv = 0;
        for (int j = 0; j < P; j++) {
            size_t off;
            if (block_table) {
                int blk = block_table[(size_t)b * max_blocks + j / block_size];
                off = (((size_t)blk * Hkv + kvh) * block_size + (size_t)(j % block_size)) * d;
            } else {
                off = (((size_t)b * P_cap + j) * Hkv + kvh) * d;
            }
            voff[nv] = off;
            vsrc[nv] = 0;
            nv++;
        }
        for (int j = 0; j < n; j++)
            if (dense[((size_t)b * T_max + k) * T_max + j]) {
                voff[nv] = (((size_t)b * T_max + j) * Hkv + kvh) * d;
                vsrc[nv] = 1;
                nv++;
            }
        size_t qoff = (((size_t)b * T_max + k) * Hq + h) * d;
        double m = -INFINITY;
        for (size_t i = 0; i < nv; i++) {
            const void *kp = vsrc[i] ? kt : k_cache;
            double acc = 0.0;
            for (int c = 0; c < d; c++) acc += load_val(q, dtype, qoff + c) * load_val(kp, dtype, voff[i] + c);
            s[i] = acc * scale;
            if (s[i] > m) m = s[i];
        }
        double denom = 0.0;
        for (size_t i = 0; i < nv; i++) {
            s[i] = exp(s[i] - m);
            denom += s[i];
        }
        for (size_t i = 0; i < nv; i++) {
            const void *vp = vsrc[i] ? vt : v_cache;
            double w = s[i] / denom;
            for (int c = 0; c < d; c++) o[c] += w * load_val(vp, dtype, voff[i] + c);
        }
        if (lse) lse[((size_t)b * Hq + h) * T_max + k] = m + log(denom);
        free(s);
        free(voff);
        free(vsrc);
    }
    return err ? ORC_ERR_NOMEM : ORC_OK;
}

/* ------------------------------------------------------------------------
 * Safe path gather.  Contribution 2 and Section 3.2 "Dummy-root indexing" /
 * "Padding and batch semantics": a padding index (negative, or outside the
 * node table) is replaced by a valid dummy row before any gather, and a
 * validity flag guards every later use.
 *   safe   = idx if 0 <= idx < T_max else dummy
 *   pvalid = 1 iff 0 <= idx < n_nodes[b]
 *   gathered[b][p][i][:] = src[b][safe][:]   (row of row_bytes bytes)
 * retrieve, safe [B,L_max,W] int32; pvalid [B,L_max,W] uint8; src
 * [B,T_max,row_bytes] bytes; gathered [B,L_max,W,row_bytes].  src/gathered nullable.
 * ---------------------------------------------------------------------- */
int orc_safe_gather_paths(const int32_t *retrieve, const int32_t *n_nodes, int B, int L_max, int W, int T_max,
                          int dummy, const void *src, size_t row_bytes, int32_t *safe, uint8_t *pvalid,
                          void *gathered) {
    if (dummy < 0 || dummy >= T_max) return ORC_ERR_ARG;
    for (int b = 0; b < B; b++)
        for (int p = 0; p < L_max; p++)
            for (int i = 0; i < W; i++) {
                size_t e = ((size_t)b * L_max + p) * W + i;
                int32_t idx = retrieve[e];
                int32_t sidx = (idx >= 0 && idx < T_max) ? idx : dummy;
                int n = n_nodes ? n_nodes[b] : T_max;
                if (safe) safe[e] = sidx;
                if (pvalid) pvalid[e] = (uint8_t)(idx >= 0 && idx < n);
                if (src && gathered)
                    memcpy((char *)gathered + e * row_bytes,
                           (const char *)src + ((size_t)b * T_max + sidx) * row_bytes, row_bytes);
            }
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Greedy posterior acceptance (temperature 0, Section 5.1 "Decoding
 * configuration"; acceptance selects a single root-to-leaf path prefix,
 * Section 2.3).  Done in the naive order: for every path and every position,
 * gather the full teacher logit row of the node at that position, take its
 * argmax (lowest index among equal maxima), and compare it with the candidate
 * token of the next node on the path.  len[p] = number of leading matches, all
 * guarded by the validity of both positions.  best = lowest p of maximal len;
 * A = len[best]; acc_nodes[0..A] = the safe node indices of the accepted
 * prefix (root first), the tail filled with dummy; bonus = the teacher's
 * greedy token after the last accepted node.  g[b][n] = argmax of node n's
 * row for valid n, -1 for padded rows.
 * ---------------------------------------------------------------------- */
static int32_t row_argmax(const float *row, int V) {
    int32_t best = 0;
    for (int v = 1; v < V; v++)
        if (row[v] > row[best]) best = v;
    return best;
}

int orc_evaluate_posterior(const float *logits, const int32_t *tokens, const int32_t *retrieve,
                           const int32_t *n_nodes, int B, int T_max, int V, int L_max, int W, int dummy, int32_t *g,
                           int32_t *len, int32_t *best, int32_t *accept_len, int32_t *acc_nodes, int32_t *bonus) {
    if (dummy < 0 || dummy >= T_max || V < 1 || W < 1 || L_max < 1) return ORC_ERR_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        int n = n_nodes[b];
        const float *lg = logits + (size_t)b * T_max * V;
        const int32_t *tok = tokens + (size_t)b * T_max;
        int bestp = 0, bestlen = -1;
        for (int p = 0; p < L_max; p++) {
            const int32_t *path = retrieve + ((size_t)b * L_max + p) * W;
            int cnt = 0;
            for (int i = 0; i + 1 < W; i++) {
                int32_t a = path[i], c = path[i + 1];
                int va = (a >= 0 && a < n), vc = (c >= 0 && c < n);
                int32_t sa = (a >= 0 && a < T_max) ? a : dummy;
                int32_t sc = (c >= 0 && c < T_max) ? c : dummy;
                /* gather the row of the node at position i, then reduce it */
                int32_t ga = row_argmax(lg + (size_t)sa * V, V);
                if (va && vc && tok[sc] == ga)
                    cnt++;
                else
                    break;
            }
            len[(size_t)b * L_max + p] = cnt;
            if (cnt > bestlen) {
                bestlen = cnt;
                bestp = p;
            }
        }
        best[b] = bestp;
        accept_len[b] = bestlen;
        const int32_t *bp = retrieve + ((size_t)b * L_max + bestp) * W;
        for (int i = 0; i < W; i++) {
            int32_t a = bp[i];
            acc_nodes[(size_t)b * W + i] = (i <= bestlen && a >= 0 && a < T_max) ? a : dummy;
        }
        for (int k = 0; k < T_max; k++) g[(size_t)b * T_max + k] = (k < n) ? row_argmax(lg + (size_t)k * V, V) : -1;
        int32_t last = acc_nodes[(size_t)b * W + bestlen];
        bonus[b] = (last < n) ? row_argmax(lg + (size_t)last * V, V) : -1;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Commit of the accepted path.  Section 3.1 "Path-index-based commit", full
 * reordering: the branch cache of sequence b is the committed prefix followed
 * by the T_max tree rows; path_indices = [0..P) ++ [P + acc_nodes[i], i = 0..A];
 * the new committed cache is the branch cache gathered along the sequence axis
 * by path_indices, for every layer, KV head and K/V alike, written back at
 * logical positions 0..P+A.  prefix_len_out = P + A + 1 (the root and A draft
 * tokens; the bonus token has no KV yet).  slot_map[b][i] = physical slot of
 * logical position P+i (block_table[(P+i)/bs]*bs + (P+i)%bs when paged, P+i
 * when contiguous), -1 for i > A.
 * A sequence that fails a check is left untouched: status bit set,
 * prefix_len_out = prefix_len, slot_map = -1.
 *
 * Layouts: kt, vt [n_layers,B,T_max,Hkv,d]; caches as in attention with a
 * leading layer axis of cache_layer_stride elements.
 *
 * In-place branch cache (kt == vt == NULL), Section 3.3 "KV-cache writes and
 * commit": the verification pass has extended the cache in place, so the tree
 * row of node j already sits at logical position P + j of the cache itself,
 * and the same gather by path_indices is taken over the cache alone (from a
 * snapshot, so no row is read after it has been overwritten).  The tail must
 * fit: P + n_nodes > capacity is a CAPACITY failure.  The tail was appended in
 * node order, so an accepted root-to-leaf path reads it front to back: its node
 * indices must increase strictly (acc_nodes[i] > acc_nodes[i-1], which holds for
 * every path of a tree numbered parents-first); a path that does not is refused
 * as BAD_NODE like any other inconsistent index, the sequence left untouched.
 * ---------------------------------------------------------------------- */
int orc_commit_accepted_kv(int B, int T_max, int Hkv, int d, int elem_bytes, int n_layers, const void *kt,
                           const void *vt, void *k_cache, void *v_cache, size_t cache_layer_stride,
                           const int32_t *block_table, int block_size, int max_blocks, int num_blocks, int P_cap,
                           const int32_t *prefix_len, const int32_t *capacity, const int32_t *n_nodes,
                           const int32_t *acc_nodes, const int32_t *accept_len, int W, int32_t *prefix_len_out,
                           int32_t *slot_map, int32_t *status) {
    if (elem_bytes != 2 && elem_bytes != 4) return ORC_ERR_ARG;
    size_t rowb = (size_t)d * elem_bytes; /* one (position, head) row */
    for (int b = 0; b < B; b++) {
        int P = prefix_len[b], A = accept_len[b], n = n_nodes[b];
        int32_t st = 0;
        if (A < 0 || A > W - 1) st |= ORC_COMMIT_BAD_LEN;
        if (!st) {
            for (int i = 0; i <= A; i++) {
                int32_t nd = acc_nodes[(size_t)b * W + i];
                if (nd < 0 || nd >= n) st |= ORC_COMMIT_BAD_NODE;
                /* in place: the path must walk the appended tail front to back */
                if (!kt && i > 0 && nd <= acc_nodes[(size_t)b * W + i - 1]) st |= ORC_COMMIT_BAD_NODE;
            }
            if ((long)P + A + 1 > (long)capacity[b]) st |= ORC_COMMIT_CAPACITY;
            if (!kt && (long)P + n > (long)capacity[b]) st |= ORC_COMMIT_CAPACITY;
            if (!(st & ORC_COMMIT_CAPACITY) && block_table)
                for (int i = 0; i < (kt ? A + 1 : (n > A + 1 ? n : A + 1)); i++) {
                    int pos = P + i;
                    if (pos / block_size >= max_blocks) {
                        st |= ORC_COMMIT_CAPACITY;
                        break;
                    }
                    int blk = block_table[(size_t)b * max_blocks + pos / block_size];
                    if (blk < 0 || blk >= num_blocks) st |= ORC_COMMIT_BAD_BLOCK;
                }
        }
        status[b] = st;
        for (int i = 0; i < W; i++) slot_map[(size_t)b * W + i] = -1;
        if (st) {
            prefix_len_out[b] = P;
            continue;
        }
        size_t newlen = (size_t)P + A + 1;
        size_t *path_idx = (size_t *)malloc(sizeof(size_t) * newlen);
        const size_t catlen = (size_t)P + (kt ? (size_t)T_max : (size_t)n); /* branch cache length */
        char *cat = (char *)malloc(catlen * rowb);
        char *neu = (char *)malloc(newlen * rowb);
        if (!path_idx || !cat || !neu) return ORC_ERR_NOMEM;
        for (int j = 0; j < P; j++) path_idx[j] = (size_t)j;
        for (int i = 0; i <= A; i++) path_idx[P + i] = (size_t)P + (size_t)acc_nodes[(size_t)b * W + i];
        for (int l = 0; l < n_layers; l++)
            for (int kv = 0; kv < 2; kv++)
                for (int hh = 0; hh < Hkv; hh++) {
                    char *cache = (char *)(kv ? v_cache : k_cache) + (size_t)l * cache_layer_stride * elem_bytes;
                    const char *tree = (const char *)(kv ? vt : kt);
                    /* branch cache of this (layer, head): prefix rows then tree rows (in place: the cache tail) */
                    for (size_t j = 0; j < catlen; j++) {
                        const char *srcp;
                        if (j < (size_t)P || !tree) {
                            size_t off;
                            if (block_table) {
                                int blk = block_table[(size_t)b * max_blocks + j / block_size];
                                off = (((size_t)blk * Hkv + hh) * block_size + j % block_size) * rowb;
                            } else {
                                off = (((size_t)b * P_cap + j) * Hkv + hh) * rowb;
                            }
                            srcp = cache + off;
                        } else {
                            srcp = tree + ((((size_t)l * B + b) * T_max + (j - P)) * Hkv + hh) * rowb;
                        }
                        memcpy(cat + j * rowb, srcp, rowb);
                    }
                    for (size_t j = 0; j < newlen; j++) memcpy(neu + j * rowb, cat + path_idx[j] * rowb, rowb);
                    for (size_t j = 0; j < newlen; j++) {
                        size_t off;
                        if (block_table) {
                            int blk = block_table[(size_t)b * max_blocks + j / block_size];
                            off = (((size_t)blk * Hkv + hh) * block_size + j % block_size) * rowb;
                        } else {
                            off = (((size_t)b * P_cap + j) * Hkv + hh) * rowb;
                        }
                        memcpy(cache + off, neu + j * rowb, rowb);
                    }
                }
        for (int i = 0; i <= A; i++) {
            int pos = P + i;
            slot_map[(size_t)b * W + i] =
                block_table ? block_table[(size_t)b * max_blocks + pos / block_size] * block_size + pos % block_size
                            : pos;
        }
        prefix_len_out[b] = P + A + 1;
        free(path_idx);
        free(cat);
        free(neu);
    }
    return ORC_OK;
}

/* Number of OpenMP threads the parallel loops above will use. */
int orc_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}

/* ------------------------------------------------------------------------
 * Teacher head + greedy choice.  Section 3.3 "Execution view" / "Mapping
 * teacher outputs to node verification scores": the teacher turns the hidden
 * state of node k into logits l[k] over the vocabulary; Section 5.1: greedy
 * decoding takes the argmax.  Plain definition: logits[r][v] = sum_c
 * hidden[r][c] * weight[v][c] in fp64 from the exact input values, argmax over
 * v with the lowest index on ties.  Rows of padded nodes give argmax -1.
 *   hidden [B, T_max, D], weight [V, D] (dtype 0 = f32, 1 = bf16 bit patterns)
 *   argmax int32 [B, T_max]; maxval double [B, T_max] (nullable);
 *   logits double [B, T_max, V] (nullable: only for small cases)
 * ---------------------------------------------------------------------- */
int orc_lm_head_argmax(const void *hidden, const void *weight, int dtype, const int32_t *n_nodes, int B, int T_max,
                       int D, int V, int32_t *argmax, double *maxval, double *logits) {
    if (B < 0 || T_max < 1 || D < 1 || V < 1) return ORC_ERR_ARG;
#pragma omp parallel for schedule(dynamic)
    for (int r = 0; r < B * T_max; r++) {
        int b = r / T_max, k = r % T_max;
        int n = n_nodes[b];
        if (n < 0) n = 0;
        if (n > T_max) n = T_max;
        if (k >= n) {
            argmax[r] = -1;
            if (maxval) maxval[r] = -INFINITY;
            if (logits)
                for (int v = 0; v < V; v++) logits[(size_t)r * V + v] = 0.0;
            continue;
        }
        double best = -INFINITY;
        int bi = -1;
        for (int v = 0; v < V; v++) {
            double acc = 0.0;
            for (int c = 0; c < D; c++) acc += load_val(hidden, dtype, (size_t)r * D + c) * load_val(weight, dtype, (size_t)v * D + c);
            if (logits) logits[(size_t)r * V + v] = acc;
            if (acc > best) {
                best = acc;
                bi = v;
            }
        }
        argmax[r] = bi;
        if (maxval) maxval[r] = best;
    }
    return ORC_OK;
}

/* status bits of the branch-cache calls below (they share the commit bits above) */
#define ORC_BRANCH_NO_BLOCKS 16 /* the free list is shorter than what the call needs      */
#define ORC_BRANCH_BAD_FREE 32  /* a free-list entry this sequence would use is no block   */

/* byte offset of (position j, KV head hh) inside one layer of a cache */
static size_t cache_row_off(const int32_t *table_row, int block_size, int Hkv, int P_cap, int b, size_t j, int hh,
                            size_t rowb) {
    if (table_row) {
        int blk = table_row[j / block_size];
        return (((size_t)blk * Hkv + hh) * block_size + j % block_size) * rowb;
    }
    return (((size_t)b * P_cap + j) * Hkv + hh) * rowb;
}

/* ------------------------------------------------------------------------
 * Branch replication on a paged cache.  Section 3.1: every speculative
 * iteration creates N branch caches B_i <- Replicate(C*), each an isolated
 * replica of the committed cache that the teacher pass then extends in place;
 * isolation means extending one branch mutates neither C* nor another branch.
 * The paper replicates by deep copy.  Here the replica is an encoding: a block
 * table per branch that SHARES the blocks lying wholly inside the committed
 * prefix (nothing writes below prefix_len) and owns private blocks from the
 * position prefix_len on - the partly filled block that holds position
 * prefix_len (its committed rows copied in) and the blocks the tail will use.
 * The pins compare the logical content against the deep copy.
 *
 * Rule (what the GPU side must reproduce exactly):
 *   first_b = P_b / bs; last_b = ceil((P_b + tail_b) / bs); need_b = last_b - first_b
 *   (0 for a sequence whose lengths are refused: negative, or beyond the table);
 *   block_base[b] = N * sum_{b' < b} need_b'; branch i of sequence b owns
 *   free_blocks[block_base[b] + i*need_b + k] as its logical block first_b + k.
 *   n_taken = N * sum_b need_b.  The accounting depends on the lengths alone: a
 *   sequence refused for what its tables hold (a committed block or a free-list
 *   entry outside the pool) keeps its share of the free list, unused.  If n_taken
 *   exceeds n_free, nothing is written to the cache, n_taken = 0 and every sequence
 *   that needs blocks reports NO_BLOCKS.  Table rows of a refused sequence are all
 *   -1; entries from last_b on are -1.
 *   block_table [B, max_blocks]; branch_table [B, N, max_blocks]; status [B]
 * ---------------------------------------------------------------------- */
int orc_replicate_branches(int B, int N, int Hkv, int d, int elem_bytes, int n_layers, void *k_cache, void *v_cache,
                           size_t cache_layer_stride, const int32_t *block_table, int block_size, int max_blocks,
                           int num_blocks, const int32_t *prefix_len, const int32_t *tail_len,
                           const int32_t *free_blocks, int n_free, int32_t *branch_table, int32_t *block_base,
                           int32_t *n_taken, int32_t *status) {
    if (B < 0 || N < 1 || block_size < 1 || max_blocks < 1 || !block_table) return ORC_ERR_ARG;
    size_t rowb = (size_t)d * elem_bytes;
    int *need = (int *)calloc((size_t)B + 1, sizeof(int));
    if (!need) return ORC_ERR_NOMEM;
    long total = 0;
    for (int b = 0; b < B; b++) {
        long P = prefix_len[b], t = tail_len[b];
        int32_t st = 0;
        if (P < 0 || t < 0) st |= ORC_COMMIT_BAD_LEN;
        if (!st) {
            long last = (P + t + block_size - 1) / block_size;
            if (last > max_blocks) st |= ORC_COMMIT_CAPACITY;
            if (!st) need[b] = (int)(last - P / block_size);
            if (!st)
                for (long k = 0; k < (P + block_size - 1) / block_size; k++) {
                    int blk = block_table[(size_t)b * max_blocks + k];
                    if (blk < 0 || blk >= num_blocks) st |= ORC_COMMIT_BAD_BLOCK;
                }
        }
        status[b] = st;
        block_base[b] = (int32_t)total;
        total += (long)N * need[b];
    }
    int fits = total <= n_free;
    *n_taken = fits ? (int32_t)total : 0;
    for (int b = 0; b < B; b++) {
        if (!fits && need[b]) status[b] |= ORC_BRANCH_NO_BLOCKS;
        if (fits && !status[b])
            for (int x = 0; x < N * need[b]; x++) {
                int blk = free_blocks[block_base[b] + x];
                if (blk < 0 || blk >= num_blocks) status[b] |= ORC_BRANCH_BAD_FREE;
            }
        int P = prefix_len[b], first = status[b] ? 0 : P / block_size;
        for (int i = 0; i < N; i++) {
            int32_t *row = branch_table + ((size_t)b * N + i) * max_blocks;
            for (int k = 0; k < max_blocks; k++) {
                if (status[b] || k >= first + need[b]) row[k] = -1;
                else if (k < first) row[k] = block_table[(size_t)b * max_blocks + k];
                else row[k] = free_blocks[block_base[b] + i * need[b] + (k - first)];
            }
            if (status[b] || P % block_size == 0) continue;
            /* the committed rows of the partly filled block move into the branch's own copy of it */
            for (int l = 0; l < n_layers; l++)
                for (int kv = 0; kv < 2; kv++)
                    for (int hh = 0; hh < Hkv; hh++) {
                        char *cache = (char *)(kv ? v_cache : k_cache) + (size_t)l * cache_layer_stride * elem_bytes;
                        for (int j = first * block_size; j < P; j++)
                            memcpy(cache + cache_row_off(row, block_size, Hkv, 0, b, (size_t)j, hh, rowb),
                                   cache + cache_row_off(block_table + (size_t)b * max_blocks, block_size, Hkv, 0, b,
                                                         (size_t)j, hh, rowb),
                                   rowb);
                    }
        }
    }
    free(need);
    return ORC_OK;
}

/* ------------------------------------------------------------------------
 * Commit by path indices.  Section 3.1 "Commit by path indices and
 * prefix-sharing fast reorder": path_indices maps the next step's prefix
 * sequence to positions of the selected branch cache; the committed cache is
 * the branch cache gathered along the sequence axis,
 *     new[j] = branch[path_indices[j]],  0 <= j < new_len,
 * for every layer, KV head, K and V ("full reordering", any index order,
 * repeats allowed).  The fast path keeps the part of the prefix whose order
 * the indices preserve and gathers only the rest; it is decided from the
 * indices themselves, so any inconsistency simply shortens what is kept, down
 * to the full reorder.
 *
 * The source (branch) and destination (committed) caches are separate storage:
 * contiguous [B, P_cap, Hkv, d] buffers, or two block tables over one pool.
 * Paged with fast != 0: keep_b = the longest j <= new_len with path_indices[k] = k
 * for all k < j, rounded down to whole blocks; the destination table takes the
 * source's block ids for those blocks (sharing them) and rows >= keep_b are
 * gathered into the destination's own blocks.  Otherwise keep_b = 0.  The source
 * is read completely before anything is written.  A sequence with an error
 * writes nothing and leaves its destination table row alone.
 *   path_indices [B, L_cap]; src_len, new_len, kept_len, status [B]
 * ---------------------------------------------------------------------- */
int orc_commit_path_indices(int B, int Hkv, int d, int elem_bytes, int n_layers, const void *src_k, const void *src_v,
                            void *dst_k, void *dst_v, size_t cache_layer_stride, const int32_t *src_table,
                            int32_t *dst_table, int block_size, int max_blocks, int num_blocks, int P_cap,
                            const int32_t *path_indices, int L_cap, const int32_t *src_len, const int32_t *new_len,
                            int fast, int32_t *kept_len, int32_t *status) {
    if (B < 0 || L_cap < 1 || (src_table != NULL) != (dst_table != NULL)) return ORC_ERR_ARG;
    if (src_table && (block_size < 1 || max_blocks < 1)) return ORC_ERR_ARG;
    size_t rowb = (size_t)d * elem_bytes;
    for (int b = 0; b < B; b++) {
        long Ls = src_len[b], Ln = new_len[b];
        long cap = src_table ? (long)max_blocks * block_size : P_cap;
        const int32_t *idx = path_indices + (size_t)b * L_cap;
        const int32_t *srow = src_table ? src_table + (size_t)b * max_blocks : NULL;
        int32_t *drow = dst_table ? dst_table + (size_t)b * max_blocks : NULL;
        int32_t st = 0;
        kept_len[b] = 0;
        if (Ln < 0 || Ln > L_cap || Ls < 0 || Ls > cap) st |= ORC_COMMIT_BAD_LEN;
        if (!st && Ln > cap) st |= ORC_COMMIT_CAPACITY;
        long keep = 0;
        if (!st) {
            for (long j = 0; j < Ln; j++)
                if (idx[j] < 0 || idx[j] >= Ls) st |= ORC_COMMIT_BAD_NODE;
            if (fast && src_table) {
                while (keep < Ln && idx[keep] == keep) keep++;
                keep = keep / block_size * block_size;
            }
            if (src_table) {
                for (long k = 0; k < (Ls + block_size - 1) / block_size; k++)
                    if (srow[k] < 0 || srow[k] >= num_blocks) st |= ORC_COMMIT_BAD_BLOCK;
                for (long k = keep / block_size; k < (Ln + block_size - 1) / block_size; k++)
                    if (drow[k] < 0 || drow[k] >= num_blocks) st |= ORC_COMMIT_BAD_BLOCK;
            }
        }
        status[b] = st;
        if (st) continue;
        kept_len[b] = (int32_t)keep;
        char *snap = (char *)malloc((size_t)(Ls ? Ls : 1) * rowb);
        if (!snap) return ORC_ERR_NOMEM;
        for (int l = 0; l < n_layers; l++)
            for (int kv = 0; kv < 2; kv++)
                for (int hh = 0; hh < Hkv; hh++) {
                    const char *src = (const char *)(kv ? src_v : src_k) + (size_t)l * cache_layer_stride * elem_bytes;
                    char *dst = (char *)(kv ? dst_v : dst_k) + (size_t)l * cache_layer_stride * elem_bytes;
                    for (long j = 0; j < Ls; j++)
                        memcpy(snap + (size_t)j * rowb,
                               src + cache_row_off(srow, block_size, Hkv, P_cap, b, (size_t)j, hh, rowb), rowb);
                    for (long j = keep; j < Ln; j++)
                        memcpy(dst + cache_row_off(drow, block_size, Hkv, P_cap, b, (size_t)j, hh, rowb),
                               snap + (size_t)idx[j] * rowb, rowb);
                }
        free(snap);
        for (long k = 0; src_table && k < keep / block_size; k++) drow[k] = srow[k];
    }
    return ORC_OK;
}
