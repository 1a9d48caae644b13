// Device code shared by the separate entry points (safe_gather_paths, evaluate_posterior, commit_accepted_kv)
// and the fused epilogue: each piece is written once and called from both.
#pragma once
#include "etv_common.h"

namespace etv {

__device__ __forceinline__ int32_t safe_index(int32_t idx, int T_max, int dummy) {
    return (idx >= 0 && idx < T_max) ? idx : dummy;
}

// One path entry e of sequence b, handled by one wavefront: safe index, validity flag, lane-strided copy of
// the gathered row.  Section 3.2 "Dummy-root indexing", "Padding and batch semantics".
__device__ __forceinline__ void gather_entry(long e, int b, int lane, const int32_t *__restrict__ retrieve, int n,
                                             int T_max, int dummy, const uint8_t *__restrict__ src, size_t row_bytes,
                                             int32_t *__restrict__ safe, uint8_t *__restrict__ pvalid,
                                             uint8_t *__restrict__ gathered) {
    const int32_t idx = retrieve[e];
    const int32_t s = safe_index(idx, T_max, dummy);
    if (lane == 0) {
        if (safe) safe[e] = s;
        if (pvalid) pvalid[e] = (uint8_t)(idx >= 0 && idx < n);
    }
    if (src && gathered) {
        const uint8_t *from = src + ((size_t)b * T_max + s) * row_bytes;
        uint8_t *to = gathered + (size_t)e * row_bytes;
        if ((row_bytes & 15) == 0 && ((((uintptr_t)src) | ((uintptr_t)gathered)) & 15) == 0) {
            for (size_t o = (size_t)lane * 16; o < row_bytes; o += 64 * 16)
                *reinterpret_cast<uint4 *>(to + o) = *reinterpret_cast<const uint4 *>(from + o);
        } else if ((row_bytes & 3) == 0 && ((((uintptr_t)src) | ((uintptr_t)gathered)) & 3) == 0) {
            for (size_t o = (size_t)lane * 4; o < row_bytes; o += 64 * 4)
                *reinterpret_cast<uint32_t *>(to + o) = *reinterpret_cast<const uint32_t *>(from + o);
        } else {
            for (size_t o = lane; o < row_bytes; o += 64) to[o] = from[o];
        }
    }
}

struct MaxIdx {
    float v;
    int32_t i;
};
// (a beats b) iff a is larger, or equal with the lower index: "lowest index of the maximum"
__device__ __forceinline__ MaxIdx better(MaxIdx a, MaxIdx b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}

constexpr int kChunk = 4096;  // floats of one logit row scanned by one workgroup (16 KiB)

// Acceptance for sequence b by one workgroup of 256 threads (thread t): finish the argmax from the per-chunk
// partials (or, with pval == nullptr, take argmax[] as given), walk every path with guarded compares, reduce to the best path (longest, lowest index on ties),
// write argmax / len / best / accept_len / acc_nodes / bonus.  Leaves the accepted length in *s_A and the
// accepted node row (W entries) in s_acc (both in LDS, valid after the call for every thread).
// Section 2.3 / 5.1: greedy acceptance of the longest root-to-leaf prefix.
__device__ __forceinline__ void posterior_for_sequence(
    int b, int t, const float *__restrict__ pval, const int32_t *__restrict__ pidx, int chunks,
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ retrieve, int n, int T_max, int L_max, int W,
    int dummy, int32_t *__restrict__ argmax, int32_t *__restrict__ len, int32_t *__restrict__ best,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ acc_nodes, int32_t *__restrict__ bonus, int32_t *s_A,
    int32_t *s_acc) {
    __shared__ int32_t s_g[ETV_MAX_TREE];
    __shared__ int32_t s_tok[ETV_MAX_TREE];
    __shared__ int32_t s_len[256];
    __shared__ int32_t s_path[256];
    if (pval && chunks > 16) {
        // many partials per node (the per-tile maxima of the fused head): one wavefront per node, lanes stride
        // over the partials, shuffle reduce
        const int lane = t & 63;
        for (int node = t >> 6; node < T_max; node += 4) {
            MaxIdx m = {-INFINITY, 0x7fffffff};
            if (node < n) {
                const size_t o = ((size_t)b * T_max + node) * chunks;
                for (int c = lane; c < chunks; c += 64) m = better(m, MaxIdx{pval[o + c], pidx[o + c]});
#pragma unroll
                for (int off = 32; off >= 1; off >>= 1) m = better(m, MaxIdx{__shfl_xor(m.v, off), __shfl_xor(m.i, off)});
            }
            if (lane == 0) {
                const int32_t g = node < n ? m.i : -1;
                s_g[node] = g;
                s_tok[node] = tokens[(size_t)b * T_max + node];
                argmax[(size_t)b * T_max + node] = g;
            }
        }
    } else {
        for (int node = t; node < T_max; node += 256) {
            int32_t g = -1;
            if (node < n) {
                if (pval) {
                    size_t o = ((size_t)b * T_max + node) * chunks;
                    MaxIdx m = {pval[o], pidx[o]};
                    for (int c = 1; c < chunks; c++) m = better(m, MaxIdx{pval[o + c], pidx[o + c]});
                    g = m.i;
                } else {  // the caller already has the teacher's choice per node (etv_lm_head_argmax)
                    g = argmax[(size_t)b * T_max + node];
                }
            }
            s_g[node] = g;
            s_tok[node] = tokens[(size_t)b * T_max + node];
            if (pval) argmax[(size_t)b * T_max + node] = g;
        }
    }
    __syncthreads();
    int my_len = -1, my_path = 0x7fffffff;
    for (int p = t; p < L_max; p += 256) {
        const int32_t *path = retrieve + ((size_t)b * L_max + p) * W;
        int cnt = 0;
        int32_t a = path[0];
        for (int i = 0; i + 1 < W; i++) {
            int32_t c = path[i + 1];
            bool va = (a >= 0 && a < n), vc = (c >= 0 && c < n);
            int32_t sa = safe_index(a, T_max, dummy), sc = safe_index(c, T_max, dummy);
            if (!(va && vc && s_tok[sc] == s_g[sa])) break;
            cnt++;
            a = c;
        }
        len[(size_t)b * L_max + p] = cnt;
        if (cnt > my_len) {  // ascending p per thread: strict '>' keeps the lowest path
            my_len = cnt;
            my_path = p;
        }
    }
    s_len[t] = my_len;
    s_path[t] = my_path;
    __syncthreads();
    for (int off = 128; off >= 1; off >>= 1) {
        if (t < off) {
            int l2 = s_len[t + off], p2 = s_path[t + off];
            if (l2 > s_len[t] || (l2 == s_len[t] && p2 < s_path[t])) {
                s_len[t] = l2;
                s_path[t] = p2;
            }
        }
        __syncthreads();
    }
    const int A = s_len[0], bp = s_path[0];
    const int32_t *path = retrieve + ((size_t)b * L_max + bp) * W;
    for (int i = t; i < W; i += 256) {
        const int32_t nd = (i <= A) ? safe_index(path[i], T_max, dummy) : dummy;
        acc_nodes[(size_t)b * W + i] = nd;
        if (s_acc) s_acc[i] = nd;
    }
    if (t == 0) {
        best[b] = bp;
        accept_len[b] = A;
        int32_t last = safe_index(path[A], T_max, dummy);
        bonus[b] = s_g[last];
        if (s_A) *s_A = A;
    }
    __syncthreads();
}

// Commit plan of sequence b by one thread: validate, physical slot of every appended position, new prefix
// length.  acc_row: the W accepted node rows of the sequence.  Section 3.1 "Commit by path indices and
// prefix-sharing fast reorder".
// in_place: the tree rows are in the cache tail (positions P .. P + n - 1), which must then exist as well.
__device__ __forceinline__ void commit_plan_for_sequence(const etv_commit_desc &dsc, int b,
                                                         const int32_t *__restrict__ block_table, int P, int cap,
                                                         int n, const int32_t *acc_row, int A,
                                                         int32_t *__restrict__ prefix_len_out,
                                                         int32_t *__restrict__ slot_map, int32_t *__restrict__ status,
                                                         bool in_place = false) {
    const int W = dsc.W;
    int32_t st = 0;
    if (A < 0 || A > W - 1) st |= ETV_COMMIT_BAD_LEN;
    if (!st) {
        for (int i = 0; i <= A; i++) {
            int32_t nd = acc_row[i];
            if (nd < 0 || nd >= n) st |= ETV_COMMIT_BAD_NODE;
        }
        if ((long)P + A + 1 > (long)cap || P < 0) st |= ETV_COMMIT_CAPACITY;
        if (in_place && (long)P + n > (long)cap) st |= ETV_COMMIT_CAPACITY;
        const int reach = in_place ? max(n, A + 1) : A + 1;  // positions behind P that are read or written
        if (!(st & ETV_COMMIT_CAPACITY) && dsc.block_size > 0) {
            for (int i = 0; i < reach; i++) {
                int lb = (P + i) / dsc.block_size;
                if (lb >= dsc.max_blocks) {
                    st |= ETV_COMMIT_CAPACITY;
                    break;
                }
                int blk = block_table[(size_t)b * dsc.max_blocks + lb];
                if (blk < 0 || blk >= dsc.num_blocks) st |= ETV_COMMIT_BAD_BLOCK;
            }
        } else if (!(st & ETV_COMMIT_CAPACITY) && (long)P + reach > (long)dsc.P_cap) {
            st |= ETV_COMMIT_CAPACITY;
        }
    }
    for (int i = 0; i < W; i++) {
        int32_t slot = -1;
        if (!st && i <= A) {
            int pos = P + i;
            slot = dsc.block_size > 0 ? block_table[(size_t)b * dsc.max_blocks + pos / dsc.block_size] * dsc.block_size +
                                            pos % dsc.block_size
                                      : pos;
        }
        slot_map[(size_t)b * W + i] = slot;
    }
    status[b] = st;
    prefix_len_out[b] = st ? P : P + A + 1;
}

// host side, defined next to the commit kernels
int32_t check_commit_args(const etv_commit_desc *h, const void *kt, const void *vt, const void *k_cache,
                          const void *v_cache, const int32_t *block_table);
int32_t launch_commit_copy(const etv_commit_desc *h, const void *kt, const void *vt, void *k_cache, void *v_cache,
                           const int32_t *acc_nodes, const int32_t *slot_map, hipStream_t s);
int32_t launch_commit_compact(const etv_commit_desc *h, void *k_cache, void *v_cache, const int32_t *block_table,
                              const int32_t *prefix_len, const int32_t *acc_nodes, const int32_t *accept_len,
                              const int32_t *slot_map, hipStream_t s);

}  // namespace etv
