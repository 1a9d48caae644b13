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
// write argmax / len / best / accept_len / acc_nodes / bonus (unless write_out is false: a workgroup that only
// needs the result for itself).  Leaves the accepted length in *s_A and the accepted node row (W entries) in
// s_acc (both in LDS, valid after the call for every thread).
// Section 2.3 / 5.1: greedy acceptance of the longest root-to-leaf prefix.
__device__ __forceinline__ void posterior_for_sequence(
    int b, int t, const float *__restrict__ pval, const int32_t *__restrict__ pidx, int chunks,
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ retrieve, int n, int T_max, int L_max, int W,
    int dummy, int32_t *__restrict__ argmax, int32_t *__restrict__ len, int32_t *__restrict__ best,
    int32_t *__restrict__ accept_len, int32_t *__restrict__ acc_nodes, int32_t *__restrict__ bonus, int32_t *s_A,
    int32_t *s_acc, bool write_out = true) {
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
                if (write_out) argmax[(size_t)b * T_max + node] = g;
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
            if (pval && write_out) argmax[(size_t)b * T_max + node] = g;
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
        if (write_out) len[(size_t)b * L_max + p] = cnt;
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
        if (write_out) acc_nodes[(size_t)b * W + i] = nd;
        if (s_acc) s_acc[i] = nd;
    }
    if (t == 0) {
        if (write_out) {
            best[b] = bp;
            accept_len[b] = A;
            int32_t last = safe_index(path[A], T_max, dummy);
            bonus[b] = s_g[last];
        }
        if (s_A) *s_A = A;
    }
    __syncthreads();
}

// Commit plan of sequence b by one thread: validate, physical slot of every appended position, new prefix
// length.  acc_row: the W accepted node rows of the sequence.  The results go to slot_row[0..W), *status_b and
// *prefix_len_out_b (global memory or LDS).  Section 3.1 "Commit by path indices and prefix-sharing fast reorder".
// in_place: the tree rows are in the cache tail (positions P .. P + n - 1), which must then exist as well, and
// the accepted path must walk that tail front to back (strictly increasing node indices), which is what lets
// the compaction run in ascending order without reading a row after it has been overwritten.
__device__ __forceinline__ void commit_plan_for_sequence(const etv_commit_desc &dsc, int b,
                                                         const int32_t *__restrict__ block_table, int P, int cap,
                                                         int n, const int32_t *acc_row, int A,
                                                         int32_t *prefix_len_out_b, int32_t *slot_row,
                                                         int32_t *status_b, bool in_place = false) {
    const int W = dsc.W;
    int32_t st = 0;
    if (A < 0 || A > W - 1) st |= ETV_COMMIT_BAD_LEN;
    if (!st) {
        for (int i = 0; i <= A; i++) {
            int32_t nd = acc_row[i];
            if (nd < 0 || nd >= n) st |= ETV_COMMIT_BAD_NODE;
            if (in_place && i > 0 && nd <= acc_row[i - 1]) st |= ETV_COMMIT_BAD_NODE;
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
        slot_row[i] = slot;
    }
    *status_b = st;
    *prefix_len_out_b = st ? P : P + A + 1;
}

// The same plan computed by a whole workgroup (thread t of nthreads, all of them call it): one position per thread
// instead of one thread walking all of them, because every position costs a dependent trip to the block table and
// a single thread pays those one after the other.  The checks are those of commit_plan_for_sequence in an order
// that does not matter: a position whose logical block lies behind the table row sets CAPACITY and skips the block
// check, exactly the positions the sequential walk never reaches.  s_status: one word of LDS; the results are in
// slot_row / *status_b / *prefix_len_out_b after the call's last barrier.
__device__ __forceinline__ void commit_plan_cooperative(const etv_commit_desc &dsc, int b,
                                                        const int32_t *__restrict__ block_table, int P, int cap, int n,
                                                        const int32_t *acc_row, int A, int32_t *prefix_len_out_b,
                                                        int32_t *slot_row, int32_t *status_b, bool in_place, int t,
                                                        int nthreads, int32_t *s_status) {
    const int W = dsc.W;
    const bool bad_len = (A < 0 || A > W - 1);
    int32_t pre = bad_len ? ETV_COMMIT_BAD_LEN : 0;
    if (!bad_len) {
        if ((long)P + A + 1 > (long)cap || P < 0) pre |= ETV_COMMIT_CAPACITY;
        if (in_place && (long)P + n > (long)cap) pre |= ETV_COMMIT_CAPACITY;
    }
    if (t == 0) *s_status = pre;
    __syncthreads();
    if (!bad_len) {
        int32_t mine = 0;
        for (int i = t; i <= A; i += nthreads) {
            const int32_t nd = acc_row[i];
            if (nd < 0 || nd >= n) mine |= ETV_COMMIT_BAD_NODE;
            if (in_place && i > 0 && nd <= acc_row[i - 1]) mine |= ETV_COMMIT_BAD_NODE;
        }
        const int reach = in_place ? max(n, A + 1) : A + 1;
        if (!(pre & ETV_COMMIT_CAPACITY)) {
            if (dsc.block_size > 0) {
                for (int i = t; i < reach; i += nthreads) {
                    const int lb = (P + i) / dsc.block_size;
                    if (lb >= dsc.max_blocks) {
                        mine |= ETV_COMMIT_CAPACITY;
                    } else {
                        const int blk = block_table[(size_t)b * dsc.max_blocks + lb];
                        if (blk < 0 || blk >= dsc.num_blocks) mine |= ETV_COMMIT_BAD_BLOCK;
                    }
                }
            } else if (t == 0 && (long)P + reach > (long)dsc.P_cap) {
                mine |= ETV_COMMIT_CAPACITY;
            }
        }
        if (mine) atomicOr(s_status, mine);
    }
    __syncthreads();
    const int32_t st = *s_status;
    for (int i = t; i < W; i += nthreads) {
        int32_t slot = -1;
        if (!st && i <= A) {
            const int pos = P + i;
            slot = dsc.block_size > 0 ? block_table[(size_t)b * dsc.max_blocks + pos / dsc.block_size] * dsc.block_size +
                                            pos % dsc.block_size
                                      : pos;
        }
        slot_row[i] = slot;
    }
    if (t == 0) {
        *status_b = st;
        *prefix_len_out_b = st ? P : P + A + 1;
    }
    __syncthreads();
}

// Byte offset, inside one layer of the cache, of 16-byte unit `part` of KV head hh at physical slot `slot`.
__device__ __forceinline__ size_t cache_unit_offset(const etv_commit_desc &dsc, int b, int slot, int hh, int part) {
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    if (dsc.block_size > 0) {
        const int blk = slot / dsc.block_size, off = slot - blk * dsc.block_size;
        return (((size_t)blk * dsc.Hkv + hh) * dsc.block_size + off) * head_bytes + (size_t)part * 16;
    }
    return (((size_t)b * dsc.P_cap + slot) * dsc.Hkv + hh) * head_bytes + (size_t)part * 16;
}

// One 16-byte unit u (0 .. 2 * Hkv * d * elem_bytes / 16: the K row, then the V row) of tree row `node` of
// sequence b in layer l, copied to cache slot `slot`.  The tree row [Hkv, d] is contiguous.
__device__ __forceinline__ void commit_copy_unit(const etv_commit_desc &dsc, int b, int l, int node, int slot, int u,
                                                 const uint8_t *__restrict__ kt, const uint8_t *__restrict__ vt,
                                                 uint8_t *__restrict__ k_cache, uint8_t *__restrict__ v_cache) {
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const int units_per_head = (int)(head_bytes / 16);
    const int units = units_per_head * dsc.Hkv;
    const bool is_v = u >= units;
    const int uu = is_v ? u - units : u;
    const int hh = uu / units_per_head, part = uu - hh * units_per_head;
    const size_t src_off = (((size_t)l * dsc.B + b) * dsc.T_max + node) * (head_bytes * dsc.Hkv);
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    const uint8_t *src = (is_v ? vt : kt) + src_off + (size_t)uu * 16;
    uint8_t *dst = (is_v ? v_cache : k_cache) + layer_off + cache_unit_offset(dsc, b, slot, hh, part);
    *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
}

// In-place branch cache, one layer of one sequence by the threads t, t + nthreads, ...: the accepted rows move
// from cache position P + acc[i] to P + i (slot[i]).  The path is strictly increasing (checked by the plan), so
// acc[i] >= i: a destination can be the tail position of a node accepted earlier, never of one accepted later,
// and the move is safe when every row is read before a later row is written.  A thread owns 16-byte columns of
// the [K row | V row] pair and moves them for all accepted positions itself, sixteen positions per batch: all
// loads of a batch, then its stores.  A batch's stores land on positions below every source of the following
// batches, and within a batch everything is read before anything is written; different threads touch different
// bytes.  acc / slot: the sequence's accepted node row and slot row (global memory or LDS).
__device__ __forceinline__ void commit_compact_layer(const etv_commit_desc &dsc, int b, int l, int P, int A,
                                                     const int32_t *acc, const int32_t *slot,
                                                     const int32_t *__restrict__ block_table,
                                                     uint8_t *__restrict__ k_cache, uint8_t *__restrict__ v_cache,
                                                     int t, int nthreads) {
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const int units_per_head = (int)(head_bytes / 16);
    const int units = units_per_head * dsc.Hkv;
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    auto slot_of = [&](int pos) {
        return dsc.block_size > 0 ? block_table[(size_t)b * dsc.max_blocks + pos / dsc.block_size] * dsc.block_size +
                                        pos % dsc.block_size
                                  : pos;
    };
    for (int u = t; u < 2 * units; u += nthreads) {
        const bool is_v = u >= units;
        const int uu = is_v ? u - units : u;
        const int hh = uu / units_per_head, part = uu - hh * units_per_head;
        uint8_t *cache = (is_v ? v_cache : k_cache) + layer_off;
        for (int i0 = 0; i0 <= A; i0 += 16) {
            uint4 val[16];
#pragma unroll
            for (int j = 0; j < 16; j++) {
                const int i = i0 + j;
                if (i <= A) val[j] = *reinterpret_cast<const uint4 *>(cache + cache_unit_offset(dsc, b, slot_of(P + acc[i]), hh, part));
            }
#pragma unroll
            for (int j = 0; j < 16; j++) {
                const int i = i0 + j;
                if (i <= A) *reinterpret_cast<uint4 *>(cache + cache_unit_offset(dsc, b, slot[i], hh, part)) = val[j];
            }
        }
    }
}

// host side, defined next to the commit kernels
int32_t check_commit_args(const etv_commit_desc *h, const void *kt, const void *vt, const void *k_cache,
                          const void *v_cache, const int32_t *block_table);

}  // namespace etv
