// Branch caches over a paged pool (Section 3.1, "Branchable KV-cache abstraction"): copy-on-write replication of
// the committed cache into N branch tables, and the commit by path indices (the general gather along the sequence
// axis, with the prefix-sharing fast path decided from the indices).  Integer and byte work only.
#include "etv_common.h"

namespace etv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // a 16-byte unit the streaming builtins accept

// --------------------------------------------------------------------------------------------------------------
// replicate_branches
// --------------------------------------------------------------------------------------------------------------
// Blocks a branch of one sequence owns: from the block that holds position P to the last block of the tail.  It
// depends on the lengths alone (0 when they are refused), so every workgroup can work out any sequence's share
// of the free list without waiting for anybody's table checks.
struct ReplNeed {
    int32_t st;   // ETV_COMMIT_BAD_LEN / ETV_COMMIT_CAPACITY or 0
    int first, need;
};
__device__ __forceinline__ ReplNeed repl_need(long P, long t, int bs, int max_blocks) {
    ReplNeed r{0, 0, 0};
    if (P < 0 || t < 0) r.st = ETV_COMMIT_BAD_LEN;
    else if ((P + t + bs - 1) / bs > max_blocks) r.st = ETV_COMMIT_CAPACITY;
    if (!r.st) {
        r.first = (int)(P / bs);
        r.need = (int)((P + t + bs - 1) / bs) - r.first;
    }
    return r;
}

// Sum of need over the sequences [0, upto) and over all of them, by one workgroup of 256 threads.
__device__ __forceinline__ void repl_sums(const etv_cache_desc &dsc, const int32_t *__restrict__ prefix_len,
                                          const int32_t *__restrict__ tail_len, int upto, long &before, long &total) {
    __shared__ long s_b[4], s_t[4];
    long mb = 0, mt = 0;
    for (int x = threadIdx.x; x < dsc.B; x += 256) {
        const int nd = repl_need(prefix_len[x], tail_len[x], dsc.block_size, dsc.max_blocks).need;
        mt += nd;
        if (x < upto) mb += nd;
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        mb += __shfl_xor(mb, off);
        mt += __shfl_xor(mt, off);
    }
    if ((threadIdx.x & 63) == 0) { s_b[threadIdx.x >> 6] = mb; s_t[threadIdx.x >> 6] = mt; }
    __syncthreads();
    before = s_b[0] + s_b[1] + s_b[2] + s_b[3];
    total = s_t[0] + s_t[1] + s_t[2] + s_t[3];
}

// Large batches: one workgroup writes block_base[] and n_taken ahead of the fill kernel, which then reads them
// instead of summing over the batch itself.  Exclusive scan in chunks of 256 sequences with a running carry.
__global__ void __launch_bounds__(256) replicate_scan_kernel(etv_cache_desc dsc, const int32_t *__restrict__ prefix_len,
                                                             const int32_t *__restrict__ tail_len, int N, int n_free,
                                                             int32_t *__restrict__ block_base,
                                                             int32_t *__restrict__ n_taken) {
    __shared__ int s_part[256];
    __shared__ long s_carry;
    const int t = threadIdx.x;
    if (t == 0) s_carry = 0;
    __syncthreads();
    for (int b0 = 0; b0 < dsc.B; b0 += 256) {
        const int b = b0 + t;
        const int mine = b < dsc.B ? repl_need(prefix_len[b], tail_len[b], dsc.block_size, dsc.max_blocks).need : 0;
        s_part[t] = mine;
        __syncthreads();
        for (int off = 1; off < 256; off <<= 1) {   // inclusive scan of the 256 entries
            const int add = t >= off ? s_part[t - off] : 0;
            __syncthreads();
            s_part[t] += add;
            __syncthreads();
        }
        const long carry = s_carry;
        if (b < dsc.B) block_base[b] = (int32_t)(N * (carry + s_part[t] - mine));
        __syncthreads();
        if (t == 255) s_carry = carry + s_part[255];
        __syncthreads();
    }
    if (t == 0) {
        const long total = (long)N * s_carry;
        n_taken[0] = total <= n_free ? (int32_t)total : 0;   // 0 with sequences that need blocks: it did not fit
    }
}

// grid (N, B, n_layers), 256 threads: branch i of sequence b in layer l.  Every workgroup derives the sequence's
// share of the free list (PRESCANNED: reads it), checks the sequence's tables, and copies the committed rows of
// the partly filled block into the branch's own block for its layer; layer 0's workgroup also writes the table
// row, and the first branch's the per-sequence outputs.
template <bool PRESCANNED>
__global__ void __launch_bounds__(256) replicate_fill_kernel(etv_cache_desc dsc, uint8_t *__restrict__ k_cache,
                                                             uint8_t *__restrict__ v_cache,
                                                             const int32_t *__restrict__ block_table,
                                                             const int32_t *__restrict__ prefix_len,
                                                             const int32_t *__restrict__ tail_len, int N,
                                                             const int32_t *__restrict__ free_blocks, int n_free,
                                                             int32_t *__restrict__ block_base,
                                                             int32_t *__restrict__ branch_table,
                                                             int32_t *__restrict__ n_taken,
                                                             int32_t *__restrict__ status) {
    const int i = blockIdx.x, b = blockIdx.y, l = blockIdx.z, t = threadIdx.x;
    const int bs = dsc.block_size;
    const int P = prefix_len[b];
    const ReplNeed rn = repl_need(P, tail_len[b], bs, dsc.max_blocks);
    long base;
    bool fits;
    if (PRESCANNED) {
        base = block_base[b];
        fits = n_taken[0] > 0 || rn.need == 0;   // the scan kernel wrote 0 if the demand exceeds the free list
    } else {
        long before, total;
        repl_sums(dsc, prefix_len, tail_len, b, before, total);
        base = (long)N * before;
        total *= N;
        fits = total <= n_free;
        if (i == 0 && b == 0 && l == 0 && t == 0) n_taken[0] = fits ? (int32_t)total : 0;
    }
    int32_t st = rn.st;
    if (!fits && rn.need > 0) st |= ETV_BRANCH_NO_BLOCKS;
    // Table checks, all loads in one go and one barrier: the committed blocks, and the sequence's share of the
    // free list (which counts only for a sequence that is good so far).  The blocks of the partial-block copy are
    // looked up here too, so that the copy does not start with another trip to memory.
    int bad = 0;
    if (!rn.st)
        for (int k = t; k < (P + bs - 1) / bs; k += 256) {
            const int blk = block_table[(size_t)b * dsc.max_blocks + k];
            bad |= (blk < 0 || blk >= dsc.num_blocks) ? 1 : 0;
        }
    if (!st)
        for (int x = t; x < N * rn.need; x += 256) {
            const int blk = free_blocks[base + x];
            bad |= (blk < 0 || blk >= dsc.num_blocks) ? 2 : 0;
        }
    const int rows0 = st ? 0 : P - rn.first * bs;   // committed rows inside the partly filled block
    const int src_blk = rows0 > 0 ? block_table[(size_t)b * dsc.max_blocks + rn.first] : 0;
    const int dst_blk = rows0 > 0 ? free_blocks[base + (size_t)i * rn.need] : 0;
    const int any_block = __syncthreads_or(bad & 1), any_free = __syncthreads_or(bad & 2);   // every load is out by now
    if (any_block) st |= ETV_COMMIT_BAD_BLOCK;
    else if (any_free) st |= ETV_BRANCH_BAD_FREE;
    const int rows = st ? 0 : rows0;
    const int32_t *mine = free_blocks + base + (size_t)i * rn.need;
    if (l == 0) {
        if (i == 0 && t == 0) {
            status[b] = st;
            if (!PRESCANNED) block_base[b] = (int32_t)base;
        }
        int32_t *row = branch_table + ((size_t)b * N + i) * dsc.max_blocks;
        for (int k = t; k < dsc.max_blocks; k += 256) {
            int32_t v = -1;
            if (!st && k < rn.first + rn.need) v = k < rn.first ? block_table[(size_t)b * dsc.max_blocks + k] : mine[k - rn.first];
            row[k] = v;
        }
    }
    if (st || rows <= 0) return;
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const int upr = (int)(head_bytes / 16);              // 16-byte units per row of one head
    const int per_head = rows * upr;                     // the rows of a head are consecutive memory
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    for (int u = t; u < 2 * dsc.Hkv * per_head; u += 256) {
        const int kvh = u / per_head, w = u - kvh * per_head;
        const bool is_v = kvh >= dsc.Hkv;
        const int hh = is_v ? kvh - dsc.Hkv : kvh;
        uint8_t *cache = (is_v ? v_cache : k_cache) + layer_off;
        const size_t so = ((size_t)src_blk * dsc.Hkv + hh) * bs * head_bytes + (size_t)w * 16;
        const size_t dof = ((size_t)dst_blk * dsc.Hkv + hh) * bs * head_bytes + (size_t)w * 16;
        *reinterpret_cast<uint4 *>(cache + dof) = *reinterpret_cast<const uint4 *>(cache + so);   // plain: streaming ones were slower here
    }
}

// --------------------------------------------------------------------------------------------------------------
// commit_path_indices
// --------------------------------------------------------------------------------------------------------------
// grid B, 256 threads: checks, the length of the preserved prefix, and the shared blocks of the destination table.
__global__ void __launch_bounds__(256) path_commit_plan_kernel(etv_cache_desc dsc, const int32_t *__restrict__ src_table,
                                                               int32_t *__restrict__ dst_table,
                                                               const int32_t *__restrict__ path_indices, int L_cap,
                                                               const int32_t *__restrict__ src_len,
                                                               const int32_t *__restrict__ new_len, int fast,
                                                               int32_t *__restrict__ kept_len,
                                                               int32_t *__restrict__ status) {
    __shared__ int s_min[4];
    const int b = blockIdx.x, t = threadIdx.x;
    const int bs = dsc.block_size;
    const bool paged = bs > 0;
    const long Ls = src_len[b], Ln = new_len[b];
    const long cap = paged ? (long)dsc.max_blocks * bs : dsc.P_cap;
    const int32_t *idx = path_indices + (size_t)b * L_cap;
    int32_t st = 0;
    if (Ln < 0 || Ln > L_cap || Ls < 0 || Ls > cap) st |= ETV_COMMIT_BAD_LEN;
    if (!st && Ln > cap) st |= ETV_COMMIT_CAPACITY;
    int bad = 0, brk = st ? 0 : (int)Ln;   // first position whose index is not the position itself
    if (!st)
        for (int j = t; j < (int)Ln; j += 256) {
            const int v = idx[j];
            bad |= (v < 0 || v >= Ls);
            if (v != j && j < brk) brk = j;
        }
    if (__syncthreads_or(bad)) st |= ETV_COMMIT_BAD_NODE;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) brk = min(brk, __shfl_xor(brk, off));
    if ((t & 63) == 0) s_min[t >> 6] = brk;
    __syncthreads();
    brk = min(min(s_min[0], s_min[1]), min(s_min[2], s_min[3]));
    const int keep = (fast && paged && !(st & (ETV_COMMIT_BAD_LEN | ETV_COMMIT_CAPACITY))) ? brk / bs * bs : 0;
    bad = 0;
    if (paged && !(st & (ETV_COMMIT_BAD_LEN | ETV_COMMIT_CAPACITY))) {
        for (int k = t; k < (int)((Ls + bs - 1) / bs); k += 256) {
            const int blk = src_table[(size_t)b * dsc.max_blocks + k];
            bad |= (blk < 0 || blk >= dsc.num_blocks);
        }
        for (int k = keep / bs + t; k < (int)((Ln + bs - 1) / bs); k += 256) {
            const int blk = dst_table[(size_t)b * dsc.max_blocks + k];
            bad |= (blk < 0 || blk >= dsc.num_blocks);
        }
    }
    if (__syncthreads_or(bad)) st |= ETV_COMMIT_BAD_BLOCK;
    if (t == 0) {
        status[b] = st;
        kept_len[b] = st ? 0 : keep;
    }
    if (!st && paged)
        for (int k = t; k < keep / bs; k += 256) dst_table[(size_t)b * dsc.max_blocks + k] = src_table[(size_t)b * dsc.max_blocks + k];
}

// grid (X, B, n_layers), 256 threads.  A chunk is one destination block (paged) or 16 rows (contiguous); workgroup x
// takes the chunks first + x, first + x + X, ... where first is the chunk that holds row kept_len, so a call that
// keeps the prefix can use a small grid whatever the prefix length.  The rows j in [kept_len, new_len) of a chunk
// are copied from source row path_indices[j], K and V, all heads.  A row consists of pieces of consecutive memory
// (one per K|V and head in a block, one per K|V in a contiguous cache); a thread owns the same 16-byte unit of
// every piece of its row, so consecutive lanes write consecutive memory and the per-row lookups (index, source
// block) are done once, ahead of the copies.  A batch is VB row positions x SB pieces = 8 loads, all issued
// before their stores; lanes past the end of the chunk load a clamped (valid) address and store nothing, so the
// batch is straight-line code and no load waits for another.  Loads and stores are streaming (nontemporal): every
// byte is touched once, and plain stores left in L2 for the write-back at the end of the kernel cost a quarter of
// the bandwidth of a full reorder and half the time of a short one.
template <bool PAGED>
__global__ void __launch_bounds__(256) path_commit_gather_kernel(etv_cache_desc dsc, const uint8_t *src_k,
                                                                 const uint8_t *src_v,
                                                                 uint8_t *dst_k, uint8_t *dst_v,
                                                                 const int32_t *__restrict__ src_table,
                                                                 const int32_t *__restrict__ dst_table,
                                                                 const int32_t *__restrict__ path_indices, int L_cap,
                                                                 const int32_t *__restrict__ new_len,
                                                                 const int32_t *__restrict__ kept_len,
                                                                 const int32_t *__restrict__ status) {
    constexpr int VB = PAGED ? 1 : 4, SB = 8 / VB;
    const int b = blockIdx.y, l = blockIdx.z, t = threadIdx.x;
    const int keep = kept_len[b], Ln = new_len[b];
    if (status[b]) return;
    const int bs = dsc.block_size;
    const int R = PAGED ? bs : 16;
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const int Hkv = dsc.Hkv;
    const int width = (int)(head_bytes / 16) * (PAGED ? 1 : Hkv);   // 16-byte units of one piece
    const int slabs = PAGED ? 2 * Hkv : 2;                          // pieces per row: (K|V, head) or (K|V)
    const size_t piece_stride = PAGED ? (size_t)bs * head_bytes : 0;
    const int wsh = (width & (width - 1)) == 0 ? __ffs(width) - 1 : -1;
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    const int32_t *idx = path_indices + (size_t)b * L_cap;
    const int32_t *srow = PAGED ? src_table + (size_t)b * dsc.max_blocks : nullptr;
    for (int c = keep / R + blockIdx.x; c * R < Ln; c += gridDim.x) {
        const int j0 = c * R;
        const int lo = max(j0, keep), hi = min(j0 + R, Ln);
        const int dst_blk = PAGED ? dst_table[(size_t)b * dsc.max_blocks + c] : 0;
        const int per = (hi - lo) * width;             // units of one piece over the chunk's rows
        for (int v0 = 0; v0 < per; v0 += 256 * VB) {
            size_t so[VB], dof[VB];
            bool live[VB];
            int sj[VB];
#pragma unroll
            for (int y = 0; y < VB; y++) {
                const int v = v0 + y * 256 + t;
                live[y] = v < per;
                const int vc = live[y] ? v : per - 1;
                const int r = wsh >= 0 ? vc >> wsh : vc / width;
                const int j = lo + r;
                sj[y] = idx[j];
                dof[y] = (size_t)(vc - r * width) * 16 +
                         (PAGED ? ((size_t)dst_blk * Hkv * bs + (j - j0)) * head_bytes
                                : ((size_t)b * dsc.P_cap + j) * Hkv * head_bytes);
                so[y] = (size_t)(vc - r * width) * 16;
            }
#pragma unroll
            for (int y = 0; y < VB; y++) {
                if (PAGED) {
                    const int sb = sj[y] / bs;
                    so[y] += ((size_t)srow[sb] * Hkv * bs + (sj[y] - sb * bs)) * head_bytes;
                } else {
                    so[y] += ((size_t)b * dsc.P_cap + sj[y]) * Hkv * head_bytes;
                }
            }
            for (int s0 = 0; s0 < slabs; s0 += SB) {
                u32x4 val[VB][SB];
#pragma unroll
                for (int x = 0; x < SB; x++) {
                    const int slab = min(s0 + x, slabs - 1);   // uniform; a repeated piece is loaded, not stored
                    const int kv = slab >= slabs / 2;
                    const size_t within = layer_off + (size_t)(slab - kv * (slabs / 2)) * piece_stride;
#pragma unroll
                    for (int y = 0; y < VB; y++)
                        val[y][x] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>((kv ? src_v : src_k) + within + so[y]));
                }
#pragma unroll
                for (int x = 0; x < SB; x++) {
                    const int slab = s0 + x;
                    if (slab >= slabs) break;
                    const int kv = slab >= slabs / 2;
                    const size_t within = layer_off + (size_t)(slab - kv * (slabs / 2)) * piece_stride;
#pragma unroll
                    for (int y = 0; y < VB; y++)
                        if (live[y]) __builtin_nontemporal_store(val[y][x], reinterpret_cast<u32x4 *>((kv ? dst_v : dst_k) + within + dof[y]));
                }
            }
        }
    }
}

static int32_t check_cache_desc(const etv_cache_desc *h, bool need_paged) {
    if (!h) return ETV_ERR_INVALID_ARG;
    if (h->B < 0 || h->Hkv < 1 || h->d < 1 || h->n_layers < 1 || h->block_size < 0) return ETV_ERR_INVALID_ARG;
    if (h->elem_bytes != 2 && h->elem_bytes != 4) return ETV_ERR_UNSUPPORTED;
    if (((size_t)h->d * h->elem_bytes) % 16 != 0) return ETV_ERR_UNSUPPORTED;
    if (need_paged && h->block_size == 0) return ETV_ERR_UNIMPLEMENTED;  // replication of a contiguous cache: not built
    if (h->block_size > 0 && (h->max_blocks < 1 || h->num_blocks < 1)) return ETV_ERR_INVALID_ARG;
    if (h->block_size == 0 && h->P_cap < 1) return ETV_ERR_INVALID_ARG;
    if (h->cache_layer_stride < 0 || ((size_t)h->cache_layer_stride * h->elem_bytes) % 16 != 0) return ETV_ERR_INVALID_ARG;
    if (h->B > 65535 || h->n_layers > 65535) return ETV_ERR_UNSUPPORTED;
    return ETV_OK;
}

}  // namespace etv

extern "C" int32_t etv_replicate_branches(const etv_cache_desc *h, void *k_cache, void *v_cache,
                                          const int32_t *block_table, const int32_t *prefix_len,
                                          const int32_t *tail_len, int32_t N, const int32_t *free_blocks,
                                          int32_t n_free, int32_t *branch_table, int32_t *block_base,
                                          int32_t *n_taken, int32_t *status, void *stream) {
    int32_t rc = etv::check_cache_desc(h, true);
    if (rc != ETV_OK) return rc;
    if (!n_taken || N < 1 || n_free < 0 || (n_free > 0 && !free_blocks)) return ETV_ERR_INVALID_ARG;
    // an empty batch needs nothing but n_taken: the scan alone runs and writes 0
    if (h->B > 0 && (!k_cache || !v_cache || !block_table || !prefix_len || !tail_len || !branch_table || !block_base ||
                     !status))
        return ETV_ERR_INVALID_ARG;
    if ((((uintptr_t)k_cache) | ((uintptr_t)v_cache)) & 15) return ETV_ERR_INVALID_ARG;
    if ((long)h->B * N * h->max_blocks > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;   // block_base is an int32
    hipStream_t s = etv::as_stream(stream);
    uint8_t *kc = static_cast<uint8_t *>(k_cache), *vc = static_cast<uint8_t *>(v_cache);
    const dim3 grid(N, h->B, h->n_layers);
    if (h->B > 0 && h->B <= 256) {
        // every workgroup sums the batch's block demand itself: one launch
        hipLaunchKernelGGL(etv::replicate_fill_kernel<false>, grid, dim3(256), 0, s, *h, kc, vc, block_table, prefix_len,
                           tail_len, N, free_blocks, n_free, block_base, branch_table, n_taken, status);
        return etv::check_launch();
    }
    // large batches (and the empty one, which only needs n_taken = 0): a one-workgroup scan first
    hipLaunchKernelGGL(etv::replicate_scan_kernel, dim3(1), dim3(256), 0, s, *h, prefix_len, tail_len, N, n_free,
                       block_base, n_taken);
    rc = etv::check_launch();
    if (rc != ETV_OK || h->B == 0) return rc;
    hipLaunchKernelGGL(etv::replicate_fill_kernel<true>, grid, dim3(256), 0, s, *h, kc, vc, block_table, prefix_len,
                       tail_len, N, free_blocks, n_free, block_base, branch_table, n_taken, status);
    return etv::check_launch();
}

extern "C" int32_t etv_commit_path_indices(const etv_cache_desc *h, const void *src_k, const void *src_v, void *dst_k,
                                           void *dst_v, const int32_t *src_table, int32_t *dst_table,
                                           const int32_t *path_indices, int32_t L_cap, const int32_t *src_len,
                                           const int32_t *new_len, int32_t fast, int32_t *kept_len, int32_t *status,
                                           void *stream) {
    int32_t rc = etv::check_cache_desc(h, false);
    if (rc != ETV_OK) return rc;
    if (h->B == 0) return ETV_OK;
    if (!src_k || !src_v || !dst_k || !dst_v || !path_indices || !src_len || !new_len || !kept_len || !status)
        return ETV_ERR_INVALID_ARG;
    if (L_cap < 1) return ETV_ERR_INVALID_ARG;
    const bool paged = h->block_size > 0;
    if (paged != (src_table != nullptr) || paged != (dst_table != nullptr)) return ETV_ERR_INVALID_ARG;
    if (paged && src_table == dst_table) return ETV_ERR_INVALID_ARG;
    if (paged && (src_k != dst_k || src_v != dst_v)) return ETV_ERR_INVALID_ARG;   // both tables index one pool
    if (!paged && (src_k == dst_k || src_v == dst_v)) return ETV_ERR_INVALID_ARG;   // a contiguous cache is rebuilt elsewhere
    if ((((uintptr_t)src_k) | ((uintptr_t)src_v) | ((uintptr_t)dst_k) | ((uintptr_t)dst_v)) & 15) return ETV_ERR_INVALID_ARG;
    hipStream_t s = etv::as_stream(stream);
    hipLaunchKernelGGL(etv::path_commit_plan_kernel, dim3(h->B), dim3(256), 0, s, *h, src_table, dst_table,
                       path_indices, L_cap, src_len, new_len, fast, kept_len, status);
    rc = etv::check_launch();
    if (rc != ETV_OK) return rc;
    const int R = paged ? h->block_size : 16;
    const long cap = paged ? (long)h->max_blocks * h->block_size : h->P_cap;
    const long rows = L_cap < cap ? L_cap : cap;
    const long chunks = (rows + R - 1) / R;
    // a full reorder gets a workgroup per chunk; a call that expects to keep the prefix gets a few per sequence and
    // layer, which loop over the chunks if the indices turn out not to preserve it
    long X = (fast && paged) ? 4 : chunks;
    X = X > chunks ? chunks : X;
    auto kern = paged ? etv::path_commit_gather_kernel<true> : etv::path_commit_gather_kernel<false>;
    hipLaunchKernelGGL(kern, dim3((unsigned)X, h->B, h->n_layers), dim3(256),
                       0, s, *h, static_cast<const uint8_t *>(src_k), static_cast<const uint8_t *>(src_v),
                       static_cast<uint8_t *>(dst_k), static_cast<uint8_t *>(dst_v), src_table, dst_table, path_indices,
                       L_cap, new_len, kept_len, status);
    return etv::check_launch();
}
