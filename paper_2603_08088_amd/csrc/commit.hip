// commit_accepted_kv: prefix-sharing fast commit (Section 3.1, "Commit by path indices and
// prefix-sharing fast reorder").  The committed prefix is never moved; the accepted rows are
// gathered from the step's tree K/V buffer and appended, for every layer in one launch.  Because
// the tree K/V lives in its own buffer and not in the cache tail, source and destination never
// overlap and every copy is independent.
#include "epilogue_parts.h"

namespace etv {

// One thread per sequence: validate, compute the physical slot of every appended position and the
// new prefix length.  The copy kernel reads only slot_map, so prefix_len_out may alias prefix_len.
__global__ void commit_plan_kernel(etv_commit_desc dsc, const int32_t *__restrict__ block_table,
                                   const int32_t *__restrict__ prefix_len, const int32_t *__restrict__ capacity,
                                   const int32_t *__restrict__ n_nodes, const int32_t *__restrict__ acc_nodes,
                                   const int32_t *__restrict__ accept_len, int32_t *__restrict__ prefix_len_out,
                                   int32_t *__restrict__ slot_map, int32_t *__restrict__ status, int in_place) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= dsc.B) return;
    commit_plan_for_sequence(dsc, b, block_table, prefix_len[b], capacity[b], clampi(n_nodes[b], 0, dsc.T_max),
                             acc_nodes + (size_t)b * dsc.W, accept_len[b], prefix_len_out, slot_map, status,
                             in_place != 0);
}

// grid (W, B, n_layers), 256 threads: one appended position of one sequence in one layer.
// The tree row [Hkv, d] is contiguous; 16-byte units are spread over the threads, K then V.
__global__ void __launch_bounds__(256) commit_copy_kernel(etv_commit_desc dsc, const uint8_t *__restrict__ kt,
                                                          const uint8_t *__restrict__ vt, uint8_t *__restrict__ k_cache,
                                                          uint8_t *__restrict__ v_cache,
                                                          const int32_t *__restrict__ acc_nodes,
                                                          const int32_t *__restrict__ slot_map) {
    const int i = blockIdx.x, b = blockIdx.y, l = blockIdx.z;
    const int slot = slot_map[(size_t)b * dsc.W + i];
    if (slot < 0) return;
    const int node = acc_nodes[(size_t)b * dsc.W + i];
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const size_t row_bytes = head_bytes * dsc.Hkv;
    const int units_per_head = (int)(head_bytes / 16);
    const int units = units_per_head * dsc.Hkv;
    const size_t src_off = (((size_t)l * dsc.B + b) * dsc.T_max + node) * row_bytes;
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    for (int u = threadIdx.x; u < 2 * units; u += 256) {
        const bool is_v = u >= units;
        const int uu = is_v ? u - units : u;
        const int hh = uu / units_per_head, part = uu - hh * units_per_head;
        size_t dst_off;
        if (dsc.block_size > 0) {
            int blk = slot / dsc.block_size, off = slot - blk * dsc.block_size;
            dst_off = (((size_t)blk * dsc.Hkv + hh) * dsc.block_size + off) * head_bytes + (size_t)part * 16;
        } else {
            dst_off = (((size_t)b * dsc.P_cap + slot) * dsc.Hkv + hh) * head_bytes + (size_t)part * 16;
        }
        const uint8_t *src = (is_v ? vt : kt) + src_off + (size_t)uu * 16;
        uint8_t *dst = (is_v ? v_cache : k_cache) + layer_off + dst_off;
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    }
}

// In-place branch cache: the accepted rows move from cache position P + acc_nodes[i] to P + i inside the cache.
// A destination P + i can be the tail position of a node accepted earlier (acc_nodes[j] == i, j < i), never of one
// accepted later (acc_nodes[j] >= j), so the copy is safe when every row is read before a later row is written.
// grid (1, B, n_layers): a thread owns 16-byte columns of the [K row | V row] pair and moves them for all accepted
// positions itself, sixteen positions per batch: all loads of a batch, then its stores.  A batch's stores land on
// positions below every source of the following batches, and within a batch everything is read before anything
// is written; different threads touch different bytes.
__global__ void __launch_bounds__(256) commit_compact_kernel(etv_commit_desc dsc, uint8_t *__restrict__ k_cache,
                                                             uint8_t *__restrict__ v_cache,
                                                             const int32_t *__restrict__ block_table,
                                                             const int32_t *__restrict__ prefix_len,
                                                             const int32_t *__restrict__ acc_nodes,
                                                             const int32_t *__restrict__ accept_len,
                                                             const int32_t *__restrict__ slot_map) {
    const int b = blockIdx.y, l = blockIdx.z;
    if (slot_map[(size_t)b * dsc.W] < 0) return;  // the sequence failed a check: untouched
    const int P = prefix_len[b], A = accept_len[b];
    const size_t head_bytes = (size_t)dsc.d * dsc.elem_bytes;
    const int units_per_head = (int)(head_bytes / 16);
    const int units = units_per_head * dsc.Hkv;
    const size_t layer_off = (size_t)l * (size_t)dsc.cache_layer_stride * dsc.elem_bytes;
    auto slot_of = [&](int pos) {
        return dsc.block_size > 0 ? block_table[(size_t)b * dsc.max_blocks + pos / dsc.block_size] * dsc.block_size +
                                        pos % dsc.block_size
                                  : pos;
    };
    auto offset_of = [&](int slot, int hh, int part) {
        if (dsc.block_size > 0) {
            const int blk = slot / dsc.block_size, off = slot - blk * dsc.block_size;
            return (((size_t)blk * dsc.Hkv + hh) * dsc.block_size + off) * head_bytes + (size_t)part * 16;
        }
        return (((size_t)b * dsc.P_cap + slot) * dsc.Hkv + hh) * head_bytes + (size_t)part * 16;
    };
    for (int u = threadIdx.x; u < 2 * units; u += 256) {
        const bool is_v = u >= units;
        const int uu = is_v ? u - units : u;
        const int hh = uu / units_per_head, part = uu - hh * units_per_head;
        uint8_t *cache = (is_v ? v_cache : k_cache) + layer_off;
        for (int i0 = 0; i0 <= A; i0 += 16) {
            uint4 val[16];
#pragma unroll
            for (int j = 0; j < 16; j++) {
                const int i = i0 + j;
                if (i <= A)
                    val[j] = *reinterpret_cast<const uint4 *>(cache + offset_of(slot_of(P + acc_nodes[(size_t)b * dsc.W + i]), hh, part));
            }
#pragma unroll
            for (int j = 0; j < 16; j++) {
                const int i = i0 + j;
                if (i <= A) *reinterpret_cast<uint4 *>(cache + offset_of(slot_map[(size_t)b * dsc.W + i], hh, part)) = val[j];
            }
        }
    }
}

}  // namespace etv

namespace etv {

int32_t check_commit_args(const etv_commit_desc *h, const void *kt, const void *vt, const void *k_cache,
                          const void *v_cache, const int32_t *block_table) {
    if (!h || !k_cache || !v_cache) return ETV_ERR_INVALID_ARG;
    if ((kt == nullptr) != (vt == nullptr)) return ETV_ERR_INVALID_ARG;  // both null: in-place branch cache
    if (h->B < 0 || h->T_max < 1 || h->Hkv < 1 || h->d < 1 || h->n_layers < 1 || h->W < 1) return ETV_ERR_INVALID_ARG;
    if (h->elem_bytes != 2 && h->elem_bytes != 4) return ETV_ERR_UNSUPPORTED;
    if (((size_t)h->d * h->elem_bytes) % 16 != 0) return ETV_ERR_UNSUPPORTED;
    if (h->block_size < 0) return ETV_ERR_INVALID_ARG;
    if (h->block_size > 0 && (!block_table || h->max_blocks < 1 || h->num_blocks < 1)) return ETV_ERR_INVALID_ARG;
    if (h->block_size == 0 && h->P_cap < 1) return ETV_ERR_INVALID_ARG;
    if (((uintptr_t)kt | (uintptr_t)vt | (uintptr_t)k_cache | (uintptr_t)v_cache) & 15) return ETV_ERR_INVALID_ARG;  // null passes
    if (((size_t)h->cache_layer_stride * h->elem_bytes) % 16 != 0) return ETV_ERR_INVALID_ARG;
    if (h->B > 65535 || h->n_layers > 65535) return ETV_ERR_UNSUPPORTED;
    return ETV_OK;
}

int32_t launch_commit_copy(const etv_commit_desc *h, const void *kt, const void *vt, void *k_cache, void *v_cache,
                           const int32_t *acc_nodes, const int32_t *slot_map, hipStream_t s) {
    hipLaunchKernelGGL(commit_copy_kernel, dim3(h->W, h->B, h->n_layers), dim3(256), 0, s, *h,
                       static_cast<const uint8_t *>(kt), static_cast<const uint8_t *>(vt),
                       static_cast<uint8_t *>(k_cache), static_cast<uint8_t *>(v_cache), acc_nodes, slot_map);
    return check_launch();
}

int32_t launch_commit_compact(const etv_commit_desc *h, void *k_cache, void *v_cache, const int32_t *block_table,
                              const int32_t *prefix_len, const int32_t *acc_nodes, const int32_t *accept_len,
                              const int32_t *slot_map, hipStream_t s) {
    hipLaunchKernelGGL(commit_compact_kernel, dim3(1, h->B, h->n_layers), dim3(256), 0, s, *h,
                       static_cast<uint8_t *>(k_cache), static_cast<uint8_t *>(v_cache), block_table, prefix_len,
                       acc_nodes, accept_len, slot_map);
    return check_launch();
}

}  // namespace etv

extern "C" int32_t etv_commit_accepted_kv(const etv_commit_desc *h, const void *kt, const void *vt, void *k_cache,
                                          void *v_cache, const int32_t *block_table, const int32_t *prefix_len,
                                          const int32_t *capacity, const int32_t *n_nodes, const int32_t *acc_nodes,
                                          const int32_t *accept_len, int32_t *prefix_len_out, int32_t *slot_map,
                                          int32_t *status, void *stream) {
    if (!prefix_len || !capacity || !n_nodes || !acc_nodes || !accept_len || !prefix_len_out || !slot_map || !status)
        return ETV_ERR_INVALID_ARG;
    int32_t rc = etv::check_commit_args(h, kt, vt, k_cache, v_cache, block_table);
    if (rc != ETV_OK) return rc;
    if (h->B == 0) return ETV_OK;
    hipStream_t s = etv::as_stream(stream);
    const bool in_place = (kt == nullptr);
    if (in_place && prefix_len_out == prefix_len) return ETV_ERR_INVALID_ARG;  // the compaction still needs the old length
    hipLaunchKernelGGL(etv::commit_plan_kernel, dim3((h->B + 63) / 64), dim3(64), 0, s, *h, block_table, prefix_len,
                       capacity, n_nodes, acc_nodes, accept_len, prefix_len_out, slot_map, status, in_place ? 1 : 0);
    rc = etv::check_launch();
    if (rc != ETV_OK) return rc;
    if (in_place)
        return etv::launch_commit_compact(h, k_cache, v_cache, block_table, prefix_len, acc_nodes, accept_len, slot_map, s);
    return etv::launch_commit_copy(h, kt, vt, k_cache, v_cache, acc_nodes, slot_map, s);
}
