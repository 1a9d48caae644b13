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
                             acc_nodes + (size_t)b * dsc.W, accept_len[b], prefix_len_out + b,
                             slot_map + (size_t)b * dsc.W, status + b, in_place != 0);
}

// grid (W, B, n_layers), 256 threads: one appended position of one sequence in one layer, 16-byte units spread
// over the threads, K then V.
__global__ void __launch_bounds__(256) commit_copy_kernel(etv_commit_desc dsc, const uint8_t *__restrict__ kt,
                                                          const uint8_t *__restrict__ vt, uint8_t *__restrict__ k_cache,
                                                          uint8_t *__restrict__ v_cache,
                                                          const int32_t *__restrict__ acc_nodes,
                                                          const int32_t *__restrict__ slot_map) {
    const int i = blockIdx.x, b = blockIdx.y, l = blockIdx.z;
    const int slot = slot_map[(size_t)b * dsc.W + i];
    if (slot < 0) return;
    const int node = acc_nodes[(size_t)b * dsc.W + i];
    const int units2 = 2 * (int)((size_t)dsc.d * dsc.elem_bytes / 16) * dsc.Hkv;
    for (int u = threadIdx.x; u < units2; u += 256) commit_copy_unit(dsc, b, l, node, slot, u, kt, vt, k_cache, v_cache);
}

// In-place branch cache, grid (1, B, n_layers): one layer of one sequence per workgroup (see commit_compact_layer).
__global__ void __launch_bounds__(256) commit_compact_kernel(etv_commit_desc dsc, uint8_t *__restrict__ k_cache,
                                                             uint8_t *__restrict__ v_cache,
                                                             const int32_t *__restrict__ block_table,
                                                             const int32_t *__restrict__ prefix_len,
                                                             const int32_t *__restrict__ acc_nodes,
                                                             const int32_t *__restrict__ accept_len,
                                                             const int32_t *__restrict__ slot_map) {
    const int b = blockIdx.y, l = blockIdx.z;
    if (slot_map[(size_t)b * dsc.W] < 0) return;  // the sequence failed a check: untouched
    commit_compact_layer(dsc, b, l, prefix_len[b], accept_len[b], acc_nodes + (size_t)b * dsc.W,
                         slot_map + (size_t)b * dsc.W, block_table, k_cache, v_cache, threadIdx.x, 256);
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

static int32_t launch_commit_copy(const etv_commit_desc *h, const void *kt, const void *vt, void *k_cache, void *v_cache,
                           const int32_t *acc_nodes, const int32_t *slot_map, hipStream_t s) {
    hipLaunchKernelGGL(commit_copy_kernel, dim3(h->W, h->B, h->n_layers), dim3(256), 0, s, *h,
                       static_cast<const uint8_t *>(kt), static_cast<const uint8_t *>(vt),
                       static_cast<uint8_t *>(k_cache), static_cast<uint8_t *>(v_cache), acc_nodes, slot_map);
    return check_launch();
}

static int32_t launch_commit_compact(const etv_commit_desc *h, void *k_cache, void *v_cache, const int32_t *block_table,
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
