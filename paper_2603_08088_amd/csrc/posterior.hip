// safe_gather_paths and evaluate_posterior.
// Section 3.2 ("Dummy-root indexing", "Padding and batch semantics"): padding indices are mapped to
// a valid dummy row before any gather and every later use is guarded by a validity flag.
// Section 2.3 / 5.1: greedy acceptance of the longest root-to-leaf prefix whose candidate tokens
// equal the teacher's argmax at the preceding node.
#include "epilogue_parts.h"
#include <algorithm>

namespace etv {

// ---------------------------------------------------------------- safe gather
// One wavefront per path entry.
__global__ void __launch_bounds__(256) safe_gather_kernel(const int32_t *__restrict__ retrieve,
                                                          const int32_t *__restrict__ n_nodes, long total,
                                                          int per_seq, int T_max, int dummy,
                                                          const uint8_t *__restrict__ src, size_t row_bytes,
                                                          int32_t *__restrict__ safe, uint8_t *__restrict__ pvalid,
                                                          uint8_t *__restrict__ gathered) {
    const int lane = threadIdx.x & 63;
    long e = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (e >= total) return;
    const int b = (int)(e / per_seq);
    const int n = n_nodes ? clampi(n_nodes[b], 0, T_max) : T_max;
    gather_entry(e, b, lane, retrieve, n, T_max, dummy, src, row_bytes, safe, pvalid, gathered);
}

// ---------------------------------------------------------------- argmax scan
// grid (chunks, T_max, B): each workgroup reduces one 16 KiB chunk of one node's logit row with
// 16-byte loads, wave shuffles, then one LDS step.  Rows of padded nodes are not read at all.
__global__ void __launch_bounds__(256) argmax_partial_kernel(const float *__restrict__ logits,
                                                             const int32_t *__restrict__ n_nodes, int T_max, int V,
                                                             int chunks, float *__restrict__ pval,
                                                             int32_t *__restrict__ pidx) {
    const int c = blockIdx.x, node = blockIdx.y, b = blockIdx.z;
    if (node >= clampi(n_nodes[b], 0, T_max)) return;
    const float *row = logits + ((size_t)b * T_max + node) * V;
    const int begin = c * kChunk;
    const int end = min(V, begin + kChunk);
    MaxIdx m = {-INFINITY, 0x7fffffff};
    if ((V & 3) == 0 && (((uintptr_t)logits) & 15) == 0) {
        // streaming loads: every logit is read once
        typedef float f32x4 __attribute__((ext_vector_type(4)));
        const f32x4 *row4 = reinterpret_cast<const f32x4 *>(row);
        for (int i = begin / 4 + threadIdx.x; i < end / 4; i += 256) {
            const f32x4 x = __builtin_nontemporal_load(row4 + i);
            int base = i * 4;
            // ascending index order with strict '>' keeps the lowest index among equals
            if (x.x > m.v || m.i == 0x7fffffff) m = {x.x, base};
            if (x.y > m.v) m = {x.y, base + 1};
            if (x.z > m.v) m = {x.z, base + 2};
            if (x.w > m.v) m = {x.w, base + 3};
        }
    } else {
        for (int i = begin + threadIdx.x; i < end; i += 256) {
            float x = row[i];
            if (x > m.v || m.i == 0x7fffffff) m = {x, i};
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        MaxIdx o = {__shfl_xor(m.v, off), __shfl_xor(m.i, off)};
        m = better(m, o);
    }
    __shared__ MaxIdx s_m[4];
    if ((threadIdx.x & 63) == 0) s_m[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        MaxIdx r = better(better(s_m[0], s_m[1]), better(s_m[2], s_m[3]));
        size_t o = ((size_t)b * T_max + node) * chunks + c;
        pval[o] = r.v;
        pidx[o] = r.i;
    }
}

// One workgroup per sequence: finish the argmax, then walk every path with guarded compares and
// reduce to the best path.  All state lives in LDS; the only global traffic is the small outputs.
__global__ void __launch_bounds__(256) posterior_paths_kernel(
    const float *__restrict__ pval, const int32_t *__restrict__ pidx, int chunks,
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ retrieve, const int32_t *__restrict__ n_nodes,
    int T_max, int L_max, int W, int dummy, int32_t *__restrict__ argmax, int32_t *__restrict__ len,
    int32_t *__restrict__ best, int32_t *__restrict__ accept_len, int32_t *__restrict__ acc_nodes,
    int32_t *__restrict__ bonus) {
    const int b = blockIdx.x;
    posterior_for_sequence(b, threadIdx.x, pval, pidx, chunks, tokens, retrieve, clampi(n_nodes[b], 0, T_max), T_max,
                           L_max, W, dummy, argmax, len, best, accept_len, acc_nodes, bonus, nullptr, nullptr);
}

// Fused epilogue: gather, acceptance and commit in ONE launch.
// Workgroups 0 .. B*G-1: sequence b = id / G, layer group g = id % G.  Every one of them runs the acceptance of
// its sequence (a few KiB of per-node maxima and path entries, all cache hits after the first reader) and, from
// the accepted row still in LDS, the commit plan; group 0 writes the results, and every group then moves the
// accepted K/V rows of its own layers (g, g + G, ...).  Recomputing the small acceptance G times costs less than
// any way of handing its result to other workgroups of the same launch (a flag in memory would cost each waiter
// a device-scope round trip and the launch a scratch word that has to start at zero), and no workgroup ever
// waits for another.  Workgroups B*G ..: the safe gather, four path entries each (it depends on the path table
// only, so it runs beside the acceptance instead of before it).
__global__ void __launch_bounds__(256) verify_epilogue_kernel(
    etv_commit_desc dsc, int G, const float *__restrict__ pval, const int32_t *__restrict__ pidx, int chunks,
    const int32_t *__restrict__ tokens, const int32_t *__restrict__ retrieve, const int32_t *__restrict__ n_nodes,
    int L_max, int dummy, const uint8_t *__restrict__ src, size_t row_bytes, int32_t *__restrict__ safe,
    uint8_t *__restrict__ pvalid, uint8_t *__restrict__ gathered, int32_t *__restrict__ argmax,
    int32_t *__restrict__ len, int32_t *__restrict__ best, int32_t *__restrict__ accept_len,
    int32_t *__restrict__ acc_nodes, int32_t *__restrict__ bonus, const uint8_t *__restrict__ kt,
    const uint8_t *__restrict__ vt, uint8_t *__restrict__ k_cache, uint8_t *__restrict__ v_cache,
    const int32_t *__restrict__ block_table, const int32_t *__restrict__ prefix_len,
    const int32_t *__restrict__ capacity, int32_t *__restrict__ prefix_len_out, int32_t *__restrict__ slot_map,
    int32_t *__restrict__ status, int in_place) {
    __shared__ int32_t s_A, s_st, s_plo, s_coop;
    __shared__ int32_t s_acc[ETV_MAX_TREE];
    __shared__ int32_t s_slot[ETV_MAX_TREE];
    const int t = threadIdx.x;
    const int T_max = dsc.T_max, W = dsc.W;
    if ((long)blockIdx.x >= (long)dsc.B * G) {  // uniform over the workgroup
        const long per_seq = (long)L_max * W;
        const long e = ((long)blockIdx.x - (long)dsc.B * G) * 4 + (t >> 6);
        if (e >= per_seq * dsc.B) return;
        const int b = (int)(e / per_seq);
        gather_entry(e, b, t & 63, retrieve, clampi(n_nodes[b], 0, T_max), T_max, dummy, src, row_bytes, safe, pvalid,
                     gathered);
        return;
    }
    const int b = blockIdx.x / G, g = blockIdx.x % G;
    const int n = clampi(n_nodes[b], 0, T_max);
    const int P = prefix_len[b];  // read before group 0 can have written anything (prefix_len_out is another buffer)
    posterior_for_sequence(b, t, pval, pidx, chunks, tokens, retrieve, n, T_max, L_max, W, dummy, argmax, len, best,
                           accept_len, acc_nodes, bonus, &s_A, s_acc, g == 0);
    commit_plan_cooperative(dsc, b, block_table, P, capacity[b], n, s_acc, s_A, &s_plo, s_slot, &s_st, in_place != 0, t, 256,
                            &s_coop);
    if (g == 0) {
        for (int i = t; i < W; i += 256) slot_map[(size_t)b * W + i] = s_slot[i];
        if (t == 0) {
            status[b] = s_st;
            prefix_len_out[b] = s_plo;
        }
    }
    if (s_st) return;  // refused: the sequence stays untouched
    const int A = s_A;
    if (in_place) {
        for (int l = g; l < dsc.n_layers; l += G)
            commit_compact_layer(dsc, b, l, P, A, s_acc, s_slot, block_table, k_cache, v_cache, t, 256);
    } else {
        const int units2 = 2 * (int)((size_t)dsc.d * dsc.elem_bytes / 16) * dsc.Hkv;
        const int total = (A + 1) * units2;
        for (int l = g; l < dsc.n_layers; l += G)
            for (int idx = t; idx < total; idx += 256) {
                const int i = idx / units2;
                commit_copy_unit(dsc, b, l, s_acc[i], s_slot[i], idx - i * units2, kt, vt, k_cache, v_cache);
            }
    }
}

}  // namespace etv

extern "C" int32_t etv_safe_gather_paths(const int32_t *retrieve, const int32_t *n_nodes, int32_t B, int32_t L_max,
                                         int32_t W, int32_t T_max, int32_t dummy, const void *src, size_t row_bytes,
                                         int32_t *safe, uint8_t *pvalid, void *gathered, void *stream) {
    if (!retrieve || B < 0 || L_max < 0 || W < 1 || T_max < 1) return ETV_ERR_INVALID_ARG;
    if (dummy < 0 || dummy >= T_max) return ETV_ERR_INVALID_ARG;
    if ((src == nullptr) != (gathered == nullptr)) return ETV_ERR_INVALID_ARG;
    if (src && row_bytes == 0) return ETV_ERR_INVALID_ARG;
    long total = (long)B * L_max * W;
    if (total == 0) return ETV_OK;
    long blocks = (total + 3) / 4;
    if (blocks > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(etv::safe_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, etv::as_stream(stream),
                       retrieve, n_nodes, total, (int)(L_max * W), (int)T_max, (int)dummy,
                       static_cast<const uint8_t *>(src), row_bytes, safe, pvalid, static_cast<uint8_t *>(gathered));
    return etv::check_launch();
}

extern "C" size_t etv_evaluate_posterior_workspace_bytes(int32_t B, int32_t T_max, int32_t V) {
    if (B < 1 || T_max < 1 || V < 1) return 0;
    size_t chunks = ((size_t)V + etv::kChunk - 1) / etv::kChunk;
    return (size_t)B * T_max * chunks * (sizeof(float) + sizeof(int32_t));
}

extern "C" int32_t etv_evaluate_posterior(const float *logits, const int32_t *tokens, const int32_t *retrieve,
                                          const int32_t *n_nodes, int32_t B, int32_t T_max, int32_t V,
                                          int32_t L_max, int32_t W, int32_t dummy, int32_t *argmax, int32_t *len,
                                          int32_t *best, int32_t *accept_len, int32_t *acc_nodes, int32_t *bonus,
                                          void *workspace, size_t workspace_bytes, void *stream) {
    if (!tokens || !retrieve || !n_nodes || !argmax || !len || !best || !accept_len || !acc_nodes || !bonus)
        return ETV_ERR_INVALID_ARG;
    if (B < 0 || T_max < 1 || (logits && V < 1) || V < 0 || L_max < 1 || W < 1) return ETV_ERR_INVALID_ARG;
    if (dummy < 0 || dummy >= T_max) return ETV_ERR_INVALID_ARG;
    if (T_max > ETV_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if (B == 0) return ETV_OK;
    if (B > 65535) return ETV_ERR_UNSUPPORTED;
    hipStream_t s = etv::as_stream(stream);
    int chunks = 0;
    float *pval = nullptr;
    int32_t *pidx = nullptr;
    int32_t rc;
    if (logits) {  // without logits, argmax[] is an input
        size_t need = etv_evaluate_posterior_workspace_bytes(B, T_max, V);
        if (!workspace || workspace_bytes < need) return ETV_ERR_WORKSPACE_TOO_SMALL;
        chunks = (V + etv::kChunk - 1) / etv::kChunk;
        pval = static_cast<float *>(workspace);
        pidx = reinterpret_cast<int32_t *>(pval + (size_t)B * T_max * chunks);
        hipLaunchKernelGGL(etv::argmax_partial_kernel, dim3(chunks, T_max, B), dim3(256), 0, s, logits, n_nodes,
                           (int)T_max, (int)V, chunks, pval, pidx);
        rc = etv::check_launch();
        if (rc != ETV_OK) return rc;
    } else if (V > 0) {  // the per-tile maxima left by etv_lm_head_argmax (argmax == NULL there) for this B, T_max, V
        size_t need = etv_lm_head_argmax_workspace_bytes(B, T_max, V);
        if (!workspace || workspace_bytes < need) return ETV_ERR_WORKSPACE_TOO_SMALL;
        chunks = (V + 127) / 128;
        pval = static_cast<float *>(workspace);
        pidx = reinterpret_cast<int32_t *>(pval + (size_t)B * T_max * chunks);
    }
    hipLaunchKernelGGL(etv::posterior_paths_kernel, dim3(B), dim3(256), 0, s, pval, pidx, chunks, tokens, retrieve,
                       n_nodes, (int)T_max, (int)L_max, (int)W, (int)dummy, argmax, len, best, accept_len, acc_nodes,
                       bonus);
    return etv::check_launch();
}

extern "C" int32_t etv_verify_epilogue(const etv_commit_desc *h, const float *logits, int32_t V, const int32_t *tokens,
                                       const int32_t *retrieve, int32_t L_max, int32_t dummy, const void *src,
                                       size_t row_bytes, int32_t *safe, uint8_t *pvalid, void *gathered,
                                       int32_t *argmax, int32_t *len, int32_t *best, int32_t *accept_len,
                                       int32_t *acc_nodes, int32_t *bonus, const void *kt, const void *vt,
                                       void *k_cache, void *v_cache, const int32_t *block_table,
                                       const int32_t *prefix_len, const int32_t *capacity, const int32_t *n_nodes,
                                       int32_t *prefix_len_out, int32_t *slot_map, int32_t *status, void *workspace,
                                       size_t workspace_bytes, void *stream) {
    if (!tokens || !retrieve || !n_nodes || !argmax || !len || !best || !accept_len || !acc_nodes ||
        !bonus || !prefix_len || !capacity || !prefix_len_out || !slot_map || !status)
        return ETV_ERR_INVALID_ARG;
    int32_t rc = etv::check_commit_args(h, kt, vt, k_cache, v_cache, block_table);
    if (rc != ETV_OK) return rc;
    if ((logits && V < 1) || V < 0 || L_max < 1) return ETV_ERR_INVALID_ARG;
    if (dummy < 0 || dummy >= h->T_max) return ETV_ERR_INVALID_ARG;
    if ((src == nullptr) != (gathered == nullptr)) return ETV_ERR_INVALID_ARG;
    if (src && row_bytes == 0) return ETV_ERR_INVALID_ARG;
    if (h->T_max > ETV_MAX_TREE || h->W > ETV_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    const bool in_place = (kt == nullptr);  // in-place branch cache, as in etv_commit_accepted_kv
    // several workgroups of the one launch read prefix_len[b] while another writes prefix_len_out[b]
    if (prefix_len_out == prefix_len) return ETV_ERR_INVALID_ARG;
    if (h->B == 0) return ETV_OK;
    const int32_t B = h->B, T_max = h->T_max;
    hipStream_t s = etv::as_stream(stream);
    int chunks = 0;
    float *pval = nullptr;
    int32_t *pidx = nullptr;
    if (logits) {  // without logits, argmax[] is an input
        size_t need = etv_evaluate_posterior_workspace_bytes(B, T_max, V);
        if (!workspace || workspace_bytes < need) return ETV_ERR_WORKSPACE_TOO_SMALL;
        chunks = (V + etv::kChunk - 1) / etv::kChunk;
        pval = static_cast<float *>(workspace);
        pidx = reinterpret_cast<int32_t *>(pval + (size_t)B * T_max * chunks);
        hipLaunchKernelGGL(etv::argmax_partial_kernel, dim3(chunks, T_max, B), dim3(256), 0, s, logits, n_nodes,
                           (int)T_max, (int)V, chunks, pval, pidx);
        rc = etv::check_launch();
        if (rc != ETV_OK) return rc;
    } else if (V > 0) {  // the per-tile maxima left by etv_lm_head_argmax (argmax == NULL there) for this B, T_max, V
        size_t need = etv_lm_head_argmax_workspace_bytes(B, T_max, V);
        if (!workspace || workspace_bytes < need) return ETV_ERR_WORKSPACE_TOO_SMALL;
        chunks = (V + 127) / 128;
        pval = static_cast<float *>(workspace);
        pidx = reinterpret_cast<int32_t *>(pval + (size_t)B * T_max * chunks);
    }
    const long gather_blocks = (safe || pvalid || gathered) ? ((long)B * L_max * h->W + 3) / 4 : 0;
    // layer groups per sequence: enough workgroups to spread the row copies over the chip, at most one per layer
    const int G = std::max(1, std::min((int)h->n_layers, 512 / B));
    if (gather_blocks + (long)B * G > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(etv::verify_epilogue_kernel, dim3((unsigned)((long)B * G + gather_blocks)), dim3(256), 0, s, *h, G,
                       pval, pidx, chunks, tokens, retrieve, n_nodes, (int)L_max, (int)dummy,
                       static_cast<const uint8_t *>(src), row_bytes, safe, pvalid, static_cast<uint8_t *>(gathered),
                       argmax, len, best, accept_len, acc_nodes, bonus, static_cast<const uint8_t *>(kt),
                       static_cast<const uint8_t *>(vt), static_cast<uint8_t *>(k_cache),
                       static_cast<uint8_t *>(v_cache), block_table, prefix_len, capacity, prefix_len_out, slot_map,
                       status, in_place ? 1 : 0);
    return etv::check_launch();
}
