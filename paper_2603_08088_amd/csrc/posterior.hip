// safe_gather_paths and evaluate_posterior.
// Section 3.2 ("Dummy-root indexing", "Padding and batch semantics"): padding indices are mapped to
// a valid dummy row before any gather and every later use is guarded by a validity flag.
// Section 2.3 / 5.1: greedy acceptance of the longest root-to-leaf prefix whose candidate tokens
// equal the teacher's argmax at the preceding node.
#include "etv_common.h"

namespace etv {

// ---------------------------------------------------------------- safe gather
__device__ __forceinline__ int32_t safe_index(int32_t idx, int T_max, int dummy) {
    return (idx >= 0 && idx < T_max) ? idx : dummy;
}

// One wavefront per path entry: lane-strided copy of the gathered row.
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
    const int32_t idx = retrieve[e];
    const int32_t s = safe_index(idx, T_max, dummy);
    const int n = n_nodes ? clampi(n_nodes[b], 0, T_max) : T_max;
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

// ---------------------------------------------------------------- argmax scan
struct MaxIdx {
    float v;
    int32_t i;
};
// (a beats b) iff a is larger, or equal with the lower index: "lowest index of the maximum"
__device__ __forceinline__ MaxIdx better(MaxIdx a, MaxIdx b) {
    return (b.v > a.v || (b.v == a.v && b.i < a.i)) ? b : a;
}

constexpr int kChunk = 4096;  // floats of one logit row scanned by one workgroup (16 KiB)

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
        const float4 *row4 = reinterpret_cast<const float4 *>(row);
        for (int i = begin / 4 + threadIdx.x; i < end / 4; i += 256) {
            float4 x = row4[i];
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
    __shared__ int32_t s_g[ETV_MAX_TREE];
    __shared__ int32_t s_tok[ETV_MAX_TREE];
    __shared__ int32_t s_len[256];
    __shared__ int32_t s_path[256];
    const int b = blockIdx.x, t = threadIdx.x;
    const int n = clampi(n_nodes[b], 0, T_max);
    for (int node = t; node < T_max; node += 256) {
        int32_t g = -1;
        if (node < n) {
            size_t o = ((size_t)b * T_max + node) * chunks;
            MaxIdx m = {pval[o], pidx[o]};
            for (int c = 1; c < chunks; c++) m = better(m, MaxIdx{pval[o + c], pidx[o + c]});
            g = m.i;
        }
        s_g[node] = g;
        s_tok[node] = tokens[(size_t)b * T_max + node];
        argmax[(size_t)b * T_max + node] = g;
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
    for (int i = t; i < W; i += 256)
        acc_nodes[(size_t)b * W + i] = (i <= A) ? safe_index(path[i], T_max, dummy) : dummy;
    if (t == 0) {
        best[b] = bp;
        accept_len[b] = A;
        int32_t last = safe_index(path[A], T_max, dummy);
        bonus[b] = s_g[last];
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
    if (!logits || !tokens || !retrieve || !n_nodes || !argmax || !len || !best || !accept_len || !acc_nodes ||
        !bonus)
        return ETV_ERR_INVALID_ARG;
    if (B < 0 || T_max < 1 || V < 1 || L_max < 1 || W < 1) return ETV_ERR_INVALID_ARG;
    if (dummy < 0 || dummy >= T_max) return ETV_ERR_INVALID_ARG;
    if (T_max > ETV_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if (B == 0) return ETV_OK;
    if (B > 65535) return ETV_ERR_UNSUPPORTED;
    size_t need = etv_evaluate_posterior_workspace_bytes(B, T_max, V);
    if (!workspace || workspace_bytes < need) return ETV_ERR_WORKSPACE_TOO_SMALL;
    int chunks = (V + etv::kChunk - 1) / etv::kChunk;
    float *pval = static_cast<float *>(workspace);
    int32_t *pidx = reinterpret_cast<int32_t *>(pval + (size_t)B * T_max * chunks);
    hipStream_t s = etv::as_stream(stream);
    hipLaunchKernelGGL(etv::argmax_partial_kernel, dim3(chunks, T_max, B), dim3(256), 0, s, logits, n_nodes,
                       (int)T_max, (int)V, chunks, pval, pidx);
    int32_t rc = etv::check_launch();
    if (rc != ETV_OK) return rc;
    hipLaunchKernelGGL(etv::posterior_paths_kernel, dim3(B), dim3(256), 0, s, pval, pidx, chunks, tokens, retrieve,
                       n_nodes, (int)T_max, (int)L_max, (int)W, (int)dummy, argmax, len, best, accept_len, acc_nodes,
                       bonus);
    return etv::check_launch();
}
