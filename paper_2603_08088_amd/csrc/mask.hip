// build_tree_mask: ancestor bitmask, dense 4D mask, depths and structural-invariant status.
// Section 3.2 ("Ancestor tables", "Structural invariants") and Section 3.3 ("Tree attention
// mask", "Implementation note": compact ancestor encoding produced on the device).
// tensorize_tree: the same launch also writes position ids (Section 3.3 "Execution view": prefix
// length + depth) and the table of root-to-leaf paths that the gather and the acceptance step
// consume, so nothing about the tree is computed on the host.
#include "etv_common.h"

namespace etv {

constexpr int kMaskWords = ETV_MAX_TREE / 64;

// One workgroup per sequence, one thread per node row.  Instead of materialising the
// (D_max+1) x T ancestor table, each thread follows its own parent chain (bounded by the
// node count) and ORs the visited rows into registers: the same relation, no table.
//
// Paths (retrieve != nullptr): a leaf is a valid node that no valid node names as its parent; leaves are
// ranked in ascending row order with one ballot per wavefront; the thread of the leaf ranked r walks its
// chain once more and writes row r back to front (entry i = the ancestor depth - i steps up), then pads
// the row with -1; rows beyond the last leaf are filled by all threads together.
__global__ void __launch_bounds__(ETV_MAX_TREE) build_tree_mask_kernel(
    const int32_t *__restrict__ parent, const int32_t *__restrict__ n_nodes, int T_max, int words,
    uint64_t *__restrict__ bitmask, uint8_t *__restrict__ dense, int32_t *__restrict__ depth,
    int32_t *__restrict__ status, const int32_t *__restrict__ prefix_len, int32_t *__restrict__ position_ids,
    int32_t *__restrict__ retrieve, int32_t *__restrict__ n_paths, int L_max, int W) {
    __shared__ int32_t s_ep[ETV_MAX_TREE];                 // effective parent after range/closure repair
    __shared__ uint64_t s_bits[ETV_MAX_TREE][kMaskWords];  // rows, for the cooperative dense write
    __shared__ int32_t s_status;
    __shared__ uint8_t s_child[ETV_MAX_TREE];
    __shared__ int32_t s_wave_leaves[ETV_MAX_TREE / 64];
    const int b = blockIdx.x;
    const int k = threadIdx.x;
    const int n = clampi(n_nodes[b], 0, T_max);
    if (k == 0) s_status = 0;
    s_child[k] = 0;
    __syncthreads();
    int32_t st = 0;
    if (k < n) {
        int32_t p = parent[(size_t)b * T_max + k];
        int32_t ep;
        if (k == 0) {
            if (p != 0) st |= ETV_TREE_RANGE;
            ep = 0;
        } else if (p < 0 || p >= T_max) {
            st |= ETV_TREE_RANGE;
            ep = 0;
        } else if (p >= n) {
            st |= ETV_TREE_CLOSURE;
            ep = 0;
        } else {
            ep = p;
        }
        s_ep[k] = ep;
    }
    __syncthreads();
    uint64_t bits[kMaskWords];
#pragma unroll
    for (int w = 0; w < kMaskWords; w++) bits[w] = 0;
    int dep = 0;
    if (k < n) {
        int cur = k, steps = 0;
        while (cur != 0 && steps < n) {
#pragma unroll
            for (int w = 0; w < kMaskWords; w++)
                if ((cur >> 6) == w) bits[w] |= 1ull << (cur & 63);
            cur = s_ep[cur];
            steps++;
        }
        if (cur == 0) {
            bits[0] |= 1ull;
            dep = steps;
        } else {  // the chain never reaches the root: a cycle.  Re-attach k to the root.
            st |= ETV_TREE_CYCLE;
#pragma unroll
            for (int w = 0; w < kMaskWords; w++) bits[w] = ((k >> 6) == w) ? (1ull << (k & 63)) : 0ull;
            bits[0] |= 1ull;
            dep = 1;
        }
    }
    const bool cyc = (st & ETV_TREE_CYCLE) != 0;
    if (st) atomicOr(&s_status, st);
    if (k < T_max) {
#pragma unroll
        for (int w = 0; w < kMaskWords; w++) {
            s_bits[k][w] = bits[w];
            if (w < words) bitmask[((size_t)b * T_max + k) * words + w] = bits[w];
        }
        if (depth) depth[(size_t)b * T_max + k] = dep;
    }
    if (position_ids && k < T_max) {
        const int P = prefix_len ? max(prefix_len[b], 0) : 0;
        position_ids[(size_t)b * T_max + k] = P + dep;
    }
    if (retrieve) {
        __syncthreads();             // every chain walk is done: the repaired parents may now change
        if (cyc) s_ep[k] = 0;        // a node on a cycle hangs off the root from here on
        __syncthreads();
        if (k >= 1 && k < n) s_child[s_ep[k]] = 1;
        __syncthreads();
        const bool leaf = k < n && !s_child[k];
        const unsigned long long lb = __ballot(leaf);
        const int wv = k >> 6;
        if ((k & 63) == 0) s_wave_leaves[wv] = __popcll(lb);
        __syncthreads();
        int rank = __popcll(lb & ((1ull << (k & 63)) - 1ull));
        int total = 0;
        for (int w = 0; w < (int)(blockDim.x >> 6); w++) {
            if (w < wv) rank += s_wave_leaves[w];
            total += s_wave_leaves[w];
        }
        int32_t *rows = retrieve + (size_t)b * L_max * W;
        if (leaf && rank < L_max) {
            int32_t *row = rows + (size_t)rank * W;
            if (dep + 1 > W) st |= ETV_TREE_DEPTH;
            int cur = k;
            for (int i = dep; i >= 0; i--) {   // dep <= n - 1: the walk above reached the root in dep steps
                if (i < W) row[i] = cur;
                cur = s_ep[cur];
            }
            for (int i = dep + 1; i < W; i++) row[i] = -1;
        }
        if (total > L_max) st |= ETV_TREE_PATHS;
        const int kept = min(total, L_max);
        for (int e = kept * W + k; e < L_max * W; e += blockDim.x) rows[e] = -1;
        if (n_paths && k == 0) n_paths[b] = kept;
        if (st & (ETV_TREE_DEPTH | ETV_TREE_PATHS)) atomicOr(&s_status, st);
    }
    __syncthreads();
    if (k == 0) status[b] = s_status;
    if (dense) {
        uint8_t *out = dense + (size_t)b * T_max * T_max;
        if ((T_max & 3) == 0 && (((uintptr_t)dense) & 3) == 0) {
            // four mask bytes per store: thread k keeps one 4-byte group of a row and walks down the rows
            // (groups = T_max / 4 <= 64 <= blockDim: one division per thread, none per element)
            const int groups = T_max >> 2;
            const int g = k % groups, rstep = blockDim.x / groups;
            uint32_t *out4 = reinterpret_cast<uint32_t *>(out);
            for (int row = k / groups; row < T_max && k < rstep * groups; row += rstep) {
                const uint32_t nib = (uint32_t)(s_bits[row][g >> 4] >> ((g & 15) * 4)) & 15u;
                // bit i of the nibble -> byte i
                out4[row * groups + g] = (nib & 1u) | ((nib & 2u) << 7) | ((nib & 4u) << 14) | ((nib & 8u) << 21);
            }
        } else {
            const int total = T_max * T_max;
            for (int e = k; e < total; e += blockDim.x) {
                int row = e / T_max, col = e - row * T_max;
                out[e] = (uint8_t)((s_bits[row][col >> 6] >> (col & 63)) & 1ull);
            }
        }
    }
}

}  // namespace etv

extern "C" int32_t etv_build_tree_mask(const int32_t *parent, const int32_t *n_nodes, int32_t B, int32_t T_max,
                                       uint64_t *bitmask, uint8_t *dense, int32_t *depth, int32_t *status,
                                       void *stream) {
    if (!parent || !n_nodes || !bitmask || !status || B < 0) return ETV_ERR_INVALID_ARG;
    if (T_max < 1) return ETV_ERR_INVALID_ARG;
    if (T_max > ETV_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if (B == 0) return ETV_OK;
    int threads = ((T_max + 63) / 64) * 64;
    int words = (T_max + 63) / 64;
    hipLaunchKernelGGL(etv::build_tree_mask_kernel, dim3(B), dim3(threads), 0, etv::as_stream(stream), parent,
                       n_nodes, (int)T_max, words, bitmask, dense, depth, status, (const int32_t *)nullptr,
                       (int32_t *)nullptr, (int32_t *)nullptr, (int32_t *)nullptr, 0, 0);
    return etv::check_launch();
}

extern "C" int32_t etv_tensorize_tree(const int32_t *parent, const int32_t *n_nodes, const int32_t *prefix_len,
                                      int32_t B, int32_t T_max, int32_t L_max, int32_t W, uint64_t *bitmask,
                                      uint8_t *dense, int32_t *depth, int32_t *position_ids, int32_t *retrieve,
                                      int32_t *n_paths, int32_t *status, void *stream) {
    if (!parent || !n_nodes || !bitmask || !retrieve || !status || B < 0) return ETV_ERR_INVALID_ARG;
    if (T_max < 1 || L_max < 1 || W < 1) return ETV_ERR_INVALID_ARG;
    if (position_ids && !prefix_len) return ETV_ERR_INVALID_ARG;
    if (T_max > ETV_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if ((long)L_max * W > (1l << 24)) return ETV_ERR_UNSUPPORTED;
    if (B == 0) return ETV_OK;
    int threads = ((T_max + 63) / 64) * 64;
    int words = (T_max + 63) / 64;
    hipLaunchKernelGGL(etv::build_tree_mask_kernel, dim3(B), dim3(threads), 0, etv::as_stream(stream), parent,
                       n_nodes, (int)T_max, words, bitmask, dense, depth, status, prefix_len, position_ids, retrieve,
                       n_paths, (int)L_max, (int)W);
    return etv::check_launch();
}
