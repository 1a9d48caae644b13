// build_tree_mask: ancestor bitmask, dense 4D mask, depths and structural-invariant status.
// Section 3.2 ("Ancestor tables", "Structural invariants") and Section 3.3 ("Tree attention
// mask", "Implementation note": compact ancestor encoding produced on the device).
#include "etv_common.h"

namespace etv {

constexpr int kMaskWords = ETV_MAX_TREE / 64;

// One workgroup per sequence, one thread per node row.  Instead of materialising the
// (D_max+1) x T ancestor table, each thread follows its own parent chain (bounded by the
// node count) and ORs the visited rows into registers: the same relation, no table.
__global__ void __launch_bounds__(ETV_MAX_TREE) build_tree_mask_kernel(
    const int32_t *__restrict__ parent, const int32_t *__restrict__ n_nodes, int T_max, int words,
    uint64_t *__restrict__ bitmask, uint8_t *__restrict__ dense, int32_t *__restrict__ depth,
    int32_t *__restrict__ status) {
    __shared__ int32_t s_ep[ETV_MAX_TREE];                 // effective parent after range/closure repair
    __shared__ uint64_t s_bits[ETV_MAX_TREE][kMaskWords];  // rows, for the cooperative dense write
    __shared__ int32_t s_status;
    const int b = blockIdx.x;
    const int k = threadIdx.x;
    const int n = clampi(n_nodes[b], 0, T_max);
    if (k == 0) s_status = 0;
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
    if (st) atomicOr(&s_status, st);
    if (k < T_max) {
#pragma unroll
        for (int w = 0; w < kMaskWords; w++) {
            s_bits[k][w] = bits[w];
            if (w < words) bitmask[((size_t)b * T_max + k) * words + w] = bits[w];
        }
        if (depth) depth[(size_t)b * T_max + k] = dep;
    }
    __syncthreads();
    if (k == 0) status[b] = s_status;
    if (dense) {
        uint8_t *out = dense + (size_t)b * T_max * T_max;
        const int total = T_max * T_max;
        for (int e = k; e < total; e += blockDim.x) {
            int row = e / T_max, col = e - row * T_max;
            out[e] = (uint8_t)((s_bits[row][col >> 6] >> (col & 63)) & 1ull);
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
                       n_nodes, (int)T_max, words, bitmask, dense, depth, status);
    return etv::check_launch();
}
