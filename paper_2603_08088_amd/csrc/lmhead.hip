// lm_head_argmax: teacher head and greedy choice in one pass, logits never written to memory.
// Section 3.3 ("Execution view", "Mapping teacher outputs to node verification scores"): the teacher turns
// the hidden state of every tree node into logits over the vocabulary; Section 5.1: greedy decoding needs only
// their argmax.  For the 60..128 rows of a verify step this is a weight-streaming product: each head weight is
// read from HBM once (2 * V * D bytes) and the arithmetic intensity is the row count, so the bound is HBM.
//
// Work unit: 128 vocabulary rows x up to 64 node rows.  The contraction runs over D in steps of 128: a step's
// weight tile (128 rows x 256 B = 32 KiB, 256 contiguous bytes of every row) and hidden tile (64 rows x 256 B)
// go to LDS with asynchronous direct-to-LDS loads into a ring of three stages, one barrier per step.
// Wavefront w of 8 owns vocabulary block w % 4 (32 rows) and node chunk w / 4 (32 rows).
// C^T[vocab, node] = W . H^T on v_mfma_f32_32x32x16_bf16: A = weight rows, B = hidden rows, so a node is an
// accumulator column and its maximum over the vocabulary stays in one lane pair.  The 16-byte chunk c of tile
// row r sits at chunk position c ^ (r & 15), which spreads the fragment reads of 32 consecutive rows over the
// LDS banks.
//
// More than 64 rows (lm_head_argmax_wide_kernel): a workgroup takes up to 128 node rows.  What bounds the stream is
// the weight bytes a compute unit keeps in flight (in flight / latency = rate), so LDS is spent on weights: a step
// is half a weight tile (64 vocabulary rows x 256 B = 16 KiB, consecutive in the packed layout) in a ring of five
// stages, and the 128 hidden rows of a contraction step (32 KiB, from L2) serve both halves and get a ring of two.
// A wavefront's loads complete in order, so the deep weight ring and the shallow hidden ring are fed by different
// wavefronts (0..3 weights, 4..7 hidden rows), each waiting on its own counter.  Wavefront w owns vocabulary block
// w % 2 of each half and node chunk w / 2, with one accumulator per half.  More than 128 rows run as further row
// groups: they stream the weights again, placed so that the groups of one vocabulary tile share an XCD and the
// repeat comes from its L2.
//
// Weight layout.  With row-major [V, D] weights a step reads 128 pieces of 256 B that lie 2 * D bytes apart,
// and the stream reaches 4.6-4.8 TB/s; with the weights packed once into tiles ([V/128][D/128][128 rows][128],
// etv_pack_lm_head) a step's tile is 32 KiB of consecutive memory and the same kernel reaches 5.5-5.8 TB/s.
// Both layouts are accepted.
#include "etv_common.h"

namespace etv {

typedef __attribute__((ext_vector_type(8))) __bf16 lh_bf16x8;
typedef __attribute__((ext_vector_type(16))) float lh_f32x16;

constexpr int LH_VT = 128;   // vocabulary rows per workgroup
constexpr int LH_RT = 64;    // node rows per workgroup (2 chunks of 32)
constexpr int LH_KC = 128;   // contraction elements per step
constexpr int LH_ROWB = LH_KC * 2;               // bytes of a tile row
constexpr int LH_W_BYTES = LH_VT * LH_ROWB;      // 32 KiB
constexpr int LH_STAGE = LH_W_BYTES + LH_RT * LH_ROWB;  // 48 KiB
constexpr int LH_NS = 3;     // ring stages (144 KiB)

extern __shared__ __attribute__((aligned(1024))) uint8_t lh_smem[];

// NT: streaming (nontemporal) load, for bytes that no other workgroup will ask for: they stream a seventh faster
// than plain loads on this machine, but do not stay in L2.
template <bool NT>
__device__ __forceinline__ void lh_async_load16(const void *sbase_in, uint32_t voff, uint32_t lds_addr_in) {
    // base and LDS address are the same in every lane; readfirstlane says so to the compiler whatever it concluded
    // about the selects and loops they came through (it folds away for values already in scalar registers)
    const uint64_t raw = (uint64_t)(uintptr_t)sbase_in;
    const uint64_t uni = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(raw >> 32)) << 32) |
                         (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)raw);
    const void *sbase = (const void *)(uintptr_t)uni;
    const uint32_t lds_addr = (uint32_t)__builtin_amdgcn_readfirstlane((int)lds_addr_in);
    if (NT)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}
template <int N>
__device__ __forceinline__ void lh_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}

struct LhParams {
    const uint8_t *hidden;   // [rows_total, D] bf16
    const uint8_t *weight;   // [V, D] bf16
    const int32_t *n_nodes;  // [B]
    float *pval;             // [rows_total, tiles]
    int32_t *pidx;
    int rows_total, T_max, D, V, tiles, groups;
    int packed;  // weight layout: 0 = [V, D] row-major, 1 = tiles of etv_pack_lm_head
};

// wait until at most n of the wavefront's loads are outstanding, n = (steps ahead) * (loads per step)
__device__ __forceinline__ void lh_wait(int n) {
    switch (n) {
    case 4: lh_wait_vmcnt<4>(); break;
    case 5: lh_wait_vmcnt<5>(); break;
    case 6: lh_wait_vmcnt<6>(); break;
    default: lh_wait_vmcnt<0>(); break;
    }
}

// 1-D grid over (vocabulary tile, row group).  Workgroups go to the 8 XCDs round-robin by id; the row groups of
// one vocabulary tile get ids that differ by 8, so they run at the same time on one XCD and the second reader
// of a weight line finds it in that XCD's L2.
__global__ void __launch_bounds__(512, 1) lm_head_argmax_kernel(LhParams p) {
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lh_smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, hh = lane >> 5;
    const int rest = blockIdx.x >> 3;
    const int group = rest % p.groups;
    const int tile = (rest / p.groups) * 8 + (blockIdx.x & 7);
    if (tile >= p.tiles) return;  // uniform over the workgroup
    const int v0 = tile * LH_VT;
    const int r0 = group * LH_RT;
    const int nrows = min(LH_RT, p.rows_total - r0);   // >= 1
    const int nchunks = (nrows + 31) >> 5;
    const int steps = p.D / LH_KC;

    // Loads.  A 1 KiB unit = 4 tile rows x 256 B; lane i fetches row i / 16 of the unit and the source chunk
    // that belongs at chunk position i % 16, i.e. chunk (i % 16) ^ (row & 15).  Units 0..31 are weight rows,
    // 32..47 hidden rows; wavefront w issues units w, w + 8, ... : the row within the tile is 4 * unit + i / 16,
    // so row & 15 = (4 * w + i / 16) & 15 for every one of them.  Rows past the end of the vocabulary / of the
    // node rows re-read the last valid row (their results are masked).
    const int l_row = lane >> 4;
    const uint32_t lane_col = (uint32_t)(((lane & 15) ^ ((4 * wave + l_row) & 15)) * 16);
    const size_t row_bytes = (size_t)p.D * 2;
    uint32_t voff[6];
    const uint8_t *sbase[6];
    bool unit_on[6];
#pragma unroll
    for (int u = 0; u < 6; u++) {
        const int unit = wave + 8 * u;
        if (u < 4) {
            if (p.packed) {  // the tile of step st: 32 KiB at (tile * steps + st) * 32 KiB, unit after unit
                sbase[u] = p.weight + (size_t)tile * steps * LH_W_BYTES + (size_t)unit * 1024;
                voff[u] = (uint32_t)(l_row * LH_ROWB) + lane_col;
            } else {
                const int vrow = min(v0 + 4 * unit + l_row, p.V - 1);
                const int vfirst = min(v0 + 4 * unit, p.V - 1);
                sbase[u] = p.weight + (size_t)vfirst * row_bytes;
                voff[u] = (uint32_t)((size_t)(vrow - vfirst) * row_bytes) + lane_col;
            }
            unit_on[u] = true;
        } else {
            const int hu = unit - 32;  // hidden unit: rows 4 * hu ..
            const int last = r0 + nrows - 1;
            const int rrow = min(r0 + 4 * hu + l_row, last);
            const int rfirst = min(r0 + 4 * hu, last);
            sbase[u] = p.hidden + (size_t)rfirst * row_bytes;
            voff[u] = (uint32_t)((size_t)(rrow - rfirst) * row_bytes) + lane_col;
            unit_on[u] = 4 * hu < nrows;  // hidden units beyond the rows of this group are not loaded at all
        }
    }
    const int loads_per_step = 4 + (unit_on[4] ? 1 : 0) + (unit_on[5] ? 1 : 0);
    auto issue = [&](int st) {
        const uint32_t dst = smem_addr + (uint32_t)(st % LH_NS) * LH_STAGE + (uint32_t)wave * 1024;
        const size_t koff = (size_t)st * LH_ROWB;                               // row-major: next 256 B of every row
        const size_t woff = p.packed ? (size_t)st * LH_W_BYTES : koff;          // packed: next 32 KiB tile
        // with a single row group each weight byte is read by one workgroup: streamed; the hidden rows are
        // read by every workgroup and stay plain
        if (p.groups == 1) {
#pragma unroll
            for (int u = 0; u < 4; u++)
                if (unit_on[u]) lh_async_load16<true>(sbase[u] + woff, voff[u], dst + u * 8192);
        } else {
#pragma unroll
            for (int u = 0; u < 4; u++)
                if (unit_on[u]) lh_async_load16<false>(sbase[u] + woff, voff[u], dst + u * 8192);
        }
#pragma unroll
        for (int u = 4; u < 6; u++)
            if (unit_on[u]) lh_async_load16<false>(sbase[u] + koff, voff[u], dst + u * 8192);
    };
    constexpr int PD = LH_NS - 1;
    for (int st = 0; st < PD && st < steps; st++) issue(st);

    // Fragment offsets: A = weight rows of vocabulary block vb, B = hidden rows of chunk cg; lane holds row
    // c32 and the 8 contraction values at 16-byte chunk 2 * kk + hh of the 128-element step.
    const int vb = wave & 3, cg = wave >> 2;
    const uint32_t a_row = (uint32_t)((32 * vb + c32) * LH_ROWB);
    const uint32_t b_row = (uint32_t)(LH_W_BYTES + (32 * cg + c32) * LH_ROWB);
    const int sw = c32 & 15;
    const bool has = cg < nchunks;

    lh_f32x16 acc0, acc1;  // two chains over the even / odd contraction steps
#pragma unroll
    for (int i = 0; i < 16; i++) { acc0[i] = 0.f; acc1[i] = 0.f; }

    for (int st = 0; st < steps; st++) {
        // loads of the younger step may stay outstanding
        lh_wait(min(PD - 1, steps - 1 - st) * loads_per_step);
        __builtin_amdgcn_s_barrier();  // step st is in LDS for everyone; the stage of step st - 1 is free
        asm volatile("" ::: "memory");
        if (st + PD < steps) issue(st + PD);
        const uint8_t *stage = lh_smem + (st % LH_NS) * LH_STAGE;
        if (!has) continue;
        lh_bf16x8 a[8], b[8];
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            const int col = ((2 * kk + hh) ^ sw) << 4;
            a[kk] = *reinterpret_cast<const lh_bf16x8 *>(stage + a_row + col);
            b[kk] = *reinterpret_cast<const lh_bf16x8 *>(stage + b_row + col);
        }
#pragma unroll
        for (int kk = 0; kk < 8; kk += 2) {
            acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], b[kk], acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk + 1], b[kk + 1], acc1, 0, 0, 0);
        }
    }

    // Epilogue: per node column the maximum over this wavefront's 32 vocabulary rows (accumulator element i of
    // lane half hh is vocabulary row 8 * (i / 4) + 4 * hh + i % 4: ascending in i), then over the two lane
    // halves, then over the four vocabulary blocks through LDS.  Lowest index wins among equals.
    __builtin_amdgcn_s_barrier();  // the ring is free
    float *s_val = reinterpret_cast<float *>(lh_smem);                    // [4 blocks][64 rows]
    int32_t *s_idx = reinterpret_cast<int32_t *>(lh_smem + 4 * LH_RT * 4);
    if (has) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int v = v0 + 32 * vb + 8 * (i >> 2) + 4 * hh + (i & 3);
            const float x = (v < p.V) ? acc0[i] + acc1[i] : -INFINITY;
            if (x > bv || (bi == 0x7fffffff && v < p.V)) { bv = x; bi = v; }
        }
        const float ov = __shfl_xor(bv, 32);
        const int oi = __shfl_xor(bi, 32);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        if (hh == 0) {
            const int rl = 32 * cg + c32;
            s_val[vb * LH_RT + rl] = bv;
            s_idx[vb * LH_RT + rl] = bi;
        }
    }
    __syncthreads();
    if (tid < nrows) {
        float bv = s_val[tid];
        int bi = s_idx[tid];
#pragma unroll
        for (int q = 1; q < 4; q++) {
            const float ov = s_val[q * LH_RT + tid];
            const int oi = s_idx[q * LH_RT + tid];
            if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        const size_t o = (size_t)(r0 + tid) * p.tiles + tile;
        p.pval[o] = bv;
        p.pidx[o] = bi;
    }
}

// ----------------------------------------------------------------------------------------------------------------
// 65..128 node rows per workgroup (see the file comment).  Step s = (contraction step k = s / 2, tile half s % 2).
// ----------------------------------------------------------------------------------------------------------------
constexpr int LHW_RT = 128;                  // node rows per workgroup
constexpr int LHW_W_STEP = 64 * LH_ROWB;     // 16 KiB: 64 vocabulary rows of a step
constexpr int LHW_H_STEP = LHW_RT * LH_ROWB; // 32 KiB: the hidden rows of a contraction step
constexpr int LHW_NSW = 5, LHW_NSH = 2;      // ring stages: weights, hidden rows
constexpr int LHW_W_RING = LHW_NSW * LHW_W_STEP;
static_assert(LHW_W_RING + LHW_NSH * LHW_H_STEP == LH_NS * LH_STAGE, "both kernels use the same 144 KiB");

__global__ void __launch_bounds__(512, 1) lm_head_argmax_wide_kernel(LhParams p) {
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lh_smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, hh = lane >> 5;
    const int rest = blockIdx.x >> 3;
    const int group = rest % p.groups;
    const int tile = (rest / p.groups) * 8 + (blockIdx.x & 7);
    if (tile >= p.tiles) return;  // uniform over the workgroup
    const int v0 = tile * LH_VT;
    const int r0 = group * LHW_RT;
    const int nrows = min(LHW_RT, p.rows_total - r0);   // >= 1
    const int nchunks = (nrows + 31) >> 5;
    const int ksteps = p.D / LH_KC;
    const int steps = 2 * ksteps;

    // Loads: 1 KiB units of 4 rows x 256 B as in the narrow kernel.  Issuing wavefront iw (of four per kind) takes
    // units iw, iw + 4, ...: the row within the tile is 4 * unit + i / 16, so row & 15 = (4 * iw + i / 16) & 15.
    const bool w_issuer = wave < 4;
    const int iw = wave & 3;
    const int l_row = lane >> 4;
    const uint32_t lane_col = (uint32_t)(((lane & 15) ^ ((4 * iw + l_row) & 15)) * 16);
    const size_t row_bytes = (size_t)p.D * 2;
    // weights: 16 units per step, 4 per issuing wavefront; row-major sources differ between the two tile halves
    uint32_t wvoff[2][4];
    const uint8_t *wbase[2][4];
#pragma unroll
    for (int h = 0; h < 2; h++)
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int unit = iw + 4 * u;
            if (p.packed) {  // the tile's bytes in step order: step s at s * 16 KiB
                wbase[h][u] = p.weight + (size_t)tile * ksteps * LH_W_BYTES + (size_t)unit * 1024;
                wvoff[h][u] = (uint32_t)(l_row * LH_ROWB) + lane_col;
            } else {
                const int vrow = min(v0 + 64 * h + 4 * unit + l_row, p.V - 1);
                const int vfirst = min(v0 + 64 * h + 4 * unit, p.V - 1);
                wbase[h][u] = p.weight + (size_t)vfirst * row_bytes;
                wvoff[h][u] = (uint32_t)((size_t)(vrow - vfirst) * row_bytes) + lane_col;
            }
        }
    // hidden rows: 32 units per contraction step, 8 per issuing wavefront
    uint32_t hvoff[8];
    const uint8_t *hbase[8];
    bool h_on[8];
#pragma unroll
    for (int u = 0; u < 8; u++) {
        const int unit = iw + 4 * u;
        const int last = r0 + nrows - 1;
        const int rrow = min(r0 + 4 * unit + l_row, last);
        const int rfirst = min(r0 + 4 * unit, last);
        hbase[u] = p.hidden + (size_t)rfirst * row_bytes;
        hvoff[u] = (uint32_t)((size_t)(rrow - rfirst) * row_bytes) + lane_col;
        h_on[u] = 4 * unit < nrows;
    }
    auto issue_w = [&](int s) {
        const uint32_t dst = smem_addr + (uint32_t)(s % LHW_NSW) * LHW_W_STEP + (uint32_t)iw * 1024;
        const int h = s & 1;
        const size_t off = p.packed ? (size_t)s * LHW_W_STEP : (size_t)(s >> 1) * LH_ROWB;
        if (p.groups == 1) {   // one reader per weight byte: streamed
#pragma unroll
            for (int u = 0; u < 4; u++) lh_async_load16<true>(wbase[h][u] + off, wvoff[h][u], dst + u * 4096);
        } else {
#pragma unroll
            for (int u = 0; u < 4; u++) lh_async_load16<false>(wbase[h][u] + off, wvoff[h][u], dst + u * 4096);
        }
    };
    auto issue_h = [&](int k) {
        const uint32_t dst = smem_addr + LHW_W_RING + (uint32_t)(k % LHW_NSH) * LHW_H_STEP + (uint32_t)iw * 1024;
        const size_t off = (size_t)k * LH_ROWB;
#pragma unroll
        for (int u = 0; u < 8; u++)
            if (h_on[u]) lh_async_load16<false>(hbase[u] + off, hvoff[u], dst + u * 4096);
    };
    // prologue: fill both rings
    if (w_issuer) {
        for (int s = 0; s < LHW_NSW && s < steps; s++) issue_w(s);
    } else {
        issue_h(0);
        if (ksteps > 1) issue_h(1);
    }

    const int vb = wave & 1, cg = wave >> 1;
    const uint32_t a_row = (uint32_t)((32 * vb + c32) * LH_ROWB);
    const uint32_t b_row = (uint32_t)(LHW_W_RING + (32 * cg + c32) * LH_ROWB);
    const int sw = c32 & 15;
    const bool has = cg < nchunks;
    lh_f32x16 acc[2];  // one per tile half (the two wavefronts of a SIMD interleave their chains)
#pragma unroll
    for (int i = 0; i < 16; i++) { acc[0][i] = 0.f; acc[1][i] = 0.f; }

    // Fragments are read one step ahead of the products that use them, so a wavefront's LDS reads of step s + 1
    // run under its matrix instructions of step s.  A = the weight rows of the step, B = the hidden rows of the
    // contraction step, read once and used for both tile halves.
    auto read_a = [&](int s, lh_bf16x8 (&a)[8]) {
        const uint8_t *wst = lh_smem + (s % LHW_NSW) * LHW_W_STEP + a_row;
#pragma unroll
        for (int kk = 0; kk < 8; kk++) a[kk] = *reinterpret_cast<const lh_bf16x8 *>(wst + (((2 * kk + hh) ^ sw) << 4));
    };
    auto read_b = [&](int k, lh_bf16x8 (&bf)[8]) {
        const uint8_t *hst = lh_smem + (k % LHW_NSH) * LHW_H_STEP + b_row;
#pragma unroll
        for (int kk = 0; kk < 8; kk++) bf[kk] = *reinterpret_cast<const lh_bf16x8 *>(hst + (((2 * kk + hh) ^ sw) << 4));
    };
    auto products = [&](const lh_bf16x8 (&a)[8], const lh_bf16x8 (&bf)[8], lh_f32x16 &c) {
#pragma unroll
        for (int kk = 0; kk < 8; kk++) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[kk], bf[kk], c, 0, 0, 0);
    };
    // Before the barrier of ring step s: this wavefront's loads of step s + 1 have landed (weights: steps s + 2 ..
    // s + 4 may stay outstanding, four loads each; hidden rows: contraction step (s + 1) / 2 is needed from an odd
    // s on and nothing younger is outstanding then), and its own fragment reads of step s are done.  After the
    // barrier: step s + 1 is visible to everyone, the weight stage of step s is free (refilled with step s + 5),
    // and on odd s so is the hidden-row stage of contraction step s / 2 (refilled with s / 2 + 2).
    auto ring_step = [&](int s) {
        if (w_issuer) {
            const int ahead = min(3, steps - 2 - s);
            if (ahead >= 3) lh_wait_vmcnt<12>();
            else if (ahead == 2) lh_wait_vmcnt<8>();
            else if (ahead == 1) lh_wait_vmcnt<4>();
            else lh_wait_vmcnt<0>();
        } else if (s & 1) {
            lh_wait_vmcnt<0>();
        }
        __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the fragment reads of step s
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (w_issuer) {
            if (s + LHW_NSW < steps) issue_w(s + LHW_NSW);
        } else if ((s & 1) && (s >> 1) + 2 < ksteps) {
            issue_h((s >> 1) + 2);
        }
    };

    lh_bf16x8 a_even[8], a_odd[8], b_cur[8], b_next[8];
    // step 0 and contraction step 0 must be in LDS before the first fragment reads
    if (w_issuer) {
        const int ahead = min(LHW_NSW - 1, steps - 1);
        if (ahead >= 4) lh_wait_vmcnt<16>();
        else if (ahead == 3) lh_wait_vmcnt<12>();
        else if (ahead == 2) lh_wait_vmcnt<8>();
        else lh_wait_vmcnt<4>();
    } else {
        lh_wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    if (has) {
        read_a(0, a_even);
        read_b(0, b_cur);
    }
    for (int k = 0; k < ksteps; k++) {
        // even step 2k: half 0
        ring_step(2 * k);
        if (has) {
            read_a(2 * k + 1, a_odd);
            products(a_even, b_cur, acc[0]);
        }
        // odd step 2k + 1: half 1; the next contraction step's fragments are read here
        ring_step(2 * k + 1);
        if (has) {
            if (k + 1 < ksteps) {
                read_a(2 * k + 2, a_even);
                read_b(k + 1, b_next);
            }
            products(a_odd, b_cur, acc[1]);
            if (k + 1 < ksteps) {
#pragma unroll
                for (int kk = 0; kk < 8; kk++) b_cur[kk] = b_next[kk];
            }
        }
    }

    // Epilogue as in the narrow kernel: per node column the maximum over this wavefront's 2 x 32 vocabulary rows
    // (ascending: half 0 then half 1, element i of lane half hh is row 8 * (i / 4) + 4 * hh + i % 4), then over
    // the two lane halves, then over the two vocabulary blocks through LDS.  Lowest index wins among equals.
    __builtin_amdgcn_s_barrier();  // the rings are free
    float *s_val = reinterpret_cast<float *>(lh_smem);                    // [2 blocks][128 rows]
    int32_t *s_idx = reinterpret_cast<int32_t *>(lh_smem + 2 * LHW_RT * 4);
    if (has) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int h = 0; h < 2; h++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int v = v0 + 64 * h + 32 * vb + 8 * (i >> 2) + 4 * hh + (i & 3);
                const float x = (v < p.V) ? acc[h][i] : -INFINITY;
                if (x > bv || (bi == 0x7fffffff && v < p.V)) { bv = x; bi = v; }
            }
        const float ov = __shfl_xor(bv, 32);
        const int oi = __shfl_xor(bi, 32);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        if (hh == 0) {
            const int rl = 32 * cg + c32;
            s_val[vb * LHW_RT + rl] = bv;
            s_idx[vb * LHW_RT + rl] = bi;
        }
    }
    __syncthreads();
    if (tid < nrows) {
        float bv = s_val[tid];
        int bi = s_idx[tid];
        const float ov = s_val[LHW_RT + tid];
        const int oi = s_idx[LHW_RT + tid];
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        const size_t o = (size_t)(r0 + tid) * p.tiles + tile;
        p.pval[o] = bv;
        p.pidx[o] = bi;
    }
}

// ----------------------------------------------------------------------------------------------------------------
// More than 256 node rows (a batch of trees): the product is no longer a weight stream but a dense
// contraction bound by the matrix cores, and the tiling is a GEMM's.  A workgroup takes 256 vocabulary rows x 256
// node rows; wavefront w of 8 owns 128 vocabulary rows (w % 2) x 64 node rows (w / 2) as 4 x 2 accumulators of
// 32 x 32, so the eight products of a 16-wide contraction step need six fragments (1.3 LDS bytes per flop less
// than the kernels above, and eight independent accumulator chains).  The contraction runs in steps of 64
// elements: a step's weight rows (256 x 128 B) and hidden rows (256 x 128 B) are 64 KiB of LDS, two stages, filled
// by direct-to-LDS loads one step ahead, one barrier per step (32 products per wavefront).  A 128-byte tile row
// holds eight 16-byte chunks; chunk c of row r sits at position c ^ ((r >> 1) & 7), so the sixteen consecutive rows
// that a 16-byte fragment read serves in one cycle fall on sixteen different bank groups.  The weights reach a
// compute unit from L2 (the row groups of one vocabulary tile run side by side on one XCD), the hidden rows from
// L2 and the memory-side cache.  C^T[vocab, node] as above: a node is an accumulator column, so a wavefront's
// maximum over its 128 vocabulary rows needs one exchange between the lane halves and is exactly one per-tile
// partial of the layout the finishing kernel (and the epilogue) reads.
// ----------------------------------------------------------------------------------------------------------------
constexpr int LHG_VT = 256, LHG_RT = 256;    // vocabulary rows, node rows per workgroup
constexpr int LHG_KC = 64;                   // contraction elements per step
constexpr int LHG_ROWB = LHG_KC * 2;         // 128 B
constexpr int LHG_W_BYTES = LHG_VT * LHG_ROWB;            // 32 KiB
constexpr int LHG_STAGE = LHG_W_BYTES + LHG_RT * LHG_ROWB;  // 64 KiB
constexpr int LHG_NS = 2;
constexpr int LHG_MIN_ROWS = 257;   // measured: from 257 rows on this tiling beats the 128-row groups (288 rows: 129 vs 143 us)

__global__ void __launch_bounds__(512, 2) lm_head_argmax_gemm_kernel(LhParams p) {
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)lh_smem;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, hh = lane >> 5;
    const int tiles256 = (p.tiles + 1) >> 1;
    const int rest = blockIdx.x >> 3;
    const int group = rest % p.groups;
    const int tile = (rest / p.groups) * 8 + (blockIdx.x & 7);   // 256-row vocabulary tile
    if (tile >= tiles256) return;  // uniform over the workgroup
    const int v0 = tile * LHG_VT;
    const int r0 = group * LHG_RT;
    const int steps = p.D / LHG_KC;
    const int ksteps128 = p.D / LH_KC;  // steps of the packed layout

    // Loads.  A 1 KiB unit = 8 tile rows x 128 B; lane i fetches row i / 8 of the unit and the source chunk that
    // belongs at position i % 8, i.e. chunk (i % 8) ^ ((row >> 1) & 7).  Units 0..31 are weight rows, 32..63 hidden
    // rows; wavefront w issues units w, w + 8, w + 16, w + 24 of each: row = 8 * unit + i / 8, so
    // (row >> 1) & 7 = (4 * (w & 1) + i / 16) & 7 for all of them.
    const int l_row = lane >> 3;
    const uint32_t lane_chunk = (uint32_t)((lane & 7) ^ ((4 * (wave & 1) + (lane >> 4)) & 7));
    const size_t row_bytes = (size_t)p.D * 2;
    const uint8_t *wbase[4], *hbase[4];
    uint32_t wvoff[4], hvoff[4];
#pragma unroll
    for (int u = 0; u < 4; u++) {
        const int unit = wave + 8 * u;          // rows 8 * unit .. + 7 of the 256
        if (p.packed) {
            // packed tiles of 128 vocabulary rows x 128 elements (32 KiB); rows past V are zero there
            const int t128 = min(2 * tile + (unit >> 4), p.tiles - 1);
            wbase[u] = p.weight + (size_t)t128 * ksteps128 * LH_W_BYTES + (size_t)(8 * (unit & 15)) * LH_ROWB;
            wvoff[u] = (uint32_t)(l_row * LH_ROWB) + lane_chunk * 16;
        } else {
            const int vrow = min(v0 + 8 * unit + l_row, p.V - 1);
            const int vfirst = min(v0 + 8 * unit, p.V - 1);
            wbase[u] = p.weight + (size_t)vfirst * row_bytes;
            wvoff[u] = (uint32_t)((size_t)(vrow - vfirst) * row_bytes) + lane_chunk * 16;
        }
        const int last = p.rows_total - 1;
        const int rrow = min(r0 + 8 * unit + l_row, last);
        const int rfirst = min(r0 + 8 * unit, last);
        hbase[u] = p.hidden + (size_t)rfirst * row_bytes;
        hvoff[u] = (uint32_t)((size_t)(rrow - rfirst) * row_bytes) + lane_chunk * 16;
    }
    auto issue = [&](int st) {
        const uint32_t dst = smem_addr + (uint32_t)(st % LHG_NS) * LHG_STAGE + (uint32_t)wave * 1024;
        const size_t koff = (size_t)st * LHG_ROWB;   // row-major: the next 128 B of every row
        const size_t woff = p.packed ? (size_t)(st >> 1) * LH_W_BYTES + (size_t)(st & 1) * LHG_ROWB : koff;
#pragma unroll
        for (int u = 0; u < 4; u++) lh_async_load16<false>(wbase[u] + woff, wvoff[u], dst + u * 8192);
#pragma unroll
        for (int u = 0; u < 4; u++) lh_async_load16<false>(hbase[u] + koff, hvoff[u], dst + LHG_W_BYTES + u * 8192);
    };
    issue(0);

    // Fragments: A = weight rows of vocabulary block vb (4 per wavefront), B = hidden rows of row block rb (2);
    // the lane holds row c32 and the 8 contraction values at chunk 2 * kk + hh of the 64-element step.
    const int wv = wave & 1, wr = wave >> 1;
    const int sw = (c32 >> 1) & 7;   // (row >> 1) & 7: block bases are multiples of 32 rows
    const uint32_t a_row = (uint32_t)((128 * wv + c32) * LHG_ROWB);
    const uint32_t b_row = (uint32_t)(LHG_W_BYTES + (64 * wr + c32) * LHG_ROWB);
    lh_f32x16 acc[4][2];
#pragma unroll
    for (int vb = 0; vb < 4; vb++)
#pragma unroll
        for (int rb = 0; rb < 2; rb++)
#pragma unroll
            for (int i = 0; i < 16; i++) acc[vb][rb][i] = 0.f;

    for (int st = 0; st < steps; st++) {
        lh_wait_vmcnt<0>();              // this wavefront's part of step st has landed
        __builtin_amdgcn_s_barrier();    // step st is in LDS for everyone; the stage of step st - 1 is free
        asm volatile("" ::: "memory");
        if (st + 1 < steps) issue(st + 1);
        const uint8_t *stage = lh_smem + (st % LHG_NS) * LHG_STAGE;
#pragma unroll
        for (int kk = 0; kk < 4; kk++) {
            const int col = ((2 * kk + hh) ^ sw) << 4;
            lh_bf16x8 a[4], b[2];
#pragma unroll
            for (int vb = 0; vb < 4; vb++) a[vb] = *reinterpret_cast<const lh_bf16x8 *>(stage + a_row + vb * (32 * LHG_ROWB) + col);
#pragma unroll
            for (int rb = 0; rb < 2; rb++) b[rb] = *reinterpret_cast<const lh_bf16x8 *>(stage + b_row + rb * (32 * LHG_ROWB) + col);
#pragma unroll
            for (int vb = 0; vb < 4; vb++)
#pragma unroll
                for (int rb = 0; rb < 2; rb++)
                    acc[vb][rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[vb], b[rb], acc[vb][rb], 0, 0, 0);
        }
    }

    // Epilogue: per node column the maximum over the wavefront's 128 vocabulary rows, ascending (block vb, then
    // element i of lane half hh = row 8 * (i / 4) + 4 * hh + i % 4), then over the two lane halves: one per-tile
    // partial.  Lowest index wins among equals.
    const int t128 = 2 * tile + wv;
    if (t128 >= p.tiles) return;
#pragma unroll
    for (int rb = 0; rb < 2; rb++) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int vb = 0; vb < 4; vb++)
#pragma unroll
            for (int i = 0; i < 16; i++) {
                const int v = v0 + 128 * wv + 32 * vb + 8 * (i >> 2) + 4 * hh + (i & 3);
                const float x = (v < p.V) ? acc[vb][rb][i] : -INFINITY;
                if (x > bv || (bi == 0x7fffffff && v < p.V)) { bv = x; bi = v; }
            }
        const float ov = __shfl_xor(bv, 32);
        const int oi = __shfl_xor(bi, 32);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        const int row = r0 + 64 * wr + 32 * rb + c32;
        if (hh == 0 && row < p.rows_total) {
            const size_t o = (size_t)row * p.tiles + t128;
            p.pval[o] = bv;
            p.pidx[o] = bi;
        }
    }
}

// One wavefront per node row: reduce the per-tile partials (lowest index among equals); padded rows give -1.
__global__ void __launch_bounds__(256) lm_head_finish_kernel(const float *__restrict__ pval,
                                                            const int32_t *__restrict__ pidx, int tiles,
                                                            const int32_t *__restrict__ n_nodes, int rows_total,
                                                            int T_max, int32_t *__restrict__ argmax,
                                                            float *__restrict__ maxval) {
    const int r = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (r >= rows_total) return;
    const int b = r / T_max, k = r - b * T_max;
    if (k >= clampi(n_nodes[b], 0, T_max)) {
        if (lane == 0) {
            argmax[r] = -1;
            if (maxval) maxval[r] = -INFINITY;
        }
        return;
    }
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int t = lane; t < tiles; t += 64) {
        const float v = pval[(size_t)r * tiles + t];
        const int i = pidx[(size_t)r * tiles + t];
        if (v > bv || (v == bv && i < bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(bv, off);
        const int oi = __shfl_xor(bi, off);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    if (lane == 0) {
        argmax[r] = bi;
        if (maxval) maxval[r] = bv;
    }
}

// Packing: out[tile][step][r][c] = weight[tile * 128 + r][step * 128 + c], zeros for rows past V.
// One thread per 16-byte piece.
__global__ void __launch_bounds__(256) lm_head_pack_kernel(const uint4 *__restrict__ weight, uint4 *__restrict__ out,
                                                          int V, int D, long pieces) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= pieces) return;
    const int steps = D / LH_KC;
    const int c16 = (int)(i & 15);                 // 16-byte piece within the 256-byte tile row
    const int r = (int)((i >> 4) & (LH_VT - 1));   // row within the tile
    const long ts = i >> 11;                       // tile * steps + step
    const int st = (int)(ts % steps);
    const long v = (ts / steps) * LH_VT + r;
    uint4 x = {0, 0, 0, 0};
    if (v < V) x = weight[(v * D + (long)st * LH_KC) / 8 + c16];
    out[i] = x;
}

}  // namespace etv

extern "C" size_t etv_lm_head_packed_bytes(int32_t V, int32_t D) {
    if (V < 1 || D < 1 || D % etv::LH_KC != 0) return 0;
    return (((size_t)V + etv::LH_VT - 1) / etv::LH_VT) * etv::LH_VT * (size_t)D * 2;
}

extern "C" int32_t etv_pack_lm_head(const void *weight, int32_t V, int32_t D, void *packed, void *stream) {
    using namespace etv;
    if (!weight || !packed || V < 1 || D < 1) return ETV_ERR_INVALID_ARG;
    if (D % LH_KC != 0) return ETV_ERR_UNSUPPORTED;
    if ((((uintptr_t)weight) | ((uintptr_t)packed)) & 15) return ETV_ERR_INVALID_ARG;
    const long pieces = (long)(etv_lm_head_packed_bytes(V, D) / 16);
    const long blocks = (pieces + 255) / 256;
    if (blocks > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(lm_head_pack_kernel, dim3((unsigned)blocks), dim3(256), 0, as_stream(stream),
                       static_cast<const uint4 *>(weight), static_cast<uint4 *>(packed), (int)V, (int)D, pieces);
    return check_launch();
}

extern "C" size_t etv_lm_head_argmax_workspace_bytes(int32_t B, int32_t T_max, int32_t V) {
    if (B < 1 || T_max < 1 || V < 1) return 0;
    const size_t tiles = ((size_t)V + etv::LH_VT - 1) / etv::LH_VT;
    return (size_t)B * T_max * tiles * (sizeof(float) + sizeof(int32_t));
}

extern "C" int32_t etv_lm_head_argmax(const void *hidden, const void *weight, int32_t weight_packed,
                                      const int32_t *n_nodes, int32_t B, int32_t T_max, int32_t D, int32_t V,
                                      int32_t *argmax, float *maxval, void *workspace, size_t workspace_bytes,
                                      void *stream) {
    using namespace etv;
    if (!hidden || !weight || !n_nodes || B < 0 || T_max < 1 || D < 1 || V < 1) return ETV_ERR_INVALID_ARG;
    if (D % LH_KC != 0) return ETV_ERR_UNSUPPORTED;
    if ((((uintptr_t)hidden) | ((uintptr_t)weight)) & 15) return ETV_ERR_INVALID_ARG;
    if ((size_t)D * 2 * 8 >= (1ull << 32)) return ETV_ERR_UNSUPPORTED;
    if (B == 0) return ETV_OK;
    const long rows_total = (long)B * T_max;
    const bool wide = rows_total > LH_RT;   // more than 64 rows: 128 per workgroup
    // from a few hundred rows on the product is bound by the matrix cores: GEMM tiling, 256 x 256 per workgroup
    const bool gemm = rows_total >= LHG_MIN_ROWS;
    const long rt = gemm ? LHG_RT : (wide ? LHW_RT : LH_RT);
    const long groups = (rows_total + rt - 1) / rt;
    const long tiles = ((long)V + LH_VT - 1) / LH_VT;
    if (groups > 65535 || rows_total > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < etv_lm_head_argmax_workspace_bytes(B, T_max, V))
        return ETV_ERR_WORKSPACE_TOO_SMALL;
    LhParams p{};
    p.hidden = static_cast<const uint8_t *>(hidden);
    p.weight = static_cast<const uint8_t *>(weight);
    p.n_nodes = n_nodes;
    p.pval = static_cast<float *>(workspace);
    p.pidx = reinterpret_cast<int32_t *>(p.pval + (size_t)rows_total * tiles);
    p.rows_total = (int)rows_total; p.T_max = T_max; p.D = D; p.V = V; p.tiles = (int)tiles; p.groups = (int)groups;
    p.packed = weight_packed ? 1 : 0;
    constexpr size_t lds = (size_t)LH_NS * LH_STAGE;
    constexpr size_t lds_gemm = (size_t)LHG_NS * LHG_STAGE;
    static const bool lds_ok = [] {
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_argmax_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_argmax_wide_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess &&
               hipFuncSetAttribute(reinterpret_cast<const void *>(&lm_head_argmax_gemm_kernel),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_gemm) == hipSuccess;
    }();
    if (!lds_ok) return ETV_ERR_HIP;
    hipStream_t s = as_stream(stream);
    const long vtiles = gemm ? (tiles + 1) / 2 : tiles;   // vocabulary tiles of the launch: 256 or 128 rows
    const long nblocks = ((vtiles + 7) / 8) * groups * 8;
    if (nblocks > 0x7fffffffL) return ETV_ERR_UNSUPPORTED;
    if (gemm) hipLaunchKernelGGL(lm_head_argmax_gemm_kernel, dim3((unsigned)nblocks), dim3(512), lds_gemm, s, p);
    else if (wide) hipLaunchKernelGGL(lm_head_argmax_wide_kernel, dim3((unsigned)nblocks), dim3(512), lds, s, p);
    else hipLaunchKernelGGL(lm_head_argmax_kernel, dim3((unsigned)nblocks), dim3(512), lds, s, p);
    int32_t rc = check_launch();
    if (rc != ETV_OK || !argmax) return rc;  // without argmax the per-tile maxima stay in the workspace for the epilogue
    hipLaunchKernelGGL(lm_head_finish_kernel, dim3((unsigned)((rows_total + 3) / 4)), dim3(256), 0, s, p.pval, p.pidx,
                       (int)tiles, n_nodes, (int)rows_total, (int)T_max, argmax, maxval);
    return check_launch();
}
