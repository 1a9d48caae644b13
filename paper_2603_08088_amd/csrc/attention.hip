// tree_verify_attention: tree-masked attention of the draft-tree query rows against the committed
// prefix cache plus the tree's own K/V (Section 3.3, "Execution view" and "Tree attention mask").
//
// Two kernels compute the per-split partial (m, l, O):
//   * attn_mfma_kernel   bf16, d = 128: K/V tiles staged through LDS, QK^T and PV on
//                        v_mfma_f32_32x32x16_bf16, online softmax in registers, the ancestor mask applied
//                        as a per-row bitmask only on the tree tile.
//   * attn_generic_kernel  any supported dtype / head dim, fp32 VALU arithmetic, one wavefront per query
//                        row.  It is the fp32 path (bit-for-bit fp32 inputs need fp32 products).
// and attn_combine_kernel merges the splits by log-sum-exp.  With a single split the partial kernels write
// the final output themselves.
//
// Scores are kept in "scaled log2 units" t = (q.k) * scale * log2(e) so that exp is a bare v_exp_f32.
#include "etv_common.h"
#include <atomic>

namespace etv {

struct AttnParams {
    const void *q, *k_cache, *v_cache, *kt, *vt;
    const int32_t *block_table, *prefix_len, *n_nodes;
    const uint64_t *bitmask;
    void *out;
    float *lse;
    float *part_o, *part_m, *part_l;
    int B, T_max, Hq, Hkv, G, d, block_size, max_blocks, P_cap, P_max, words;
    int chunk;   // prefix keys per split, multiple of 64
    int nsplit;  // splits the launch provides; sequence b uses max(1, ceil(P_b / chunk)) of them
    // partial results, split-major so that one workgroup writes one contiguous region:
    //   part_o [B][nsplit][Hq][T_max][d], part_m / part_l [B][nsplit][Hq][T_max]
    int pairs;   // mfma kernel: 32-row chunks of the packed query rows of a KV head
    int wgp;     // mfma kernel: workgroups per (b, kv head, split) = ceil(pairs / 4)
    float scale_log2;
    // mfma kernel, batches of 2 .. 64 sequences with splits: the B * nsplit split slots are shared out among the
    // sequences by their lengths (on the device, where the lengths are), slot-major partials
    //   part_o [B * nsplit][Hq][T_max][d]; split_tab[b] = (first slot, splits in use) for the combine kernel
    int balanced;
    int2 *split_tab;
};

constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int seq_prefix_len(const AttnParams &p, int b) { return clampi(p.prefix_len[b], 0, p.P_max); }
__device__ __forceinline__ int seq_nsplit(const AttnParams &p, int P) { return max(1, (P + p.chunk - 1) / p.chunk); }
// partial row of split slot `slot` (= b * nsplit + s where every sequence owns nsplit slots)
__device__ __forceinline__ size_t part_row(const AttnParams &p, int slot, int h, int k) {
    return ((size_t)slot * p.Hq + h) * p.T_max + k;
}

// element offset of prefix row `key` of KV head kvh (contiguous or paged cache)
__device__ __forceinline__ size_t prefix_row_offset(const AttnParams &p, int b, int kvh, int key) {
    if (p.block_size > 0) {
        int blk = p.block_table[(size_t)b * p.max_blocks + key / p.block_size];
        return (((size_t)blk * p.Hkv + kvh) * p.block_size + (key % p.block_size)) * (size_t)p.d;
    }
    return (((size_t)b * p.P_cap + key) * p.Hkv + kvh) * (size_t)p.d;
}
__device__ __forceinline__ size_t tree_row_offset(const AttnParams &p, int b, int kvh, int j) {
    return (((size_t)b * p.T_max + j) * p.Hkv + kvh) * (size_t)p.d;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
    return v;
}
__device__ __forceinline__ int wave_max_i(int v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = max(v, __shfl_xor(v, off));
    return v;
}

// Balanced splits.  With one split size for the whole batch a ragged batch leaves the split slots of its short
// sequences empty while the workgroups of its longest sequence decide the launch time.  Here the launch's
// S = B * nsplit slots are shared out by length: L = the smallest tile count with sum_b max(1, ceil(tiles_b / L))
// <= S (tiles_b: 64-key tiles of the prefix and of the tree), sequence b gets ceil(tiles_b / L) consecutive slots
// and cuts its prefix evenly over them; its last split in use also takes the tree.  Every wavefront works this
// out for itself, lane i holding sequence i (B <= 64): integer arithmetic only, so all of them agree.
struct SplitShare {
    int b, j, nvalid, start, tps, P_raw, n_raw;  // sequence, split within it, splits in use, first slot, tiles per split
    bool live;
};
__device__ __forceinline__ int uni(int v) { return __builtin_amdgcn_readfirstlane(v); }
__device__ inline SplitShare balanced_share(const AttnParams &p, int x, int lane) {
    const bool has = lane < p.B;
    const int P_raw = has ? p.prefix_len[lane] : 0, n_raw = has ? p.n_nodes[lane] : 0;
    const int P = clampi(P_raw, 0, p.P_max), n = clampi(n_raw, 0, p.T_max);
    const int pt = (P + 63) >> 6;
    const int tt = pt + ((n + 63) >> 6);
    const int S = p.B * p.nsplit;
    const int total = uni(wave_sum_i(tt));
    int hi = max(1, uni(wave_max_i(tt)));                                   // one slot per sequence always fits
    if (S > p.B) hi = min(hi, max(1, (total + (S - p.B) - 1) / (S - p.B)));  // sum (tiles_b / L + 1) <= S
    int lo = min(hi, max(1, (total + S - 1) / S));
    while (lo < hi) {  // sum_b max(1, ceil(tiles_b / L)) falls as L grows
        const int mid = (lo + hi) >> 1;
        const int cnt = uni(wave_sum_i(has ? max(1, (tt + mid - 1) / mid) : 0));
        if (cnt <= S) hi = mid;
        else lo = mid + 1;
    }
    const int ns = has ? max(1, (tt + lo - 1) / lo) : 0;  // slots of the lane's sequence
    const int tps = max(1, (tt + max(ns, 1) - 1) / max(ns, 1));
    const int nv = max(1, (pt + tps - 1) / tps);          // of them in use: those that hold prefix keys
    int incl = ns;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    const int start = incl - ns;  // strictly increasing over the sequences
    const int owner = uni(__popcll(__ballot(has && start <= x)) - 1);
    SplitShare r;
    r.b = owner;
    r.start = uni(__shfl(start, owner));
    r.j = x - r.start;
    r.nvalid = uni(__shfl(nv, owner));
    r.tps = uni(__shfl(tps, owner));
    r.P_raw = uni(__shfl(P_raw, owner));
    r.n_raw = uni(__shfl(n_raw, owner));
    r.live = owner >= 0 && r.j < r.nvalid;
    return r;
}

template <typename T>
__device__ __forceinline__ float load_elem(const T *p, size_t i);
template <>
__device__ __forceinline__ float load_elem<float>(const float *p, size_t i) { return p[i]; }
template <>
__device__ __forceinline__ float load_elem<uint16_t>(const uint16_t *p, size_t i) { return bf16_bits_to_float(p[i]); }

template <typename T>
__device__ __forceinline__ void store_elem(T *p, size_t i, float v);
template <>
__device__ __forceinline__ void store_elem<float>(float *p, size_t i, float v) { p[i] = v; }
template <>
__device__ __forceinline__ void store_elem<uint16_t>(uint16_t *p, size_t i, float v) { p[i] = float_to_bf16_bits(v); }

template <typename T, int D>
__device__ __forceinline__ float dot_row(const float *sq, const T *row) {
    float acc = 0.f;
    if constexpr (sizeof(T) == 4) {
        const float4 *r4 = reinterpret_cast<const float4 *>(row);
#pragma unroll 4
        for (int c = 0; c < D / 4; c++) {
            float4 x = r4[c];
            acc = fmaf(sq[4 * c], x.x, acc);
            acc = fmaf(sq[4 * c + 1], x.y, acc);
            acc = fmaf(sq[4 * c + 2], x.z, acc);
            acc = fmaf(sq[4 * c + 3], x.w, acc);
        }
    } else {
        const uint4 *r8 = reinterpret_cast<const uint4 *>(row);
#pragma unroll 4
        for (int c = 0; c < D / 8; c++) {
            uint4 x = r8[c];
            uint32_t w[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 4; e++) {
                acc = fmaf(sq[8 * c + 2 * e], __uint_as_float(w[e] << 16), acc);
                acc = fmaf(sq[8 * c + 2 * e + 1], __uint_as_float(w[e] & 0xffff0000u), acc);
            }
        }
    }
    return acc;
}

// ----------------------------------------------------------------------------------------------
// Generic kernel: grid (T_max, Hq, B * nsplit), one wavefront per (query row, head, split).
// QK: lane = key (row dot product against q held in LDS); PV: lane = head-dim column, the weight of
// key j broadcast by a lane read.
// ----------------------------------------------------------------------------------------------
template <typename T, int D>
__global__ void __launch_bounds__(64) attn_generic_kernel(AttnParams p) {
    constexpr int DPL = D / 64;
    const int k = blockIdx.x, h = blockIdx.y;
    const int b = blockIdx.z / p.nsplit, s = blockIdx.z % p.nsplit;
    const int lane = threadIdx.x;
    const int n = clampi(p.n_nodes[b], 0, p.T_max);
    const int P = seq_prefix_len(p, b);
    const int nvalid = seq_nsplit(p, P);
    if (s >= nvalid) return;
    const bool direct = (p.nsplit == 1);
    T *out = static_cast<T *>(p.out);
    const size_t orow = (((size_t)b * p.T_max + k) * p.Hq + h) * D;
    if (k >= n) {
        if (direct) {
#pragma unroll
            for (int i = 0; i < DPL; i++) store_elem<T>(out, orow + lane + 64 * i, 0.f);
            if (p.lse && lane == 0) p.lse[((size_t)b * p.Hq + h) * p.T_max + k] = -INFINITY;
        }
        return;
    }
    __shared__ float sq[D];
    const T *q = static_cast<const T *>(p.q);
#pragma unroll
    for (int i = 0; i < DPL; i++) sq[lane + 64 * i] = load_elem<T>(q, orow + lane + 64 * i);
    __syncthreads();
    const int kvh = h / p.G;
    const T *kc = static_cast<const T *>(p.k_cache), *vc = static_cast<const T *>(p.v_cache);
    const T *kt = static_cast<const T *>(p.kt), *vt = static_cast<const T *>(p.vt);
    float m = -INFINITY, l = 0.f;
    float o[DPL];
#pragma unroll
    for (int i = 0; i < DPL; i++) o[i] = 0.f;

    auto tile = [&](float sc, bool valid, int count, auto v_row_of) {
        float tmax = wave_max(valid ? sc : -INFINITY);
        float m_new = fmaxf(m, tmax);
        if (m_new == -INFINITY) return;  // nothing visible yet
        float alpha = exp2f(m - m_new);
        float pv = valid ? exp2f(sc - m_new) : 0.f;
        l = l * alpha + wave_sum(pv);
#pragma unroll
        for (int i = 0; i < DPL; i++) o[i] *= alpha;
        m = m_new;
        for (int j = 0; j < count; j++) {
            float pj = __shfl(pv, j);
            if (pj == 0.f) continue;  // wave-uniform
            const T *vr = v_row_of(j);
#pragma unroll
            for (int i = 0; i < DPL; i++) o[i] = fmaf(pj, load_elem<T>(vr, lane + 64 * i), o[i]);
        }
    };

    const int k0 = s * p.chunk, k1 = min(P, k0 + p.chunk);
    for (int t0 = k0; t0 < k1; t0 += 64) {
        const int key = t0 + lane;
        const bool valid = key < k1;
        float sc = 0.f;
        if (valid) sc = dot_row<T, D>(sq, kc + prefix_row_offset(p, b, kvh, key)) * p.scale_log2;
        tile(sc, valid, min(64, k1 - t0), [&](int j) { return vc + prefix_row_offset(p, b, kvh, t0 + j); });
    }
    if (s == nvalid - 1) {
        const uint64_t *mrow = p.bitmask + ((size_t)b * p.T_max + k) * p.words;
        for (int t0 = 0; t0 < n; t0 += 64) {
            const int j = t0 + lane;
            const bool valid = (j < n) && ((mrow[t0 >> 6] >> lane) & 1ull);
            float sc = 0.f;
            // tree rows: the step's own buffer, or (kt null) the cache tail, node j at position P + j
            if (valid)
                sc = (kt ? dot_row<T, D>(sq, kt + tree_row_offset(p, b, kvh, j))
                         : dot_row<T, D>(sq, kc + prefix_row_offset(p, b, kvh, P + j))) * p.scale_log2;
            tile(sc, valid, min(64, n - t0), [&](int jj) {
                return kt ? vt + tree_row_offset(p, b, kvh, t0 + jj) : vc + prefix_row_offset(p, b, kvh, P + t0 + jj);
            });
        }
    }
    if (direct) {
        const float inv = 1.f / l;
#pragma unroll
        for (int i = 0; i < DPL; i++) store_elem<T>(out, orow + lane + 64 * i, o[i] * inv);
        if (p.lse && lane == 0) p.lse[((size_t)b * p.Hq + h) * p.T_max + k] = (m + log2f(l)) * kLn2;
    } else {
        const size_t pr = part_row(p, b * p.nsplit + s, h, k);
#pragma unroll
        for (int i = 0; i < DPL; i++) p.part_o[pr * D + lane + 64 * i] = o[i];
        if (lane == 0) {
            p.part_m[pr] = m;
            p.part_l[pr] = l;
        }
    }
}

// ----------------------------------------------------------------------------------------------
// Combine: grid (T_max, Hq, B), D threads.  out = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
// ----------------------------------------------------------------------------------------------
// WPR wavefronts per query row (b, k, h), 4 / WPR rows per workgroup; a lane owns D / (64 * WPR) consecutive output
// elements (two wavefronts per row for small launches, where the latency of a row's chain is what counts).  Two
// trips to memory: the sequence's sizes, then the row's first U splits (only splits that exist are read; all loads of
// a batch are in flight together).  Further batches of U splits, for launches with more splits than that, update a
// running (M, L, acc) that is rescaled when a later batch raises the maximum.
template <typename T, int D, int WPR, int U>
__global__ void __launch_bounds__(256) attn_combine_kernel(AttnParams p) {
    constexpr int E = D / (64 * WPR);
    static_assert(E >= 1, "at least one element per lane");
    const int wv = threadIdx.x >> 6;
    const long row = (long)blockIdx.x * (4 / WPR) + wv / WPR;
    const int lane = (wv % WPR) * 64 + (threadIdx.x & 63);  // position within the row, in units of E elements
    const long rows_total = (long)p.B * p.T_max * p.Hq;
    if (row >= rows_total) return;
    const int h = (int)(row % p.Hq);
    const long bk = row / p.Hq;
    const int k = (int)(bk % p.T_max), b = (int)(bk / p.T_max);
    const int n_raw = p.n_nodes[b], P_raw = p.prefix_len[b];  // all before any is used: one trip
    int2 share = {0, 0};
    if (p.balanced) share = p.split_tab[b];
    T *out = static_cast<T *>(p.out);
    const size_t orow = (((size_t)b * p.T_max + k) * p.Hq + h) * D + (size_t)lane * E;
    const size_t lrow = ((size_t)b * p.Hq + h) * p.T_max + k;
    const int nvalid = p.balanced ? share.y : seq_nsplit(p, clampi(P_raw, 0, p.P_max));
    if (k >= clampi(n_raw, 0, p.T_max)) {
#pragma unroll
        for (int e = 0; e < E; e++) store_elem<T>(out, orow + e, 0.f);
        if (p.lse && lane == 0) p.lse[lrow] = -INFINITY;
        return;
    }
    const size_t pr0 = part_row(p, p.balanced ? share.x : b * p.nsplit, h, k);
    const size_t sstride = (size_t)p.Hq * p.T_max;  // rows between consecutive splits
    float M = -INFINITY, L = 0.f, acc[E];
#pragma unroll
    for (int e = 0; e < E; e++) acc[e] = 0.f;
    for (int s0 = 0; s0 < nvalid; s0 += U) {
        float ms[U], ls[U], os[U][E];
#pragma unroll
        for (int u = 0; u < U; u++) {
            const bool ok = s0 + u < nvalid;
            const size_t r = pr0 + (size_t)(ok ? s0 + u : 0) * sstride;
            ms[u] = ok ? p.part_m[r] : -INFINITY;
            ls[u] = ok ? p.part_l[r] : 0.f;
#pragma unroll
            for (int e = 0; e < E; e++) os[u][e] = ok ? p.part_o[r * D + (size_t)lane * E + e] : 0.f;
        }
        float Mb = M;
#pragma unroll
        for (int u = 0; u < U; u++) Mb = fmaxf(Mb, ms[u]);
        if (Mb == -INFINITY) continue;  // nothing visible in this batch or before
        const float keep = exp2f(M - Mb);  // 0 while M is still -inf
        L *= keep;
#pragma unroll
        for (int e = 0; e < E; e++) acc[e] *= keep;
        M = Mb;
#pragma unroll
        for (int u = 0; u < U; u++) {
            if (ms[u] != -INFINITY) {  // absent or empty split: its l/O may be uninitialised memory
                const float w = exp2f(ms[u] - M);
                L = fmaf(w, ls[u], L);
#pragma unroll
                for (int e = 0; e < E; e++) acc[e] = fmaf(w, os[u][e], acc[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < E; e++) store_elem<T>(out, orow + e, acc[e] / L);
    if (p.lse && lane == 0) p.lse[lrow] = (M + log2f(L)) * kLn2;
}

// ----------------------------------------------------------------------------------------------
// MFMA kernel (bf16, d = 128).
//
// Work unit: (split, KV head x row group, sequence).  A workgroup has NW wavefronts (8, or 4 for small
// trees); wavefront w owns one 32-row chunk of the KV head's packed query rows and all of them share the K/V tiles of
// their KV head through LDS, so each prefix K/V byte is fetched from HBM once per G*T query rows.  Two
// wavefronts are resident per SIMD: while one runs the softmax on the vector ALU the other feeds the
// matrix cores.
//
// K/V tiles (64 keys x 256 B each) travel HBM -> LDS with asynchronous direct-to-LDS loads
// (global_load_lds_dwordx4: no registers, completion tracked by vmcnt) into a ring of NS stages, so
// NS-1 tiles (32 KiB each) are in flight per workgroup while one is being consumed; one workgroup
// barrier per tile.  A direct-to-LDS load writes lane i's 16 bytes at (base + 16 i), so rows cannot be
// padded; instead the 16-byte chunk c of key row r is stored at chunk position c ^ (r & 15) in the K tile
// and c ^ (((r & 3) << 1) | ((r >> 2) & 1)) in the V tile, which spreads the 16-byte K reads (consecutive rows,
// same chunk) and the 8-byte transpose reads of V (4 consecutive rows x 32 B) over the LDS banks.
//
// The two wavefronts of a SIMD (w and w+4) run one phase apart: wavefronts 0..3 do QK(t), softmax(t),
// PV(t) inside ring step t, wavefronts 4..7 do PV(t-1), QK(t), softmax(t).  The tile barrier would otherwise
// keep them in lockstep, both wanting the matrix core, then both the vector ALU; shifted, one wavefront's
// softmax overlaps the other's products.  A V tile therefore lives one ring step longer than a K tile, and
// the ring refills the stage of tile t-2 (two tiles in flight) rather than that of tile t-1.
//
// Per 64-key tile and wavefront (32x32x16 MFMA, 64-lane layouts: A/B operand lane = (row|col l%32,
// 8 contraction values at 8*(l/32)); accumulator lane = (col l%32, rows 8*(i/4) + 4*(l/32) + i%4)):
//   S^T[key, q] = K[key, :] . Q[q, :]      A = K rows from LDS (16-byte reads), B = Q held in registers
//   online softmax down each accumulator column (a query row lives in lanes l and l^32)
//   O^T[d, q]  += V^T[d, key] P^T[key, q]  A = V^T via the LDS transpose read (ds_read_b64_tr_b16),
//                                          B = P^T taken straight from the S^T accumulator registers
// Both products keep the query index on the accumulator column, so the softmax statistics and the
// rescale of O never cross lanes.
// ----------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(4))) const int32_t *const_i32_ptr;

constexpr int KT = 64;                      // keys per tile
constexpr int ROW_BYTES = 256;              // one K or V row of a KV head (d = 128, bf16)
constexpr int TILE_BYTES = KT * ROW_BYTES;  // 16 KiB
constexpr int STAGE_BYTES = 2 * TILE_BYTES; // K tile then V tile

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

// acc + the two bf16 values of a packed pair, in fp32: one instruction for two probabilities.  The row sum is
// taken over the probabilities as rounded to bf16, i.e. over exactly the weights the PV product uses.
__device__ __forceinline__ float pair_sum(uint32_t packed, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, packed), __builtin_bit_cast(bf16x2, 0x3f803f80u),
                                           acc, false);
}

// 16 bytes per lane from global memory straight into LDS at (lds_addr + 16 * lane); asynchronous.
__device__ __forceinline__ void async_load16(const void *gptr, uint32_t lds_addr) {
    // lds_addr is the same in every lane; readfirstlane says so to the compiler whatever it concluded about the loop
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off\n" ::"v"(gptr),
                 "s"(__builtin_amdgcn_readfirstlane(lds_addr)) : "memory");
}
// wait until at most N of this wavefront's vector-memory loads are outstanding (N < 64)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | (0x7 << 4) | (0xF << 8));
}
// max / sum of a value with its partner in the other half of the wavefront (lane ^ 32) without touching
// LDS: v_permlane32_swap exchanges the upper 32 lanes of one register with the lower 32 of another.  (A
// ds_bpermute shuffle here would make the wavefront wait for its pending V-fragment LDS reads as well.)
__device__ __forceinline__ float half_swap_max(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
// three-input max as one instruction.  (fmaxf would first canonicalise each MFMA result with an extra v_max,
// doubling the instruction count of the row-max reduction; scores are never NaN here.)
__device__ __forceinline__ float max3(float a, float b, float c) {
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ float half_swap_sum(float v) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// chunk-position swizzles (measured on gfx950: 16-byte reads reach the full 256 B/clk only with a 4-bit
// row term; the 8-byte transpose reads are fastest with the 3-bit term below)
__device__ __forceinline__ int kswz_of_row(int r) { return r & 15; }
__device__ __forceinline__ int vswz_of_row(int r) { return ((r & 3) << 1) | ((r >> 2) & 1); }

extern __shared__ __attribute__((aligned(1024))) uint8_t attn_smem[];

// Asynchronous loads of one 64-key K/V tile into ring stage (ti % NS).  A tile is 16 chunk pairs of
// 1 KiB (4 key rows of K, the same 4 rows of V).  Issuing wavefront w takes pairs w, w+4, w+8, w+12; in a chunk
// lane i fetches key row 4j + i/16 and the 16-byte piece that belongs at chunk position i%16 of that row.
// Pair w + 4u holds rows 16u + 4w .. +3: the lane's place within those 16 rows (and with it both swizzles)
// does not depend on u, so a load is a scalar base per u plus one per-lane 32-bit offset, and the address
// arithmetic of a tile is scalar (a wavefront's instruction issue rate is what bounds a tile step).
template <int NW>
struct TileLoader {
    // wavefronts that issue loads: all 4 of a small workgroup; of 8, only wavefronts 0..3, which otherwise
    // idle at the tile barrier while wavefronts 4..7 (one phase behind) finish their longer chain
    static constexpr int NI = 4;
    static constexpr int U = 16 / NI;  // chunk pairs per issuing wavefront and tile
    const uint8_t *kc, *vc, *kt, *vt;
    const uint8_t *kf, *vf;  // full tiles: kc / vc advanced by head_off (paged) or seq_off (contiguous)
    const int32_t *bt;
    size_t row_stride, seq_off, blk_stride, head_off;  // strides are below 2^32
    uint32_t smem_addr;
    int wave, l_row, l_pos, k0, k1, npt, n;
    int P;      // prefix length of the sequence
    bool tail;  // the tree rows live in the cache itself, node j at position P + j (no separate tree buffer)
    uint32_t kcol, vcol;  // per-lane source column (bytes) for the K tile / the V tile swizzle
    uint32_t koff, voff;  // per-lane byte offset from the scalar base of a chunk pair (full tiles)
};

// 16 bytes per lane from (uniform base + per-lane 32-bit offset) into LDS at (lds_addr + 16 * lane)
// NT: streaming (nontemporal) load.  Plain loads sustain 6.0-6.4 TB/s on this machine, streaming ones 7.1 TB/s, but
// a streamed line does not stay in L2 for another workgroup: used only when one workgroup reads each K/V byte.
template <bool NT>
__device__ __forceinline__ void async_load16_s(const void *sbase, uint32_t voff, uint32_t lds_addr) {
    if (NT)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}

// full prefix tile (all 64 keys exist): straight-line address arithmetic.  For a paged cache the physical
// block ids are fetched with scalar loads by fetch_blocks() ahead of the wait and barrier of the ring step,
// so their latency is hidden; the block table is read-only for the kernel (constant address space).
template <int NW>
__device__ __forceinline__ void fetch_blocks(const TileLoader<NW> &ld, int ti, int (&blk)[TileLoader<NW>::U]) {
    const int lb0 = (ld.k0 + ti * KT) >> 4;
#pragma unroll
    for (int u = 0; u < TileLoader<NW>::U; u++)
        blk[u] = ((const_i32_ptr)(uintptr_t)ld.bt)[lb0 + ((ld.wave + TileLoader<NW>::NI * u) >> 2)];
}

template <int NW, int NS, bool PAGED, bool NT>
__device__ __forceinline__ void issue_full_tile(const TileLoader<NW> &ld, int ti, const int (&blk)[TileLoader<NW>::U]) {
    constexpr int U = TileLoader<NW>::U, NI = TileLoader<NW>::NI;
    static_assert(NI == 4 && U == 4, "pair w + 4u lies in 16-key block u of the tile");
    const uint32_t dst = ld.smem_addr + (uint32_t)(ti % NS) * STAGE_BYTES + (uint32_t)ld.wave * 1024;
#pragma unroll
    for (int u = 0; u < U; u++) {
        // kf / vf: the cache pointers advanced to this KV head's part of block 0 (paged) or of row 0 of the sequence
        const size_t off = PAGED ? (size_t)(uint32_t)blk[u] * (size_t)(uint32_t)ld.blk_stride
                                 : (size_t)(uint32_t)(ld.k0 + ti * KT + 16 * u) * (size_t)(uint32_t)ld.row_stride;
        async_load16_s<NT>(ld.kf + off, ld.koff, dst + u * (NI * 1024));
        async_load16_s<NT>(ld.vf + off, ld.voff, dst + TILE_BYTES + u * (NI * 1024));
    }
}

// ragged last prefix tile or tree tile: rows past the end re-read the last valid row (masked later)
template <int NW, int NS>
__device__ __forceinline__ void issue_edge_tile(const TileLoader<NW> &ld, int ti) {
    constexpr int U = TileLoader<NW>::U, NI = TileLoader<NW>::NI;
    const bool tree = ti >= ld.npt;
    const int base = tree ? (ti - ld.npt) * KT : ld.k0 + ti * KT;
    const int last = (tree ? ld.n : ld.k1) - 1;
    const uint32_t stage = ld.smem_addr + (uint32_t)(ti % NS) * STAGE_BYTES;
    const bool own = tree && !ld.tail;  // rows of the step's own tree buffer
    const uint8_t *ksrc = own ? ld.kt : ld.kc;
    const uint8_t *vsrc = own ? ld.vt : ld.vc;
#pragma unroll
    for (int u = 0; u < U; u++) {
        const int j = ld.wave + NI * u;
        const int r_in = 4 * j + ld.l_row;
        const int key = min(base + r_in, last);
        size_t off;
        if (own) {
            off = (size_t)key * ld.row_stride;
        } else if (tree) {
            // in-place branch cache: node `key` sits at cache position P + key.  P is arbitrary, so the four rows
            // of a chunk may lie in two blocks: the block id is looked up per lane.
            const int pos = ld.P + key;
            if (ld.bt) off = (size_t)ld.bt[pos >> 4] * ld.blk_stride + ld.head_off + (size_t)(pos & 15) * ROW_BYTES;
            else off = ld.seq_off + (size_t)pos * ld.row_stride;
        } else if (ld.bt) {
            // the logical block is the same for the whole chunk (its rows are clamped into one block)
            const int lb = __builtin_amdgcn_readfirstlane(min(base + 4 * j, last) >> 4);
            const int blk = ((const_i32_ptr)(uintptr_t)ld.bt)[lb];
            off = (size_t)blk * ld.blk_stride + ld.head_off + (size_t)(key & 15) * ROW_BYTES;
        } else {
            off = ld.seq_off + (size_t)key * ld.row_stride;
        }
        async_load16(ksrc + off + ld.kcol, stage + j * 1024);
        async_load16(vsrc + off + ld.vcol, stage + TILE_BYTES + j * 1024);
    }
}

// LDS view of one staged tile plus the per-lane fragment offsets (bytes) that do not depend on the tile.
struct TileView {
    int krow;          // K fragment row offset: row (lane%32) of key block 0; block 1 is 32 rows further
    int ksw;           // swizzle term of that row (the same for row + 32)
    int vrow, vsw, vchunk, vsub;  // V transpose-read row within a 16-key step, its swizzle, chunk, sub-offset
    int hh;            // lane / 32
};

// How far the running reference of a row may lag behind its true maximum (log2 units) before the
// accumulators are rescaled: exp2 arguments stay <= kLazy, so P <= 256 and nothing overflows, and the
// rescale of the O registers (which live in accumulator registers and cost three instructions each to
// touch) becomes rare after the first tiles.
constexpr float kLazy = 8.0f;

// V^T fragments of 32 keys (key block kb) of the V tile at lv.
__device__ __forceinline__ void load_v_frags(const TileView &tv, const uint8_t *lv, int kb, bf16x8 (&vf)[2][4]) {
#pragma unroll
    for (int st = 0; st < 2; st++) {
        const uint8_t *vr = lv + (32 * kb + 16 * st + tv.vrow) * ROW_BYTES + tv.vsub;
#pragma unroll
        for (int db = 0; db < 4; db++) {
            const int cpos = ((4 * db + tv.vchunk) ^ tv.vsw) << 4;
            const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vr + cpos));
            const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(vr + 8 * ROW_BYTES + cpos));
            const bf16x4 a0 = __builtin_bit_cast(bf16x4, v0), a1 = __builtin_bit_cast(bf16x4, v1);
            vf[st][db] = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
        }
    }
}

// First half of a 64-key tile for one wavefront (32 query rows): S^T = K Q^T, mask, running reference,
// P^T = exp2(S^T * scale - m) packed to bf16 in pf[key block][16-key step].  MASKED: key kin of the tile is
// visible to the lane's row iff bit kin of `vis`.
template <bool MASKED>
__device__ __forceinline__ void qk_softmax(const TileView &tv, const uint8_t *lk, const bf16x8 (&qreg)[8],
                                           f32x16 (&oacc)[4], float &m_run, float &l_run, float scale_log2,
                                           uint64_t vis, bf16x8 (&pf)[2][2]) {
    // two independent accumulator chains (keys 0..31 and 32..63)
    f32x16 s0, s1;
#pragma unroll
    for (int i = 0; i < 16; i++) { s0[i] = 0.f; s1[i] = 0.f; }
    {
        bf16x8 ka[8], kb[8];
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            const int col = (((2 * kk + tv.hh) ^ tv.ksw) << 4);
            ka[kk] = *reinterpret_cast<const bf16x8 *>(lk + tv.krow + col);
            kb[kk] = *reinterpret_cast<const bf16x8 *>(lk + tv.krow + 32 * ROW_BYTES + col);
        }
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[kk], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kb[kk], qreg[kk], s1, 0, 0, 0);
        }
    }
    if (MASKED) {
        const uint32_t lo = (uint32_t)(vis >> (4 * tv.hh)), hi = (uint32_t)(vis >> (32 + 4 * tv.hh));
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int bit = 8 * (i >> 2) + (i & 3);
            s0[i] = ((lo >> bit) & 1u) ? s0[i] : -INFINITY;
            s1[i] = ((hi >> bit) & 1u) ? s1[i] : -INFINITY;
        }
    }
    float rmax = max3(s0[0], s1[0], s0[1]);
    rmax = max3(rmax, s1[1], s0[2]);
    rmax = max3(rmax, s1[2], s0[3]);
    rmax = max3(rmax, s1[3], s1[15]);
#pragma unroll
    for (int i = 4; i < 15; i += 1) rmax = max3(rmax, s0[i], s1[i]);
    rmax = fmaxf(rmax, s0[15]);
    rmax = half_swap_max(rmax);
    const float tmax = rmax * scale_log2;  // scale_log2 > 0
    const bool lift = tmax > m_run + kLazy;  // also true for the first visible keys (reference -inf)
    if (__any(lift)) {
        // only the rows that need it move their reference; the others multiply by exactly 1, so a row's
        // arithmetic never depends on what the other rows of the wavefront see
        const float m_new = lift ? tmax : m_run;
        const float alpha = lift ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[db][i] *= alpha;
    }
    const float neg_m = (MASKED && m_run == -INFINITY) ? 0.f : -m_run;
    float psum = 0.f, psum2 = 0.f;  // two chains
    uint32_t pk0[8], pk1[8];
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        const float a0 = __builtin_amdgcn_exp2f(fmaf(s0[i], scale_log2, neg_m));
        const float a1 = __builtin_amdgcn_exp2f(fmaf(s0[i + 1], scale_log2, neg_m));
        const float b0 = __builtin_amdgcn_exp2f(fmaf(s1[i], scale_log2, neg_m));
        const float b1 = __builtin_amdgcn_exp2f(fmaf(s1[i + 1], scale_log2, neg_m));
        pk0[i >> 1] = pack_bf16x2(a0, a1);
        pk1[i >> 1] = pack_bf16x2(b0, b1);
        psum = pair_sum(pk0[i >> 1], psum);
        psum2 = pair_sum(pk1[i >> 1], psum2);
    }
    const uint4 l0 = {pk0[0], pk0[1], pk0[2], pk0[3]}, h0 = {pk0[4], pk0[5], pk0[6], pk0[7]};
    const uint4 l1 = {pk1[0], pk1[1], pk1[2], pk1[3]}, h1 = {pk1[4], pk1[5], pk1[6], pk1[7]};
    pf[0][0] = __builtin_bit_cast(bf16x8, l0); pf[0][1] = __builtin_bit_cast(bf16x8, h0);
    pf[1][0] = __builtin_bit_cast(bf16x8, l1); pf[1][1] = __builtin_bit_cast(bf16x8, h1);
    l_run += psum + psum2;
}

// Second half: O^T += V^T P^T over the 64 keys of the V tile at lv; four independent accumulator chains.
// The first 32 keys' fragments may have been read ahead (vf0_ready).
__device__ __forceinline__ void pv_accumulate(const TileView &tv, const uint8_t *lv, const bf16x8 (&pf)[2][2],
                                              f32x16 (&oacc)[4], bf16x8 (&vf)[2][4], bool vf0_ready) {
    if (!vf0_ready) load_v_frags(tv, lv, 0, vf);
#pragma unroll
    for (int kb = 0; kb < 2; kb++) {
        bf16x8 va[2][4];
#pragma unroll
        for (int st = 0; st < 2; st++)
#pragma unroll
            for (int db = 0; db < 4; db++) va[st][db] = vf[st][db];
        if (kb == 0) load_v_frags(tv, lv, 1, vf);  // the second half's fragments fly during the first half's products
#pragma unroll
        for (int st = 0; st < 2; st++)
#pragma unroll
            for (int db = 0; db < 4; db++)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[st][db], pf[kb][st], oacc[db], 0, 0, 0);
    }
}

// Key-halves variants: a wavefront takes 32 of the 64 keys of a tile (key block kb); two wavefronts share a
// 32-row chunk and keep independent running (m, l, O), merged once after the last tile.  Halves the
// per-tile dependency chain of a wavefront, which is what bounds the rate when a workgroup has fewer chunks
// than wavefronts.  vis32: visibility bits of the wavefront's 32 keys.
template <bool MASKED>
__device__ __forceinline__ void qk_softmax_half(const TileView &tv, const uint8_t *lk, int kb, const bf16x8 (&qreg)[8],
                                                f32x16 (&oacc)[4], float &m_run, float &l_run, float scale_log2,
                                                uint32_t vis32, bf16x8 (&pf)[2]) {
    // two accumulator chains over the even / odd 16-wide d steps, summed afterwards
    f32x16 s0, s1;
#pragma unroll
    for (int i = 0; i < 16; i++) { s0[i] = 0.f; s1[i] = 0.f; }
    {
        bf16x8 ka[8];
        const uint8_t *kr = lk + tv.krow + kb * (32 * ROW_BYTES);
#pragma unroll
        for (int kk = 0; kk < 8; kk++)
            ka[kk] = *reinterpret_cast<const bf16x8 *>(kr + (((2 * kk + tv.hh) ^ tv.ksw) << 4));
#pragma unroll
        for (int kk = 0; kk < 8; kk += 2) {
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk], qreg[kk], s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[kk + 1], qreg[kk + 1], s1, 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < 16; i++) s0[i] += s1[i];
    if (MASKED) {
        const uint32_t lo = vis32 >> (4 * tv.hh);
#pragma unroll
        for (int i = 0; i < 16; i++) {
            const int bit = 8 * (i >> 2) + (i & 3);
            s0[i] = ((lo >> bit) & 1u) ? s0[i] : -INFINITY;
        }
    }
    float rmax = max3(s0[0], s0[1], s0[2]);
#pragma unroll
    for (int i = 3; i < 15; i += 2) rmax = max3(rmax, s0[i], s0[i + 1]);
    rmax = fmaxf(rmax, s0[15]);
    rmax = half_swap_max(rmax);
    const float tmax = rmax * scale_log2;
    const bool lift = tmax > m_run + kLazy;
    if (__any(lift)) {
        const float m_new = lift ? tmax : m_run;
        const float alpha = lift ? __builtin_amdgcn_exp2f(m_run - m_new) : 1.f;
        m_run = m_new;
        l_run *= alpha;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[db][i] *= alpha;
    }
    const float neg_m = (MASKED && m_run == -INFINITY) ? 0.f : -m_run;
    float psum = 0.f;
    uint32_t pk[8];
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        const float a0 = __builtin_amdgcn_exp2f(fmaf(s0[i], scale_log2, neg_m));
        const float a1 = __builtin_amdgcn_exp2f(fmaf(s0[i + 1], scale_log2, neg_m));
        pk[i >> 1] = pack_bf16x2(a0, a1);
        psum = pair_sum(pk[i >> 1], psum);
    }
    const uint4 l0 = {pk[0], pk[1], pk[2], pk[3]}, h0 = {pk[4], pk[5], pk[6], pk[7]};
    pf[0] = __builtin_bit_cast(bf16x8, l0);
    pf[1] = __builtin_bit_cast(bf16x8, h0);
    l_run += psum;
}

__device__ __forceinline__ void pv_accumulate_half(const TileView &tv, const uint8_t *lv, int kb, const bf16x8 (&pf)[2],
                                                   f32x16 (&oacc)[4]) {
    bf16x8 vf[2][4];
    load_v_frags(tv, lv, kb, vf);
#pragma unroll
    for (int st = 0; st < 2; st++)
#pragma unroll
        for (int db = 0; db < 4; db++)
            oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[st][db], pf[st], oacc[db], 0, 0, 0);
}

template <int NW, int NS, bool PAGED, bool KH>
__global__ void __launch_bounds__(NW * 64, 2) attn_mfma_kernel(AttnParams p) {
    constexpr int D = 128;
    constexpr int LPW = 2 * TileLoader<NW>::U;  // direct-to-LDS loads an issuing wavefront issues per tile
    uint8_t *const smem = attn_smem;
    const uint32_t smem_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) uint8_t *)attn_smem;

    // Row groups (wg) of one KV head read the same K/V.  Workgroups go to the 8 XCDs round-robin by linear id;
    // with wg as the slow index the ids of one (split, KV head) differ by multiples of nsplit * Hkv, i.e. (for
    // Hkv a multiple of 8) they share an XCD and the second reader of a K/V line finds it in that XCD's L2.
    const int wg = blockIdx.y / p.Hkv, kvh = blockIdx.y % p.Hkv;
    const int tid = threadIdx.x, lane = tid & 63;
    SplitShare share{};
    if (p.balanced) {  // grid (B * nsplit slots, Hkv * row groups): which sequence and split is this slot?
        share = balanced_share(p, (int)blockIdx.x, lane);
        if (!share.live) return;  // uniform over the workgroup
        if (share.j == 0 && blockIdx.y == 0 && tid == 0) p.split_tab[share.b] = make_int2(share.start, share.nvalid);
    }
    const int b = p.balanced ? share.b : (int)blockIdx.z;
    // The split index is rotated by the sequence index.  Unrotated, split s of every sequence lands on XCD s
    // (mod 8 with the head): in a ragged batch the first splits are all full and the last ones short or absent,
    // so some XCDs carry all the long workgroups and finish half as late again as the others.  (Not rotated by
    // the KV head: in a contiguous cache the heads of a key row are neighbours in memory, and the XCD that
    // reads one of them should read all of them at about the same time.)
    const int s = p.balanced ? share.j : (int)((blockIdx.x + blockIdx.z) % p.nsplit);
    const int chunk = p.balanced ? share.tps * KT : p.chunk;  // prefix keys per split of this sequence
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c32 = lane & 31, hh = lane >> 5;

    // Start-up.  The caches are cold when a kernel starts and every dependent trip to memory costs the better
    // part of a microsecond, so the trips before the first tile load are made as few as possible: one for the
    // kernel arguments (all of them, not a few at a time as they come up), one for the sequence's sizes
    // together with the physical block ids of the first tiles.  Those ids are read before it is known how long
    // the prefix is: the index is clamped into the table row, and an id is used only if its tile turns out to
    // be a full prefix tile.
    constexpr bool kShifted = (NW == 8);
    constexpr int PD = kShifted ? NS - 2 : NS - 1;  // tiles in flight behind the one being consumed
    static_assert(PD >= 1 && PD <= 3, "ring depth");
    asm volatile("" ::"s"(p.q), "s"(p.k_cache), "s"(p.v_cache), "s"(p.kt), "s"(p.vt), "s"(p.block_table),
                 "s"(p.prefix_len), "s"(p.n_nodes), "s"(p.bitmask), "s"(p.T_max), "s"(p.Hq), "s"(p.G),
                 "s"(p.max_blocks), "s"(p.P_cap), "s"(p.P_max), "s"(p.words), "s"(p.chunk), "s"(p.pairs));
    int n_raw, P_raw;
    if (p.balanced) {
        n_raw = share.n_raw; P_raw = share.P_raw;
    } else {
        n_raw = ((const_i32_ptr)(uintptr_t)p.n_nodes)[b]; P_raw = ((const_i32_ptr)(uintptr_t)p.prefix_len)[b];
    }
    // (an issuing wavefront needs ids lb, lb+1, lb+2, lb+3 of each tile: 4 * PD consecutive table entries)
    static_assert(TileLoader<NW>::U == 4 && TileLoader<NW>::NI == 4, "block ids of a tile: four consecutive entries");
    int blk_pro[PD][4];
    const int lb_first = (s * p.chunk) >> 4;
    const bool spec = PAGED && !p.balanced && lb_first + 4 * PD <= p.max_blocks;  // the whole range lies inside the table row
    if (spec) {
        const const_i32_ptr bt_row = (const_i32_ptr)(uintptr_t)(p.block_table + (size_t)b * p.max_blocks + lb_first);
#pragma unroll
        for (int t = 0; t < PD; t++)
#pragma unroll
            for (int u = 0; u < 4; u++) blk_pro[t][u] = bt_row[4 * t + u];
    } else {
#pragma unroll
        for (int t = 0; t < PD; t++)
#pragma unroll
            for (int u = 0; u < 4; u++) blk_pro[t][u] = 0;
    }
    // one wait for all of them
    if constexpr (PD == 3)
        asm volatile("" ::"s"(n_raw), "s"(P_raw), "s"(blk_pro[0][0]), "s"(blk_pro[0][1]), "s"(blk_pro[0][2]), "s"(blk_pro[0][3]),
                     "s"(blk_pro[1][0]), "s"(blk_pro[1][1]), "s"(blk_pro[1][2]), "s"(blk_pro[1][3]),
                     "s"(blk_pro[2][0]), "s"(blk_pro[2][1]), "s"(blk_pro[2][2]), "s"(blk_pro[2][3]));
    else if constexpr (PD == 2)
        asm volatile("" ::"s"(n_raw), "s"(P_raw), "s"(blk_pro[0][0]), "s"(blk_pro[0][1]), "s"(blk_pro[0][2]), "s"(blk_pro[0][3]),
                     "s"(blk_pro[1][0]), "s"(blk_pro[1][1]), "s"(blk_pro[1][2]), "s"(blk_pro[1][3]));
    else
        asm volatile("" ::"s"(n_raw), "s"(P_raw), "s"(blk_pro[0][0]), "s"(blk_pro[0][1]), "s"(blk_pro[0][2]), "s"(blk_pro[0][3]));

    const int n = clampi(n_raw, 0, p.T_max);
    const int P = clampi(P_raw, 0, p.P_max);
    const int nvalid = p.balanced ? share.nvalid : seq_nsplit(p, P);
    if (s >= nvalid) return;  // uniform over the workgroup
    const bool direct = (p.nsplit == 1);

    // The G * T_max query rows of a KV head are numbered r = k * G + g (node k, head-in-group g) and cut into
    // chunks of 32: a small tree fills whole MFMA tiles with rows of several heads instead of padding every
    // head to 32 rows.  Wavefront `wave` of row group `wg` owns chunk `pair`; with key halves (KH) a chunk
    // belongs to two wavefronts, wave and wave + NW/2, which take key block kb = 0 / 1 of every tile.
    constexpr int CW = KH ? NW / 2 : NW;  // chunks per workgroup
    const int kb = KH ? wave / CW : 0;
    const int pair = wg * CW + (KH ? wave % CW : wave);
    const bool active = pair < p.pairs;
    const int r = (active ? pair : 0) * 32 + c32;
    const int kq = r / p.G;              // the lane's node
    const int h = kvh * p.G + (r - kq * p.G);  // and query head
    // wavefront-uniform: does the chunk hold any valid row?  If not the wavefront only takes part in loads and barriers
    const bool wactive = active && pair * 32 < n * p.G;

    const int k0 = s * chunk, k1 = min(P, k0 + chunk);
    const int nfull = (k1 > k0) ? (k1 - k0) / KT : 0;               // full prefix tiles
    const int npt = (k1 > k0) ? (k1 - k0 + KT - 1) / KT : 0;        // prefix tiles incl. a ragged last one
    const int ntt = (s == nvalid - 1) ? (n + KT - 1) / KT : 0;      // tree tiles
    const int nt = npt + ntt;

    TileLoader<NW> ld;
    ld.kc = static_cast<const uint8_t *>(p.k_cache); ld.vc = static_cast<const uint8_t *>(p.v_cache);
    ld.kt = static_cast<const uint8_t *>(p.kt) + ((size_t)b * p.T_max * p.Hkv + kvh) * ROW_BYTES;
    ld.vt = static_cast<const uint8_t *>(p.vt) + ((size_t)b * p.T_max * p.Hkv + kvh) * ROW_BYTES;
    ld.bt = PAGED ? p.block_table + (size_t)b * p.max_blocks : nullptr;
    ld.row_stride = (size_t)p.Hkv * ROW_BYTES;
    ld.seq_off = ((size_t)b * p.P_cap * p.Hkv + kvh) * ROW_BYTES;   // contiguous cache: row 0 of (b, kvh)
    ld.blk_stride = (size_t)p.Hkv * 16 * ROW_BYTES;                  // paged cache: one block, all heads
    ld.head_off = (size_t)kvh * 16 * ROW_BYTES;
    ld.kf = ld.kc + (PAGED ? ld.head_off : ld.seq_off); ld.vf = ld.vc + (PAGED ? ld.head_off : ld.seq_off);
    ld.smem_addr = smem_addr; ld.wave = wave; ld.l_row = lane >> 4; ld.l_pos = lane & 15;
    ld.k0 = k0; ld.k1 = k1; ld.npt = npt; ld.n = n; ld.P = P; ld.tail = (p.kt == nullptr);
    {
        // the lane's row within the 16 rows that pair `wave` + 4u covers, the same for every u
        const int r_in = 4 * wave + ld.l_row;
        ld.kcol = (uint32_t)((ld.l_pos ^ kswz_of_row(r_in)) * 16);
        ld.vcol = (uint32_t)((ld.l_pos ^ vswz_of_row(r_in)) * 16);
        const uint32_t rowpart = PAGED ? (uint32_t)((r_in & 15) * ROW_BYTES) : (uint32_t)r_in * (uint32_t)ld.row_stride;
        ld.koff = rowpart + ld.kcol;
        ld.voff = rowpart + ld.vcol;
    }
    const bool issuer = wave < TileLoader<NW>::NI;
    // one workgroup per (split, KV head): nobody else reads these K/V bytes, so they are streamed past L2
    const bool stream_kv = p.wgp == 1;
    // prologue: fill the ring, then fetch Q and the mask row while those loads fly
#pragma unroll
    for (int t = 0; t < PD; t++) {
        if (t >= nt || !issuer) continue;
        if (t < nfull) {
            if (PAGED && !spec) fetch_blocks<NW>(ld, t, blk_pro[t]);
            if (stream_kv) issue_full_tile<NW, NS, PAGED, true>(ld, t, blk_pro[t]);
            else issue_full_tile<NW, NS, PAGED, false>(ld, t, blk_pro[t]);
        } else {
            issue_edge_tile<NW, NS>(ld, t);
        }
    }

    const uint16_t *qp = static_cast<const uint16_t *>(p.q);
    // Q as B operand: lane holds query row kq, d values 16*kk + 8*hh .. +7
    bf16x8 qreg[8];
    uint64_t mbits0 = 0, mbits1 = 0, mbits2 = 0, mbits3 = 0;  // the row's ancestor bits, one word per tree tile
    const bool rv = active && kq < n;
    if (rv) {
        const uint64_t *mrow = p.bitmask + ((size_t)b * p.T_max + kq) * p.words;
        mbits0 = mrow[0];
        if (p.words > 1) mbits1 = mrow[1];
        if (p.words > 2) mbits2 = mrow[2];
        if (p.words > 3) mbits3 = mrow[3];
    }
#pragma unroll
    for (int kk = 0; kk < 8; kk++) {
        uint4 v = {0, 0, 0, 0};
        if (rv) v = *reinterpret_cast<const uint4 *>(qp + (((size_t)b * p.T_max + kq) * p.Hq + h) * D + 16 * kk + 8 * hh);
        qreg[kk] = __builtin_bit_cast(bf16x8, v);
    }

    f32x16 oacc[4];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int db = 0; db < 4; db++)
#pragma unroll
        for (int i = 0; i < 16; i++) oacc[db][i] = 0.f;

    // Q and the mask row must have arrived before the loop: a wait the compiler can see here keeps it from
    // placing a vmcnt(0) inside the loop, which would also drain the asynchronous tile loads every iteration
    wait_vmcnt<0>();

    // per-lane LDS offsets (bytes within a tile) that do not depend on the tile
    const int g16 = lane >> 4, i16 = lane & 15;
    const int vrow = 4 * hh + (i16 >> 2);  // V row within a 16-key step (second read: +8)
    TileView tv{c32 * ROW_BYTES, kswz_of_row(c32), vrow, vswz_of_row(vrow),
                2 * (g16 & 1) + ((i16 & 3) >> 1), 8 * (i16 & 1), hh};

    // Ring step: wait for tile ti, barrier, refill.  PD = tiles in flight behind the one being consumed.
    // With 8 wavefronts the V tile of step ti-1 is still being read by wavefronts 4..7 during step ti, so
    // the stage that is refilled is the one of tile ti-2.
    auto ring_step = [&](int ti) {
        const int tn = ti + PD;  // tile to issue in this step
        int blk[TileLoader<NW>::U];
        const bool full_next = issuer && tn < nfull;
        if (PAGED && full_next) fetch_blocks<NW>(ld, tn, blk);  // scalar loads fly during the wait below
        const int ahead = min(PD - 1, nt - 1 - ti);  // younger tiles whose loads may still be outstanding
        if (PD >= 3 && ahead >= 2) wait_vmcnt<2 * LPW>();
        else if (PD >= 2 && ahead == 1) wait_vmcnt<LPW>();
        else wait_vmcnt<0>();
        __builtin_amdgcn_s_barrier();  // everyone's part of tile ti is in LDS; the refilled stage is no longer read
        asm volatile("" ::: "memory");
        if (full_next) {
            if (stream_kv) issue_full_tile<NW, NS, PAGED, true>(ld, tn, blk);
            else issue_full_tile<NW, NS, PAGED, false>(ld, tn, blk);
        }
        else if (issuer && tn < nt) issue_edge_tile<NW, NS>(ld, tn);
    };
    auto tile_vis = [&](int ti) -> uint64_t {
        if (ti < npt) return (1ull << (k1 - k0 - nfull * KT)) - 1ull;  // ragged last prefix tile: 1..63 keys
        const int w = ti - npt;                                         // tree tile: the row's ancestor bits
        const uint64_t lo = (w & 1) ? mbits1 : mbits0, hi = (w & 1) ? mbits3 : mbits2;
        return (w & 2) ? hi : lo;
    };
    bf16x8 pf[2][2], vf[2][4];
    // one tile for one wavefront, in two parts (the parts run in different ring steps for late wavefronts)
    auto part_qk = [&](int t, bool masked) {
        const uint8_t *lk = smem + (t % NS) * STAGE_BYTES;
        if (KH) {
            const uint32_t v32 = masked ? (uint32_t)(tile_vis(t) >> (32 * kb)) : ~0u;
            if (masked) qk_softmax_half<true>(tv, lk, kb, qreg, oacc, m_run, l_run, p.scale_log2, v32, pf[0]);
            else qk_softmax_half<false>(tv, lk, kb, qreg, oacc, m_run, l_run, p.scale_log2, v32, pf[0]);
        } else {
            if (masked) qk_softmax<true>(tv, lk, qreg, oacc, m_run, l_run, p.scale_log2, tile_vis(t), pf);
            else qk_softmax<false>(tv, lk, qreg, oacc, m_run, l_run, p.scale_log2, ~0ull, pf);
        }
    };
    auto part_pv = [&](int t) {
        const uint8_t *lv = smem + (t % NS) * STAGE_BYTES + TILE_BYTES;
        if (KH) pv_accumulate_half(tv, lv, kb, pf[0], oacc);
        else pv_accumulate(tv, lv, pf, oacc, vf, false);
    };
    int ti = 0;
    if (!kShifted || wave < 4) {
        // QK(t), softmax(t), PV(t) within ring step t
        for (; ti < nfull; ti++) {  // full prefix tiles: no masking code at all
            ring_step(ti);
            if (!wactive) continue;
            part_qk(ti, false);
            part_pv(ti);
        }
        for (; ti < nt; ti++) {     // ragged last prefix tile and tree tiles
            ring_step(ti);
            if (!wactive) continue;
            part_qk(ti, true);
            part_pv(ti);
        }
    } else {
        // one phase behind: PV(t-1), QK(t), softmax(t) within ring step t; the last PV after the loop
        for (; ti < nfull; ti++) {
            ring_step(ti);
            if (!wactive) continue;
            if (ti > 0) part_pv(ti - 1);
            part_qk(ti, false);
        }
        for (; ti < nt; ti++) {
            ring_step(ti);
            if (!wactive) continue;
            if (ti > 0) part_pv(ti - 1);
            part_qk(ti, true);
        }
        if (nt > 0 && wactive) part_pv(nt - 1);
    }

    if (KH) {
        // Merge the two key halves of a chunk through LDS (the ring is no longer needed): the kb = 1
        // wavefront hands its (m, l, O) to its kb = 0 partner, which rescales both to the larger reference.
        __builtin_amdgcn_s_barrier();  // every wavefront has finished reading tiles; no tile load is outstanding
        asm volatile("" ::: "memory");
        float4 *mx = reinterpret_cast<float4 *>(smem) + (size_t)(wave % CW) * (17 * 64);
        if (kb == 1 && wactive) {
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int ig = 0; ig < 4; ig++)
                    mx[(4 * db + ig) * 64 + lane] = float4{oacc[db][4 * ig], oacc[db][4 * ig + 1], oacc[db][4 * ig + 2], oacc[db][4 * ig + 3]};
            mx[16 * 64 + lane] = float4{m_run, l_run, 0.f, 0.f};
        }
        __syncthreads();
        if (kb == 1) return;
        if (wactive) {
            const float4 ml = mx[16 * 64 + lane];
            const float m_new = fmaxf(m_run, ml.x);
            const float fa = (m_run == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(m_run - m_new);
            const float fb = (ml.x == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(ml.x - m_new);
            m_run = m_new;
            l_run = l_run * fa + ml.y * fb;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int ig = 0; ig < 4; ig++) {
                    const float4 o = mx[(4 * db + ig) * 64 + lane];
                    oacc[db][4 * ig] = oacc[db][4 * ig] * fa + o.x * fb;
                    oacc[db][4 * ig + 1] = oacc[db][4 * ig + 1] * fa + o.y * fb;
                    oacc[db][4 * ig + 2] = oacc[db][4 * ig + 2] * fa + o.z * fb;
                    oacc[db][4 * ig + 3] = oacc[db][4 * ig + 3] * fa + o.w * fb;
                }
        }
    }

    // ---- epilogue
    if (!active || kq >= p.T_max) return;
    uint16_t *out = static_cast<uint16_t *>(p.out);
    const float l_tot = half_swap_sum(l_run);
    const size_t lrow = ((size_t)b * p.Hq + h) * p.T_max + kq;
    if (direct) {
        const size_t orow = (((size_t)b * p.T_max + kq) * p.Hq + h) * D;
        const float inv = rv ? 1.f / l_tot : 0.f;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int ig = 0; ig < 4; ig++) {
                const int dcol = 32 * db + 8 * ig + 4 * hh;
                uint2 w;
                w.x = rv ? pack_bf16x2(oacc[db][4 * ig] * inv, oacc[db][4 * ig + 1] * inv) : 0u;
                w.y = rv ? pack_bf16x2(oacc[db][4 * ig + 2] * inv, oacc[db][4 * ig + 3] * inv) : 0u;
                *reinterpret_cast<uint2 *>(out + orow + dcol) = w;
            }
        if (p.lse && hh == 0) p.lse[lrow] = rv ? (m_run + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
    } else if (rv) {
        const size_t pr = part_row(p, p.balanced ? (int)blockIdx.x : b * p.nsplit + s, h, kq);
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int ig = 0; ig < 4; ig++) {
                const int dcol = 32 * db + 8 * ig + 4 * hh;
                float4 w = {oacc[db][4 * ig], oacc[db][4 * ig + 1], oacc[db][4 * ig + 2], oacc[db][4 * ig + 3]};
                *reinterpret_cast<float4 *>(p.part_o + pr * D + dcol) = w;
            }
        if (hh == 0) {
            p.part_m[pr] = m_run;
            p.part_l[pr] = l_tot;
        }
    }
}

// ----------------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------------
struct Plan {
    bool mfma, kh;
    int nw, ns, pairs, wgp, chunk, nsplit;
    bool balanced;  // split slots shared out among the sequences by their lengths, on the device
};

static bool supported(const etv_attn_desc *h) {
    if (h->B < 0 || h->T_max < 1 || h->Hq < 1 || h->Hkv < 1 || h->d < 1) return false;
    if (h->Hq > 65536) return false;  // keeps the byte strides of a cache row and of a block below 2^32
    return true;
}

// Launch shape.  Cost model in microseconds, fitted on MI355X: workgroups run in rounds of the slots the chip
// offers; a round costs its tiles plus tree tiles and ramp-up; every extra split writes and re-reads one
// (m, l, O) set per query row and needs the combine launch.  A tile costs about 2.8 us for an 8-wavefront
// workgroup (two wavefronts per SIMD), the same for two 4-wavefront workgroups sharing a compute unit, and
// about 1.7 us for a 4-wavefront workgroup that has a compute unit to itself (1.5 us when at most two of its
// wavefronts hold valid rows).
constexpr double kTileKhAlone = 1.1, kTileKhShared = 2.2, kTileKh8 = 1.65;
// whole tiles: one 8-wavefront workgroup per compute unit (its two wavefronts per SIMD run one phase apart and it
// fetches each tile once) is 4-7 % faster in sustained runs than two 4-wavefront workgroups, which cost 2.8 together
constexpr double kTileWhole8 = 2.65;
static Plan make_plan(const etv_attn_desc *h) {
    Plan pl{};
    const int tiles = max(1, (h->P_max + KT - 1) / KT);
    const int B = max(1, h->B);
    pl.mfma = (h->dtype == ETV_BF16 && h->d == 128 && !(h->flags & ETV_ATTN_FLAG_GENERIC));
    if (!pl.mfma) {
        const long units = ((long)B * h->Hq * h->T_max + 7) / 8;  // 8 resident wavefronts ~ one workgroup slot
        int tps;
        if (h->kv_split > 0) {
            tps = (h->kv_split + KT - 1) / KT;
        } else {
            long want = (256 + units - 1) / units;
            want = want < 1 ? 1 : (want > tiles ? tiles : want);
            tps = (int)((tiles + want - 1) / want);
        }
        pl.chunk = tps * KT;
        pl.nsplit = (tiles + tps - 1) / tps;
        return pl;
    }
    pl.pairs = ((h->Hq / h->Hkv) * h->T_max + 31) / 32;  // 32-row chunks of the G * T_max packed rows of a KV head
    const double part_us = 2.0 * B * h->Hq * h->T_max * (h->d + 2.0) * 4.0 / 3.0e6;
    double best = 1e30;
    for (int nw = 4; nw <= 8; nw += 4) {
        for (int kh = 0; kh <= 1; kh++) {
            const int cw = kh ? nw / 2 : nw;  // chunks per workgroup
            // key halves pay when a workgroup would otherwise have idle wavefronts
            if (kh && (h->flags & ETV_ATTN_FLAG_WHOLE_TILE)) continue;
            if (!kh && (h->flags & ETV_ATTN_FLAG_KEY_HALVES)) continue;
            if (nw == 8 && (pl.pairs <= (kh ? 2 : 4) || (h->flags & ETV_ATTN_FLAG_SMALL_WG))) continue;
            if (nw == 4 && (h->flags & ETV_ATTN_FLAG_LARGE_WG) && pl.pairs > (kh ? 2 : 4)) continue;
            const int wgp = (pl.pairs + cw - 1) / cw;
            const long units = (long)B * h->Hkv * wgp;
            // candidates: every distinct number of splits, or the one split size the caller asks for
            const int forced_tps = h->kv_split > 0 ? min(tiles, (h->kv_split + KT - 1) / KT) : 0;
            for (int ns = 1; ns <= tiles; ns++) {
                const int tps = forced_tps ? forced_tps : (tiles + ns - 1) / ns;
                if ((tiles + tps - 1) / tps != ns) continue;
                const long wgs = units * ns;
                const bool alone = (nw == 4 && wgs <= 256);
                const double slots = nw == 8 ? 256.0 : 512.0;
                double t_tile;
                if (kh) t_tile = alone ? kTileKhAlone : (nw == 8 ? kTileKh8 : kTileKhShared);
                else t_tile = alone ? (pl.pairs <= 2 ? 1.5 : 1.7) : (nw == 8 ? kTileWhole8 : 2.8);
                const double rounds = ceil((double)wgs / slots);
                const double est = rounds * (tps + 1.5) * t_tile + 4.0 + (ns > 1 ? 4.6 + ns * part_us : 0.0);
                if (est < best) {
                    best = est;
                    pl.nw = nw; pl.kh = kh; pl.wgp = wgp; pl.chunk = tps * KT; pl.nsplit = ns;
                    pl.ns = nw == 8 ? 4 : (alone ? 4 : 2);  // ring stages: a lone small workgroup can afford four
                }
            }
        }
    }
    // a batch with splits: the slots go to the sequences by length (lane i of a wavefront plans sequence i)
    pl.balanced = pl.nsplit > 1 && B >= 2 && B <= 64 && !(h->flags & ETV_ATTN_FLAG_UNIFORM_SPLITS);
    if (best == 1e30) {  // kv_split larger than the prefix: a single split
        pl.nw = (pl.pairs > 4 && !(h->flags & ETV_ATTN_FLAG_SMALL_WG)) ? 8 : 4;
        pl.kh = false;
        pl.wgp = (pl.pairs + pl.nw - 1) / pl.nw;
        pl.chunk = tiles * KT; pl.nsplit = 1; pl.ns = pl.nw == 8 ? 4 : 2;
    }
    return pl;
}

template <int NW, int NS, bool PAGED, bool KH>
static int32_t launch_mfma(const AttnParams &p, dim3 grid, hipStream_t st) {
    constexpr size_t lds = (size_t)NS * STAGE_BYTES;
    static const bool lds_ok = [] {  // opt in to more than 64 KiB of dynamic LDS, once per process
        return hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_mfma_kernel<NW, NS, PAGED, KH>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess;
    }();
    if (!lds_ok) return ETV_ERR_HIP;
    hipLaunchKernelGGL((attn_mfma_kernel<NW, NS, PAGED, KH>), grid, dim3(NW * 64), lds, st, p);
    return check_launch();
}

}  // namespace etv

extern "C" int32_t etv_tree_verify_attention_plan(const etv_attn_desc *h, etv_attn_plan *out) {
    if (!h || !out || !etv::supported(h) || h->Hq % h->Hkv != 0) return ETV_ERR_INVALID_ARG;
    const etv::Plan pl = etv::make_plan(h);
    out->mfma = pl.mfma ? 1 : 0;
    out->wavefronts = pl.mfma ? pl.nw : 1;
    out->key_halves = pl.mfma && pl.kh ? 1 : 0;
    out->ring_stages = pl.mfma ? pl.ns : 0;
    out->row_groups = pl.mfma ? pl.wgp : 0;
    out->kv_split = pl.chunk;
    out->n_splits = pl.nsplit;
    out->balanced_splits = pl.mfma && pl.balanced ? 1 : 0;
    out->workgroups = pl.mfma ? (int64_t)pl.nsplit * h->Hkv * pl.wgp * (h->B > 0 ? h->B : 0)
                              : (int64_t)h->T_max * h->Hq * (h->B > 0 ? h->B : 0) * pl.nsplit;
    return ETV_OK;
}

extern "C" size_t etv_tree_verify_attention_workspace_bytes(const etv_attn_desc *h) {
    if (!h || !etv::supported(h) || h->B == 0) return 0;
    etv::Plan pl = etv::make_plan(h);
    if (pl.nsplit <= 1) return 256;
    size_t rows = (size_t)h->B * h->Hq * h->T_max * pl.nsplit;
    return rows * ((size_t)h->d + 2) * sizeof(float) + 1024;  // partials, then 64 (first slot, splits) pairs
}

namespace etv {
// argument checks and launches shared by the two entry points (caller's workspace / the library's static one)
static int32_t attention_run(const etv_attn_desc *h, const void *q, const void *k_cache, const void *v_cache,
                             const int32_t *block_table, const int32_t *prefix_len, const void *kt, const void *vt,
                             const uint64_t *bitmask, const int32_t *n_nodes, void *out, float *lse, void *workspace,
                             size_t workspace_bytes, void *stream) {
    if (!h || !q || !prefix_len || !bitmask || !n_nodes || !out) return ETV_ERR_INVALID_ARG;
    if ((kt == nullptr) != (vt == nullptr)) return ETV_ERR_INVALID_ARG;
    const bool tail = (kt == nullptr);  // in-place branch cache: the tree rows are in the cache behind the prefix
    if (!supported(h)) return ETV_ERR_INVALID_ARG;
    if (h->Hq % h->Hkv != 0) return ETV_ERR_INVALID_ARG;
    if (h->dtype != ETV_F32 && h->dtype != ETV_BF16) return ETV_ERR_UNSUPPORTED;
    if (h->d != 64 && h->d != 128) return ETV_ERR_UNSUPPORTED;
    if (h->T_max > ETV_ATTN_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if (h->P_max < 0) return ETV_ERR_INVALID_ARG;
    if (h->block_size != 0 && h->block_size != 16) return ETV_ERR_UNSUPPORTED;
    if (h->block_size > 0 && (!block_table || h->max_blocks < 1)) return ETV_ERR_INVALID_ARG;
    const long reach = (long)h->P_max + (tail ? h->T_max : 0);  // cache positions the kernel may read
    if (h->block_size > 0 && reach > (long)h->max_blocks * h->block_size) return ETV_ERR_INVALID_ARG;
    if (h->block_size == 0 && reach > h->P_cap) return ETV_ERR_INVALID_ARG;
    if (reach > 0 && (!k_cache || !v_cache)) return ETV_ERR_INVALID_ARG;
    if (h->kv_split < 0) return ETV_ERR_INVALID_ARG;
    const uintptr_t align = (uintptr_t)q | (uintptr_t)k_cache | (uintptr_t)v_cache | (uintptr_t)kt | (uintptr_t)vt |
                            (uintptr_t)out | (uintptr_t)workspace;
    if (align & 15) return ETV_ERR_INVALID_ARG;
    if (h->B == 0) return ETV_OK;
    if (h->B > 65535) return ETV_ERR_UNSUPPORTED;

    Plan pl = make_plan(h);
    if ((long)h->B * pl.nsplit > 65535 && !pl.mfma) return ETV_ERR_UNSUPPORTED;
    if (pl.nsplit > 1) {
        if (!workspace || workspace_bytes < etv_tree_verify_attention_workspace_bytes(h))
            return ETV_ERR_WORKSPACE_TOO_SMALL;
    }
    AttnParams p{};
    p.q = q; p.k_cache = k_cache; p.v_cache = v_cache; p.kt = kt; p.vt = vt;
    p.block_table = block_table; p.prefix_len = prefix_len; p.n_nodes = n_nodes; p.bitmask = bitmask;
    p.out = out; p.lse = lse;
    p.B = h->B; p.T_max = h->T_max; p.Hq = h->Hq; p.Hkv = h->Hkv; p.G = h->Hq / h->Hkv; p.d = h->d;
    p.block_size = h->block_size; p.max_blocks = h->max_blocks; p.P_cap = h->P_cap; p.P_max = h->P_max;
    p.words = (h->T_max + 63) / 64;
    p.chunk = pl.chunk; p.nsplit = pl.nsplit; p.pairs = pl.pairs; p.wgp = pl.wgp;
    const float scale = (h->scale == 0.f) ? 1.0f / sqrtf((float)h->d) : h->scale;
    p.scale_log2 = scale * 1.4426950408889634f;
    if (pl.nsplit > 1) {
        size_t rows = (size_t)h->B * h->Hq * h->T_max * pl.nsplit;
        p.part_o = static_cast<float *>(workspace);
        p.part_m = p.part_o + rows * h->d;
        p.part_l = p.part_m + rows;
        p.split_tab = reinterpret_cast<int2 *>(p.part_l + rows);  // 8-byte aligned: rows * (d + 2) floats in
        p.balanced = pl.mfma && pl.balanced;
    }
    hipStream_t st = as_stream(stream);
    int32_t rc;
    if (pl.mfma) {
        const dim3 grid = pl.balanced ? dim3(pl.nsplit * h->B, h->Hkv * pl.wgp, 1) : dim3(pl.nsplit, h->Hkv * pl.wgp, h->B);
        const bool paged = h->block_size > 0;
        // 8 wavefronts: one workgroup per compute unit with a 4-stage ring (128 KiB of LDS);
        // 4 wavefronts: two workgroups per compute unit with 2 stages each, or 4 stages when the grid is small
        const int shape = (pl.nw == 8 ? 0 : (pl.ns == 4 ? 1 : 2)) * 4 + (paged ? 2 : 0) + (pl.kh ? 1 : 0);
        switch (shape) {
        case 0: rc = launch_mfma<8, 4, false, false>(p, grid, st); break;
        case 1: rc = launch_mfma<8, 4, false, true>(p, grid, st); break;
        case 2: rc = launch_mfma<8, 4, true, false>(p, grid, st); break;
        case 3: rc = launch_mfma<8, 4, true, true>(p, grid, st); break;
        case 4: rc = launch_mfma<4, 4, false, false>(p, grid, st); break;
        case 5: rc = launch_mfma<4, 4, false, true>(p, grid, st); break;
        case 6: rc = launch_mfma<4, 4, true, false>(p, grid, st); break;
        case 7: rc = launch_mfma<4, 4, true, true>(p, grid, st); break;
        case 8: rc = launch_mfma<4, 2, false, false>(p, grid, st); break;
        case 9: rc = launch_mfma<4, 2, false, true>(p, grid, st); break;
        case 10: rc = launch_mfma<4, 2, true, false>(p, grid, st); break;
        default: rc = launch_mfma<4, 2, true, true>(p, grid, st); break;
        }
    } else {
        dim3 grid(h->T_max, h->Hq, h->B * pl.nsplit);
        if (h->dtype == ETV_F32 && h->d == 64)
            hipLaunchKernelGGL((attn_generic_kernel<float, 64>), grid, dim3(64), 0, st, p);
        else if (h->dtype == ETV_F32)
            hipLaunchKernelGGL((attn_generic_kernel<float, 128>), grid, dim3(64), 0, st, p);
        else if (h->d == 64)
            hipLaunchKernelGGL((attn_generic_kernel<uint16_t, 64>), grid, dim3(64), 0, st, p);
        else
            hipLaunchKernelGGL((attn_generic_kernel<uint16_t, 128>), grid, dim3(64), 0, st, p);
        rc = check_launch();
    }
    if (rc != ETV_OK || pl.nsplit == 1) return rc;
    const long crows = (long)h->B * h->T_max * h->Hq;
    const bool two = h->d == 128 && crows <= 512;  // very few rows: two wavefronts per row
    const bool wide = pl.nsplit > 8;                // many splits: sixteen per batch of loads
    dim3 cgrid((unsigned)((crows + (two ? 1 : 3)) / (two ? 2 : 4)));
#define ETV_COMBINE(TY, DD, WPR) \
    do { \
        if (wide) hipLaunchKernelGGL((attn_combine_kernel<TY, DD, WPR, 16>), cgrid, dim3(256), 0, st, p); \
        else hipLaunchKernelGGL((attn_combine_kernel<TY, DD, WPR, 8>), cgrid, dim3(256), 0, st, p); \
    } while (0)
    if (h->dtype == ETV_F32 && h->d == 64) ETV_COMBINE(float, 64, 1);
    else if (h->dtype == ETV_F32 && two) ETV_COMBINE(float, 128, 2);
    else if (h->dtype == ETV_F32) ETV_COMBINE(float, 128, 1);
    else if (h->d == 64) ETV_COMBINE(uint16_t, 64, 1);
    else if (two) ETV_COMBINE(uint16_t, 128, 2);
    else ETV_COMBINE(uint16_t, 128, 1);
#undef ETV_COMBINE
    return check_launch();
}
}  // namespace etv

extern "C" int32_t etv_tree_verify_attention(const etv_attn_desc *h, const void *q, const void *k_cache,
                                             const void *v_cache, const int32_t *block_table,
                                             const int32_t *prefix_len, const void *kt, const void *vt,
                                             const uint64_t *bitmask, const int32_t *n_nodes, void *out, float *lse,
                                             void *workspace, size_t workspace_bytes, void *stream) {
    return etv::attention_run(h, q, k_cache, v_cache, block_table, prefix_len, kt, vt, bitmask, n_nodes, out, lse,
                              workspace, workspace_bytes, stream);
}

// ----------------------------------------------------------------------------------------------
// The same call for callers that cannot allocate or carry a workspace (code under graph capture, serving loops):
// the split partials go to a fixed array in device memory that the library owns.  Each GPU holds its own copy
// of the array at its own address; the address is asked for once per device and only that pointer is ever
// handed to a kernel (the array's name is a host-side stand-in in host code, not a device address).
// ----------------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[ETV_ATTN_STATIC_WORKSPACE_BYTES];

namespace etv {
constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];           // per device, filled on the first call on that device
static std::atomic<int> g_scratch_state[kMaxDevices];  // 0 unset, 1 being set, 2 set

static int32_t static_scratch(void **ptr) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ETV_ERR_HIP;
    if (g_scratch_state[dev].load(std::memory_order_acquire) != 2) {
        int expect = 0;
        if (g_scratch_state[dev].compare_exchange_strong(expect, 1, std::memory_order_acq_rel)) {
            void *d = nullptr;
            const hipError_t e = hipGetSymbolAddress(&d, HIP_SYMBOL(scratch));  // device `dev` is current
            if (e != hipSuccess || d == nullptr) {
                g_last_hip_error = (int32_t)e;
                g_scratch_state[dev].store(0, std::memory_order_release);
                return ETV_ERR_HIP;
            }
            g_scratch_ptr[dev] = d;
            g_scratch_state[dev].store(2, std::memory_order_release);
        } else {
            while (g_scratch_state[dev].load(std::memory_order_acquire) == 1) { /* another thread is asking */ }
            if (g_scratch_state[dev].load(std::memory_order_acquire) != 2) return ETV_ERR_HIP;
        }
    }
    *ptr = g_scratch_ptr[dev];
    return ETV_OK;
}
}  // namespace etv

extern "C" int32_t etv_tree_verify_attention_static(const etv_attn_desc *h, const void *q, const void *k_cache,
                                                    const void *v_cache, const int32_t *block_table,
                                                    const int32_t *prefix_len, const void *kt, const void *vt,
                                                    const uint64_t *bitmask, const int32_t *n_nodes, void *out,
                                                    float *lse, void *stream) {
    if (!h) return ETV_ERR_INVALID_ARG;
    // sizes beyond the array are refused before anything is launched
    if (etv_tree_verify_attention_workspace_bytes(h) > (size_t)ETV_ATTN_STATIC_WORKSPACE_BYTES)
        return ETV_ERR_WORKSPACE_TOO_SMALL;
    void *ws = nullptr;
    const int32_t rc = etv::static_scratch(&ws);
    if (rc != ETV_OK) return rc;
    // Nothing in the array has to start at zero: a launch writes every (m, l, O) partial it later merges, and
    // never reads one it has not written (absent splits and padded rows are skipped), so the last call's
    // contents are harmless.
    return etv::attention_run(h, q, k_cache, v_cache, block_table, prefix_len, kt, vt, bitmask, n_nodes, out, lse, ws,
                              (size_t)ETV_ATTN_STATIC_WORKSPACE_BYTES, stream);
}
