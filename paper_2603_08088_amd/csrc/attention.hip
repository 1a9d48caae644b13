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
    int pairs;   // mfma kernel: (head-in-group, row chunk) pairs per KV head
    int wgp;     // mfma kernel: workgroups per (b, kv head, split) = ceil(pairs / 4)
    float scale_log2;
};

constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ int seq_prefix_len(const AttnParams &p, int b) { return clampi(p.prefix_len[b], 0, p.P_max); }
__device__ __forceinline__ int seq_nsplit(const AttnParams &p, int P) { return max(1, (P + p.chunk - 1) / p.chunk); }

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
            if (valid) sc = dot_row<T, D>(sq, kt + tree_row_offset(p, b, kvh, j)) * p.scale_log2;
            tile(sc, valid, min(64, n - t0), [&](int jj) { return vt + tree_row_offset(p, b, kvh, t0 + jj); });
        }
    }
    if (direct) {
        const float inv = 1.f / l;
#pragma unroll
        for (int i = 0; i < DPL; i++) store_elem<T>(out, orow + lane + 64 * i, o[i] * inv);
        if (p.lse && lane == 0) p.lse[((size_t)b * p.Hq + h) * p.T_max + k] = (m + log2f(l)) * kLn2;
    } else {
        const size_t pr = (((size_t)b * p.Hq + h) * p.T_max + k) * p.nsplit + s;
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
template <typename T, int D>
__global__ void __launch_bounds__(D) attn_combine_kernel(AttnParams p) {
    const int k = blockIdx.x, h = blockIdx.y, b = blockIdx.z, c = threadIdx.x;
    const int n = clampi(p.n_nodes[b], 0, p.T_max);
    T *out = static_cast<T *>(p.out);
    const size_t orow = (((size_t)b * p.T_max + k) * p.Hq + h) * D;
    const size_t lrow = ((size_t)b * p.Hq + h) * p.T_max + k;
    if (k >= n) {
        store_elem<T>(out, orow + c, 0.f);
        if (p.lse && c == 0) p.lse[lrow] = -INFINITY;
        return;
    }
    const int nvalid = seq_nsplit(p, seq_prefix_len(p, b));
    const size_t pr = lrow * p.nsplit;
    float M = -INFINITY;
    for (int s = 0; s < nvalid; s++) M = fmaxf(M, p.part_m[pr + s]);
    float L = 0.f, acc = 0.f;
    for (int s = 0; s < nvalid; s++) {
        float ms = p.part_m[pr + s];
        float w = (ms == -INFINITY) ? 0.f : exp2f(ms - M);
        L = fmaf(w, p.part_l[pr + s], L);
        acc = fmaf(w, p.part_o[(pr + s) * D + c], acc);
    }
    store_elem<T>(out, orow + c, acc / L);
    if (p.lse && c == 0) p.lse[lrow] = (M + log2f(L)) * kLn2;
}

// ----------------------------------------------------------------------------------------------
// MFMA kernel (bf16, d = 128).
//
// Work unit: (split, KV head x row group, sequence).  A workgroup has 4 wavefronts; wavefront w owns one
// (query head, row chunk) pair = 32*MT query rows of one head, and all 4 share the K/V tiles of their
// KV head through LDS, so each prefix K/V byte is fetched from HBM once per G*T query rows.
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

constexpr int KT = 64;          // keys per tile
constexpr int K_STRIDE = 272;   // LDS bytes per K row: 256 + 16 (row-to-row bank rotation for 16-byte reads)
constexpr int V_STRIDE = 288;   // LDS bytes per V row: 256 + 32 (bank rotation for the 8-byte transpose reads)
constexpr int LDS_K_BYTES = KT * K_STRIDE;
constexpr int LDS_V_BYTES = KT * V_STRIDE;

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);
    return __builtin_bit_cast(uint32_t, r);
}

template <int MT>
__global__ void __launch_bounds__(256) attn_mfma_kernel(AttnParams p) {
    constexpr int D = 128;
    __shared__ __attribute__((aligned(16))) uint8_t lds_k[LDS_K_BYTES];
    __shared__ __attribute__((aligned(16))) uint8_t lds_v[LDS_V_BYTES];

    const int s = blockIdx.x;
    const int kvh = blockIdx.y / p.wgp, wg = blockIdx.y % p.wgp;
    const int b = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int c32 = lane & 31, hh = lane >> 5;

    const int n = clampi(p.n_nodes[b], 0, p.T_max);
    const int P = seq_prefix_len(p, b);
    const int nvalid = seq_nsplit(p, P);
    if (s >= nvalid) return;  // uniform over the workgroup
    const bool direct = (p.nsplit == 1);

    const int pair = wg * 4 + wave;
    const bool active = pair < p.pairs;
    const int g = active ? pair % p.G : 0;
    const int rc = active ? pair / p.G : 0;
    const int h = kvh * p.G + g;
    const int row0 = rc * 32 * MT;

    const uint16_t *qp = static_cast<const uint16_t *>(p.q);
    // Q as B operand: lane holds query row (row0 + 32*mt + c32), d values 16*kk + 8*hh .. +7
    bf16x8 qreg[MT][8];
    uint64_t mbits[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int kq = row0 + 32 * mt + c32;
        const bool rv = active && kq < n;
        mbits[mt][0] = 0;
        mbits[mt][1] = 0;
        if (rv) {
            const uint64_t *mrow = p.bitmask + ((size_t)b * p.T_max + kq) * p.words;
            mbits[mt][0] = mrow[0];
            if (p.words > 1) mbits[mt][1] = mrow[1];
        }
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            uint4 v = {0, 0, 0, 0};
            if (rv) v = *reinterpret_cast<const uint4 *>(qp + (((size_t)b * p.T_max + kq) * p.Hq + h) * D + 16 * kk + 8 * hh);
            qreg[mt][kk] = __builtin_bit_cast(bf16x8, v);
        }
    }

    f32x16 oacc[MT][4];
    float m_run[MT], l_run[MT];
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        m_run[mt] = -INFINITY;
        l_run[mt] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; db++)
#pragma unroll
            for (int i = 0; i < 16; i++) oacc[mt][db][i] = 0.f;
    }

    const int k0 = s * p.chunk, k1 = min(P, k0 + p.chunk);
    const int npt = (k1 > k0) ? (k1 - k0 + KT - 1) / KT : 0;
    const int ntt = (s == nvalid - 1) ? (n + KT - 1) / KT : 0;
    const int nt = npt + ntt;

    const uint8_t *kc = static_cast<const uint8_t *>(p.k_cache), *vc = static_cast<const uint8_t *>(p.v_cache);
    const uint8_t *ktp = static_cast<const uint8_t *>(p.kt), *vtp = static_cast<const uint8_t *>(p.vt);

    uint4 kreg[4], vreg[4];
    // global -> registers for tile `ti`: thread handles 16-byte part (c & 15) of key (c >> 4), c = tid + 256 j
    auto load_tile = [&](int ti) {
        const bool tree = ti >= npt;
        const int base = tree ? (ti - npt) * KT : k0 + ti * KT;
        const int limit = tree ? n : k1;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int c = tid + 256 * j;
            const int key = base + (c >> 4);
            uint4 kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
            if (key < limit) {
                const size_t off = (tree ? tree_row_offset(p, b, kvh, key) : prefix_row_offset(p, b, kvh, key)) * 2 +
                                   (size_t)(c & 15) * 16;
                kv = *reinterpret_cast<const uint4 *>((tree ? ktp : kc) + off);
                vv = *reinterpret_cast<const uint4 *>((tree ? vtp : vc) + off);
            }
            kreg[j] = kv;
            vreg[j] = vv;
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const int c = tid + 256 * j;
            *reinterpret_cast<uint4 *>(lds_k + (c >> 4) * K_STRIDE + (c & 15) * 16) = kreg[j];
            *reinterpret_cast<uint4 *>(lds_v + (c >> 4) * V_STRIDE + (c & 15) * 16) = vreg[j];
        }
    };

    if (nt > 0) load_tile(0);
    for (int ti = 0; ti < nt; ti++) {
        __syncthreads();  // previous tile fully consumed
        store_tile();
        __syncthreads();
        if (ti + 1 < nt) load_tile(ti + 1);  // in flight during the compute below

        const bool tree = ti >= npt;
        const int base = tree ? (ti - npt) * KT : k0 + ti * KT;
        const int limit = tree ? n : k1;

        // ---- S^T = K Q^T
        f32x16 sacc[2][MT];
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
            for (int mt = 0; mt < MT; mt++)
#pragma unroll
                for (int i = 0; i < 16; i++) sacc[kb][mt][i] = 0.f;
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(lds_k + (32 * kb + c32) * K_STRIDE + (16 * kk + 8 * hh) * 2);
#pragma unroll
                for (int mt = 0; mt < MT; mt++)
                    sacc[kb][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[mt][kk], sacc[kb][mt], 0, 0, 0);
            }
        }

        // ---- mask + online softmax (per query column), P^T packed to bf16
        bf16x8 pfrag[2][MT][2];
        const bool need_mask = tree || (base + KT > limit);
#pragma unroll
        for (int mt = 0; mt < MT; mt++) {
            float tmax = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; kb++)
#pragma unroll
                for (int i = 0; i < 16; i++) {
                    float t = sacc[kb][mt][i] * p.scale_log2;
                    if (need_mask) {
                        const int kin = 32 * kb + 8 * (i >> 2) + 4 * hh + (i & 3);
                        bool vis;
                        if (tree) {
                            const int j = base + kin;  // < 128
                            vis = (mbits[mt][j >> 6] >> (j & 63)) & 1ull;
                        } else {
                            vis = (base + kin) < limit;
                        }
                        t = vis ? t : -INFINITY;
                    }
                    sacc[kb][mt][i] = t;
                    tmax = fmaxf(tmax, t);
                }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float m_new = fmaxf(m_run[mt], tmax);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[mt] - m_use);
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; kb++) {
                uint32_t pk[8];
#pragma unroll
                for (int i = 0; i < 16; i += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(sacc[kb][mt][i] - m_use);
                    const float p1 = __builtin_amdgcn_exp2f(sacc[kb][mt][i + 1] - m_use);
                    psum += p0 + p1;
                    pk[i >> 1] = pack_bf16x2(p0, p1);
                }
                uint4 lo = {pk[0], pk[1], pk[2], pk[3]}, hi = {pk[4], pk[5], pk[6], pk[7]};
                pfrag[kb][mt][0] = __builtin_bit_cast(bf16x8, lo);
                pfrag[kb][mt][1] = __builtin_bit_cast(bf16x8, hi);
            }
            l_run[mt] = l_run[mt] * alpha + psum;
            m_run[mt] = m_new;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int i = 0; i < 16; i++) oacc[mt][db][i] *= alpha;
        }

        // ---- O^T += V^T P^T
        const int g16 = lane >> 4, i16 = lane & 15;
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
            for (int st = 0; st < 2; st++) {
                const int keyb = 32 * kb + 16 * st + 4 * hh + (i16 >> 2);
#pragma unroll
                for (int db = 0; db < 4; db++) {
                    const int col = (32 * db + 16 * (g16 & 1) + 4 * (i16 & 3)) * 2;
                    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
                    const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4 *)(lds_v + keyb * V_STRIDE + col));
                    const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (lds_s16x4 *)(lds_v + (keyb + 8) * V_STRIDE + col));
                    const bf16x4 a0 = __builtin_bit_cast(bf16x4, v0), a1 = __builtin_bit_cast(bf16x4, v1);
                    const bf16x8 a = __builtin_shufflevector(a0, a1, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int mt = 0; mt < MT; mt++)
                        oacc[mt][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pfrag[kb][mt][st], oacc[mt][db], 0, 0, 0);
                }
            }
    }

    // ---- epilogue
    if (!active) return;
    uint16_t *out = static_cast<uint16_t *>(p.out);
#pragma unroll
    for (int mt = 0; mt < MT; mt++) {
        const int kq = row0 + 32 * mt + c32;
        if (kq >= p.T_max) continue;
        const float l_tot = l_run[mt] + __shfl_xor(l_run[mt], 32);
        const size_t lrow = ((size_t)b * p.Hq + h) * p.T_max + kq;
        if (direct) {
            const size_t orow = (((size_t)b * p.T_max + kq) * p.Hq + h) * D;
            const bool rv = kq < n;
            const float inv = rv ? 1.f / l_tot : 0.f;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int ig = 0; ig < 4; ig++) {
                    const int dcol = 32 * db + 8 * ig + 4 * hh;
                    uint2 w;
                    w.x = rv ? pack_bf16x2(oacc[mt][db][4 * ig] * inv, oacc[mt][db][4 * ig + 1] * inv) : 0u;
                    w.y = rv ? pack_bf16x2(oacc[mt][db][4 * ig + 2] * inv, oacc[mt][db][4 * ig + 3] * inv) : 0u;
                    *reinterpret_cast<uint2 *>(out + orow + dcol) = w;
                }
            if (p.lse && hh == 0) p.lse[lrow] = rv ? (m_run[mt] + __builtin_amdgcn_logf(l_tot)) * kLn2 : -INFINITY;
        } else if (kq < n) {
            const size_t pr = lrow * p.nsplit + s;
#pragma unroll
            for (int db = 0; db < 4; db++)
#pragma unroll
                for (int ig = 0; ig < 4; ig++) {
                    const int dcol = 32 * db + 8 * ig + 4 * hh;
                    float4 w = {oacc[mt][db][4 * ig], oacc[mt][db][4 * ig + 1], oacc[mt][db][4 * ig + 2],
                                oacc[mt][db][4 * ig + 3]};
                    *reinterpret_cast<float4 *>(p.part_o + pr * D + dcol) = w;
                }
            if (hh == 0) {
                p.part_m[pr] = m_run[mt];
                p.part_l[pr] = l_tot;
            }
        }
    }
}

// ----------------------------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------------------------
struct Plan {
    bool mfma;
    int mt, pairs, wgp, chunk, nsplit;
};

static bool supported(const etv_attn_desc *h) {
    if (h->B < 0 || h->T_max < 1 || h->Hq < 1 || h->Hkv < 1 || h->d < 1) return false;
    return true;
}

static Plan make_plan(const etv_attn_desc *h) {
    Plan pl{};
    const int tiles = max(1, (h->P_max + KT - 1) / KT);
    pl.mfma = (h->dtype == ETV_BF16 && h->d == 128 && !(h->flags & ETV_ATTN_FLAG_GENERIC));
    long units;
    if (pl.mfma) {
        pl.mt = h->T_max <= 32 ? 1 : 2;
        const int nrc = (h->T_max + 32 * pl.mt - 1) / (32 * pl.mt);
        pl.pairs = (h->Hq / h->Hkv) * nrc;
        pl.wgp = (pl.pairs + 3) / 4;
        units = (long)max(1, h->B) * h->Hkv * pl.wgp;
    } else {
        units = ((long)max(1, h->B) * h->Hq * h->T_max + 7) / 8;  // 8 resident wavefronts ~ one workgroup slot
    }
    int tiles_per_split;
    if (h->kv_split > 0) {
        tiles_per_split = (h->kv_split + KT - 1) / KT;
    } else {
        const long target = 512;  // workgroups wanted in flight: two per compute unit
        long want = (target + units - 1) / units;
        if (want < 1) want = 1;
        if (want > tiles) want = tiles;
        tiles_per_split = (int)((tiles + want - 1) / want);
    }
    pl.chunk = tiles_per_split * KT;
    pl.nsplit = (tiles + tiles_per_split - 1) / tiles_per_split;
    return pl;
}

}  // namespace etv

extern "C" size_t etv_tree_verify_attention_workspace_bytes(const etv_attn_desc *h) {
    if (!h || !etv::supported(h) || h->B == 0) return 0;
    etv::Plan pl = etv::make_plan(h);
    if (pl.nsplit <= 1) return 256;
    size_t rows = (size_t)h->B * h->Hq * h->T_max * pl.nsplit;
    return rows * ((size_t)h->d + 2) * sizeof(float) + 512;
}

extern "C" int32_t etv_tree_verify_attention(const etv_attn_desc *h, const void *q, const void *k_cache,
                                             const void *v_cache, const int32_t *block_table,
                                             const int32_t *prefix_len, const void *kt, const void *vt,
                                             const uint64_t *bitmask, const int32_t *n_nodes, void *out, float *lse,
                                             void *workspace, size_t workspace_bytes, void *stream) {
    using namespace etv;
    if (!h || !q || !prefix_len || !kt || !vt || !bitmask || !n_nodes || !out) return ETV_ERR_INVALID_ARG;
    if (!supported(h)) return ETV_ERR_INVALID_ARG;
    if (h->Hq % h->Hkv != 0) return ETV_ERR_INVALID_ARG;
    if (h->dtype != ETV_F32 && h->dtype != ETV_BF16) return ETV_ERR_UNSUPPORTED;
    if (h->d != 64 && h->d != 128) return ETV_ERR_UNSUPPORTED;
    if (h->T_max > ETV_ATTN_MAX_TREE) return ETV_ERR_UNSUPPORTED;
    if (h->P_max < 0) return ETV_ERR_INVALID_ARG;
    if (h->block_size != 0 && h->block_size != 16) return ETV_ERR_UNSUPPORTED;
    if (h->block_size > 0 && (!block_table || h->max_blocks < 1)) return ETV_ERR_INVALID_ARG;
    if (h->block_size > 0 && (long)h->P_max > (long)h->max_blocks * h->block_size) return ETV_ERR_INVALID_ARG;
    if (h->block_size == 0 && h->P_max > h->P_cap) return ETV_ERR_INVALID_ARG;
    if (h->P_max > 0 && (!k_cache || !v_cache)) return ETV_ERR_INVALID_ARG;
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
    }
    hipStream_t st = as_stream(stream);
    if (pl.mfma) {
        dim3 grid(pl.nsplit, h->Hkv * pl.wgp, h->B);
        if (pl.mt == 1)
            hipLaunchKernelGGL(attn_mfma_kernel<1>, grid, dim3(256), 0, st, p);
        else
            hipLaunchKernelGGL(attn_mfma_kernel<2>, grid, dim3(256), 0, st, p);
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
    }
    int32_t rc = check_launch();
    if (rc != ETV_OK || pl.nsplit == 1) return rc;
    dim3 cgrid(h->T_max, h->Hq, h->B);
    if (h->dtype == ETV_F32 && h->d == 64)
        hipLaunchKernelGGL((attn_combine_kernel<float, 64>), cgrid, dim3(64), 0, st, p);
    else if (h->dtype == ETV_F32)
        hipLaunchKernelGGL((attn_combine_kernel<float, 128>), cgrid, dim3(128), 0, st, p);
    else if (h->d == 64)
        hipLaunchKernelGGL((attn_combine_kernel<uint16_t, 64>), cgrid, dim3(64), 0, st, p);
    else
        hipLaunchKernelGGL((attn_combine_kernel<uint16_t, 128>), cgrid, dim3(128), 0, st, p);
    return check_launch();
}
