// Measurement aids (libeagletv_probe.so): a streaming read of device memory and a register-only MFMA loop.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "eagletv_probe.h"

namespace etvp {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// Streaming read with 16-byte nontemporal loads, 8 in flight per lane.
__global__ void __launch_bounds__(256) hbm_read_probe_kernel(const u32x4 *__restrict__ src, size_t n16, u32x4 *sink) {
    const size_t per_wg = n16 / gridDim.x;
    const u32x4 *p = src + per_wg * blockIdx.x;
    u32x4 acc = {0, 0, 0, 0};
    for (size_t i = threadIdx.x; i + 7 * 256 < per_wg; i += 256 * 8) {
        u32x4 v[8];
#pragma unroll
        for (int u = 0; u < 8; u++) v[u] = __builtin_nontemporal_load(p + i + u * 256);
#pragma unroll
        for (int u = 0; u < 8; u++) acc ^= v[u];
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u) sink[0] = acc;  // keeps the loads alive
}

constexpr int kMfmaGrid = 2048;         // workgroups of 4 wavefronts: 8 per compute unit, two resident per SIMD
constexpr int kMfmaPerIter = 16;

__device__ __forceinline__ uint32_t mix(uint32_t x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}

// Operands: bf16 values with random sign and mantissa and an exponent that keeps |x| in [0.5, 2), so the
// multipliers see realistic bit activity (an all-zero loop draws less power and clocks higher than real work).
__global__ void __launch_bounds__(256, 2) mfma_bf16_probe_kernel(int iters, float *sink) {
    bf16x8 a[4], b[4];
    const uint32_t id = blockIdx.x * 256u + threadIdx.x;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        uint32_t wa[4], wb[4];
#pragma unroll
        for (int j = 0; j < 4; j++) {
            const uint32_t ra = mix(id * 64u + i * 8u + j), rb = mix(id * 64u + 32u + i * 8u + j);
            // two bf16 per word: sign 1, exponent 126 or 127, 7 mantissa bits
            wa[j] = (ra & 0x80ff80ffu) | 0x3f003f00u;
            wb[j] = (rb & 0x80ff80ffu) | 0x3f003f00u;
        }
        const u32x4 va = {wa[0], wa[1], wa[2], wa[3]}, vb = {wb[0], wb[1], wb[2], wb[3]};
        a[i] = __builtin_bit_cast(bf16x8, va);
        b[i] = __builtin_bit_cast(bf16x8, vb);
    }
    f32x16 acc[4];
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
        for (int i = 0; i < 16; i++) acc[c][i] = 0.f;
    for (int it = 0; it < iters; it++) {
#pragma unroll
        for (int u = 0; u < 4; u++)
#pragma unroll
            for (int c = 0; c < 4; c++)
                acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(u + c) & 3], b[u], acc[c], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
        for (int i = 0; i < 16; i++) s += acc[c][i];
    if (iters < 0) sink[0] = s;  // never true: keeps the products alive
}

// The matrix instructions of an attention launch and nothing else: 512 workgroups of 8 wavefronts, one workgroup per
// compute unit (two wavefronts per SIMD, two rounds on 256 compute units); per 64-key "tile" a wavefront issues 16 score
// products (two fresh chains of eight) and 16 value products (four running chains), as the attention kernel does for
// 32 query rows.  Unlike the loop above the operands change from product to product and from tile to tile: the "K"
// and "V" fragments are re-randomised every tile (sign and mantissa bits), the "P" operands are made from the bits of
// the scores just computed.  No memory traffic, no barrier, nothing to wait for.
constexpr int kLiveGrid = 512;
__global__ void __launch_bounds__(512, 2) mfma_bf16_live_probe_kernel(int tiles, float *sink) {
    extern __shared__ uint32_t occupy[];     // 96 KiB of dynamic LDS: keeps a second workgroup off the compute unit
    const uint32_t id = blockIdx.x * 512u + threadIdx.x;
    if (tiles < 0) occupy[threadIdx.x] = id;  // never true
    u32x4 kf[8], vf[8], q[8];
#pragma unroll
    for (int i = 0; i < 8; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) {
            kf[i][j] = (mix(id * 128u + i * 4u + j) & 0x80ff80ffu) | 0x3f003f00u;
            vf[i][j] = (mix(id * 128u + 32u + i * 4u + j) & 0x80ff80ffu) | 0x3f003f00u;
            q[i][j] = (mix(id * 128u + 64u + i * 4u + j) & 0x80ff80ffu) | 0x3f003f00u;
        }
    f32x16 o[4];
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
        for (int i = 0; i < 16; i++) o[c][i] = 0.f;
    uint32_t salt = mix(id);
    for (int t = 0; t < tiles; t++) {
        f32x16 s0, s1;
#pragma unroll
        for (int i = 0; i < 16; i++) { s0[i] = 0.f; s1[i] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < 8; kk++) {
            s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, kf[kk]), __builtin_bit_cast(bf16x8, q[kk]), s0, 0, 0, 0);
            s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[kk]), __builtin_bit_cast(bf16x8, q[kk]), s1, 0, 0, 0);
        }
        // "probabilities": bf16 pairs in [0.5, 2) with the sign and mantissa bits of the scores
        u32x4 pf[4];
#pragma unroll
        for (int i = 0; i < 4; i++)
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float x = (i & 1) ? s1[4 * (i >> 1) + j] : s0[4 * (i >> 1) + j];
                pf[i][j] = (__float_as_uint(x) & 0x807f807fu) | 0x3f003f00u;
            }
#pragma unroll
        for (int st = 0; st < 4; st++)
#pragma unroll
            for (int c = 0; c < 4; c++)
                o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, (st & 1) ? vf[(st + c) & 7] : kf[(st + c) & 7]),
                                                               __builtin_bit_cast(bf16x8, pf[st]), o[c], 0, 0, 0);
        // the next tile's fragments: new sign and mantissa bits
        salt = salt * 1664525u + 1013904223u;
#pragma unroll
        for (int i = 0; i < 8; i++) {
            kf[i][i & 3] ^= (salt >> i) & 0x807f807fu;
            vf[i][(i + 1) & 3] ^= (salt << i) & 0x807f807fu;
        }
    }
    float acc = 0.f;
#pragma unroll
    for (int c = 0; c < 4; c++)
#pragma unroll
        for (int i = 0; i < 16; i++) acc += o[c][i];
    if (tiles < 0) sink[0] = acc + (float)occupy[0];  // never true: keeps the products alive
}

}  // namespace etvp

extern "C" int32_t etvp_hbm_read_probe(const void *buf, size_t bytes, void *sink, void *stream) {
    if (!buf || !sink || bytes < (size_t)1 << 20 || ((uintptr_t)buf & 15) || ((uintptr_t)sink & 15)) return -1;
    hipLaunchKernelGGL(etvp::hbm_read_probe_kernel, dim3(4096), dim3(256), 0, reinterpret_cast<hipStream_t>(stream),
                       static_cast<const etvp::u32x4 *>(buf), bytes / 16, static_cast<etvp::u32x4 *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" double etvp_mfma_bf16_probe_flops(int32_t iters) {
    return (double)etvp::kMfmaGrid * 4.0 * (double)iters * etvp::kMfmaPerIter * (2.0 * 32 * 32 * 16);
}

extern "C" int32_t etvp_mfma_bf16_probe(int32_t iters, void *sink, void *stream) {
    if (!sink || iters < 1 || iters > (1 << 20)) return -1;
    hipLaunchKernelGGL(etvp::mfma_bf16_probe_kernel, dim3(etvp::kMfmaGrid), dim3(256), 0,
                       reinterpret_cast<hipStream_t>(stream), iters, static_cast<float *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -4;
}

extern "C" double etvp_mfma_bf16_live_probe_flops(int32_t tiles) {
    return (double)etvp::kLiveGrid * 8.0 * (double)tiles * 32.0 * (2.0 * 32 * 32 * 16);
}

extern "C" int32_t etvp_mfma_bf16_live_probe(int32_t tiles, void *sink, void *stream) {
    if (!sink || tiles < 1 || tiles > (1 << 20)) return -1;
    constexpr int lds = 96 * 1024;
    static const bool lds_ok = hipFuncSetAttribute(reinterpret_cast<const void *>(&etvp::mfma_bf16_live_probe_kernel),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, lds) == hipSuccess;
    if (!lds_ok) return -4;
    hipLaunchKernelGGL(etvp::mfma_bf16_live_probe_kernel, dim3(etvp::kLiveGrid), dim3(512), lds,
                       reinterpret_cast<hipStream_t>(stream), tiles, static_cast<float *>(sink));
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
