/*
 * eagletv_probe - measurement aids for the MI355X (gfx950) this library runs on.  No part of the verification
 * step: two kernels of known work whose timing gives the ceilings that the machine actually sustains, to be quoted
 * beside the published peaks when a kernel of libeagletv is placed on its roofline (HBM stream for the prefix
 * K/V of tree_verify_attention, bf16 matrix rate for its two contractions).  Built as its own library
 * (libeagletv_probe.so); libeagletv.so does not depend on it.
 *
 * Conventions as in eagletv.h: device pointers, asynchronous on `stream` (a hipStream_t passed as void*), return
 * 0 or a negative code (-1 invalid argument, -4 launch failure).
 */
#ifndef EAGLETV_PROBE_H
#define EAGLETV_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(ETV_BUILDING)
#define ETVP_API __attribute__((visibility("default")))
#else
#define ETVP_API
#endif

/* One kernel that streams `bytes` (>= 1 MiB, 16-byte aligned) of device memory through 16-byte streaming
 * (nontemporal) loads and discards them: the read bandwidth a read-once stream reaches on this machine.
 * sink: 16 bytes of device memory (written only in a practically impossible case, to keep the loads alive). */
ETVP_API int32_t etvp_hbm_read_probe(const void *buf, size_t bytes, void *sink, void *stream);

/* One kernel in which every wavefront of the chip issues v_mfma_f32_32x32x16_bf16 back to back from registers
 * (four independent accumulator chains, operands with random bits, no memory traffic): the matrix rate the
 * machine sustains at the clock it settles to under this load.  `iters` loop trips of 16 products per wavefront
 * (1 <= iters <= 2^20); etvp_mfma_bf16_probe_flops(iters) is the flop count of one launch (2 * 32*32*16 per
 * product).  sink: at least 4 bytes of device memory, never written in practice. */
ETVP_API double etvp_mfma_bf16_probe_flops(int32_t iters);
ETVP_API int32_t etvp_mfma_bf16_probe(int32_t iters, void *sink, void *stream);

/* The matrix instructions of an attention launch and nothing else (no memory traffic, no barrier, no softmax): 512
 * workgroups of 8 wavefronts, one per compute unit, each wavefront issuing per "tile" the 16 score products (two
 * fresh chains) and 16 value products (four running chains) that the attention kernel issues for 32 query rows and
 * 64 keys, on operands that change from product to product and from tile to tile.  The clock of the chip falls
 * with the switching activity in the matrix cores, so this rate is lower than the loop above reaches on operands
 * that never change; it is what the matrix part of the attention launch costs on this machine.  `tiles`: 1 ..
 * 2^20 (66 is the headline sweep cell: 283 GFLOP per launch); sink as above. */
ETVP_API double etvp_mfma_bf16_live_probe_flops(int32_t tiles);
ETVP_API int32_t etvp_mfma_bf16_live_probe(int32_t tiles, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EAGLETV_PROBE_H */
