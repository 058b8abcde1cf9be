/*
 * moe_int4.h -- C ABI of the INT4 per-group backup of expert weights (gfx950).
 *
 * The paper's dynamic parallelism transition ("The Dynamic Parallelism Transition Strategy")
 * keeps a 4-bit quantised copy of the expert weights, uploads the part a device needs under the
 * next Expert-module strategy, and dequantises it to the native precision (BF16); of per-tensor,
 * per-channel and per-group quantisation it adopts per-group.  The time of the dequantisation,
 * T_dequant, enters the switching cost and is tabulated against the number of dequantised
 * parameters, V_dequant.  This header is the device side of that: dequantise (the operation on
 * the switching path) and quantise (to build the backup).
 *
 * Format (the paper fixes neither group size nor code book): groups of MOE_INT4_GROUP = 64
 * consecutive weights of the flat tensor, uniform affine codes
 *     scale = bf16((max - min) / 15),  code = clamp(rint((w - min) / scale), 0, 15),
 *     w'    = bf16(min + code * scale)
 * with all arithmetic in fp32 (round to nearest even everywhere); a group whose scale rounds to 0
 * gets code 0 for every weight.
 *   codes   uint8 [n/2]: weight 2i in the low nibble of byte i, weight 2i+1 in the high nibble
 *   qparams bf16  [n/64][2]: (scale, min) of each group
 *
 * Conventions as in moe_shard.h: status codes (MOE_OK / MOE_ERR_*), validation on the host before
 * any HIP call, no allocation, no synchronisation, work enqueued on `stream`; all pointers are
 * DEVICE pointers owned by the caller, 16-byte aligned.  Weights must be finite.
 */
#ifndef MOE_INT4_H
#define MOE_INT4_H

#include "moe_shard.h"

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_INT4_GROUP 64

/*
 * codes [n/2] uint8, qparams [n/64][2] bf16  ->  w_bf16 [n] bf16.
 * Requires n_elems >= 0 and n_elems % 64 == 0.  Reads 0.5625 and writes 2 bytes per weight.
 */
int moe_int4_dequantize(const void* codes, const void* qparams, int64_t n_elems, void* w_bf16, void* stream);

/*
 * w_bf16 [n] bf16  ->  codes [n/2] uint8, qparams [n/64][2] bf16.
 * Requires n_elems >= 0 and n_elems % 64 == 0.
 */
int moe_int4_quantize(const void* w_bf16, int64_t n_elems, void* codes, void* qparams, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_INT4_H */
