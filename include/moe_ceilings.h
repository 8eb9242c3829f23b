/*
 * moe_ceilings.h -- measurement aids, NOT part of the MoE path: the practical ceilings that the
 * benchmark prints beside the published peaks (libmoe_ceilings.so, separate from libmoe_hip.so).
 *
 *   - a register-only MFMA loop: what the matrix cores sustain when nothing but MFMAs runs, on
 *     operand bits of the caller's choice (constants toggle few wires; random data draws more
 *     power and the chip lowers its clock);
 *   - a plain streaming copy and a streaming read: what HBM sustains for the simplest kernels.
 *
 * All pointers are device pointers owned by the caller; calls only enqueue on `stream`
 * (a hipStream_t as void*) and return 0 or a negative value (-1 bad argument, -4 HIP error).
 */
#ifndef MOE_HIP_MOE_CEILINGS_H
#define MOE_HIP_MOE_CEILINGS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Bytes of `operands` below: 2 fragment sets x 6 fragments x 64 lanes x 32 bytes. */
#define MOE_CEILING_OPERAND_BYTES (2 * 6 * 64 * 32)

/* `workgroups` workgroups of 8 waves (two per SIMD, as in the grouped GEMM); every wave keeps a
 * 2 x 4 grid of 32x32 fp32 accumulators and issues 8 MFMAs per iteration, alternating between
 * two fragment sets read once from `operands` (each lane's 32 bytes: 8 bf16 in the first 16
 * bytes, or 32 e4m3 codes).  fp8 = 0: v_mfma_f32_32x32x16_bf16; fp8 = 1: the 32x32x64 f8f6f4
 * form with both block scales 1.  FLOPs = workgroups * 8 * iters * 8 * 2*32*32*K (K = 16 or 64).
 * sink [workgroups * 512] receives one float per lane (keeps the loop alive). */
int moe_ceiling_mfma_loop(int fp8, const void* operands, int iters, int workgroups, float* sink,
                          void* stream);

/* The bf16 loop above with its operands streamed from LDS at the grouped GEMM's ratio (6 fragment
 * reads of 16 bytes per lane for 8 MFMAs): every MFMA sees fresh operand bits and the LDS read path
 * runs beside the matrix cores, still without global loads, barriers or an epilogue.  lds_image:
 * 128 KiB of bf16 values copied into every workgroup's LDS first.  Same FLOP count (K = 16). */
int moe_ceiling_mfma_lds_loop(const void* lds_image, int iters, int workgroups, float* sink,
                              void* stream);

/* The LDS-fed loop with the grouped GEMM's global -> LDS traffic beside it.  Every four iterations
 * (one k-step) the lower four waves of a workgroup issue sixteen 1 KiB direct-to-LDS loads each
 * (64 KiB per workgroup and step) from slice (step mod src_bytes/64 KiB) of src, which all workgroups
 * read alike (L2 hits after the first touch), into the half of the LDS image given by the step's
 * parity.  flags: 1 = issue the loads; 2 = the loading waves wait for their loads at the end of each
 * step; 4 = a workgroup barrier per step.  src [src_bytes] bf16 values, src_bytes a multiple of
 * 64 KiB, at most 1 GiB; iters a multiple of 4.  Same FLOP count as the loops above (K = 16). */
int moe_ceiling_mfma_lds_dma_loop(const void* lds_image, const void* src, size_t src_bytes, int iters,
                                  int flags, int workgroups, float* sink, void* stream);

/* dst[i] = src[i] for `bytes` bytes (multiple of 16), 16 bytes per lane, streaming loads/stores. */
int moe_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream);

/* Reads `bytes` bytes (multiple of 16) once; sink [4096] receives partial sums. */
int moe_ceiling_read(const void* src, size_t bytes, float* sink, void* stream);

#ifdef __cplusplus
}
#endif
#endif
