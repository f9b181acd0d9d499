/*
 * sparsed_diag.h - diagnostics of the MI355X (gfx950) SparseD attention library.
 *
 * Nothing here is part of the method (arXiv 2509.24014) or of the hot path: these calls measure the
 * machine, for reports that put the attention kernels' rates next to what the hardware sustains.
 * Same conventions as sparsed.h (C11, device pointers owned by the caller, status codes).
 */
#ifndef SPARSED_DIAG_H
#define SPARSED_DIAG_H

#include "sparsed.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * The rate (TFLOP/s) this GPU sustains on bf16 32x32x16 matrix instructions alone, operands in
 * registers, 8 waves on every compute unit for `iters` x 32 instructions per wave (iters in
 * [1, 1000000]). random_operands == 0 uses all-zero operands (reaches the published peak); != 0 uses
 * operands with random signs and mantissas, for which the chip settles at a lower clock: the
 * practical ceiling for kernels that multiply real data. SYNCHRONISES the stream. Needs
 * ex->workspace of at least 512 KiB (SPARSED_ERR_WORKSPACE otherwise).
 */
sparsed_status sparsed_probe_mfma_bf16(int32_t random_operands, int32_t iters, double* tflops_out,
                                       const sparsed_exec* ex);

/*
 * The rate this GPU sustains on one kind of fp32 vector instruction alone, in 1e9 lane-operations per
 * second (64 per wave instruction): op 0 = fused multiply-add, op 1 = base-2 exponential. 8 waves on
 * every compute unit issue `iters` x 64 independent instructions each (iters in [1, 1000000]). The
 * softmax side of attention needs one exponential per logit (Sec. 3.1, Eq. 1); the ratio of the two
 * rates says how many ordinary vector instructions that exponential displaces. SYNCHRONISES the
 * stream. Needs ex->workspace of at least 512 KiB (SPARSED_ERR_WORKSPACE otherwise).
 */
sparsed_status sparsed_probe_valu_f32(int32_t op, int32_t iters, double* gops_out, const sparsed_exec* ex);

/*
 * The matrix rate (TFLOP/s) of an attention-like instruction mix with nothing else in the way: the
 * launch of sparsed_probe_mfma_bf16 with random operands, where every matrix instruction is
 * accompanied by `vector_per_mfma` independent fp32 vector instructions (one of 0, 2, 3, 4, 5, 6, 8;
 * every fourth an exp2, the rest fma) and, if lds_operands != 0, takes one operand from a 1 KiB LDS
 * read issued one group earlier. The softmax between the two products of Eq. 1 costs the attention
 * kernels about 5 vector instructions per matrix instruction and K, V reach the matrix cores through
 * LDS, so (5, 1) is the ceiling for such a kernel on this chip: no dependencies, barriers or global
 * loads are in this probe. SYNCHRONISES the stream. Needs ex->workspace of at least 512 KiB
 * (SPARSED_ERR_WORKSPACE otherwise); SPARSED_ERR_RANGE for other values of vector_per_mfma or iters
 * outside [1, 1000000].
 */
sparsed_status sparsed_probe_mix_bf16(int32_t vector_per_mfma, int32_t lds_operands, int32_t iters,
                                      double* tflops_out, const sparsed_exec* ex);

#ifdef __cplusplus
}
#endif
#endif /* SPARSED_DIAG_H */
