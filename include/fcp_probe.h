/*
 * fcp_probe.h -- measurement aids of the MI355X block-attention library.  Not part of the method and not
 * needed by any caller of fcp.h: these entry points launch synthetic kernels whose only purpose is to show what
 * one unit of the chip sustains (matrix pipes, LDS, vector ALU, memory atomics), so that the design choices of
 * the attention kernels can be checked against numbers measured on the machine they run on.  bench.py reports
 * them; nothing in the product path calls them.
 *
 * Conventions as in fcp.h: C ABI, FCP_OK or a negative fcp_status, text via fcp_last_error(); every kernel is
 * enqueued on the given hipStream_t and the call returns without waiting; the caller times the launch.
 */
#ifndef FCP_PROBE_H_
#define FCP_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * fcp_mfma_probe -- measurement aid, not part of the method: what the matrix pipes of this chip
 * sustain on the attention kernels' MFMA (v_mfma_f32_32x32x16_bf16) for given operand VALUES.
 *
 * Launches one kernel on `stream`: one workgroup of 8 waves per compute unit (two waves per SIMD,
 * as in the attention kernels), each wave issuing iters x 16 back-to-back MFMAs on operands held in
 * registers -- no LDS, no memory traffic, no other vector work.  The caller times the launch;
 * FLOPs = n_compute_units x 8 x iters x 16 x 32768.  The rate depends on the operand values because
 * the chip lowers its clock to stay inside its power limit: zeros or constants run near the published
 * peak, random values well below it.
 * operand_kind: 0 = zeros, 1 = every element 0.5, 2 = pseudo-random, approximately N(0,1).
 * out: device, at least 8 x n_compute_units floats (one checksum per wave; contents meaningless).
 * Errors: FCP_ERR_INVALID_ARG (NULL out, iters <= 0, unknown kind), FCP_ERR_HIP.
 */
int fcp_mfma_probe(int32_t operand_kind, int32_t iters, float* out, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FCP_PROBE_H_ */
