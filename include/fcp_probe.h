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

/*
 * fcp_mfma_valu_probe -- fcp_mfma_probe with vector-ALU work beside the MFMAs: after every MFMA the wave issues
 * valu_per_mfma (0, 2, 4, 6, 8 or 12) independent fp32 FMAs.  Shows what the vector work that an attention kernel
 * has to place between its MFMAs (exponentials, masks, packing) costs the matrix pipe: a SIMD issues one
 * instruction per wave every few cycles, and both kinds share those slots.  FLOPs counted = the MFMAs only.
 */
int fcp_mfma_valu_probe(int32_t operand_kind, int32_t valu_per_mfma, int32_t iters, float* out, void* stream);

/*
 * fcp_lds_probe -- raw LDS throughput of a compute unit for the access patterns of the attention kernels.
 * One workgroup of n_waves (4 or 8) waves per compute unit; every wave issues iters x 16 instructions of one kind:
 *   mode 0: ds_read_b128, 1 KB per instruction (row operands of a swizzled tile)
 *   mode 1: ds_read_b64_tr_b16, 512 B per instruction (transposed operands)
 *   mode 2: ds_write_b128, 1 KB     mode 3: ds_write_b64, 512 B
 *   mode 4: LDS-DMA (global_load_lds_dwordx4), 1 KB per instruction, from `src`, a 64 KB device buffer that stays in
 *           the L2 cache: what a tile load costs on the LDS side.
 * Bytes per compute unit = n_waves x iters x 16 x (bytes per instruction); the caller times the launch.
 * src: device, 64 KB (read in mode 4 only, but required); out: device, one float (contents meaningless).
 */
int fcp_lds_probe(int32_t mode, int32_t n_waves, int32_t iters, const void* src, float* out, void* stream);

/*
 * fcp_atomic_probe -- fp32 atomic adds to memory in the pattern with which a KV-stationary backward would
 * accumulate dQ (per wave and iteration 16 rows of 32 consecutive floats, rows row_stride floats apart): the
 * measurement behind the choice of a backward without atomics.
 * workgroups_per_cu (1..8) workgroups of 4 waves per compute unit, iters iterations each; payload bytes =
 * n_compute_units x workgroups_per_cu x 256 x iters x 16 x 4.  buf: device, n_rows x row_stride floats
 * (n_rows >= 2048, row_stride >= 256), accumulated into.
 */
int fcp_atomic_probe(float* buf, int64_t n_rows, int32_t row_stride, int32_t iters, int32_t workgroups_per_cu, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FCP_PROBE_H_ */
