/*
 * pdelta_probes.h - bench helpers of the pdelta library: small kernels that measure what the
 * GPU itself sustains, built with the same toolchain and flags as the product kernels, so that
 * "fraction of peak" can be read next to "fraction of what this box achieves".  They are not
 * part of the method (nothing of the paper is computed here) and no product entry point calls
 * them; bench.py does.
 *
 * Conventions as in pdelta.h: device pointers owned by the caller, `stream` is a hipStream_t
 * passed as void*, the call enqueues and returns, a pdelta_status comes back, arguments are
 * checked on the host before any HIP call.
 */
#ifndef PDELTA_PROBES_H
#define PDELTA_PROBES_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Read-only stream: every byte of [src, src + bytes) is loaded exactly once with 16-byte loads
 * (consecutive lanes on consecutive 16 bytes, several loads in flight per lane) and folded into
 * a checksum that is written to `sink` only if it equals a value it cannot take, so the kernel
 * reads and never writes.  The achieved read bandwidth is bytes / kernel time.
 *   src    in   device memory, 16-byte aligned; bytes must be a positive multiple of 16
 *   sink   out  device memory of at least 16 bytes, 16-byte aligned (practically never written)
 * PDELTA_EINVAL / PDELTA_EALIGN / PDELTA_ESHAPE (bytes not a multiple of 16) as elsewhere.
 */
int pdelta_probe_read_stream(const void* src, size_t bytes, void* sink, void* stream);

/*
 * Matrix-core ceiling: every wave of a grid that fills the chip (256 workgroups) issues `iters`
 * groups of four independent v_mfma_f32_32x32x16_f16 and nothing else.  Rate = 256 workgroups x
 * waves x iters x 4 x 32768 flop / kernel time.
 *   waves_per_simd   1, 2 or 4 (workgroups of 4, 8 or 16 waves, one workgroup per compute unit)
 *   random_operands  0: every operand element is 1.0 (the rate the nameplate figure assumes);
 *                    1: operands are pseudo-random fp16 values in [-2, 2) from a hash of lane and
 *                       register index (what a multiplication of real data toggles)
 *   sink             device memory of at least 16 bytes (practically never written)
 * PDELTA_EINVAL for other waves_per_simd / random_operands values or iters < 1.
 */
int pdelta_probe_mfma(int waves_per_simd, int random_operands, int iters, void* sink, void* stream);

/*
 * Where a prefill launch spends its time: the product's prefill kernel for more than 128 tokens
 * (bf16 X and W_b, row scales; the operation is the delta linear layer of paper Eq. 1, arguments as
 * pdelta_linear_row) built with parts of its inner loop compiled out.  `parts` is a bit mask of
 * what stays: 1 the global loads of the steady loop, 2 the bf16 -> fp16 conversion, sign / scale
 * add and LDS writes, 4 the fragment reads from LDS, 8 the MFMAs.  15 is the product kernel itself
 * and writes the same Y as pdelta_linear_row, bit for bit; with any other mask Y is written with
 * meaningless values (all accesses stay in bounds).  Built masks: 0, 1, 2, 3, 4, 8, 12, 13, 14, 15.
 *   M > 128 (PDELTA_ESHAPE otherwise); other checks and status values as pdelta_linear_row;
 *   PDELTA_EINVAL for a mask that is not built.
 */
int pdelta_probe_prefill_parts(int parts, const void* X, const void* W_b, const uint32_t* B_packed,
                               const uint16_t* v_row, void* Y, int64_t M, int64_t d_out, int64_t d_in,
                               int y_dtype, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* PDELTA_PROBES_H */
