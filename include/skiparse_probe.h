/*
 * skiparse_probe.h -- C ABI of the measurement library (libskiparse_probe.so).  NOT part of the attention library: these are
 * micro-kernels that the benchmark times to state what the matrix pipe of the chip sustains by itself, next to the nominal
 * peak, and a helper that reads the device's compute-unit count and clock.  Nothing here computes any part of the method.
 *
 * Conventions: operands / sink are DEVICE pointers owned by the caller (operands 16-byte aligned, sink 4-byte aligned); a call only
 * enqueues one kernel on `stream` (a hipStream_t passed as void*; NULL = the default stream), never allocates, never synchronises.
 * Return value: the error codes of skiparse.h (SKIPARSE_OK, SKIPARSE_EINVAL: null / misaligned pointer or non-positive count,
 * SKIPARSE_EUNSUPPORTED: no such probe, SKIPARSE_EWORKSPACE: a buffer is too small, SKIPARSE_EHIP: the launch failed).
 * Arguments are validated before the first HIP call.
 */
#ifndef SKIPARSE_PROBE_H
#define SKIPARSE_PROBE_H

#include <stddef.h>

#include "skiparse.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * A kernel that issues nothing but matrix-core instructions (32x32x16 bf16 for SKIPARSE_BF16, 32x32x64 fp8 for SKIPARSE_FP8_E4M3)
 * on the caller's operand bytes held in registers: `blocks` workgroups of 4 wavefronts, iters * 4 instructions per wavefront.
 * operands: >= 2048 * 8 bytes of device memory (random values of the element type); sink: >= blocks * 256 floats, overwritten.
 * *flop (host pointer, may be NULL) receives the floating-point operations of one launch.
 */
int skiparse_mfma_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int dtype, int blocks, int iters,
                        double* flop, void* stream);

/*
 * The bf16 loop (iters * 2 instructions per wavefront) with valu_per_mfma (0, 2, 4, 6 or 8) independent v_fma_f32 after every
 * MFMA: shows how much vector-ALU work the matrix pipe hides, which is what limits a softmax placed between two matrix products.
 */
int skiparse_mfma_valu_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int valu_per_mfma, int blocks,
                             int iters, double* flop, void* stream);

/*
 * The bf16 loop (iters * 8 instructions per wavefront) in which the A operand of every MFMA is read from LDS with a 16-byte read
 * per lane: the rate of a loop whose operands come from LDS, under the board's power management.
 */
int skiparse_mfma_lds_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int blocks, int iters, double* flop,
                            void* stream);

/* The same with the 8-bit instruction (32x32x64 fp8, iters * 2 per wavefront) and valu_per_mfma in {0, 4, 8, 12, 16}. */
int skiparse_mfma8_valu_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int valu_per_mfma, int blocks,
                              int iters, double* flop, void* stream);

/*
 * The bf16 loop with `chain` (1, 2, 4 or 8) consecutive MFMAs on the same accumulator before moving to the next of four
 * (iters * 4 * chain instructions per wavefront): whether accumulator reuse inside the matrix pipe changes its sustained rate.
 */
int skiparse_mfma_chain_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int chain, int blocks, int iters,
                              double* flop, void* stream);

/*
 * LDS read instructions only, addressed as the attention kernels address a staged tile of 64 rows of 128 bf16 values: kind 0 = the
 * 16-byte fragment reads (ds_read_b128), kind 1 = the transposing reads (ds_read_b64_tr_b16), kind 2 = plain 8-byte reads at the
 * transposing reads' addresses.  `blocks` workgroups of 8 wavefronts, iters * 16 reads per wavefront.  sink: >= blocks * 512 floats.
 * *bytes (host pointer, may be NULL) receives the bytes read from LDS by one launch.
 */
int skiparse_lds_read_probe(const void* operands, size_t operand_bytes, float* sink, size_t sink_bytes, int kind, int blocks, int iters,
                            double* bytes, void* stream);

/* Compute units and nominal engine clock (kHz) of HIP device `device`, as the runtime reports them (host pointers). */
int skiparse_probe_device_info(int device, int* compute_units, int* clock_khz);

/* The hipError_t (as int) of the last failed call of this library on this thread, 0 if none. */
int skiparse_probe_last_hip_error(void);

#ifdef __cplusplus
}
#endif
#endif /* SKIPARSE_PROBE_H */
