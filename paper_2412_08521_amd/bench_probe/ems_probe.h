/*
 * ems_probe.h -- measurement kernels for the benchmark, built into their own shared object
 * (libems_probe.so): they are not part of the product library or its interface.  They give the
 * machine's own ceilings next to the datasheet figures: a loop of bf16 MFMA instructions (on
 * constant operands, or on operands read from a caller's buffer: random data toggles far more
 * logic, and the power limit then sets a lower clock) and a plain vector copy.  Run in the same
 * process as the kernels they are compared with, so both see the same clocks.  Device pointers
 * owned by the caller, work enqueued on the caller's stream, nothing allocated or synchronised.
 * Return values: 0 ok, -1 invalid argument, -4 launch failed.
 */
#ifndef EMS_PROBE_H
#define EMS_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EMS_PROBE_OPERAND_BYTES 65536   /* size of the operand buffer ems_probe_mfma reads */

/*
 * Enqueues `blocks` blocks of 256 threads; every wave issues iters * 32 v_mfma_f32_32x32x16_bf16
 * (four accumulators in rotation over 8 A and 8 B operand fragments) and stores one value so
 * that the loop is not removed.  Work: blocks * 4 waves * iters * 32 * 32768 flops.
 *   operands  in: device, EMS_PROBE_OPERAND_BYTES of bf16 values the fragments are read from,
 *             or NULL for built-in constants
 *   sink      out: device f32 [blocks * 256]
 */
int ems_probe_mfma(int32_t blocks, int32_t iters, const void* operands, float* sink, void* hip_stream);

/*
 * Copies `bytes` (a multiple of 16) from src to dst with 16-byte loads and stores, one
 * grid-stride pass: bytes read + bytes written of HBM traffic.
 */
int ems_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EMS_PROBE_H */
