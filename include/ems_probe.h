/*
 * ems_probe.h -- two measurement kernels that give the machine's own ceilings next to the
 * datasheet figures: a loop of independent bf16 MFMA instructions and a plain vector copy.
 * They are run by the benchmark in the same process as the kernels they are compared with,
 * so both see the same clocks.  Same conventions as ems.h: device pointers owned by the
 * caller, work enqueued on the caller's stream, nothing allocated or synchronised.
 */
#ifndef EMS_PROBE_H
#define EMS_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Enqueues `blocks` blocks of 256 threads; every wave issues iters * 4 independent
 * v_mfma_f32_32x32x16_bf16 (four accumulators in rotation) and stores one value so that the
 * loop is not removed.  Work: blocks * 4 waves * iters * 4 * 32768 flops.
 *   sink   out: device f32 [blocks * 256]
 * Returns an ems_status (ems.h).
 */
int ems_probe_mfma(int32_t blocks, int32_t iters, float* sink, void* hip_stream);

/*
 * Copies `bytes` (a multiple of 16) from src to dst with 16-byte loads and stores, one
 * grid-stride pass: bytes read + bytes written of HBM traffic.
 */
int ems_probe_copy(const void* src, void* dst, size_t bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EMS_PROBE_H */
