/*
 * vmonarch_bench.h -- measurement aids of libvmonarch (not part of the method's interface): phase
 * timing of vmonarch_attention and a probe of the bare matrix instruction.  Conventions as in
 * vmonarch.h (device pointers unless "host", stream as void*, negative error codes).
 */
#ifndef VMONARCH_BENCH_H_
#define VMONARCH_BENCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* While enabled, vmonarch_attention[_f32] records a HIP event on the caller's
 * stream before each of its phases ("r_update", "l_update", "r_update_last", "l_update_last",
 * "first_frame" or "sink_average") and one at the end.  vmonarch_get_phase_timing waits for the last call's
 * final event and writes, for up to `cap` phases, the elapsed milliseconds to ms_host[i] and
 * the phase name to names_host + 32*i (HOST buffers of cap floats / cap*32 chars).  A phase
 * may span more than one kernel launch.  Not thread-safe; off by default. */
int vmonarch_set_phase_timing(int enable);
int vmonarch_get_phase_timing(int* n_phases, float* ms_host, char* names_host, int cap);

/*
 * The sustained rate of the bf16 matrix instruction the MFMA kernels are built
 * on (v_mfma_f32_32x32x16_bf16) with nothing else running, on operand data the caller
 * supplies.  Launches `blocks` workgroups of 8 waves; every lane reads 8 x 16 bytes from
 * `operands` (device, blocks * 512 * 128 bytes: 4 A and 4 B operands per lane) and issues
 * 8 * iters MFMAs on four accumulators; one float per lane goes to `out` (device,
 * blocks * 512 floats) so that the work is not optimised away.  *flops_host (HOST, may be
 * NULL) receives the floating-point operations of the launch.  The matrix pipe is
 * power-limited: the rate measured with random operands is lower than with zeros.
 */
int vmonarch_mfma_probe(const void* operands, float* out, int blocks, int iters, double* flops_host,
                        void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VMONARCH_BENCH_H_ */
