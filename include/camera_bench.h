/*
 * camera_bench.h -- measured ceilings of the machine, for benchmark reports only.
 *
 * Not part of the product ABI (include/camera.h): nothing here is a step of the method.  The two calls
 * give the measured peaks that the roofline fractions of the grouped contraction (bf16 MFMA) and of the
 * column-norm pass (HBM reads) are set beside.  Built into libcamera_bench.so.
 *
 * Both calls allocate their own device buffer, run on the default stream of `device`, wait for their
 * kernels and free the buffer.  Return 0, or -1 (bad argument), -4 (allocation failed), -5 (HIP error).
 *
 * camera_bench_mfma_bf16: `launches` back-to-back launches (about 4 ms each) of a register-resident
 *   v_mfma_f32_16x16x32_bf16 loop (the instruction of the grouped contraction) on every CU, no LDS and no
 *   memory traffic.  random_operands == 0: all operand elements 1.0 (reaches the published peak); != 0:
 *   random operand values as in a contraction of real data, for which the chip lowers its clock to hold
 *   its power limit.
 *     tflops     HOST out: 10^12 floating-point operations per second over all launches
 *     shader_mhz HOST out: mean shader clock during the kernels (cycle counter / 100 MHz reference)
 * camera_bench_hbm_read: `launches` streaming reads of a `bytes`-long buffer (choose it much larger than
 *   the 256 MB memory-side cache; a multiple of 16 in [2^20, 2^36]); gb_per_s HOST out: 10^9 bytes per second.
 */
#ifndef CAMERA_BENCH_H_
#define CAMERA_BENCH_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

int camera_bench_mfma_bf16(int device, int random_operands, int launches, double* tflops, double* shader_mhz);
int camera_bench_hbm_read(int device, int64_t bytes, int launches, double* gb_per_s);

#ifdef __cplusplus
}
#endif
#endif /* CAMERA_BENCH_H_ */
