/*
 * mfma_rate_probe.h - a measurement aid for benchmarks on MI355X (gfx950): what the matrix cores
 * of the machine at hand sustain.  Not part of the GRASS library or of its C ABI; it is built
 * into libgrass_probe.so and loaded by the benchmark only.
 *
 * mfma_rate_probe launches a kernel that does nothing but issue the bf16 matrix instruction of
 * the compressed-gradient GEMM (v_mfma_f32_32x32x16_bf16) on every compute unit: 256 workgroups
 * x 4 wavefronts x `iters` x 32 instructions, no global memory traffic inside the loop.  The
 * clock the chip sustains under this load depends on what the instructions are fed, hence three
 * operand sources:
 *   MFMA_PROBE_CONSTANTS  small constants held in registers (`operands` is not read);
 *   MFMA_PROBE_REGISTERS  the caller's values, two sets of eight fragments held in registers
 *                         and used alternately;
 *   MFMA_PROBE_LDS        the caller's values staged in LDS once; every group of 16
 *                         instructions reads its eight fragments from there (16 bytes per lane
 *                         and fragment: the LDS read traffic of the GEMM).
 * `operands` (device, 16-byte aligned, at least 65536 bytes, `operand_bytes` says how many):
 * bf16 values; thread t of a workgroup takes elements [(256 f + t) 8, +8) as fragment f = 0..15,
 * fragments 0-3 and 8-11 on the left side of the products, 4-7 and 12-15 on the right.
 * `out` (device, at least 65536 floats, `out_floats` says how many) receives one value per
 * thread so that the work cannot be optimised away; `*flops` (host) receives the number of
 * floating-point operations the launch performs.  `stream`: a hipStream_t as void*; the caller
 * times the launch on it.  Returns MFMA_PROBE_OK or an error code; an error launches nothing.
 */
#ifndef MFMA_RATE_PROBE_H
#define MFMA_RATE_PROBE_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { MFMA_PROBE_CONSTANTS = 0, MFMA_PROBE_REGISTERS = 1, MFMA_PROBE_LDS = 2 };
enum {
    MFMA_PROBE_OK = 0,
    MFMA_PROBE_ERR_NULL = 1,   /* a required pointer is NULL                      */
    MFMA_PROBE_ERR_SIZE = 2,   /* iters < 1, a buffer too small or misaligned     */
    MFMA_PROBE_ERR_SOURCE = 3, /* unknown operand source                          */
    MFMA_PROBE_ERR_DEVICE = 4  /* the launch failed                               */
};

int mfma_rate_probe(int source, const void* operands, size_t operand_bytes, float* out,
                    size_t out_floats, int iters, double* flops, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MFMA_RATE_PROBE_H */
