/*
 * libtsa -- measurement support.  Nothing here is a step of Token Sparse Attention: these entry points
 * exist for benchmarks that want to state what the chip itself sustains next to a kernel's rate.
 * Same conventions as tsa.h (device pointers owned by the caller, status codes, tsa_last_error()).
 */
#ifndef TSA_BENCH_H
#define TSA_BENCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Matrix-pipe calibration: runs a bare loop of 8 * iters bf16 MFMAs
 * (32x32x16) per wavefront, 4 wavefronts per workgroup, `blocks` workgroups, with operand values taken
 * from `operands`, and records the shader clock it ran at.  The sustained matrix rate of the chip
 * depends on the operand values (clock under power limit); a benchmark uses this to report the
 * rate a pure MFMA stream reaches on the workload's own data beside the published peak.
 *   operands: device, at least 64 KiB of bf16 values;  sink: device, blocks * 256 fp32 (scratch output)
 *   clocks: device int64[2], out: {shader-clock cycles, wall-clock ticks} of workgroup 0's loop
 *   flops (host, out, may be NULL): floating-point operations of the whole launch
 *   wall_clock_khz (host, out, may be NULL): rate of the wall clock in kHz
 * The caller times the launch (events on `stream`) and divides. */
int tsa_mfma_probe(const void* operands, int32_t iters, int32_t blocks, float* sink, int64_t* clocks,
                   double* flops, int32_t* wall_clock_khz, void* stream);


/* Instruction-mix calibration: the MFMA and vector instruction streams of the library's two matrix loops with
 * every operand in registers (no LDS traffic, no global memory, no barrier), two wavefronts per SIMD as in the
 * kernels: what the loops could reach on the given operand values if staging, fragment reads and
 * synchronisation were free.  mix 0: attention, MFMAs alone (per iteration a chain of 8 into one accumulator
 * and 8 into four); 1: attention with its vector work (per MFMA one exp2, one add, half a pack, one fma, half
 * a max3); 2: scoring, MFMAs alone (a chain of 8); 3: scoring with its vector work (per MFMA two fma, two
 * exp2, two adds).  `blocks` workgroups of 4 wavefronts, each pinned to half a CU's LDS (launch 2 per CU);
 *   operands: device, at least 16 KiB of bf16 values;  sink: device, blocks * 256 fp32 (scratch output)
 *   flops (host, out, may be NULL): floating-point operations of the MFMAs of the whole launch
 * The caller times the launch and divides. */
int tsa_mix_probe(int32_t mix, const void* operands, int32_t iters, int32_t blocks, float* sink, double* flops, void* stream);

/* Read-bandwidth calibration: streams `bytes` bytes (a multiple of 16, device, 16-byte aligned) through the
 * chip without writing anything (sink: 4 bytes of device memory that are practically never written): the
 * rate a kernel that only consumes a tensor can reach, as the scoring passes do with K. */
int tsa_read_probe(const void* src, size_t bytes, void* sink, void* stream);

/* Memory-bandwidth calibration: a plain streaming copy dst[i] = src[i] of `bytes` bytes (a multiple of
 * 16; both pointers 16-byte aligned, device) in 16-byte pieces with non-temporal stores, the access
 * pattern of the library's gather / scatter kernels without their indirection.  The caller times the
 * launch; 2 * bytes / time is the rate a mover can reach on this chip. */
int tsa_copy_probe(const void* src, void* dst, size_t bytes, void* stream);

/* Form of the attention kernel for the launches that follow, process-wide: 0 = chosen per launch from
 * the problem size (the default), 1 = 256 query rows per workgroup, 2 = 128 query rows per workgroup with
 * the keys of every tile split over two groups of wavefronts.  Both forms compute the same attention
 * (results agree within rounding, not bit for bit); a benchmark uses this to time one against the other. */
int tsa_bench_set_attend_form(int32_t form);

#ifdef __cplusplus
}
#endif
#endif /* TSA_BENCH_H */
