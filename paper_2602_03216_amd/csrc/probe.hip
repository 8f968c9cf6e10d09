// Calibration of the matrix-core roofline: the rate of a bare v_mfma_f32_32x32x16_bf16 loop (no
// memory traffic, every SIMD busy) and the shader clock it runs at, for operand values the
// caller supplies.  The published dense peak assumes the maximum clock; the clock the chip
// sustains under matrix load depends on how many operand bits toggle, so the same loop is
// slower on N(0,1)-like data than on zeros.  A benchmark runs this beside the attention kernel
// to report what fraction of the peak a pure MFMA stream reaches on the workload's own values.
#include "tsa_internal.h"

namespace tsa {

namespace {

__global__ __launch_bounds__(256) void mfma_probe_kernel(const u32x4* __restrict__ operands, float* __restrict__ sink,
                                                          long long* __restrict__ clocks, int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {            // 8 x 16 bytes per thread out of the first 64 KiB
    a[i] = __builtin_bit_cast(bf16x8, operands[(threadIdx.x * 8 + i) & 4095]);
    b[i] = __builtin_bit_cast(bf16x8, operands[(threadIdx.x * 8 + 4 + i) & 4095]);
  }
  f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
  const long long t0 = clock64(), w0 = wall_clock64();
  for (int i = 0; i < iters; ++i) {
    c0 = mfma32(a[0], b[0], c0); c1 = mfma32(a[1], b[1], c1); c2 = mfma32(a[2], b[2], c2); c3 = mfma32(a[3], b[3], c3);
    c0 = mfma32(a[1], b[2], c0); c1 = mfma32(a[2], b[3], c1); c2 = mfma32(a[3], b[0], c2); c3 = mfma32(a[0], b[1], c3);
  }
  const long long t1 = clock64(), w1 = wall_clock64();
  sink[blockIdx.x * 256 + threadIdx.x] = c0[0] + c1[1] + c2[2] + c3[3];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    clocks[0] = t1 - t0;                   // shader-clock cycles of the loop
    clocks[1] = w1 - w0;                   // ticks of the constant-rate wall clock over the same span
  }
}

// Streaming copy in 16-byte pieces, grid-stride, non-temporal stores: what a pure mover reaches.
__global__ __launch_bounds__(256) void copy_probe_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, long long n) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < n; i += stride)
    __builtin_nontemporal_store(src[i], dst + i);
}

}  // namespace

hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st) {
  const long long n = (long long)(bytes / 16);
  if (n == 0) return hipSuccess;
  long long blocks = (n + 256 * 4 - 1) / (256 * 4);      // about four pieces per thread
  if (blocks > 65536) blocks = 65536;
  copy_probe_kernel<<<(unsigned)blocks, 256, 0, st>>>((const u32x4*)src, (u32x4*)dst, n);
  return hipGetLastError();
}

hipError_t launch_mfma_probe(const void* operands, int iters, int blocks, float* sink, long long* clocks, hipStream_t st) {
  mfma_probe_kernel<<<blocks, 256, 0, st>>>((const u32x4*)operands, sink, clocks, iters);
  return hipGetLastError();
}

}  // namespace tsa
