// Inter-Layer Representation Drift (Eq. 1 of the paper):
//   R = mean over tokens t of  ||h_out[t] - h_in[t]||_2 / (||h_in[t]||_2 + eps)
// for the hidden states entering and leaving one layer.  A streaming reduction bound by HBM
// bandwidth: one wavefront per token row, 16 bytes per lane per step, fp32 sums of squares,
// per-workgroup partial sums in a fixed order (the result is deterministic), a last small
// kernel adds the partials in fp64.
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kRowsPerBlock = 64;     // rows per workgroup (16 per wavefront)

__global__ __launch_bounds__(kThreads) void drift_rows_kernel(const u32x4* __restrict__ hin, const u32x4* __restrict__ hout,
                                                              long long n_tokens, int width, float eps, double* partial) {
  __shared__ double wsum[kWaves];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int units = width / 8;                      // 16-byte units per row
  double acc = 0.0;
  for (int r = wave; r < kRowsPerBlock; r += kWaves) {
    const long long t = (long long)blockIdx.x * kRowsPerBlock + r;
    if (t >= n_tokens) break;
    float d2 = 0.f, n2 = 0.f;
    for (int u = lane; u < units; u += 64) {
      const u32x4 a = hin[t * units + u], b = hout[t * units + u];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const float a0 = __uint_as_float(a[j] << 16), a1 = __uint_as_float(a[j] & 0xffff0000u);
        const float b0 = __uint_as_float(b[j] << 16), b1 = __uint_as_float(b[j] & 0xffff0000u);
        const float e0 = b0 - a0, e1 = b1 - a1;
        d2 = fmaf(e0, e0, d2); d2 = fmaf(e1, e1, d2);
        n2 = fmaf(a0, a0, n2); n2 = fmaf(a1, a1, n2);
      }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) { d2 += __shfl_xor(d2, d); n2 += __shfl_xor(n2, d); }
    acc += (double)(sqrtf(d2) / (sqrtf(n2) + eps));
  }
  if (lane == 0) wsum[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < kWaves; ++w) s += wsum[w];
    partial[blockIdx.x] = s;
  }
}

__global__ void drift_final_kernel(const double* partial, int n_partial, long long n_tokens, float* out) {
  __shared__ double sh[256];
  double s = 0.0;
  for (int i = threadIdx.x; i < n_partial; i += 256) s += partial[i];
  sh[threadIdx.x] = s;
  __syncthreads();
  for (int d = 128; d >= 1; d >>= 1) {
    if ((int)threadIdx.x < d) sh[threadIdx.x] += sh[threadIdx.x + d];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = (float)(sh[0] / (double)n_tokens);
}

}  // namespace

size_t drift_ws_bytes(long long n_tokens) {
  const size_t blocks = (size_t)((n_tokens + kRowsPerBlock - 1) / kRowsPerBlock);
  return (blocks * sizeof(double) + 255) & ~(size_t)255;
}

hipError_t launch_drift(const void* h_in, const void* h_out, long long n_tokens, int width, float eps, float* out,
                        void* ws, hipStream_t st) {
  const int blocks = (int)((n_tokens + kRowsPerBlock - 1) / kRowsPerBlock);
  drift_rows_kernel<<<blocks, kThreads, 0, st>>>((const u32x4*)h_in, (const u32x4*)h_out, n_tokens, width, eps, (double*)ws);
  drift_final_kernel<<<1, 256, 0, st>>>((const double*)ws, blocks, n_tokens, out);
  return hipGetLastError();
}

}  // namespace tsa
