// Internal declarations shared by the kernel files and the C-ABI layer of libtsa.
// Device code here is written for gfx950 (CDNA4) only: 64-lane wavefronts, bf16 MFMA.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

namespace tsa {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Register layout of v_mfma_f32_32x32x16_bf16 (one wavefront, lane l, lo = l % 32, hi = l / 32):
//   A operand: 8 bf16 = A[row lo][k = 8*hi .. 8*hi+7]
//   B operand: 8 bf16 = B[k = 8*hi .. 8*hi+7][col lo]
//   C/D:       16 fp32, register r = D[row 8*(r/4) + 4*hi + (r%4)][col lo]
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ int c_row(int r, int hi) { return 8 * (r >> 2) + 4 * hi + (r & 3); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Shapes every launcher gets (validated by the C-ABI layer before any launch).
// Element (b, h, t, c) of a full-length tensor sits at b * b_ + h * h_ + t * l_ + c (elements).
struct Strides {
  long long b, h, l;
  __host__ __device__ long long head(long long bi, long long hi) const { return bi * b + hi * h; }
};

struct Dims {
  int B, Hq, Hkv, L, d, last_q, pool_w, group_mode, force_first, force_last, block_list_per_head;
  float scale;
  Strides q, kv, o;            // Q; K and V; O
};

// ---- launchers (each returns hipGetLastError() after queuing its kernels) ----

// score.hip
size_t score_ws_bytes(const Dims& dm);
hipError_t launch_score(const Dims& dm, const void* Q, const void* K, float* scores, void* ws, hipStream_t st);

hipError_t launch_score_queries(const Dims& dm, const void* Qsel, const int32_t* qpos_host, const void* K, float* scores,
                                void* ws, hipStream_t st);
hipError_t launch_gather_queries(const Dims& dm, const void* Q, const int32_t* qpos_host, int n, void* Qsel, hipStream_t st);
size_t pool_queries_ws_bytes(const Dims& dm, int n_pool);
hipError_t launch_pool_queries(const Dims& dm, const void* Q, int n_pool, void* Qsel, void* ws, hipStream_t st);

// select.hip
size_t select_ws_bytes(const Dims& dm);
// k_dev (device, [B], may be NULL): the count of every batch entry as decided on the device; k_keep is
// then the capacity (row stride of idx), and entries of idx past a row's count are left untouched.
hipError_t launch_select(const Dims& dm, const float* scores, int k_keep, int32_t* idx, int32_t* inv,
                         void* ws, hipStream_t st, const int32_t* k_dev = nullptr);

// budget.hip
size_t budget_ws_bytes(const Dims& dm);
// k_max > 0: the result is clamped to it (the capacity of the buffers that will hold the selection);
// k_min: the result is at least max(1, k_min) (the always-kept tokens of the selection that follows)
hipError_t launch_budget(const Dims& dm, const float* scores, double tau_cov, int32_t* k_keep, void* ws, hipStream_t st,
                         int k_max = 0, int k_min = 0);

// drift.hip
size_t drift_ws_bytes(long long n_tokens);
hipError_t launch_drift(const void* h_in, const void* h_out, long long n_tokens, int width, float eps, float* out,
                        void* ws, hipStream_t st);

// gather_scatter.hip
hipError_t launch_compress(const Dims& dm, const void* Q, const void* K, const void* V, const int32_t* idx,
                           int k_keep, void* Qc, void* Kc, void* Vc, hipStream_t st);
// idx may be NULL (rows are then located through inv alone)
hipError_t launch_decompress(const Dims& dm, const void* Oc, const int32_t* idx, const int32_t* inv, int k_keep, void* O,
                             hipStream_t st);
hipError_t launch_residual(const Dims& dm, const void* Oc, const int32_t* idx, int k_keep, void* residual, hipStream_t st);

// The attention kernel reads V as tiled V^T: [B*kv_heads][ceil(Lc/kKeyTile)][d][kKeyTile] bf16 (one d-row
// of a tile = kKeyTile consecutive keys = 128 contiguous bytes), keys past Lc zero.
constexpr int kKeyTile = 64;
inline size_t v_tiles_bytes(int B, int kv_heads, int Lc, int d) {
  return (size_t)B * kv_heads * ((Lc + kKeyTile - 1) / kKeyTile) * kKeyTile * d * 2;
}

// gather_scatter.hip (continued): row-major V -> tiled V^T; and Stage 1 compression writing
// Qc, Kc row-major and V directly as tiled V^T (the form tsa_forward uses).
hipError_t launch_v_tiles(int B, int kv_heads, int Lc, int d, const void* V, void* Vt, hipStream_t st);
hipError_t launch_compress_tiled(const Dims& dm, const void* Q, const void* K, const void* V, const int32_t* idx,
                                 int k_keep, void* Qc, void* Kc, void* Vt, hipStream_t st, const int32_t* k_dev = nullptr);

// attend.hip
hipError_t launch_attend(int B, int Hq, int kv_heads, int Lc, int d, float scale, const void* Qc, const void* Kc,
                         const void* Vt, const int32_t* block_list, int block_size, int max_blocks_per_row,
                         int block_list_per_head, void* Oc, float* lse, hipStream_t st);

// attend.hip, fused form used by tsa_forward: Q and K are the original tensors, rows are gathered
// through idx inside the kernel's loads; Vt = tiles of the gathered V (launch_compress_tiled with
// Qc = Kc = NULL); O [B,Hq,L,d] (may be NULL) receives the rows of selected tokens from the
// epilogue and zeros elsewhere; Oc [B,Hq,k,d] (may be NULL) the compacted output; residual [B,L,Hq*d]
// (may be NULL) gets the output rows added in place.
hipError_t launch_attend_fused(const Dims& dm, const void* Q, const void* K, const void* Vt, const int32_t* idx,
                               const int32_t* inv, int k_keep, const int32_t* block_list, int block_size,
                               int max_blocks_per_row, void* Oc, void* O, void* residual, hipStream_t st,
                               const int32_t* k_dev = nullptr);

// attend.hip: 0 = the form of the attention kernel is chosen per launch (default), 1 = 256 query rows per
// workgroup always, 2 = 128 rows with split keys always (measurement support)
void set_attend_form(int form);

// probe.hip: bare MFMA loop, 8 * iters MFMAs per wavefront, 4 wavefronts per workgroup
hipError_t launch_mfma_probe(const void* operands, int iters, int blocks, float* sink, long long* clocks, hipStream_t st);
// probe.hip: the MFMA / vector instruction streams of the attention (mix 0, 1) and scoring (mix 2, 3) loops on
// register operands; 16 (mix 0, 1) or 8 (mix 2, 3) MFMAs per iteration and wavefront, 4 wavefronts per workgroup
hipError_t launch_mix_probe(int mix, const void* operands, int iters, int blocks, float* sink, hipStream_t st);
// probe.hip: streaming read of `bytes` bytes (a multiple of 16); sink: 4 bytes of device memory
hipError_t launch_read_probe(const void* src, size_t bytes, void* sink, hipStream_t st);
// probe.hip: streaming copy of `bytes` bytes (a multiple of 16)
hipError_t launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t st);

}  // namespace tsa
