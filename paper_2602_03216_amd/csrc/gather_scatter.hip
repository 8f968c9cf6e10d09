// Stage 1 compression (row gather of Q, K, V by S_h) and Stage 2 decompression (scatter of
// the compressed output into a zero-filled full-length tensor, or into the residual stream).
// Section 2.2 of the paper.  All three are pure data movement, bound by HBM bandwidth:
// every lane moves 16 bytes, a row of d bf16 values is covered by d/8 adjacent lanes, so a
// wavefront reads and writes whole rows as contiguous 128- or 256-byte segments.
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 256;

// strides of a full-length tensor in 16-byte pieces (the kernels below move u32x4)
inline Strides pieces(const Strides& s) { return Strides{s.b / 8, s.h / 8, s.l / 8}; }

// Where row (bh, t) of the full-length output starts, in 16-byte pieces.  The contiguous layout keeps the
// plain product (no division by the head count in kernels that run at the memory rate).
struct OutMap {
  Strides s;
  int H, L, contiguous;
  __device__ __forceinline__ long long row(long long bh, int t) const {
    if (contiguous) return (bh * L + t) * s.l;
    const int i = (int)bh;                    // B * Hq is at most 65535
    return s.head(i / H, i % H) + t * s.l;
  }
  __device__ __forceinline__ long long flat(long long task) const {   // task = bh * L + t
    if (contiguous) return task * s.l;
    const int i = (int)(task / L);
    return s.head(i / H, i % H) + (task - (long long)i * L) * s.l;
  }
};
inline OutMap out_map(const Dims& dm) {
  OutMap m;
  m.s = pieces(dm.o); m.H = dm.Hq; m.L = dm.L;
  m.contiguous = dm.o.h == (long long)dm.L * dm.o.l && dm.o.b == (long long)dm.Hq * dm.o.h;
  return m;
}

// One task = one compacted row (b, h, r): copy Q[b,h,S[r],:] -> Qc[b,h,r,:] and the K, V rows
// of KV head h/g.  LPR lanes per row (d/8).
template <int LPR>
__global__ __launch_bounds__(kThreads) void compress_kernel(
    const u32x4* __restrict__ Q, const u32x4* __restrict__ K, const u32x4* __restrict__ V,
    const int32_t* __restrict__ idx, u32x4* __restrict__ Qc, u32x4* __restrict__ Kc, u32x4* __restrict__ Vc,
    int Hq, int Hkv, int L, int k, int group_mode, long long n_tasks, Strides qs, Strides ks) {
  const long long gtid = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long task = gtid / LPR;
  const int lane = (int)(gtid % LPR);
  if (task >= n_tasks) return;
  const int r = (int)(task % k);
  const long long bh = task / k;            // b * Hq + h
  const int h = (int)(bh % Hq);
  const long long b = bh / Hq;
  const int g = Hq / Hkv;
  const int kv = h / g;
  const long long bkv = b * Hkv + kv;
  const long long sel_head = group_mode ? bkv : bh;
  const int t = idx[sel_head * k + r];
  // LPR 16-byte units per row
  const long long kv_at = ks.head(b, kv) + t * ks.l + lane;
  Qc[(bh * k + r) * LPR + lane] = Q[qs.head(b, h) + t * qs.l + lane];
  if (group_mode == 0) {
    Kc[(bh * k + r) * LPR + lane] = K[kv_at];
    Vc[(bh * k + r) * LPR + lane] = V[kv_at];
  } else if (h % g == 0) {
    Kc[(bkv * k + r) * LPR + lane] = K[kv_at];
    Vc[(bkv * k + r) * LPR + lane] = V[kv_at];
  }
}

// One task = one output row (b, h, t): O[b,h,t,:] = inv[t] >= 0 ? Oc[b,h,inv[t],:] : 0.
// A thread serves kRowsPerThread rows a quarter of the tensor apart (independent loads in
// flight); O is written once and not read again by this kernel: streaming stores.
constexpr int kRowsPerThread = 4;
constexpr int kStrideSkew = 1000;   // rows added to the quarter-tensor spacing of a thread's rows
template <int LPR>
__global__ __launch_bounds__(kThreads) void decompress_kernel(
    const u32x4* __restrict__ Oc, const int32_t* __restrict__ inv, u32x4* __restrict__ O,
    int Hq, int g_sel, int L, int k, long long n_tasks, long long stride_tasks, OutMap om) {
  const long long gtid = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long task0 = gtid / LPR;
  const int lane = (int)(gtid % LPR);
  if (task0 >= stride_tasks) return;
  int r[kRowsPerThread];
  long long bh[kRowsPerThread];
  int t[kRowsPerThread];
#pragma unroll
  for (int j = 0; j < kRowsPerThread; ++j) {
    const long long task = task0 + j * stride_tasks;
    r[j] = -1;
    if (task < n_tasks) {
      t[j] = (int)(task % L);
      bh[j] = task / L;
      r[j] = inv[(bh[j] / g_sel) * L + t[j]];           // g_sel = 1 (per-head sets) or Hq/Hkv (per-group sets)
    }
  }
  u32x4 v[kRowsPerThread];
#pragma unroll
  for (int j = 0; j < kRowsPerThread; ++j) {
    v[j] = u32x4{0u, 0u, 0u, 0u};
    if (r[j] >= 0) v[j] = Oc[(bh[j] * k + r[j]) * LPR + lane];
  }
#pragma unroll
  for (int j = 0; j < kRowsPerThread; ++j) {
    const long long task = task0 + j * stride_tasks;
    if (task < n_tasks) __builtin_nontemporal_store(v[j], &O[om.row(bh[j], t[j]) + lane]);
  }
}

// The same result from two independent streams, for callers that also have S_h: workgroups of
// the first part copy compacted row r to O[S_h[r]] (the row's load does not wait for the index
// look-up, only its store does); workgroups of the second part write zeros to the rows inv marks
// unselected.  No thread has two dependent loads in a row.
template <int LPR>
__global__ __launch_bounds__(kThreads) void decompress_split_kernel(
    const u32x4* __restrict__ Oc, const int32_t* __restrict__ idx, const int32_t* __restrict__ inv, u32x4* __restrict__ O,
    int g_sel, int L, int k, long long n_copy, long long n_rows, unsigned copy_blocks, OutMap om) {
  if (blockIdx.x < copy_blocks) {
    const long long gtid = (long long)blockIdx.x * kThreads + threadIdx.x;
    const long long task = gtid / LPR;               // (bh, r)
    const int lane = (int)(gtid % LPR);
    if (task >= n_copy) return;
    const int r = (int)(task % k);
    const long long bh = task / k;
    const int t = idx[(bh / g_sel) * k + r];
    const u32x4 v = Oc[task * LPR + lane];
    __builtin_nontemporal_store(v, &O[om.row(bh, t) + lane]);
    return;
  }
  const long long gtid = (long long)(blockIdx.x - copy_blocks) * kThreads + threadIdx.x;
  const long long stride = (n_rows + kRowsPerThread - 1) / kRowsPerThread + kStrideSkew;
  const long long task0 = gtid / LPR;
  const int lane = (int)(gtid % LPR);
  if (task0 >= stride) return;
  int r[kRowsPerThread];
#pragma unroll
  for (int j = 0; j < kRowsPerThread; ++j) {
    const long long task = task0 + j * stride;       // (bh, t)
    r[j] = 0;
    if (task < n_rows) r[j] = inv[(task / L / g_sel) * L + task % L];
  }
#pragma unroll
  for (int j = 0; j < kRowsPerThread; ++j) {
    const long long task = task0 + j * stride;
    if (r[j] < 0) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, &O[om.flat(task) + lane]);
  }
}

__device__ __forceinline__ uint32_t add_bf16_pair(uint32_t x, uint32_t o) {
  // two bf16 in one dword: widen to fp32 (exact), add, round each sum to bf16 (nearest even)
  const float x0 = __uint_as_float(x << 16), x1 = __uint_as_float(x & 0xffff0000u);
  const float o0 = __uint_as_float(o << 16), o1 = __uint_as_float(o & 0xffff0000u);
  bf16x2 s;
  s[0] = (__bf16)(x0 + o0);
  s[1] = (__bf16)(x1 + o1);
  return __builtin_bit_cast(uint32_t, s);
}

// One task = one compacted row (b, h, r): residual[b, S[r], h*d:(h+1)*d] += Oc[b,h,r,:].
template <int LPR>
__global__ __launch_bounds__(kThreads) void residual_kernel(
    const u32x4* __restrict__ Oc, const int32_t* __restrict__ idx, u32x4* __restrict__ X,
    int Hq, int g_sel, int L, int k, long long n_tasks) {
  const long long gtid = (long long)blockIdx.x * kThreads + threadIdx.x;
  const long long task = gtid / LPR;
  const int lane = (int)(gtid % LPR);
  if (task >= n_tasks) return;
  const int r = (int)(task % k);
  const long long bh = task / k;
  const int h = (int)(bh % Hq);
  const long long b = bh / Hq;
  const int t = idx[(bh / g_sel) * k + r];
  const u32x4 o = Oc[(bh * k + r) * LPR + lane];
  u32x4* px = X + ((b * L + t) * Hq + h) * LPR + lane;
  u32x4 x = *px;
  x[0] = add_bf16_pair(x[0], o[0]);
  x[1] = add_bf16_pair(x[1], o[1]);
  x[2] = add_bf16_pair(x[2], o[2]);
  x[3] = add_bf16_pair(x[3], o[3]);
  *px = x;
}

// ---- tiled V^T.  One workgroup builds one tile: kKeyTile rows of V land in LDS with coalesced
// 16-byte loads (row stride an odd number of 4-byte words, so the column reads below are free of
// bank conflicts), then every thread assembles 16-byte pieces of a d-row from 2-byte column reads
// and stores them coalesced.  Rows past the end are zeros.
constexpr int kTileRowStride(int D) { return D + 2; }

template <int D>
__device__ __forceinline__ void tile_put(__bf16* tile, int r, int col, u32x4 v) {
  uint32_t* w = (uint32_t*)(&tile[r * kTileRowStride(D) + 8 * col]);
  w[0] = v[0]; w[1] = v[1]; w[2] = v[2]; w[3] = v[3];
}

template <int D>
__device__ __forceinline__ void tile_write_transposed(const __bf16* tile, __bf16* dst) {
  constexpr int RS = kTileRowStride(D), KC = kKeyTile / 8;
#pragma unroll
  for (int c = threadIdx.x; c < D * KC; c += kThreads) {
    const int dd = c / KC, kc = c % KC;
    const uint16_t* col = (const uint16_t*)(&tile[(8 * kc) * RS + dd]);
    u32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = (uint32_t)col[(2 * j) * RS] | ((uint32_t)col[(2 * j + 1) * RS] << 16);
    *(u32x4*)(dst + dd * kKeyTile + 8 * kc) = v;
  }
}

// V [heads][Lc][D] row-major -> V^T tiles [heads][nk_tiles][D][kKeyTile].
template <int D>
__global__ __launch_bounds__(kThreads) void v_tile_kernel(const u32x4* __restrict__ V, __bf16* __restrict__ Vt, int Lc, int nk_tiles) {
  __shared__ __attribute__((aligned(16))) __bf16 tile[kKeyTile * kTileRowStride(D)];
  constexpr int LPR = D / 8;
  const int t = blockIdx.x;
  const long long head = blockIdx.y;
  const int rows = min(kKeyTile, Lc - t * kKeyTile);
#pragma unroll
  for (int c = threadIdx.x; c < kKeyTile * LPR; c += kThreads) {
    const int r = c / LPR, col = c % LPR;
    u32x4 v = {0u, 0u, 0u, 0u};
    if (r < rows) v = V[(head * Lc + (long long)t * kKeyTile + r) * LPR + col];
    tile_put<D>(tile, r, col, v);
  }
  __syncthreads();
  tile_write_transposed<D>(tile, Vt + (head * nk_tiles + t) * (long long)(D * kKeyTile));
}

// Stage 1 compression for the fused layer: one workgroup = kKeyTile consecutive compacted rows of one
// query head: Q and K rows are copied as in compress_kernel, V rows go through LDS into the
// tile of V^T the attention kernel will read.  With per-group sets only the first query head
// of a group moves K and V.  With Qc == NULL only the V tiles are built (the attention kernel then
// gathers Q and K rows itself).
struct CompressTiledArgs {
  const u32x4* Q; const u32x4* K; const u32x4* V; const int32_t* idx;
  u32x4* Qc; u32x4* Kc; __bf16* Vt;
  int Hq, Hkv, L, k, group_mode, nk_tiles;
  const int32_t* k_dev;       // count per batch entry decided on the device (NULL: k); rows of idx and the tile
                              // arrays keep the stride of k
  Strides qs, ks;             // layouts of Q and of K / V, in 16-byte pieces
};

template <int D>
__global__ __launch_bounds__(kThreads) void compress_tiled_kernel(CompressTiledArgs a) {
  __shared__ __attribute__((aligned(16))) __bf16 tile[kKeyTile * kTileRowStride(D)];
  __shared__ int tok[kKeyTile];
  constexpr int LPR = D / 8;
  const int t = blockIdx.x;
  const long long bh = blockIdx.y;
  const int h = (int)(bh % a.Hq);
  const long long b = bh / a.Hq;
  const int g = a.Hq / a.Hkv;
  const long long bkv = b * a.Hkv + h / g;
  const long long sel_head = a.group_mode ? bkv : bh;
  const bool kv_owner = a.group_mode == 0 || h % g == 0;
  if (!a.Qc && !kv_owner) return;            // nothing to do; the same for every thread of the workgroup
  const int r0 = t * kKeyTile;
  const int k_here = a.k_dev ? a.k_dev[b] : a.k;
  if (r0 >= k_here) return;                  // tiles past this batch entry's count; the same for every thread
  if (threadIdx.x < kKeyTile) tok[threadIdx.x] = r0 + (int)threadIdx.x < k_here ? a.idx[sel_head * a.k + r0 + threadIdx.x] : -1;
  __syncthreads();
#pragma unroll
  for (int c = threadIdx.x; c < kKeyTile * LPR; c += kThreads) {
    const int r = c / LPR, col = c % LPR;
    const int tk = tok[r];
    u32x4 v = {0u, 0u, 0u, 0u};
    if (tk >= 0) {
      if (a.Qc) a.Qc[(bh * a.k + r0 + r) * LPR + col] = a.Q[a.qs.head(b, h) + tk * a.qs.l + col];
      if (kv_owner) {
        const long long kv_at = a.ks.head(b, h / g) + tk * a.ks.l + col;
        if (a.Qc) a.Kc[(sel_head * a.k + r0 + r) * LPR + col] = a.K[kv_at];
        v = a.V[kv_at];
      }
    }
    tile_put<D>(tile, r, col, v);
  }
  if (!kv_owner) return;                     // the same for every thread of the workgroup
  __syncthreads();
  tile_write_transposed<D>(tile, a.Vt + (sel_head * a.nk_tiles + t) * (long long)(D * kKeyTile));
}

inline unsigned blocks_for(long long n_tasks, int lpr) {
  return (unsigned)((n_tasks * lpr + kThreads - 1) / kThreads);
}

}  // namespace

hipError_t launch_compress(const Dims& dm, const void* Q, const void* K, const void* V, const int32_t* idx,
                           int k_keep, void* Qc, void* Kc, void* Vc, hipStream_t st) {
  const long long n = (long long)dm.B * dm.Hq * k_keep;
  auto q = (const u32x4*)Q; auto k = (const u32x4*)K; auto v = (const u32x4*)V;
  auto qc = (u32x4*)Qc; auto kc = (u32x4*)Kc; auto vc = (u32x4*)Vc;
  if (dm.d == 128)
    compress_kernel<16><<<blocks_for(n, 16), kThreads, 0, st>>>(q, k, v, idx, qc, kc, vc, dm.Hq, dm.Hkv, dm.L, k_keep, dm.group_mode, n, pieces(dm.q), pieces(dm.kv));
  else
    compress_kernel<8><<<blocks_for(n, 8), kThreads, 0, st>>>(q, k, v, idx, qc, kc, vc, dm.Hq, dm.Hkv, dm.L, k_keep, dm.group_mode, n, pieces(dm.q), pieces(dm.kv));
  return hipGetLastError();
}

hipError_t launch_v_tiles(int B, int kv_heads, int Lc, int d, const void* V, void* Vt, hipStream_t st) {
  const int nk_tiles = (Lc + kKeyTile - 1) / kKeyTile;
  const dim3 grid((unsigned)nk_tiles, (unsigned)(B * kv_heads));
  if (d == 128) v_tile_kernel<128><<<grid, kThreads, 0, st>>>((const u32x4*)V, (__bf16*)Vt, Lc, nk_tiles);
  else v_tile_kernel<64><<<grid, kThreads, 0, st>>>((const u32x4*)V, (__bf16*)Vt, Lc, nk_tiles);
  return hipGetLastError();
}

hipError_t launch_compress_tiled(const Dims& dm, const void* Q, const void* K, const void* V, const int32_t* idx,
                                 int k_keep, void* Qc, void* Kc, void* Vt, hipStream_t st, const int32_t* k_dev) {
  CompressTiledArgs a;
  a.k_dev = k_dev;
  a.qs = pieces(dm.q); a.ks = pieces(dm.kv);
  a.Q = (const u32x4*)Q; a.K = (const u32x4*)K; a.V = (const u32x4*)V; a.idx = idx;
  a.Qc = (u32x4*)Qc; a.Kc = (u32x4*)Kc; a.Vt = (__bf16*)Vt;
  a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.L = dm.L; a.k = k_keep; a.group_mode = dm.group_mode;
  a.nk_tiles = (k_keep + kKeyTile - 1) / kKeyTile;
  const dim3 grid((unsigned)a.nk_tiles, (unsigned)(dm.B * dm.Hq));
  if (dm.d == 128) compress_tiled_kernel<128><<<grid, kThreads, 0, st>>>(a);
  else compress_tiled_kernel<64><<<grid, kThreads, 0, st>>>(a);
  return hipGetLastError();
}

hipError_t launch_decompress(const Dims& dm, const void* Oc, const int32_t* idx, const int32_t* inv, int k_keep, void* O,
                             hipStream_t st) {
  const long long n = (long long)dm.B * dm.Hq * dm.L;
  // the rows of one thread are a quarter of the tensor apart, plus a few rows: with power-of-two
  // sequence lengths an exact quarter puts all four on the same memory channel
  const long long stride = (n + kRowsPerThread - 1) / kRowsPerThread + kStrideSkew;
  const int g_sel = dm.group_mode ? dm.Hq / dm.Hkv : 1;
  // Which of the two kernels: measured at 128K tokens x 32 heads, the two-stream kernel wins while
  // between 22 % and 75 % of the rows are kept (0.22 against 0.33 ms at a quarter kept, where the
  // compacted output no longer fits the Infinity Cache and the dependent look-up -> row load chain of
  // the inv-driven kernel is exposed to HBM latency twice); the inv-driven one when nearly all rows
  // are zeros (0.18 against 0.21 ms at a fifth kept) or nearly all are copies.
  const bool split = idx != nullptr && 9LL * k_keep >= 2LL * dm.L && 4LL * k_keep <= 3LL * dm.L;
  if (split) {
    const long long n_copy = (long long)dm.B * dm.Hq * k_keep;
    if (dm.d == 128) {
      const unsigned cb = blocks_for(n_copy, 16);
      decompress_split_kernel<16><<<cb + blocks_for(stride, 16), kThreads, 0, st>>>((const u32x4*)Oc, idx, inv, (u32x4*)O, g_sel, dm.L, k_keep, n_copy, n, cb, out_map(dm));
    } else {
      const unsigned cb = blocks_for(n_copy, 8);
      decompress_split_kernel<8><<<cb + blocks_for(stride, 8), kThreads, 0, st>>>((const u32x4*)Oc, idx, inv, (u32x4*)O, g_sel, dm.L, k_keep, n_copy, n, cb, out_map(dm));
    }
    return hipGetLastError();
  }
  if (dm.d == 128)
    decompress_kernel<16><<<blocks_for(stride, 16), kThreads, 0, st>>>((const u32x4*)Oc, inv, (u32x4*)O, dm.Hq, g_sel, dm.L, k_keep, n, stride, out_map(dm));
  else
    decompress_kernel<8><<<blocks_for(stride, 8), kThreads, 0, st>>>((const u32x4*)Oc, inv, (u32x4*)O, dm.Hq, g_sel, dm.L, k_keep, n, stride, out_map(dm));
  return hipGetLastError();
}

hipError_t launch_residual(const Dims& dm, const void* Oc, const int32_t* idx, int k_keep, void* residual, hipStream_t st) {
  const long long n = (long long)dm.B * dm.Hq * k_keep;
  const int g_sel = dm.group_mode ? dm.Hq / dm.Hkv : 1;
  if (dm.d == 128)
    residual_kernel<16><<<blocks_for(n, 16), kThreads, 0, st>>>((const u32x4*)Oc, idx, (u32x4*)residual, dm.Hq, g_sel, dm.L, k_keep, n);
  else
    residual_kernel<8><<<blocks_for(n, 8), kThreads, 0, st>>>((const u32x4*)Oc, idx, (u32x4*)residual, dm.Hq, g_sel, dm.L, k_keep, n);
  return hipGetLastError();
}

}  // namespace tsa
