// Causal attention over the compacted token set (Section 2.2, Stage 1: the attention
// operation on Q^, K^, V^ with cost O(L'^2 d)), also used unchanged as the dense baseline.
// Flash-style: one workgroup owns 128 query rows (4 wavefronts x 32 rows), streams 64-key
// tiles of K and V through LDS, keeps the running max / sum and the output accumulator in
// registers (online softmax), and never materialises the score matrix.
//
// Both products run on v_mfma_f32_32x32x16_bf16 in the TRANSPOSED orientation:
//   S^T = K Q^T   rows = keys, cols = queries  -> a lane owns ONE query (col) and 32 of the 64
//                 keys of the tile, so the row max / row sum of the softmax need a single
//                 cross-lane step (lane <-> lane^32);
//   O^T = V^T P^T rows = d, cols = queries     -> the P^T operand is exactly what the lane
//                 already holds (its query, eight keys per MFMA step), no shuffle or LDS
//                 round trip for P, and the rescale factor of O is the lane's own.
// The price is that V must be read with the key index contiguous.  V tiles are transposed on
// their way into LDS (4 keys x 8 d per thread, 16-bit shuffles in registers) and stored with
// the keys of each group of 16 permuted into the order in which the S^T accumulator holds
// them, so that one 16-byte LDS read yields one MFMA operand.
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 256;
constexpr int BM = 128;        // query rows per workgroup
constexpr int BN = 64;         // keys per tile
constexpr float kNegBig = -1.0e30f;

struct AttendArgs {
  const __bf16* Q;
  const __bf16* K;
  const __bf16* V;
  __bf16* O;
  float* lse;
  const int32_t* block_list;
  int max_blocks;
  int BH, Hq, kvh, Lc, nq_tiles;
  float c;                     // scale * log2(e)
};

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

template <int D>
__global__ __launch_bounds__(kThreads, 2) void attend_kernel(AttendArgs a) {
  constexpr int KS = D + 8;            // K tile row stride (elements): 16-byte pad spreads rows over banks
  constexpr int VS = BN + 8;           // V^T tile row stride
  constexpr int KCH = BN * (D / 8) / kThreads;   // 16-byte K chunks per thread per tile
  constexpr bool kVAll = (D == 128);   // every thread has a V transpose task (D=64: half of them)
  __shared__ __attribute__((aligned(16))) __bf16 Ks[BN * KS];
  __shared__ __attribute__((aligned(16))) __bf16 Vt[D * VS];

  // ---- workgroup -> (head, query tile).  Consecutive workgroup ids go to different XCDs, so
  // id % 8 picks the XCD; all tiles of a head (and all heads of a KV group) stay on one XCD to
  // share its L2, and the longest (last) query tiles are scheduled first.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int heads_per_xcd = (a.BH + 7) >> 3;
  const int hp = (slot % heads_per_xcd) * 8 + xcd;
  if (hp >= a.BH) return;
  const int qt = a.nq_tiles - 1 - slot / heads_per_xcd;
  const int b = hp / a.Hq, hr = hp % a.Hq;
  const int g = a.Hq / a.kvh;
  const int h = (hr % a.kvh) * g + hr / a.kvh;           // heads of one KV group are 8 apart in hp
  const long long bh = (long long)b * a.Hq + h;
  const long long bkv = (long long)b * a.kvh + h / g;

  const __bf16* Qh = a.Q + bh * a.Lc * D;
  const __bf16* Kh = a.K + bkv * a.Lc * D;
  const __bf16* Vh = a.V + bkv * a.Lc * D;

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int q0 = qt * BM;
  const int qrow = q0 + 32 * wave + lo;                 // this lane's query (column of S^T and O^T)

  // Q^T operand fragments stay in registers for the whole kernel
  bf16x8 qf[D / 16];
  {
    const bool ok = qrow < a.Lc;
    const __bf16* row = Qh + (long long)(ok ? qrow : 0) * D + 8 * hi;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      bf16x8 v = *(const bf16x8*)(row + 16 * s);
      if (!ok) v = bf16x8{};
      qf[s] = v;
    }
  }

  // ---- which key tiles this workgroup visits
  int n_tiles;
  const int32_t* bl_row = nullptr;
  if (a.block_list) {
    bl_row = a.block_list + (long long)qt * a.max_blocks;
    int cnt = 0;
    while (cnt < a.max_blocks) {
      const int kb = bl_row[cnt];
      if (kb < 0 || kb > qt) break;
      ++cnt;
    }
    n_tiles = 2 * cnt;                                   // a 128-token block is two key tiles
  } else {
    n_tiles = (min(q0 + BM, a.Lc) + BN - 1) / BN;
  }
  auto tile_start = [&](int it) -> int {
    return bl_row ? (bl_row[it >> 1] * 2 + (it & 1)) * BN : it * BN;
  };

  // ---- staging: global -> registers (prefetch) -> LDS
  u32x4 kreg[KCH];
  u32x4 vreg[4];
  const int v_kq = tid & 15, v_do = tid >> 4;            // key quad 0..15, d octet
  const bool v_on = kVAll || v_do < D / 8;
  auto load_tile = [&](int k0) {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = tid + kThreads * i;
      const int row = c / (D / 8), col8 = c % (D / 8);
      const int key = k0 + row;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (key < a.Lc) v = *(const u32x4*)(Kh + (long long)key * D + 8 * col8);
      kreg[i] = v;
    }
    if (v_on) {
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        const int key = k0 + 4 * v_kq + cc;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (key < a.Lc) v = *(const u32x4*)(Vh + (long long)key * D + 8 * v_do);
        vreg[cc] = v;
      }
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int i = 0; i < KCH; ++i) {
      const int c = tid + kThreads * i;
      const int row = c / (D / 8), col8 = c % (D / 8);
      *(u32x4*)(&Ks[row * KS + 8 * col8]) = kreg[i];
    }
    if (v_on) {
      // 4 keys x 8 d  ->  8 d x 4 keys; the quad goes to its permuted slot inside the group of 16 keys
      const int grp = v_kq >> 2, c4 = v_kq & 3;
      const int col = 16 * grp + 4 * (2 * (c4 & 1) + (c4 >> 1));
#pragma unroll
      for (int e2 = 0; e2 < 4; ++e2) {                   // dword e2 holds d = 2*e2, 2*e2+1
        const uint32_t k0 = vreg[0][e2], k1 = vreg[1][e2], k2 = vreg[2][e2], k3 = vreg[3][e2];
        u32x2 even, odd;
        even[0] = __builtin_amdgcn_perm(k1, k0, 0x05040100u);   // (k0.lo, k1.lo)
        even[1] = __builtin_amdgcn_perm(k3, k2, 0x05040100u);
        odd[0] = __builtin_amdgcn_perm(k1, k0, 0x07060302u);    // (k0.hi, k1.hi)
        odd[1] = __builtin_amdgcn_perm(k3, k2, 0x07060302u);
        *(u32x2*)(&Vt[(8 * v_do + 2 * e2) * VS + col]) = even;
        *(u32x2*)(&Vt[(8 * v_do + 2 * e2 + 1) * VS + col]) = odd;
      }
    }
  };

  f32x16 o[D / 32];
#pragma unroll
  for (int dt = 0; dt < D / 32; ++dt) o[dt] = f32x16{0};
  float m = kNegBig, l = 0.f;

  if (n_tiles > 0) load_tile(tile_start(0));
  for (int it = 0; it < n_tiles; ++it) {
    const int k0 = tile_start(it);
    __syncthreads();                                     // everyone is done reading the previous tile
    store_tile();
    __syncthreads();
    if (it + 1 < n_tiles) load_tile(tile_start(it + 1)); // in flight during the math below

    if (k0 > q0 + 32 * wave + 31) continue;              // every key of the tile is after this wave's rows
    // ---- S^T = K Q^T : two 32-key sub-tiles
    f32x16 st[2];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
      f32x16 acc = {0};
#pragma unroll
      for (int s = 0; s < D / 16; ++s) {
        const bf16x8 kf = *(const bf16x8*)(&Ks[(32 * kt + lo) * KS + 16 * s + 8 * hi]);
        acc = mfma32(kf, qf[s], acc);
      }
      st[kt] = acc;
    }
    if (k0 + BN - 1 > q0 + 32 * wave) {                  // tile crosses this wave's diagonal
#pragma unroll
      for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (k0 + 32 * kt + c_row(r, hi) > qrow) st[kt][r] = -INFINITY;
    }
    // ---- online softmax (log2 domain); lane and lane^32 share the query
    float mx = st[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, st[kt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float mn = fmaxf(m, mx * a.c);
    const float alpha = fast_exp2(m - mn);
    m = mn;
    float psum = 0.f;
    uint32_t pb[2][8];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float p0 = fast_exp2(fmaf(st[kt][r], a.c, -mn));
        const float p1 = fast_exp2(fmaf(st[kt][r + 1], a.c, -mn));
        psum += p0 + p1;
        pb[kt][r >> 1] = pack_bf16(p0, p1);
      }
    l = l * alpha + psum;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[dt][r] *= alpha;
    // ---- O^T += V^T P^T : four steps of 16 keys
#pragma unroll
    for (int s4 = 0; s4 < 4; ++s4) {
      const int kt = s4 >> 1, half = s4 & 1;
      u32x4 pw = {pb[kt][4 * half + 0], pb[kt][4 * half + 1], pb[kt][4 * half + 2], pb[kt][4 * half + 3]};
      const bf16x8 pf = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
      for (int dt = 0; dt < D / 32; ++dt) {
        const bf16x8 vf = *(const bf16x8*)(&Vt[(32 * dt + lo) * VS + 16 * s4 + 8 * hi]);
        o[dt] = mfma32(vf, pf, o[dt]);
      }
    }
  }

  // ---- epilogue: normalise, round to bf16, store O[query][d] (this lane: 4 consecutive d per register quad)
  const float lt = l + __shfl_xor(l, 32);
  const float inv_l = 1.0f / lt;
  if (qrow < a.Lc) {
    __bf16* orow = a.O + (bh * a.Lc + qrow) * D;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt)
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        u32x2 w;
        w[0] = pack_bf16(o[dt][4 * q4 + 0] * inv_l, o[dt][4 * q4 + 1] * inv_l);
        w[1] = pack_bf16(o[dt][4 * q4 + 2] * inv_l, o[dt][4 * q4 + 3] * inv_l);
        *(u32x2*)(orow + 32 * dt + 8 * q4 + 4 * hi) = w;
      }
    if (a.lse && hi == 0) a.lse[bh * a.Lc + qrow] = (m + log2f(lt)) * kLn2;
  }
}

}  // namespace

hipError_t launch_attend(int B, int Hq, int kv_heads, int Lc, int d, float scale, const void* Qc, const void* Kc,
                         const void* Vc, const int32_t* block_list, int max_blocks_per_row, void* Oc, float* lse,
                         hipStream_t st) {
  AttendArgs a;
  a.Q = (const __bf16*)Qc; a.K = (const __bf16*)Kc; a.V = (const __bf16*)Vc; a.O = (__bf16*)Oc;
  a.lse = lse; a.block_list = block_list; a.max_blocks = max_blocks_per_row;
  a.BH = B * Hq; a.Hq = Hq; a.kvh = kv_heads; a.Lc = Lc;
  a.nq_tiles = (Lc + BM - 1) / BM;
  a.c = scale * kLog2e;
  const unsigned grid = 8u * (unsigned)((a.BH + 7) / 8) * (unsigned)a.nq_tiles;
  if (d == 128) attend_kernel<128><<<grid, kThreads, 0, st>>>(a);
  else attend_kernel<64><<<grid, kThreads, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace tsa
