// Pieces shared by the two forms of the attention kernel (attend.hip: 256 query rows per workgroup;
// attend_split.hip: 128 query rows per workgroup with the keys of every tile split over two groups of
// wavefronts): launch arguments, the tile generator that walks plain causal tiles or a block list,
// the half-tile products on v_mfma_f32_32x32x16_bf16 and the online-softmax steps.
#pragma once

#include "tsa_internal.h"

#include <climits>

namespace tsa {

namespace attend_detail {

constexpr int BM = 256;        // query rows per workgroup
constexpr int BN = kKeyTile;   // keys per tile
#ifndef TSA_PF
#define TSA_PF 3
#define TSA_RING 4
#endif
#ifndef TSA_QS
#define TSA_QS 1
#endif


constexpr int kQS = TSA_QS;    // query sub-tiles per wavefront (see attend_kernel)
constexpr int kMaxLists = BM / BN;   // row blocks of a query tile at the smallest block size (64): 4
constexpr float kNegBig = -1.0e30f;
constexpr float kLazy = 8.0f;  // log2 units the running max may lag behind

struct AttendArgs {
  const __bf16* Q;
  const __bf16* K;
  const __bf16* Vt;            // tiled V^T: [B * kvh][nk_tiles][d][64]
  __bf16* O;
  float* lse;
  const int32_t* block_list;
  long long bl_head_stride;    // elements between the block lists of consecutive (b, h); 0 = one shared list
  int max_blocks;
  int block;                   // block size of the list: 64, 128 or 256 tokens
  int BH, Hq, kvh, Lc, nq_tiles, nk_tiles;
  int head_split, vheads_per_xcd;   // workgroup -> (head, query tile) map, see map_workgroups()
  const int32_t* k_dev;        // fused form: compacted rows per batch entry, decided on the device (NULL: Lc)
  Strides qs, ks, os;          // fused form: layouts of the original Q, K and of the full-length output (elements)
  float c;                     // scale * log2(e)
  // Fused form (gather in the loads, scatter in the epilogue): Q and K are the ORIGINAL tensors of
  // L tokens (K with Hkv heads), compacted row r of selection row `sel` is token idx[sel][r];
  // Vt holds the tiles of the gathered V.  Of (may be NULL) is the full-length output
  // [B,Hq,L,d]: rows of selected tokens are written by the epilogue, all other rows are
  // zero-filled by the workgroup that owns their token range (inv[sel][t] < 0).  O (the compacted
  // output) may be NULL in this form.
  // X (may be NULL) is the residual stream [B,L,Hq*d]: the epilogue adds output row r, as rounded
  // to bf16, into X[b, idx[r], h*d .. (h+1)*d) (fp32 add, one rounding); every (token, head) slice
  // has exactly one writer.
  const int32_t* idx;
  const int32_t* inv;
  __bf16* Of;
  __bf16* X;
  int L, Hkv;
};

// Workgroup -> (head, query tile).  Consecutive workgroup ids go to different XCDs, so id % 8 picks the XCD.
// A head's query tiles stay on one XCD (they stream the same K / V through its L2), consecutive heads (the
// heads of a KV group) share an XCD, and the longest (last) query tiles are scheduled first.  When the number
// of heads is no multiple of 8, whole heads per XCD would leave some XCDs with one head more than others (28
// heads: four against three, a launch 14 % longer than its work); every head is then cut into `head_split`
// parts (query tiles qt with (nq - 1 - qt) % head_split == part), so that the B * Hq * head_split parts
// divide evenly: XCD x takes parts [x * vheads_per_xcd, (x + 1) * vheads_per_xcd), i.e. whole heads and at
// most two partial ones.
inline void map_workgroups(AttendArgs& a) {
  int g = 8;
  while (a.BH % g) g >>= 1;                       // gcd(BH, 8)
  a.head_split = 8 / g;
  a.vheads_per_xcd = a.BH / g;
}
inline unsigned grid_for(const AttendArgs& a) {
  return 8u * (unsigned)a.vheads_per_xcd * (unsigned)((a.nq_tiles + a.head_split - 1) / a.head_split);
}

// two bf16 in one dword: widen to fp32 (exact), add, round each sum to bf16 (nearest even)
__device__ __forceinline__ uint32_t add_bf16_pairs(uint32_t x, uint32_t o) {
  const float x0 = __uint_as_float(x << 16), x1 = __uint_as_float(x & 0xffff0000u);
  const float o0 = __uint_as_float(o << 16), o1 = __uint_as_float(o & 0xffff0000u);
  bf16x2 s;
  s[0] = (__bf16)(x0 + o0);
  s[1] = (__bf16)(x1 + o1);
  return __builtin_bit_cast(uint32_t, s);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2 v;
  v[0] = (__bf16)lo;
  v[1] = (__bf16)hi;
  return __builtin_bit_cast(uint32_t, v);
}

// Workgroup barrier that waits for this wavefront's LDS traffic only.  __syncthreads() also waits
// for every outstanding global load, which would expose the latency of the tile prefetch that
// was issued just before it; those loads land in registers and are consumed a tile later.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Row stride (elements) of a V^T tile in LDS: [d][64 keys + pad].  A fragment read takes 16 bytes
// per lane from 16 consecutive d-rows: 144-byte rows walk those lanes over all 64 banks.
constexpr int VS = BN + 8;

// Keys sit in the LDS tile in a permuted row order (bits 2 and 3 of the row swapped), so
// that accumulator register r of lane half hi holds key 16*(r/8) + 8*hi + r%8 of its 32-key
// half tile: the eight probabilities a lane packs for one PV step are then eight CONSECUTIVE
// keys, and the matching V^T operand is one contiguous 16-byte read.
__device__ __forceinline__ int k_row_perm(int lo) { return (lo & ~12) | ((lo & 4) << 1) | ((lo & 8) >> 1); }
__device__ __forceinline__ int key_of(int r, int hi) { return 16 * (r >> 3) + 8 * hi + (r & 7); }

// Key tiles a workgroup visits, in order.  A block list cuts the workgroup's 256 query rows into
// row blocks of `block` tokens (4, 2 or 1 of them); `use` bit j: row block j takes part in the tile
// (they can differ only under a block list; plain causal attention is one row block of 256).
struct Tile {
  int k0;      // first key of the tile, < 0: no more tiles
  int use;
};

struct TileGen {
  const int32_t* list[kMaxLists];   // the lists of the workgroup's row blocks, merged on the fly
  int cnt[kMaxLists], pos[kMaxLists];
  int cur[kMaxLists];               // next unread entry of each list (INT_MAX: exhausted), read one block ahead
  int n_lists, block, tiles_per_block, full;
  int sub, kb, use;
  int plain_n, plain_i;
  bool plain;
  __device__ Tile next() {
    if (plain) {
      if (plain_i >= plain_n) return Tile{-1, 0};
      Tile t{plain_i * BN, 1};
      ++plain_i;
      return t;
    }
    if (sub == 0) {
      // cur[] was read from the lists when the previous block was handed out, at least a tile ago:
      // the look-up is never waited for
      kb = INT_MAX;
#pragma unroll
      for (int j = 0; j < kMaxLists; ++j) kb = min(kb, cur[j]);
      if (kb == INT_MAX) return Tile{-1, 0};
      use = 0;
#pragma unroll
      for (int j = 0; j < kMaxLists; ++j)
        if (cur[j] == kb) {
          use |= 1 << j;
          ++pos[j];
          cur[j] = pos[j] < cnt[j] ? list[j][pos[j]] : INT_MAX;
        }
    }
    const Tile t{kb * block + sub * BN, use};
    sub = sub + 1 == tiles_per_block ? 0 : sub + 1;
    return t;
  }
};

__device__ __forceinline__ int count_valid(const int32_t* row, int max_blocks, int qb) {
  int cnt = 0;
  while (cnt < max_blocks) {
    const int kb = row[cnt];
    if (kb < 0 || kb > qb) break;
    ++cnt;
  }
  return cnt;
}

// One 32-key half tile of S^T for the wavefront's two query sub-tiles: s[qs] (16 fp32 each).
template <int D, int QS>
__device__ __forceinline__ void qk_half(const __bf16* Kt_half, int k_rd, const bf16x8 (&qf)[QS][D / 16], f32x16 (&s)[QS]) {
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) s[qs] = f32x16{0};
#pragma unroll
  for (int st = 0; st < D / 16; ++st) {
    const bf16x8 kf = *(const bf16x8*)(&Kt_half[k_rd + 16 * st]);
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) s[qs] = mfma32(kf, qf[qs][st], s[qs]);
  }
}

// O^T += V^T P^T for one 32-key half tile (two MFMA k-steps of 16 keys), both query sub-tiles.
// Vt_half points at the half's first key inside a [d][VS] tile.
__device__ __forceinline__ bf16x8 p_operand(const uint32_t (&pb)[8], int hf) {
  const u32x4 pw = {pb[4 * hf + 0], pb[4 * hf + 1], pb[4 * hf + 2], pb[4 * hf + 3]};
  return __builtin_bit_cast(bf16x8, pw);
}

template <int D, int QS>
__device__ __forceinline__ void pv_half(const __bf16* Vt_half, int v_rd, const uint32_t (&pb)[QS][8], f32x16 (&o)[QS][D / 32]) {
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) {
      const bf16x8 vf = *(const bf16x8*)(&Vt_half[v_rd + (32 * dt) * VS + 16 * hf]);
#pragma unroll
      for (int qs = 0; qs < QS; ++qs) o[qs][dt] = mfma32(vf, p_operand(pb[qs], hf), o[qs][dt]);
    }
  }
}

// Row max of one half tile (per query sub-tile), in scaled log2 units.
template <int QS>
__device__ __forceinline__ void row_max(const f32x16 (&s)[QS], float c, float (&mxc)[QS]) {
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    float mx = s[qs][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qs][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    mxc[qs] = mx * c;
  }
}

// Raises the running max (and rescales l, O) only when some row outgrew it by more than kLazy.
template <int ND, int QS>
__device__ __forceinline__ void raise_max(const float (&mxc)[QS], float (&m)[QS], float (&l)[QS], f32x16 (&o)[QS][ND]) {
  bool grow = false;
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) grow = grow || mxc[qs] > m[qs] + kLazy;
  if (__any(grow)) {
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      const float mn = fmaxf(m[qs], mxc[qs]);
      const float alpha = fast_exp2(m[qs] - mn);
      m[qs] = mn;
      l[qs] *= alpha;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qs][dt][r] *= alpha;
    }
  }
}

// The same for a half tile held as s * c - m (the form the pipelined iteration keeps between a QK block
// and its exponentials): mx is the row max relative to m.  A raise also shifts the pending half tile.
template <int ND, int QS>
__device__ __forceinline__ void raise_max_rel(const float (&mx)[QS], float (&m)[QS], float (&l)[QS],
                                              f32x16 (&o)[QS][ND], f32x16 (&pending)[QS]) {
  bool grow = false;
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) grow = grow || mx[qs] > kLazy;
  if (__any(grow)) {
#pragma unroll
    for (int qs = 0; qs < QS; ++qs) {
      const float dlt = fmaxf(mx[qs], 0.f);
      const float alpha = fast_exp2(-dlt);
      m[qs] += dlt;
      l[qs] *= alpha;
#pragma unroll
      for (int r = 0; r < 16; ++r) pending[qs][r] -= dlt;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[qs][dt][r] *= alpha;
    }
  }
}

template <int ND, int QS>
__device__ __forceinline__ void softmax_max(const f32x16 (&s)[QS], float c, float (&m)[QS], float (&l)[QS], f32x16 (&o)[QS][ND]) {
  float mxc[QS];
  row_max<QS>(s, c, mxc);
  raise_max<ND, QS>(mxc, m, l, o);
}

// p = exp2(s*c - m), packed to bf16 pairs in accumulator order; row sums into l.  (c is 1 in the
// kernel, whose scores come out of the MFMAs already scaled.)
template <int QS>
__device__ __forceinline__ void softmax_exp(const f32x16 (&s)[QS], float c, const float (&m)[QS], float (&l)[QS], uint32_t (&pb)[QS][8]) {
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    const float mq = m[qs];
    float ps0 = 0.f, ps1 = 0.f;
#pragma unroll
    for (int r = 0; r < 16; r += 2) {
      const float p0 = fast_exp2(fmaf(s[qs][r], c, -mq));
      const float p1 = fast_exp2(fmaf(s[qs][r + 1], c, -mq));
      ps0 += p0;
      ps1 += p1;
      pb[qs][r >> 1] = pack_bf16(p0, p1);
    }
    l[qs] += ps0 + ps1;
  }
}

template <int QS>
__device__ __forceinline__ void mask_half(f32x16 (&s)[QS], int key0, int hi, int qrow0) {
#pragma unroll
  for (int qs = 0; qs < QS; ++qs)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (key0 + key_of(r, hi) > qrow0 + 32 * qs) s[qs][r] = -INFINITY;
}

// Raw buffer descriptor over one head's rows: loads past `bytes` return zero, so ragged tails
// and tiles beyond the end need no bounds arithmetic in the loop.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t head_rsrc(const __bf16* base, long long bytes) {
  return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, (int)bytes, 0x00020000);
}

}  // namespace attend_detail

// attend_split.hip: the 128-row form (launch with a.nq_tiles / a.nk_tiles unset; it sizes its own grid)
hipError_t launch_attend_split(attend_detail::AttendArgs& a, int d, bool fused, hipStream_t st);

}  // namespace tsa
