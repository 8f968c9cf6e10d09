// Causal attention over the compacted token set (Section 2.2, Stage 1: the attention
// operation on Q^, K^, V^ with cost O(L'^2 d)), also used unchanged as the dense baseline.
//
// Flash-style: one workgroup owns 256 query rows (8 wavefronts x 32 rows, two wavefronts per
// SIMD), streams 64-key tiles through LDS (K in a ring of three tiles, V in a ring of two, one
// barrier per tile), keeps the running max / sum and the output accumulator in registers
// (online softmax) and never materialises the score matrix.
//
// Both products run on v_mfma_f32_32x32x16_bf16 in the TRANSPOSED orientation:
//   S^T = K Q^T   rows = keys, cols = queries  -> a lane owns ONE query of the wavefront's 32
//                 and 32 of the 64 keys of the tile: the row max / row sum of the softmax need
//                 a single cross-lane step (lane <-> lane^32);
//   O^T = V^T P^T rows = d, cols = queries     -> the P^T operand is exactly what the lane
//                 already holds (its query, eight keys per MFMA step): no shuffle and no LDS
//                 round trip for P, and the rescale factor of O is the lane's own.
// V arrives as 64-key transposed tiles ([d][64 keys]) and K rows sit in LDS in a permuted order, so
// that each V^T operand is one 16-byte LDS read holding exactly the eight keys whose probabilities
// the lane has just packed.
// The loop is software-pipelined: the QK product of the next half tile is issued together with
// the softmax arithmetic of the current one, so the matrix pipe and the vector ALU overlap.
// The O rescale is lazy: the running max is only raised when a row's new max exceeds it by
// more than 2^8, so most tiles skip the multiply over the whole accumulator; the final
// division by the row sum makes the result independent of the max actually used.
// The exponent s * scale * log2(e) - m is formed in the PV block that follows a QK block (one fma per
// score, in fp32, in place, next to MFMAs that have little other vector work beside them), so the
// blocks with the exponentials apply exp2 to the half tile as it is; a raise of m in between shifts the
// waiting half tile by the same amount.
// Very short compacted sets (about 2000 tokens at 32 heads) take the 128-row form of attend_split.hip
// instead (use_split_form below).
// The template also holds the layout with 64 rows per wavefront (QS = 2: four wavefronts, one
// per SIMD, every LDS fragment feeds two MFMAs); it measures slower and is not instantiated
// by default.
#include "attend_common.h"

namespace tsa {

using namespace attend_detail;

namespace {

// QS = query sub-tiles (of 32 rows) per wavefront.  QS = 2: 4 wavefronts of 64 rows, one per SIMD,
// every LDS fragment feeds two MFMAs.  QS = 1: 8 wavefronts of 32 rows, two per SIMD, which share
// the SIMD's issue slots (a lone wavefront issues one vector instruction every ~8 clocks, two
// together one every ~5) at the price of one LDS fragment per MFMA.
// LISTS: the launch has a block list.  The plain causal form is a kernel of its own: the look-ups of the tile
// generator would otherwise sit in the tile loop as loads that may be pending, and the compiler's wait for
// them (before it reuses their registers) also waits for the K / V prefetches of the tile just requested.
template <int D, int QS, bool FUSED, bool LISTS>
__global__ __launch_bounds__(512 / QS, 2 / QS) void attend_kernel(AttendArgs a) {
  constexpr int kThreads = 512 / QS;
  constexpr int RW = 32 * QS;                     // query rows per wavefront
  // LDS row stride of a K tile in elements.  K rows are read 16 bytes per lane by 16 lanes of
  // different keys: a 16-byte pad walks them over all 64 banks.
  constexpr int KS = D + 8;
  constexpr int KTILE = BN * KS, VTILE = D * VS;  // elements of one staged tile (K: [key][d], V: [d][key])
  constexpr int CH = BN * (D / 8) / kThreads;     // 16-byte chunks per thread per tile
  constexpr int NS = D / 16;                      // MFMA k-steps of the QK product
  constexpr int ND = D / 32;                      // d sub-tiles of the output
  constexpr int ROWB = D * 2;                     // bytes of one row in global memory
  __shared__ __attribute__((aligned(16))) __bf16 smem[3 * KTILE + 2 * VTILE];   // K ring [3], V ring [2]

  // ---- workgroup -> (head, query tile).  Consecutive workgroup ids go to different XCDs, so
  // id % 8 picks the XCD; all tiles of a head (and all heads of a KV group) stay on one XCD to
  // share its L2, and the longest (last) query tiles are scheduled first.
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int vhead = xcd * a.vheads_per_xcd + slot % a.vheads_per_xcd;
  const int hp = vhead / a.head_split, part = vhead % a.head_split;
  const int b = hp / a.Hq, h = hp % a.Hq;
  // Rows of this batch entry's compacted set: the launch's count, or (fused form with a coverage
  // budget decided on the device) the count read from k_dev; a.Lc stays the capacity, i.e. the row
  // stride of idx and of the tile arrays, and the grid is sized for it.
  int Lc = a.Lc, nq_tiles = a.nq_tiles;
  if (FUSED && a.k_dev) {
    Lc = a.k_dev[b];
    nq_tiles = (Lc + BM - 1) / BM;
  }
  const int qt = nq_tiles - 1 - ((slot / a.vheads_per_xcd) * a.head_split + part);
  if (qt < 0) return;
  const int g = a.Hq / a.kvh;
  const int n_grp = FUSED ? a.Hkv : a.kvh, g_grp = a.Hq / n_grp;
  const long long bh = (long long)b * a.Hq + h;
  const long long bkv = (long long)b * a.kvh + h / g;    // head of K^ / V^ (fused: of the index set and the V tiles)
  // rows of Q and K: the compacted tensors, or (fused) the original ones addressed through idx
  // (fused: row pitch and head offsets come from the caller's layout; byte offsets of a row fit 32 bits
  // and both factors of token * pitch fit 24 bits, checked on the host)
  const int q_pitch = FUSED ? (int)a.qs.l * 2 : ROWB, k_pitch = FUSED ? (int)a.ks.l * 2 : ROWB;
  const __bf16* q_head = FUSED ? a.Q + a.qs.head(b, h) : a.Q + bh * Lc * D;
  const __bf16* k_head = FUSED ? a.K + a.ks.head(b, h / g_grp) : a.K + bkv * Lc * D;
  const int n_rows = FUSED ? a.L : Lc;
  const __amdgpu_buffer_rsrc_t Qr = head_rsrc(q_head, (long long)n_rows * q_pitch);
  const __amdgpu_buffer_rsrc_t Kr = head_rsrc(k_head, (long long)n_rows * k_pitch);
  const long long vt_bytes = (long long)a.nk_tiles * BN * ROWB;
  const __amdgpu_buffer_rsrc_t Vr = head_rsrc(a.Vt + bkv * (vt_bytes / 2), vt_bytes);
  const int32_t* idx_row = FUSED ? a.idx + bkv * a.Lc : nullptr;
  // index loads past the end of the set return 0 (token 0): such rows are only ever read as keys
  // beyond every query of the workgroup, which causality masks
  const __amdgpu_buffer_rsrc_t Ir = __builtin_amdgcn_make_buffer_rsrc((void*)idx_row, 0, FUSED ? Lc * 4 : 0, 0x00020000);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int q0 = qt * BM;
  const int wrow0 = q0 + RW * wave;                      // first query row of this wavefront
  const int row_block = LISTS ? a.block : BM;
  const int half_bit = 1 << ((RW * wave) / row_block);   // which row block of the query tile the wavefront is in
  const float c = a.c;
  const float c_ = c;
  const float inv_c = 1.0f / c;                                    // (the chunk loop of the pipelined iteration has its own c)

  // ---- fused form: zero rows of the full-length output.  The workgroup owns a range of the head's
  // tokens (see below) and clears those that inv marks unselected.  The work is
  // spread over the tile loop, one pass of kThreads / (d/8) rows every z_every iterations (the
  // look-up in inv for the next pass is in flight meanwhile), so the stores drain under the compute
  // instead of holding up the start of the workgroup; what is left when the tiles run out is flushed
  // before the epilogue.
  constexpr int LPR = D / 8, RPP = kThreads / LPR;
  const bool zfill = FUSED && a.Of != nullptr;
  const long long o_pitch16 = FUSED ? a.os.l / 8 : LPR;          // 16-byte pieces between rows of the full-length output
  const int32_t* inv_row = nullptr;
  u32x4* zrow = nullptr;
  int z_hi = 0, zt = 0, zr = 0;                          // end of the range, next row of this thread, its inv entry
  int z_every = 1, z_count = 1, z_passes = 1;
  if (zfill) {
    inv_row = a.inv + bkv * a.L;
    // Token range of this workgroup.  Any partition of [0, L) over the query tiles of a head works (a row is
    // cleared iff inv marks it unselected, whoever looks).  The shares grow linearly with the query tile,
    // as the number of tile iterations does, so that every workgroup can clear its share inside its loop.
    const long long nq = nq_tiles, wt = nq * (nq + 1) / 2;
    const int tok_lo = (int)((long long)a.L * ((long long)qt * (qt + 1) / 2) / wt);
    z_hi = (int)((long long)a.L * ((long long)(qt + 1) * (qt + 2) / 2) / wt);
    zrow = (u32x4*)(a.Of + a.os.head(b, h)) + (tid % LPR);
    zt = tok_lo + tid / LPR;
    zr = zt < z_hi ? inv_row[zt] : 0;
    z_passes = (z_hi - tok_lo + RPP - 1) / RPP;
  }
  auto zero_step = [&]() {
    if (zr < 0) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, zrow + (long long)zt * o_pitch16);
    zt += RPP;
    zr = zt < z_hi ? inv_row[zt] : 0;
  };

  // Q^T operand fragments (two 32-row sub-tiles) stay in registers for the whole kernel
  bf16x8 qf[QS][NS];
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    int qrow_off = (wrow0 + 32 * qs + lo) * ROWB;
    if (FUSED) {
      const int qr = wrow0 + 32 * qs + lo;
      qrow_off = qr < Lc ? (int)__umul24(idx_row[qr], q_pitch) : a.L * q_pitch;   // past the end: out of the buffer's range, reads zeros
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(Qr, qrow_off + 16 * hi + 32 * s, 0, 0);
      qf[qs][s] = __builtin_bit_cast(bf16x8, v);
    }
  }
  // Wait for Q here, on every path: otherwise the compiler's wait-count bookkeeping carries these
  // loads as "possibly pending" into the main loop and makes every MFMA that reads a Q fragment
  // wait for the oldest in-flight K/V prefetch as well.
  __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0)

  TileGen gen;
  gen.plain = !LISTS;
  gen.plain_i = 0;
  gen.plain_n = (min(q0 + BM, Lc) + BN - 1) / BN;
  gen.sub = gen.kb = gen.use = 0;
  gen.n_lists = 1;
  gen.block = BM;
  gen.tiles_per_block = BM / BN;
  gen.full = 1;
  int longest_list = 0;
#pragma unroll
  for (int j = 0; j < kMaxLists; ++j) { gen.list[j] = nullptr; gen.cnt[j] = gen.pos[j] = 0; gen.cur[j] = INT_MAX; }
  if (!gen.plain) {
    gen.block = a.block;
    gen.n_lists = BM / a.block;
    gen.tiles_per_block = a.block / BN;
    gen.full = 0;
    const int nqb = (Lc + a.block - 1) / a.block;
    const int32_t* bl = a.block_list + bh * a.bl_head_stride;
#pragma unroll
    for (int j = 0; j < kMaxLists; ++j) {
      const int qb = qt * gen.n_lists + j;
      if (j < gen.n_lists && qb < nqb) {
        gen.list[j] = bl + (long long)qb * a.max_blocks;
        gen.cnt[j] = count_valid(gen.list[j], a.max_blocks, qb);
        if (gen.cnt[j] > 0) gen.cur[j] = gen.list[j][0];
        gen.full |= 1 << j;
        longest_list = max(longest_list, gen.cnt[j]);
      }
    }
  }

  // zero rows: as evenly over the pipelined iterations as their number allows
  if (zfill) {
    const int n_pipelined = gen.plain ? q0 / BN - 1 : gen.tiles_per_block * longest_list - 6;
    z_every = max(1, n_pipelined / max(1, z_passes));
  }

  // ---- staging: global -> registers -> LDS in 16-byte chunks.  A K tile is 64 rows of the
  // row-major tensor: thread chunk i covers row st_row + i * kRowsPerPass, columns 8*st_col.. .
  // A V tile is one contiguous [d][64] block of the tiled V^T tensor (64 keys = 64 * ROWB bytes as
  // well): thread chunk i is 16-byte piece tid + i * kThreads, i.e. d-row piece / 8, keys
  // 8 * (piece % 8).. .  The tile's first key goes into the scalar offset of the buffer load.
  constexpr int kRowsPerPass = kThreads / (D / 8);
  const int st_row = tid / (D / 8), st_col = tid % (D / 8);
  const int lk_off = k_row_perm(st_row) * KS + 8 * st_col;        // elements, LDS side (K): permuted row order
  const int gv_off = 16 * tid;                                    // bytes, global side (V^T)
  const int lv_off = (tid >> 3) * VS + 8 * (tid & 7);             // elements, LDS side (V^T)
  constexpr int kVRowsPerPass = kThreads / 8;
  // Rows of the next K tile to be loaded: ktok[i] = row of thread chunk i (fused: the token the
  // compacted row stands for, fetched from idx one tile ahead of the K load that uses it).
  int ktok[CH];
  auto row_off = [&](int tok) -> int { return FUSED ? (int)__umul24(tok, k_pitch) : tok * ROWB; };
  auto fetch_tok = [&](int k0) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      if (FUSED) ktok[i] = __builtin_amdgcn_raw_buffer_load_b32(Ir, (st_row + i * kRowsPerPass) * 4, k0 * 4, 0);
      else ktok[i] = k0 + st_row + i * kRowsPerPass;
    }
  };
  auto load_k = [&](u32x4 (&reg)[CH]) {
#pragma unroll
    for (int i = 0; i < CH; ++i)
      reg[i] = __builtin_amdgcn_raw_buffer_load_b128(Kr, row_off(ktok[i]) + 16 * st_col, 0, 0);
  };
  auto load_v = [&](int k0, u32x4 (&reg)[CH]) {
#pragma unroll
    for (int i = 0; i < CH; ++i)
      reg[i] = __builtin_amdgcn_raw_buffer_load_b128(Vr, gv_off + i * kThreads * 16, k0 * ROWB, 0);
  };
  auto store_k = [&](__bf16* dst, const u32x4 (&reg)[CH]) {
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u32x4*)(&dst[lk_off + i * kRowsPerPass * KS]) = reg[i];
  };
  auto store_v = [&](__bf16* dst, const u32x4 (&reg)[CH]) {
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u32x4*)(&dst[lv_off + i * kVRowsPerPass * VS]) = reg[i];
  };

  // LDS read bases.  K operand (A of S^T): MFMA row lo = LDS row lo = key k_row_perm(lo) of the
  // half tile, 8 d-values at 8*hi.  (The permutation is applied when the tile is written: eight
  // adjacent lanes must read eight adjacent LDS rows to stay free of bank conflicts.)
  const int k_rd = lo * KS + 8 * hi;
  // V^T operand (A of O^T): row = d (lo within the 32-row d sub-tile), 8 keys at 8*hi.
  const int v_rd = lo * VS + 8 * hi;

  f32x16 o[QS][ND];
  float m[QS], l[QS];
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    m[qs] = kNegBig;
    l[qs] = 0.f;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt) o[qs][dt] = f32x16{0};
  }

  // ring slots: K(t) in kc, K(t+1) in kn, K(t+2) goes to kf; V(t) in vc, V(t+1) goes to vn
  __bf16* kc = smem;
  __bf16* kn = smem + KTILE;
  __bf16* kf = smem + 2 * KTILE;
  __bf16* vc = smem + 3 * KTILE;
  __bf16* vn = smem + 3 * KTILE + VTILE;
  auto rotate = [&]() {
    __bf16* t = kc; kc = kn; kn = kf; kf = t;
    t = vc; vc = vn; vn = t;
  };

  // ---- prologue
  Tile T0 = gen.next(), T1 = gen.next(), T2 = gen.next(), T3 = gen.next();
  u32x4 kreg[CH], vreg[CH];
  f32x16 sA[QS], sB[QS];
  uint32_t pA[QS][8], pB[QS][8];
  if (T0.k0 >= 0) {
    fetch_tok(T0.k0);
    load_k(kreg);
    load_v(T0.k0, vreg);
    store_k(kc, kreg);
    store_v(vc, vreg);
    if (T1.k0 >= 0) {
      fetch_tok(T1.k0);
      load_k(kreg);
      store_k(kn, kreg);
    }
  }
  __syncthreads();
  auto wave_active = [&](const Tile& t) -> bool { return t.k0 >= 0 && (t.use & half_bit) && t.k0 <= wrow0 + RW - 1; };
  if (T0.k0 >= 0) qk_half<D, QS>(kc, k_rd, qf, sA);
  if (T2.k0 >= 0) {
    fetch_tok(T2.k0);
    load_k(kreg);
  }
  if (T1.k0 >= 0) load_v(T1.k0, vreg);
  if (T3.k0 >= 0) fetch_tok(T3.k0);
  if (wave_active(T0)) {
    if (T0.k0 + 31 > wrow0) mask_half<QS>(sA, T0.k0, hi, wrow0 + lo);
    softmax_max<ND, QS>(sA, c, m, l, o);
  }

  // Invariant at the top of an iteration: sA = S^T of the first half of tile T0, already masked
  // and already covered by the running max m (if this wavefront takes part in T0); K(T0) in kc,
  // K(T1) in kn, V(T0) in vc; kreg = K(T2) and vreg = V(T1) are in flight; ktok = rows of T3.
  //
  // Order inside an iteration: every block of 16 MFMAs is issued next to vector work that does
  // not depend on it, so the matrix pipe and the VALU overlap within the wavefront:
  //   QK(T0, half 1)      with  exp(sA)
  //   PV(T0, half 0)      with  max(sB)            [then the rare raise of m, rescale of O]
  //   QK(T1, half 0)      with  exp(sB)
  //   PV(T0, half 1)      with  max(sA of T1), staging  [then the rare raise of m]

  // ---- the pipelined iteration: one key tile that lies entirely below the workgroup's first
  // row and is used by all its wavefronts (as is the tile after it) needs no mask and no
  // per-wavefront decisions; loads past the end return zeros, so nothing in it is conditional
  // except the rare raise of the running max.
  // The iteration is a stream of 32 chunks of two MFMAs each:
  //    0.. 7  S^T(T0, half 1) -> sB      with  exp(sA) -> pA
  //    8..15  O^T += V^T(T0, half 0) pA  with  row max of sB          [then the rare raise of m]
  //   16..23  S^T(T1, half 0) -> sA      with  exp(sB) -> pB
  //   24..31  O^T += V^T(T0, half 1) pB  with  row max of sA, staging  [barrier, rare raise of m]
  // Inside this loop sA and sB hold s * c - m by the time their exponentials are due (formed by an fma
  // per element in the PV block after the chain, or, with scaled Q, by a chain that starts from -m), so the
  // exponent is the register itself and the row max is relative to m; a raise of m between the two shifts
  // the pending half tile by the same amount.
  // Each chunk consumes one 16-byte LDS fragment per lane (a K fragment or a V^T fragment);
  // fragments are fetched kPF chunks ahead through a small register ring that runs across the
  // blocks and across iterations, so the LDS latency is hidden.
  constexpr int kPF = TSA_PF, kRing = TSA_RING, kChunks = 4 * NS;
  static_assert(NS == 8 || NS == 4, "chunk stream is laid out for d = 128 or 64");
  constexpr int CPB = kChunks / 4;                       // chunks per block
  // slot = chunk % kRing must mean the same slot in consecutive iterations; a fragment must not be
  // overwritten before it is consumed; and the fragments fetched across the iteration boundary
  // must all belong to block 0 (K of the next tile, complete since the previous barrier), not to
  // the V tile that this iteration is still writing
  static_assert(kChunks % kRing == 0 && kRing > kPF && kPF <= CPB, "fragment ring does not fit the chunk stream");
  bf16x8 kfr[kRing];
  // fragment fetch for chunk c of the iteration whose tiles sit in (kc_, kn_, vc_)
  auto fetch = [&](int c, const __bf16* kc_, const __bf16* kn_, const __bf16* vc_) {
    const int blk = c / CPB, i = c % CPB, slot = c % kRing;
    if (blk == 0) kfr[slot] = *(const bf16x8*)(&kc_[32 * KS + k_rd + 16 * i]);
    else if (blk == 2) kfr[slot] = *(const bf16x8*)(&kn_[k_rd + 16 * i]);
    else {
      const int hf = i / ND, dt = i % ND;
      kfr[slot] = *(const bf16x8*)(&vc_[v_rd + (32 * dt) * VS + (blk == 3 ? 32 : 0) + 16 * hf]);
    }
  };
  auto prime_ring = [&]() {
#pragma unroll
    for (int c = 0; c < kPF; ++c) fetch(c, kc, kn, vc);
  };
  // vload: byte offset of the V tile to prefetch (tile T2), tokload: first compacted row of the
  // K tile whose rows are looked up (tile T4)
  auto fast_iter = [&](const int vload, const int tokload) {
    float mxc[QS], mx[QS], ps0[QS], ps1[QS];
    f32x16 acc[QS];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int blk = c / CPB, i = c % CPB, slot = c % kRing;
      // A wavefront in a block with exponentials has the longer chain of vector instructions between
      // its MFMAs: it takes precedence over the other wavefront of its SIMD while it is there
      // (measured: 3 % faster on random values, 5 % on zeros, against equal priorities).
      if (i == 0) {
        if (blk == 0 || blk == 2) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(0);
      }
      // prefetch kPF chunks ahead; the first chunks of the next iteration read the rotated slots
      if (c + kPF < kChunks) fetch(c + kPF, kc, kn, vc);
      else fetch(c + kPF - kChunks, kn, kf, vn);
      if (blk == 0 || blk == 2) {
        const f32x16 (&s_in)[QS] = blk == 0 ? sA : sB;
        uint32_t (&p_out)[QS][8] = blk == 0 ? pA : pB;
        constexpr int EPS = 16 / NS;
        // one MFMA, then the exponentials of one query sub-tile: the vector work runs in the
        // shadow of the MFMA that was just issued
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
          if (i == 0) acc[qs] = f32x16{0};
          acc[qs] = mfma32(kfr[slot], qf[qs][i], acc[qs]);
#pragma unroll
          for (int e = 0; e < EPS; e += 2) {
            const int r = EPS * i + e;
            const float p0 = fast_exp2(s_in[qs][r]);
            const float p1 = fast_exp2(s_in[qs][r + 1]);
            if (r == 0) { ps0[qs] = p0; ps1[qs] = p1; }
            else { ps0[qs] += p0; ps1[qs] += p1; }
            p_out[qs][r >> 1] = pack_bf16(p0, p1);
          }
          if (qs + 1 < QS) __builtin_amdgcn_sched_barrier(0);
        }
        if (i == CPB - 1) {
          f32x16 (&s_out)[QS] = blk == 0 ? sB : sA;
#pragma unroll
          for (int qs = 0; qs < QS; ++qs) {
            s_out[qs] = acc[qs];
            l[qs] += ps0[qs] + ps1[qs];
          }
        }
      } else {
        f32x16 (&s_in)[QS] = blk == 1 ? sB : sA;
        const uint32_t (&pb)[QS][8] = blk == 1 ? pA : pB;
        const int hf = i / ND, dt = i % ND;
        constexpr int EPC = 16 / CPB;
        const bf16x8 vf = kfr[slot];
#pragma unroll
        for (int qs = 0; qs < QS; ++qs) {
          o[qs][dt] = mfma32(vf, p_operand(pb[qs], hf), o[qs][dt]);
          // the half tile that the last QK block left as plain scores becomes s * c - m here, two elements
          // per chunk, next to the MFMAs of a PV block that has little else to do
#pragma unroll
          for (int e = 0; e < EPC; ++e) s_in[qs][EPC * i + e] = fmaf(s_in[qs][EPC * i + e], c_, -m[qs]);
          if (i == 0) mx[qs] = s_in[qs][0];
          if (EPC == 2) mx[qs] = __builtin_fmaxf(__builtin_fmaxf(mx[qs], s_in[qs][2 * i]), s_in[qs][2 * i + 1]);
          else {
#pragma unroll
            for (int e = 0; e < EPC; ++e) mx[qs] = fmaxf(mx[qs], s_in[qs][EPC * i + e]);
          }
          if (qs + 1 < QS) __builtin_amdgcn_sched_barrier(0);
        }
        if (blk == 3) {                 // K(t+2) -> kf, V(t+1) -> vn, then refill the registers
          if (i < CH) {
            *(u32x4*)(&kf[lk_off + i * kRowsPerPass * KS]) = kreg[i];
            kreg[i] = __builtin_amdgcn_raw_buffer_load_b128(Kr, row_off(ktok[i]) + 16 * st_col, 0, 0);
            if (FUSED) ktok[i] = __builtin_amdgcn_raw_buffer_load_b32(Ir, (st_row + i * kRowsPerPass) * 4, tokload * 4, 0);
            else ktok[i] = tokload + st_row + i * kRowsPerPass;
          } else if (i < 2 * CH) {
            *(u32x4*)(&vn[lv_off + (i - CH) * kVRowsPerPass * VS]) = vreg[i - CH];
            vreg[i - CH] = __builtin_amdgcn_raw_buffer_load_b128(Vr, gv_off + (i - CH) * kThreads * 16, vload, 0);
          }
        }
        if (FUSED && blk == 3 && i == (2 * CH < CPB ? 2 * CH : CPB - 1) && zfill && --z_count <= 0) {
          zero_step();
          z_count = z_every;
        }
        if (i == CPB - 1) {
#pragma unroll
          for (int qs = 0; qs < QS; ++qs) mxc[qs] = fmaxf(mx[qs], __shfl_xor(mx[qs], 32));
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (c == 2 * CPB - 1) {
        raise_max_rel<ND, QS>(mxc, m, l, o, sB);
      }
    }
    lds_barrier();
    raise_max_rel<ND, QS>(mxc, m, l, o, sA);
    rotate();
    };

  // ---- tile loop.  A tile takes the pipelined iteration when it and the tile after it lie below
  // the workgroup's first row and are used by both halves of the workgroup (plain causal: every
  // tile but the last five; sink + window lists: all but the first and last few); diagonal tiles,
  // tiles only one half visits and the tile in front of either take the general iteration, with
  // masks and per-wavefront decisions.  Both keep the same invariant, so they alternate freely.
  auto pipelined = [&](const Tile& t) -> bool { return t.k0 >= 0 && t.use == gen.full && t.k0 + BN <= q0; };
  while (T0.k0 >= 0) {
    if (pipelined(T0) && pipelined(T1)) {
      // the pipelined iterations hold their half tiles as s * c - m: sA enters and leaves in that form
#pragma unroll
      for (int qs = 0; qs < QS; ++qs)
#pragma unroll
        for (int r = 0; r < 16; ++r) sA[qs][r] = fmaf(sA[qs][r], c_, -m[qs]);
      prime_ring();
      do {
        const Tile T4 = gen.next();
        // tiles that do not exist are replaced by tile 0 in the prefetches: loaded, never used
        fast_iter(max(T2.k0, 0) * ROWB, max(T4.k0, 0));
        T0 = T1; T1 = T2; T2 = T3; T3 = T4;
      } while (pipelined(T0) && pipelined(T1));
      if (T0.k0 < 0) break;
#pragma unroll
      for (int qs = 0; qs < QS; ++qs)
#pragma unroll
        for (int r = 0; r < 16; ++r) sA[qs][r] = (sA[qs][r] + m[qs]) * inv_c;
    }
    qk_half<D, QS>(kc + 32 * KS, k_rd, qf, sB);
    if (wave_active(T0)) {
      if (T0.k0 + BN - 1 > wrow0) mask_half<QS>(sB, T0.k0 + 32, hi, wrow0 + lo);
      softmax_exp<QS>(sA, c, m, l, pA);
      pv_half<D, QS>(vc, v_rd, pA, o);
      softmax_max<ND, QS>(sB, c, m, l, o);
      softmax_exp<QS>(sB, c, m, l, pB);
      pv_half<D, QS>(vc + 32, v_rd, pB, o);
    }
    if (T1.k0 >= 0) qk_half<D, QS>(kn, k_rd, qf, sA);
    if (wave_active(T1)) {
      if (T1.k0 + 31 > wrow0) mask_half<QS>(sA, T1.k0, hi, wrow0 + lo);
      softmax_max<ND, QS>(sA, c, m, l, o);
    }
    if (T2.k0 >= 0) store_k(kf, kreg);
    if (T1.k0 >= 0) store_v(vn, vreg);
    if (T3.k0 >= 0) load_k(kreg);
    if (T2.k0 >= 0) load_v(T2.k0, vreg);
    const Tile T4 = gen.next();
    if (T4.k0 >= 0) fetch_tok(T4.k0);
    lds_barrier();
    T0 = T1; T1 = T2; T2 = T3; T3 = T4;
    rotate();
  }

  // ---- fused form: the zero rows the tile loop did not get to
  if (zfill) {
    // Latency-bound: a batch of look-ups is a memory round trip.  Sixteen rows per thread and batch, the
    // look-ups of the next batch requested before the stores of the current one (so that waiting for them
    // never includes waiting for those stores to be acknowledged).
    constexpr int kBatch = 16;
    if (zr < 0) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, zrow + (long long)zt * o_pitch16);
    int t0 = zt + RPP;
    int r[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) r[j] = t0 + j * RPP < z_hi ? inv_row[t0 + j * RPP] : 0;
    while (t0 < z_hi) {
      const int t1 = t0 + kBatch * RPP;
      int rn[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) rn[j] = t1 + j * RPP < z_hi ? inv_row[t1 + j * RPP] : 0;
#pragma unroll
      for (int j = 0; j < kBatch; ++j)
        if (r[j] < 0) __builtin_nontemporal_store(u32x4{0u, 0u, 0u, 0u}, zrow + (long long)(t0 + j * RPP) * o_pitch16);
#pragma unroll
      for (int j = 0; j < kBatch; ++j) r[j] = rn[j];
      t0 = t1;
    }
  }

  // ---- epilogue: normalise, round to bf16, store O[query][d] (a lane holds 4 consecutive d per register quad)
#pragma unroll
  for (int qs = 0; qs < QS; ++qs) {
    const int qrow = wrow0 + 32 * qs + lo;
    const float lt = l[qs] + __shfl_xor(l[qs], 32);
    const float inv_l = lt > 0.f ? 1.0f / lt : 0.f;
    if (qrow < Lc) {
      __bf16* orow = a.O ? a.O + (bh * a.Lc + qrow) * D : nullptr;
      __bf16* frow = nullptr;                       // fused: the token's row of the full-length output
      __bf16* xrow = nullptr;                       // fused: the token's slice of the residual stream
      if (FUSED && a.Of) frow = a.Of + a.os.head(b, h) + idx_row[qrow] * a.os.l;
      if (FUSED && a.X) xrow = a.X + (((long long)b * a.L + idx_row[qrow]) * a.Hq + h) * D;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(o[qs][dt][4 * q4 + 0] * inv_l, o[qs][dt][4 * q4 + 1] * inv_l);
          w[1] = pack_bf16(o[qs][dt][4 * q4 + 2] * inv_l, o[qs][dt][4 * q4 + 3] * inv_l);
          if (orow) *(u32x2*)(orow + 32 * dt + 8 * q4 + 4 * hi) = w;
          if (FUSED && frow) *(u32x2*)(frow + 32 * dt + 8 * q4 + 4 * hi) = w;
          if (FUSED && xrow) {
            u32x2* px = (u32x2*)(xrow + 32 * dt + 8 * q4 + 4 * hi);
            u32x2 x = *px;
            x[0] = add_bf16_pairs(x[0], w[0]);
            x[1] = add_bf16_pairs(x[1], w[1]);
            *px = x;
          }
        }
      if (a.lse && hi == 0) a.lse[bh * a.Lc + qrow] = (m[qs] + log2f(lt)) * kLn2;
    }
  }
}

}  // namespace

namespace {

#ifndef TSA_SPLIT_RATIO
#define TSA_SPLIT_RATIO 1.5
#endif
constexpr double kSplitRatio = TSA_SPLIT_RATIO;

// Which form runs: 0 = chosen per launch, 1 = always 256 rows per workgroup, 2 = always 128 rows with
// the keys split over two groups of wavefronts (measurement support: set_attend_form).
int g_attend_form = 0;

// The 128-row form pays when the longest chain of a launch (the last query tile of a head: 4 nq tiles
// of 64 keys for nq tiles of 256 rows) is long against the work the chip has per CU (BH * 2 nq (nq + 1)
// tile steps over 256 CUs), i.e. for very short compacted sets.  Its iteration stages every K / V tile
// for half as many rows, which costs about 15 % of the rate: measured at 32 heads, d = 128, it wins up
// to 2048 compacted tokens (0.064 against 0.071 ms) and loses from 3277 on (0.139 against 0.118 ms), and
// it loses on sink + window block lists at every block size.
bool use_split_form(const AttendArgs& a) {
  if (g_attend_form == 1) return false;
  if (g_attend_form == 2) return true;
  const long long nq = (a.Lc + BM - 1) / BM;
  return 512 >= kSplitRatio * (long long)a.BH * (nq + 1);          // chain / work per CU = 512 / (BH (nq + 1))
}

template <bool FUSED>
hipError_t launch_any(AttendArgs& a, int d, hipStream_t st) {
  if (kQS == 1 && use_split_form(a)) return launch_attend_split(a, d, FUSED, st);
  a.nq_tiles = (a.Lc + BM - 1) / BM;
  a.nk_tiles = (a.Lc + BN - 1) / BN;
  map_workgroups(a);
  const unsigned grid = grid_for(a);
  if (a.block_list) {
    if (d == 128) attend_kernel<128, kQS, FUSED, true><<<grid, 512 / kQS, 0, st>>>(a);
    else attend_kernel<64, kQS, FUSED, true><<<grid, 512 / kQS, 0, st>>>(a);
  } else {
    if (d == 128) attend_kernel<128, kQS, FUSED, false><<<grid, 512 / kQS, 0, st>>>(a);
    else attend_kernel<64, kQS, FUSED, false><<<grid, 512 / kQS, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace

void set_attend_form(int form) { g_attend_form = form; }

hipError_t launch_attend(int B, int Hq, int kv_heads, int Lc, int d, float scale, const void* Qc, const void* Kc,
                         const void* Vt, const int32_t* block_list, int block_size, int max_blocks_per_row,
                         int block_list_per_head, void* Oc, float* lse, hipStream_t st) {
  AttendArgs a;
  a.block = block_list ? block_size : BM;
  a.bl_head_stride = block_list_per_head ? (long long)((Lc + a.block - 1) / a.block) * max_blocks_per_row : 0;
  a.Q = (const __bf16*)Qc; a.K = (const __bf16*)Kc; a.Vt = (const __bf16*)Vt; a.O = (__bf16*)Oc;
  a.lse = lse; a.block_list = block_list; a.max_blocks = max_blocks_per_row;
  a.BH = B * Hq; a.Hq = Hq; a.kvh = kv_heads; a.Lc = Lc;
  a.c = scale * kLog2e;
  a.idx = nullptr; a.inv = nullptr; a.Of = nullptr; a.X = nullptr; a.L = Lc; a.Hkv = kv_heads;
  a.k_dev = nullptr;
  a.qs = a.ks = a.os = Strides{0, 0, 0};
  return launch_any<false>(a, d, st);
}

hipError_t launch_attend_fused(const Dims& dm, const void* Q, const void* K, const void* Vt, const int32_t* idx,
                               const int32_t* inv, int k_keep, const int32_t* block_list, int block_size,
                               int max_blocks_per_row, void* Oc, void* O, void* residual, hipStream_t st,
                               const int32_t* k_dev) {
  AttendArgs a;
  a.k_dev = k_dev;
  a.qs = dm.q; a.ks = dm.kv; a.os = dm.o;
  a.block = block_list ? block_size : BM;
  a.Q = (const __bf16*)Q; a.K = (const __bf16*)K; a.Vt = (const __bf16*)Vt; a.O = (__bf16*)Oc;
  a.lse = nullptr; a.block_list = block_list; a.max_blocks = max_blocks_per_row;
  a.bl_head_stride = dm.block_list_per_head ? (long long)((k_keep + a.block - 1) / a.block) * max_blocks_per_row : 0;
  a.BH = dm.B * dm.Hq; a.Hq = dm.Hq; a.kvh = dm.group_mode ? dm.Hkv : dm.Hq; a.Lc = k_keep;
  a.c = dm.scale * kLog2e;
  a.idx = idx; a.inv = inv; a.Of = (__bf16*)O; a.X = (__bf16*)residual; a.L = dm.L; a.Hkv = dm.Hkv;
  return launch_any<true>(a, dm.d, st);
}

}  // namespace tsa
