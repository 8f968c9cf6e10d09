// Causal attention over the compacted token set (Section 2.2, Stage 1), the form for VERY SHORT sets
// (a couple of thousand compacted tokens): one workgroup owns 128 query rows, and its eight
// wavefronts are four row groups (32 rows) x two key groups: of every 64-key tile, key group 0 takes
// keys 0..31 and key group 1 keys 32..63, each with its own running max / sum / output accumulator;
// the two partial results of a row group are merged once, at the end, through LDS.
//
// Why: a wavefront walks its key tiles one after the other, so the time of a launch cannot fall
// below the longest chain (the last query tile of a head).  With 256 rows per workgroup and a few
// thousand compacted tokens that chain, not the chip's throughput, is the makespan.  Splitting the
// keys of a tile over two wavefronts halves the chain per row (a workgroup finishes 128 keys per
// iteration instead of 64) and doubles the number of workgroups, at the price of staging every K / V
// tile for 128 instead of 256 rows.
//
// The iteration is the one of the 256-row kernel (attend.hip): per wavefront a stream of 32 chunks,
//    S^T(half 1) with exp(half 0) | PV(half 0) with the row max of half 1 | S^T(next half 0) with
//    exp(half 1) | PV(half 1) with the row max of the next half 0 and the staging,
// where "half 0 / half 1" of an iteration are the wavefront's 32 keys of the step's first / second
// tile: one step = two 64-key tiles (a, b) = 128 keys, one barrier per step.
// LDS: K tiles of three steps are resident (ring of five tiles: b of the current step, a and b of the
// next one readable, a and b of the step after being written), V tiles of two steps (ring of four):
// what an iteration prefetches across its closing barrier was written an iteration earlier.
#include "attend_common.h"

namespace tsa {

using namespace attend_detail;

namespace {

constexpr int BMS = 128;                // query rows per workgroup
constexpr int kThreadsS = 512;

struct Step {
  Tile a, b;                            // the two 64-key tiles of a step; b.k0 < 0: the step has one tile
};

template <int D, bool FUSED>
__global__ __launch_bounds__(kThreadsS, 2) void attend_split_kernel(AttendArgs a) {
  constexpr int QS = 1;
  constexpr int kThreads = kThreadsS;
  constexpr int RW = 32;
  constexpr int KS = D + 8;
  constexpr int KTILE = BN * KS, VTILE = D * VS;
  constexpr int CH = BN * (D / 8) / kThreads;     // 16-byte chunks per thread per tile
  constexpr int NS = D / 16;
  constexpr int ND = D / 32;
  constexpr int ROWB = D * 2;
  constexpr int NKT = 5, NVT = 4;                 // ring slots
  __shared__ __attribute__((aligned(16))) __bf16 smem[NKT * KTILE + NVT * VTILE];

  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int vhead = xcd * a.vheads_per_xcd + slot % a.vheads_per_xcd;
  const int hp = vhead / a.head_split, part = vhead % a.head_split;
  const int b = hp / a.Hq, h = hp % a.Hq;
  int Lc = a.Lc, nq_tiles = a.nq_tiles;
  if (FUSED && a.k_dev) {
    Lc = a.k_dev[b];
    nq_tiles = (Lc + BMS - 1) / BMS;
  }
  const int qt = nq_tiles - 1 - ((slot / a.vheads_per_xcd) * a.head_split + part);
  if (qt < 0) return;
  const int g = a.Hq / a.kvh;
  const int n_grp = FUSED ? a.Hkv : a.kvh, g_grp = a.Hq / n_grp;
  const long long bh = (long long)b * a.Hq + h;
  const long long bkv = (long long)b * a.kvh + h / g;
  const int q_pitch = FUSED ? (int)a.qs.l * 2 : ROWB, k_pitch = FUSED ? (int)a.ks.l * 2 : ROWB;
  const __bf16* q_head = FUSED ? a.Q + a.qs.head(b, h) : a.Q + bh * Lc * D;
  const __bf16* k_head = FUSED ? a.K + a.ks.head(b, h / g_grp) : a.K + bkv * Lc * D;
  const int n_rows = FUSED ? a.L : Lc;
  const __amdgpu_buffer_rsrc_t Qr = head_rsrc(q_head, (long long)n_rows * q_pitch);
  const __amdgpu_buffer_rsrc_t Kr = head_rsrc(k_head, (long long)n_rows * k_pitch);
  const long long vt_bytes = (long long)a.nk_tiles * BN * ROWB;
  const __amdgpu_buffer_rsrc_t Vr = head_rsrc(a.Vt + bkv * (vt_bytes / 2), vt_bytes);
  const int32_t* idx_row = FUSED ? a.idx + bkv * a.Lc : nullptr;
  const __amdgpu_buffer_rsrc_t Ir = __builtin_amdgcn_make_buffer_rsrc((void*)idx_row, 0, FUSED ? Lc * 4 : 0, 0x00020000);

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const int rg = wave & 3, kg = wave >> 2;               // row group, key group
  const int koff = 32 * kg;                              // this wavefront's keys inside a 64-key tile
  const int q0 = qt * BMS;
  const int wrow0 = q0 + RW * rg;
  const int half_bit = (a.block_list && a.block < BMS) ? 1 << ((RW * rg) / a.block) : 1;
  const float c = a.c;
  const float c_ = c;
  const float inv_c = 1.0f / c;

  // ---- fused form: zero rows of the full-length output between this workgroup's first selected token
  // and the next workgroup's, paced over the tile loop (see attend.hip)
  constexpr int LPR = D / 8, RPP = kThreads / LPR;
  const bool zfill = FUSED && a.Of != nullptr;
  const long long o_pitch16 = FUSED ? a.os.l / 8 : LPR;
  const int32_t* inv_row = nullptr;
  u32x4* zrow = nullptr;
  int z_hi = 0, zt = 0, zr = 0;
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

  // Q^T operand fragments of the wavefront's 32 rows (both key groups hold the same rows)
  bf16x8 qf[QS][NS];
  {
    int qrow_off = (wrow0 + lo) * ROWB;
    if (FUSED) {
      const int qr = wrow0 + lo;
      qrow_off = qr < Lc ? (int)__umul24(idx_row[qr], q_pitch) : a.L * q_pitch;
    }
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(Qr, qrow_off + 16 * hi + 32 * s, 0, 0);
      qf[0][s] = __builtin_bit_cast(bf16x8, v);
    }
  }
  __builtin_amdgcn_s_waitcnt(0x0F70);                    // vmcnt(0), see attend.hip

  // ---- key tiles, two per step
  TileGen gen;
  gen.plain = a.block_list == nullptr;
  gen.plain_i = 0;
  gen.plain_n = (min(q0 + BMS, Lc) + BN - 1) / BN;
  gen.sub = gen.kb = gen.use = 0;
  gen.n_lists = 1;
  gen.block = BMS;
  gen.tiles_per_block = BMS / BN;
  gen.full = 1;
  int longest_list = 0;
#pragma unroll
  for (int j = 0; j < kMaxLists; ++j) { gen.list[j] = nullptr; gen.cnt[j] = gen.pos[j] = 0; gen.cur[j] = INT_MAX; }
  if (!gen.plain) {
    gen.block = a.block;
    gen.n_lists = a.block >= BMS ? 1 : BMS / a.block;    // row blocks of the list inside the 128 rows: 1 or 2
    gen.tiles_per_block = a.block / BN;
    gen.full = 0;
    const int nqb = (Lc + a.block - 1) / a.block;
    const int32_t* bl = a.block_list + bh * a.bl_head_stride;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int qb = q0 / a.block + j;
      if (j < gen.n_lists && qb < nqb) {
        gen.list[j] = bl + (long long)qb * a.max_blocks;
        gen.cnt[j] = count_valid(gen.list[j], a.max_blocks, qb);
        if (gen.cnt[j] > 0) gen.cur[j] = gen.list[j][0];
        gen.full |= 1 << j;
        longest_list = max(longest_list, gen.cnt[j]);
      }
    }
  }
  auto next_step = [&]() -> Step {
    Step s;
    s.a = gen.next();
    s.b = s.a.k0 >= 0 ? gen.next() : Tile{-1, 0};
    return s;
  };
  if (zfill) {
    const int n_pipelined = gen.plain ? q0 / (2 * BN) - 1 : gen.tiles_per_block * longest_list / 2 - 3;
    z_every = max(1, n_pipelined / max(1, z_passes));
  }

  // ---- staging: global -> registers -> LDS in 16-byte chunks, two K tiles and two V tiles per step
  constexpr int kRowsPerPass = kThreads / (D / 8);
  const int st_row = tid / (D / 8), st_col = tid % (D / 8);
  const int lk_off = k_row_perm(st_row) * KS + 8 * st_col;
  const int gv_off = 16 * tid;
  const int lv_off = (tid >> 3) * VS + 8 * (tid & 7);
  constexpr int kVRowsPerPass = kThreads / 8;
  int ktok[2][CH];
  u32x4 kreg[2][CH], vreg[2][CH];
  auto row_off = [&](int tok) -> int { return FUSED ? (int)__umul24(tok, k_pitch) : tok * ROWB; };
  // tiles that do not exist are replaced by tile 0 in the look-ups and loads: loaded, never used
  auto fetch_tok = [&](int j, int k0) {
    k0 = max(k0, 0);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      if (FUSED) ktok[j][i] = __builtin_amdgcn_raw_buffer_load_b32(Ir, (st_row + i * kRowsPerPass) * 4, k0 * 4, 0);
      else ktok[j][i] = k0 + st_row + i * kRowsPerPass;
    }
  };
  auto load_k = [&](int j) {
#pragma unroll
    for (int i = 0; i < CH; ++i)
      kreg[j][i] = __builtin_amdgcn_raw_buffer_load_b128(Kr, row_off(ktok[j][i]) + 16 * st_col, 0, 0);
  };
  auto load_v = [&](int j, int k0) {
    k0 = max(k0, 0);
#pragma unroll
    for (int i = 0; i < CH; ++i)
      vreg[j][i] = __builtin_amdgcn_raw_buffer_load_b128(Vr, gv_off + i * kThreads * 16, k0 * ROWB, 0);
  };
  auto store_k = [&](__bf16* dst, int j) {
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u32x4*)(&dst[lk_off + i * kRowsPerPass * KS]) = kreg[j][i];
  };
  auto store_v = [&](__bf16* dst, int j) {
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u32x4*)(&dst[lv_off + i * kVRowsPerPass * VS]) = vreg[j][i];
  };

  // LDS read bases: the wavefront's 32 keys are rows koff.. of a K tile and columns koff.. of a V^T tile
  const int k_rd = (koff + lo) * KS + 8 * hi;
  const int v_rd = lo * VS + 8 * hi + koff;

  f32x16 o[QS][ND];
  float m[QS], l[QS];
  m[0] = kNegBig;
  l[0] = 0.f;
#pragma unroll
  for (int dt = 0; dt < ND; ++dt) o[0][dt] = f32x16{0};

  // Ring roles at the top of the iteration of step j:
  //   K: kb0 = b_j, ka1 = a_(j+1), kb1 = b_(j+1) readable; kwa, kwb receive a_(j+2), b_(j+2) during the iteration
  //   V: va0 = a_j, vb0 = b_j readable; vwa, vwb receive a_(j+1), b_(j+1)
  __bf16* kb0 = smem;
  __bf16* ka1 = smem + KTILE;
  __bf16* kb1 = smem + 2 * KTILE;
  __bf16* kwa = smem + 3 * KTILE;
  __bf16* kwb = smem + 4 * KTILE;
  __bf16* va0 = smem + NKT * KTILE;
  __bf16* vb0 = va0 + VTILE;
  __bf16* vwa = va0 + 2 * VTILE;
  __bf16* vwb = va0 + 3 * VTILE;
  auto rotate = [&]() {
    __bf16* r0 = kb0; __bf16* r1 = ka1;
    kb0 = kb1; ka1 = kwa; kb1 = kwb; kwa = r0; kwb = r1;
    __bf16* t = va0; va0 = vwa; vwa = t;
    t = vb0; vb0 = vwb; vwb = t;
  };

  // ---- prologue: K of steps 0 and 1 and V of step 0 into LDS, S^T of the first half
  Step S0 = next_step(), S1 = next_step(), S2 = next_step(), S3 = next_step();
  f32x16 sA[QS], sB[QS];
  uint32_t pA[QS][8], pB[QS][8];
  // half tile h of step S: first key and whether this wavefront takes part in it
  auto act = [&](const Tile& t) -> bool { return t.k0 >= 0 && (t.use & half_bit) && t.k0 + koff <= wrow0 + RW - 1; };
  if (S0.a.k0 >= 0) {
    fetch_tok(0, S0.a.k0);
    fetch_tok(1, S0.b.k0);
    load_k(0);
    load_k(1);
    load_v(0, S0.a.k0);
    load_v(1, S0.b.k0);
    store_k(kwa, 0);                 // a_0 only serves the first S^T below; the slot is free again after the second barrier
    store_k(kb0, 1);
    store_v(va0, 0);
    store_v(vb0, 1);
    if (S1.a.k0 >= 0) {
      fetch_tok(0, S1.a.k0);
      fetch_tok(1, S1.b.k0);
      load_k(0);
      load_k(1);
      store_k(ka1, 0);
      store_k(kb1, 1);
    }
  }
  __syncthreads();
  if (S0.a.k0 >= 0) qk_half<D, QS>(kwa, k_rd, qf, sA);
  __syncthreads();
  // in flight from here on: K of step 2, V of step 1; token ids of step 3
  fetch_tok(0, S2.a.k0);
  fetch_tok(1, S2.b.k0);
  load_k(0);
  load_k(1);
  load_v(0, S1.a.k0);
  load_v(1, S1.b.k0);
  fetch_tok(0, S3.a.k0);
  fetch_tok(1, S3.b.k0);
  if (act(S0.a)) {
    if (S0.a.k0 + koff + 31 > wrow0) mask_half<QS>(sA, S0.a.k0 + koff, hi, wrow0 + lo);
    softmax_max<ND, QS>(sA, c, m, l, o);
  }

  // ---- the pipelined iteration (all four tiles of this step and the next lie below the workgroup's first
  // row and are used by all its wavefronts): the chunk stream of attend.hip with this kernel's pointers
  constexpr int kPF = TSA_PF, kRing = TSA_RING, kChunks = 4 * NS;
  static_assert(NS == 8 || NS == 4, "chunk stream is laid out for d = 128 or 64");
  constexpr int CPB = kChunks / 4;
  static_assert(kChunks % kRing == 0 && kRing > kPF && kPF <= CPB, "fragment ring does not fit the chunk stream");
  static_assert(4 * CH <= CPB, "staging of a step does not fit the last block");
  bf16x8 kfr[kRing];
  // fragment fetch for chunk c: block 0 reads b of the current step (kb_), block 2 a of the next (ka_),
  // blocks 1 and 3 the V tiles a and b of the current step
  auto fetch = [&](int c, const __bf16* kb_, const __bf16* ka_, const __bf16* va_, const __bf16* vb_) {
    const int blk = c / CPB, i = c % CPB, slot = c % kRing;
    if (blk == 0) kfr[slot] = *(const bf16x8*)(&kb_[k_rd + 16 * i]);
    else if (blk == 2) kfr[slot] = *(const bf16x8*)(&ka_[k_rd + 16 * i]);
    else {
      const int hf = i / ND, dt = i % ND;
      kfr[slot] = *(const bf16x8*)(&(blk == 1 ? va_ : vb_)[v_rd + (32 * dt) * VS + 16 * hf]);
    }
  };
  auto prime_ring = [&]() {
#pragma unroll
    for (int c = 0; c < kPF; ++c) fetch(c, kb0, ka1, va0, vb0);
  };
  // vload_*: byte offsets of the V tiles of step 2; tok_*: first compacted rows of the K tiles of step 4
  auto fast_iter = [&](const int vload_a, const int vload_b, const int tok_a, const int tok_b) {
    float mxc[QS], mx[QS], ps0[QS], ps1[QS];
    f32x16 acc[QS];
#pragma unroll
    for (int c = 0; c < kChunks; ++c) {
      const int blk = c / CPB, i = c % CPB, slot = c % kRing;
      if (i == 0) {
        if (blk == 0 || blk == 2) __builtin_amdgcn_s_setprio(2);
        else __builtin_amdgcn_s_setprio(0);
      }
      // the first chunks of the next iteration read b of the next step: complete since the previous barrier
      if (c + kPF < kChunks) fetch(c + kPF, kb0, ka1, va0, vb0);
      else fetch(c + kPF - kChunks, kb1, kwa, vwa, vwb);
      if (blk == 0 || blk == 2) {
        const f32x16 (&s_in)[QS] = blk == 0 ? sA : sB;
        uint32_t (&p_out)[QS][8] = blk == 0 ? pA : pB;
        constexpr int EPS = 16 / NS;
        if (i == 0) acc[0] = f32x16{0};
        acc[0] = mfma32(kfr[slot], qf[0][i], acc[0]);
#pragma unroll
        for (int e = 0; e < EPS; e += 2) {
          const int r = EPS * i + e;
          const float p0 = fast_exp2(s_in[0][r]);
          const float p1 = fast_exp2(s_in[0][r + 1]);
          if (r == 0) { ps0[0] = p0; ps1[0] = p1; }
          else { ps0[0] += p0; ps1[0] += p1; }
          p_out[0][r >> 1] = pack_bf16(p0, p1);
        }
        if (i == CPB - 1) {
          f32x16 (&s_out)[QS] = blk == 0 ? sB : sA;
          s_out[0] = acc[0];
          l[0] += ps0[0] + ps1[0];
        }
      } else {
        f32x16 (&s_in)[QS] = blk == 1 ? sB : sA;
        const uint32_t (&pb)[QS][8] = blk == 1 ? pA : pB;
        const int hf = i / ND, dt = i % ND;
        constexpr int EPC = 16 / CPB;
        const bf16x8 vf = kfr[slot];
        o[0][dt] = mfma32(vf, p_operand(pb[0], hf), o[0][dt]);
#pragma unroll
        for (int e = 0; e < EPC; ++e) s_in[0][EPC * i + e] = fmaf(s_in[0][EPC * i + e], c_, -m[0]);
        if (i == 0) mx[0] = s_in[0][0];
        if (EPC == 2) mx[0] = __builtin_fmaxf(__builtin_fmaxf(mx[0], s_in[0][2 * i]), s_in[0][2 * i + 1]);
        else {
#pragma unroll
          for (int e = 0; e < EPC; ++e) mx[0] = fmaxf(mx[0], s_in[0][EPC * i + e]);
        }
        if (blk == 3) {                 // K of step 2 -> kwa, kwb; V of step 1 -> vwa, vwb; then refill the registers
          if (i < 2 * CH) {
            const int j = i / CH, ii = i % CH;
            *(u32x4*)(&(j == 0 ? kwa : kwb)[lk_off + ii * kRowsPerPass * KS]) = kreg[j][ii];
            kreg[j][ii] = __builtin_amdgcn_raw_buffer_load_b128(Kr, row_off(ktok[j][ii]) + 16 * st_col, 0, 0);
            const int tk = j == 0 ? tok_a : tok_b;
            if (FUSED) ktok[j][ii] = __builtin_amdgcn_raw_buffer_load_b32(Ir, (st_row + ii * kRowsPerPass) * 4, tk * 4, 0);
            else ktok[j][ii] = tk + st_row + ii * kRowsPerPass;
          } else if (i < 4 * CH) {
            const int j = (i - 2 * CH) / CH, ii = (i - 2 * CH) % CH;
            *(u32x4*)(&(j == 0 ? vwa : vwb)[lv_off + ii * kVRowsPerPass * VS]) = vreg[j][ii];
            vreg[j][ii] = __builtin_amdgcn_raw_buffer_load_b128(Vr, gv_off + ii * kThreads * 16, j == 0 ? vload_a : vload_b, 0);
          }
        }
        if (FUSED && blk == 3 && i == CPB - 1 && zfill && --z_count <= 0) {
          zero_step();
          z_count = z_every;
        }
        if (i == CPB - 1) mxc[0] = fmaxf(mx[0], __shfl_xor(mx[0], 32));
      }
      __builtin_amdgcn_sched_barrier(0);
      if (c == 2 * CPB - 1) raise_max_rel<ND, QS>(mxc, m, l, o, sB);
    }
    lds_barrier();
    raise_max_rel<ND, QS>(mxc, m, l, o, sA);
    rotate();
  };

  // ---- step loop
  auto tile_pipelined = [&](const Tile& t) -> bool { return t.k0 >= 0 && t.use == gen.full && t.k0 + BN <= q0; };
  auto pipelined = [&](const Step& s) -> bool { return tile_pipelined(s.a) && tile_pipelined(s.b); };
  while (S0.a.k0 >= 0) {
    if (pipelined(S0) && pipelined(S1)) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sA[0][r] = fmaf(sA[0][r], c_, -m[0]);
      prime_ring();
      do {
        const Step S4 = next_step();
        fast_iter(max(S2.a.k0, 0) * ROWB, max(S2.b.k0, 0) * ROWB, max(S4.a.k0, 0), max(S4.b.k0, 0));
        S0 = S1; S1 = S2; S2 = S3; S3 = S4;
      } while (pipelined(S0) && pipelined(S1));
      if (S0.a.k0 < 0) break;
#pragma unroll
      for (int r = 0; r < 16; ++r) sA[0][r] = (sA[0][r] + m[0]) * inv_c;
    }
    // general iteration: masks and per-wavefront decisions
    if (S0.b.k0 >= 0) qk_half<D, QS>(kb0, k_rd, qf, sB);
    if (act(S0.a)) {
      softmax_exp<QS>(sA, c, m, l, pA);
      pv_half<D, QS>(va0, v_rd, pA, o);
    }
    if (act(S0.b)) {
      if (S0.b.k0 + koff + 31 > wrow0) mask_half<QS>(sB, S0.b.k0 + koff, hi, wrow0 + lo);
      softmax_max<ND, QS>(sB, c, m, l, o);
      softmax_exp<QS>(sB, c, m, l, pB);
      pv_half<D, QS>(vb0, v_rd, pB, o);
    }
    if (S1.a.k0 >= 0) qk_half<D, QS>(ka1, k_rd, qf, sA);
    if (act(S1.a)) {
      if (S1.a.k0 + koff + 31 > wrow0) mask_half<QS>(sA, S1.a.k0 + koff, hi, wrow0 + lo);
      softmax_max<ND, QS>(sA, c, m, l, o);
    }
    if (S2.a.k0 >= 0) {
      store_k(kwa, 0);
      store_k(kwb, 1);
    }
    if (S1.a.k0 >= 0) {
      store_v(vwa, 0);
      store_v(vwb, 1);
    }
    if (S3.a.k0 >= 0) {
      load_k(0);
      load_k(1);
    }
    if (S2.a.k0 >= 0) {
      load_v(0, S2.a.k0);
      load_v(1, S2.b.k0);
    }
    const Step S4 = next_step();
    if (S4.a.k0 >= 0) {
      fetch_tok(0, S4.a.k0);
      fetch_tok(1, S4.b.k0);
    }
    lds_barrier();
    S0 = S1; S1 = S2; S2 = S3; S3 = S4;
    rotate();
  }

  // ---- fused form: the zero rows the loop did not get to
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

  // ---- merge of the two key groups: group 1 hands (m, l, O) of its rows to group 0 through LDS
  constexpr int NF = 2 + 16 * ND;                        // floats per lane
  float* mrg = (float*)smem + (rg * NF) * 64 + lane;     // field f of this lane: mrg[f * 64]
  static_assert(4 * NF * 64 * 4 <= (NKT * KTILE + NVT * VTILE) * 2, "merge buffer does not fit the tile rings");
  __syncthreads();                                       // every wavefront is done with the tiles
  if (kg == 1) {
    mrg[0] = m[0];
    mrg[64] = l[0];
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) mrg[(2 + 16 * dt + r) * 64] = o[0][dt][r];
  }
  __syncthreads();
  if (kg == 1) return;
  {
    const float m1 = mrg[0], l1 = mrg[64];
    const float mn = fmaxf(m[0], m1);
    const float a0 = fast_exp2(m[0] - mn), a1 = fast_exp2(m1 - mn);
    l[0] = l[0] * a0 + l1 * a1;
    m[0] = mn;
#pragma unroll
    for (int dt = 0; dt < ND; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[0][dt][r] = o[0][dt][r] * a0 + mrg[(2 + 16 * dt + r) * 64] * a1;
  }

  // ---- epilogue (key group 0): normalise, round to bf16, store
  {
    const int qrow = wrow0 + lo;
    const float lt = l[0] + __shfl_xor(l[0], 32);
    const float inv_l = lt > 0.f ? 1.0f / lt : 0.f;
    if (qrow < Lc) {
      __bf16* orow = a.O ? a.O + (bh * a.Lc + qrow) * D : nullptr;
      __bf16* frow = nullptr;
      __bf16* xrow = nullptr;
      if (FUSED && a.Of) frow = a.Of + a.os.head(b, h) + idx_row[qrow] * a.os.l;
      if (FUSED && a.X) xrow = a.X + (((long long)b * a.L + idx_row[qrow]) * a.Hq + h) * D;
#pragma unroll
      for (int dt = 0; dt < ND; ++dt)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          u32x2 w;
          w[0] = pack_bf16(o[0][dt][4 * q4 + 0] * inv_l, o[0][dt][4 * q4 + 1] * inv_l);
          w[1] = pack_bf16(o[0][dt][4 * q4 + 2] * inv_l, o[0][dt][4 * q4 + 3] * inv_l);
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
      if (a.lse && hi == 0) a.lse[bh * a.Lc + qrow] = (m[0] + log2f(lt)) * kLn2;
    }
  }
}

}  // namespace

hipError_t launch_attend_split(AttendArgs& a, int d, bool fused, hipStream_t st) {
  a.nq_tiles = (a.Lc + BMS - 1) / BMS;
  a.nk_tiles = (a.Lc + BN - 1) / BN;
  map_workgroups(a);
  const unsigned grid = grid_for(a);
  if (d == 128) {
    if (fused) attend_split_kernel<128, true><<<grid, kThreadsS, 0, st>>>(a);
    else attend_split_kernel<128, false><<<grid, kThreadsS, 0, st>>>(a);
  } else {
    if (fused) attend_split_kernel<64, true><<<grid, kThreadsS, 0, st>>>(a);
    else attend_split_kernel<64, false><<<grid, kThreadsS, 0, st>>>(a);
  }
  return hipGetLastError();
}

}  // namespace tsa
