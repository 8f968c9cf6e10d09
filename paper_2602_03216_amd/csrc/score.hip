// Token scoring: Algorithm 1 of the paper, its first two steps (proxy attention of the most recent
// queries, then the per-head column sums):  A = softmax(Q[-last_q:] K^T * scale) (causal inside the
// window), s[h,t] = sum_i A[i,t].
//
// Exact two-pass softmax, both passes on bf16 MFMA with fp32 accumulation:
//   pass 1  S^T = K Q^T   (lane = query, registers = keys): per-query running max / sum of
//           exponentials over a chunk of keys -> partial (max, sum) per (head, query, chunk)
//   lse     combine the chunk partials into one log2-sum-exp per (head, query)
//   pass 2  S = Q K^T     (lane = key, registers = queries): p = exp2(x - lse) summed over the
//           queries inside the lane, one cross-half add, coalesced store of s[h, t]
// The two orientations use the same register fragments (a lane holds 8 consecutive d-values of
// one row), only the operand order of the MFMA is swapped, so neither pass needs a cross-lane
// reduction longer than one step.  A workgroup serves one KV head and one chunk of keys for all
// the query heads of the group: K tiles are staged in LDS once and every wavefront (one query
// head each) reads its fragments from there.
// Staging: tiles of 128 keys go from global memory straight into LDS (buffer loads with the LDS
// modifier: no staging registers, no LDS store instructions, no address arithmetic in the loop), into a
// ring of two tiles, the load of tile t + 1 in flight while tile t is computed.  Such a load writes the
// 64 lanes' 16-byte pieces to consecutive LDS addresses, so rows cannot be padded; instead the 16-byte
// pieces of a row are stored in an order that depends on the row (piece p of row r sits at position
// p ^ swz(r)), chosen on the global side of the load, which makes the fragment reads (16 bytes per lane,
// 16 consecutive rows at a time) free of bank conflicts.
// Tiles that every scoring query sees in full (all but the last few of a sequence) take a
// software-pipelined body: a "unit" is one 32-key x 32-query block (D/16 MFMAs, 16 scores per
// lane); the MFMAs of the next unit are issued chunk by chunk between the exponentials of the
// current one, so the matrix pipe and the vector ALU overlap inside the wavefront, and the pipeline
// runs on across tile boundaries (the wait for the next tile and the workgroup barrier sit between the
// last two units of a tile).  In pass 1 that body does not compute a row max at all: the running max only
// has to keep the exponentials in range, so the sum itself is the detector (a unit whose sum leaves the
// range is redone the exact way, with the true max; this happens once per row in practice).
#include "tsa_internal.h"

#include <type_traits>

namespace tsa {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kMinChunk = 256;               // keys per workgroup: at least this, a multiple of 128 (every tile size divides it)
constexpr float kNegBig = -1.0e30f;
constexpr float kSumLimit = 1073741824.0f;   // 2^30: a unit's sum of exponentials beyond this means the running max lags too far

constexpr int kMaxQueries = 128;

struct ScoreArgs {
  const __bf16* Q;             // scoring queries: row i of head (b, h) at Q + qs.head(b, h) + (q_row0 + i) * qs.l
  Strides qs, ks;              // layout of Q (or of the caller's query rows) and of K
  int q_row0;
  int min_pos;                 // smallest entry of qpos
  int qpos[kMaxQueries];       // position of scoring query i (ascending; query i sees keys t <= qpos[i]); padded with L - 1
  const __bf16* K;
  float* scores;
  float2* part;       // [B*Hq][nchunks][QP] (max, sum) in the log2 domain
  float* lse2;        // [B*Hq][QP]
  int Hq, Hkv, L, Lq, nchunks, chunk;      // chunk = keys per workgroup
  int pool_w;
  float* pooled;      // final output when pool_w > 1 (scores then points at a raw buffer)
  float c;            // scale * log2(e)
};

// Q fragments of one head: rows q_row0 .. q_row0 + Lq - 1 through a buffer descriptor that ends after row
// Lq - 1, so the padding rows of the last query sub-tile arrive as zeros without a select (nothing here
// waits for the loads).
template <int D, int NQT>
__device__ __forceinline__ void load_q_frags(const ScoreArgs& a, int b, int h, int lo, int hi, bf16x8 (&qf)[NQT][D / 16]) {
  const int pitch = (int)a.qs.l * 2;
  const __bf16* base = a.Q + a.qs.head(b, h) + (long long)a.q_row0 * a.qs.l;
  const __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, a.Lq * pitch, 0x00020000);
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int off = (32 * qt + lo) * pitch + 16 * hi;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) qf[qt][s] = __builtin_bit_cast(bf16x8, __builtin_amdgcn_raw_buffer_load_b128(r, off + 32 * s, 0, 0));
  }
}

// How a workgroup of (KV head, chunk of keys) spreads its four wavefronts over the g query heads
// that share the KV head: `hpw` heads are processed at a time, one per wavefront, and the
// remaining factor splits the keys of every staged tile.  Heads beyond hpw take further rounds.
struct WaveRole {
  int hpw, ksplit, hslot, kpart;
};
__device__ __forceinline__ WaveRole wave_role(int g, int wave) {
  WaveRole r;
  r.hpw = g >= 4 ? 4 : (g >= 2 ? 2 : 1);
  r.ksplit = kWaves / r.hpw;
  r.hslot = wave % r.hpw;
  r.kpart = wave / r.hpw;
  return r;
}

// ---- K tiles in LDS.  A tile is TK rows of 2 D bytes, unpadded; the 16-byte piece p of row r is stored
// at piece position p ^ swz(r).  A fragment read takes piece (hi + 2 i) of 32 consecutive rows: within
// every group of 16 lanes (16 consecutive rows, the same piece) the positions differ in the bits that
// select the bank, for D = 128 (256-byte rows: swz = r mod 16) and for D = 64 (128-byte rows, two per 256
// bytes: swz = (r / 2) mod 8) alike.
template <int D, int TK>
struct Geo {
  static constexpr int RB = 2 * D;               // bytes of a row
  static constexpr int CPR = D / 8;              // 16-byte pieces of a row
  static constexpr int RPW = 64 / CPR;           // rows one wavefront-wide load covers (1 KiB)
  static constexpr int RPI = kWaves * RPW;       // rows one workgroup-wide round of loads covers
  static constexpr int NLD = TK / RPI;           // loads per thread and tile
  static constexpr int TILE = TK * D;            // elements of a tile
  static_assert(TK % RPI == 0 && RPI % 16 == 0, "a round of loads covers whole periods of the swizzle");
  __device__ static __forceinline__ int swz(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
  // byte offset inside a 32-row sub-tile of the lane's fragment for k-step 0; k-step i is at frag_base ^ (i << 5)
  __device__ static __forceinline__ int frag_base(int lo, int hi) { return lo * RB + ((hi ^ swz(lo)) << 4); }
};

typedef __attribute__((address_space(3))) void* lds_void_ptr;

template <int D>
__device__ __forceinline__ bf16x8 frag(const __bf16* tile, int fbase, int sub, int i) {
  return *(const bf16x8*)((const char*)tile + 32 * sub * 2 * D + (fbase ^ (i << 5)));
}

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Waits until at most N of this wavefront's vector memory operations are outstanding (they complete in
// the order of issue, loads and stores alike).
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N <= 63, "the counter has six bits");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// The ring of staged tiles of one workgroup and chunk: tile t (keys c_begin + t TK ..) lives in slot
// t % NB, and up to NB - 1 tiles are in flight ahead of the one being read.  Lane l of wavefront w asks, in
// round j of a tile, for the piece that belongs at LDS byte (j kWaves + w) 1024 + 16 l of the tile: row
// j RPI + w RPW + l / CPR, position l % CPR.  Rows at or beyond L lie outside the buffer descriptor and
// arrive as zeros.
template <int D, int TK, int NB>
struct Ring {
  using G = Geo<D, TK>;
  __amdgpu_buffer_rsrc_t rsrc;
  __bf16* tiles;               // LDS, NB tiles
  int voff, pitch, wave, c_begin, n_tiles;
  __device__ __forceinline__ void init(const __bf16* Kh, long long row_stride, int L, int tid, __bf16* lds, int c_begin_, int n_tiles_) {
    pitch = (int)row_stride * 2;
    rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)Kh, 0, L * pitch, 0x00020000);
    wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63, r = wave * G::RPW + lane / G::CPR;
    voff = r * pitch + (((lane % G::CPR) ^ G::swz(r)) << 4);
    tiles = lds; c_begin = c_begin_; n_tiles = n_tiles_;
  }
  __device__ __forceinline__ void issue(int t, int slot) const {
#if defined(__HIP_DEVICE_COMPILE__)                        // the host pass has no such builtin and no LDS address space
    const int k0 = c_begin + t * TK;
#pragma unroll
    for (int j = 0; j < G::NLD; ++j)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void_ptr)((char*)(tiles + slot * G::TILE) + (j * kWaves + wave) * 1024), 16,
                                               voff, (k0 + j * G::RPI) * pitch, 0, 0);
#endif
  }
  // first tiles of a sweep (the ring must be idle: a workgroup barrier since its last read); the slot that
  // stays empty is filled when tile 0 is entered
  __device__ __forceinline__ void start() const {
#pragma unroll
    for (int t = 0; t < NB - 1; ++t)
      if (t < n_tiles) issue(t, t);
  }
  // Before the first read of tile t (slot SLOT = t % NB): this wavefront's loads of the tile have landed,
  // every wavefront is past its last read of tile t - 1 and has its part of tile t in place; the slot of tile
  // t - 1 then takes tile t + NB - 1.  Outstanding at the wait may be: the loads of the tiles t + 1 .. t + NB - 2
  // (as far as the chunk has them), issued after those of tile t, and NVM further vector memory operations
  // that the caller has issued after the loads of tile t.
  template <int SLOT, int NVM>
  __device__ __forceinline__ void enter(int t) const {
    if (NB == 2) {
      wait_vm<NVM>();
    } else {
      static_assert(NB == 2 || NB == 4, "the list below is for two tiles ahead");
      const int ahead = min(NB - 2, n_tiles - 1 - t);
      if (ahead >= 2) wait_vm<NVM + 2 * G::NLD>();
      else if (ahead == 1) wait_vm<NVM + G::NLD>();
      else wait_vm<NVM>();
    }
    lds_barrier();
    const int tn = t + NB - 1;
    if (tn < n_tiles) issue(tn, (SLOT + NB - 1) % NB);
  }
};

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// ---- pipelined tile bodies (tiles without any mask).  SPT = 32-key sub-tiles of the staged tile
// that this wavefront owns, starting at sub-tile `first_sub`.  Units run in the order
// (sub-tile, query sub-tile); while unit u is in the vector ALU the MFMAs of unit u + 1 are issued;
// the unit after the last one of a tile is unit 0 of the next tile, entered (Ring::enter) in between.
// The K fragments live in ONE set of registers: right after the MFMA that uses fragment i of a
// sub-tile for the last time, the register is reloaded with fragment i of the next sub-tile, which is
// consumed a whole unit later (across a tile boundary: all fragments right after the tile is entered).
template <int D, int NQT, int SPT, bool KEYS_ARE_ROWS>
struct UnitPipe {
  static constexpr int NS = D / 16, U = SPT * NQT;
  int fbase, first_sub;
  bf16x8 kf[NS];
  __device__ __forceinline__ void load_all(const __bf16* tile) {
#pragma unroll
    for (int i = 0; i < NS; ++i) kf[i] = frag<D>(tile, fbase, first_sub, i);
  }
  // MFMA i of unit `nu` (compile-time) of the tile `tile`, then the in-place reload if unit nu + 1 starts a
  // new sub-tile of the same tile
  __device__ __forceinline__ void step(const __bf16* tile, int nu, int i, const bf16x8 (&qf)[NQT][NS], f32x16& nxt) {
    const bf16x8 q = qf[nu % NQT][i];
    nxt = KEYS_ARE_ROWS ? mfma32(kf[i], q, nxt) : mfma32(q, kf[i], nxt);
    if (nu + 1 < U && (nu + 1) / NQT != nu / NQT) kf[i] = frag<D>(tile, fbase, first_sub + (nu + 1) / NQT, i);
  }
  // unit 0 of `tile` with nothing beside it (start of a sweep, or after a masked tile)
  __device__ __forceinline__ void prime(const __bf16* tile, const bf16x8 (&qf)[NQT][NS], f32x16& acc) {
    load_all(tile);
    acc = f32x16{0};
#pragma unroll
    for (int i = 0; i < NS; ++i) step(tile, 0, i, qf, acc);
  }
};

// Pass 1, lane = query: z[qt] += sum over the tile's keys of exp2(x c - m[qt]).  `acc` holds unit 0 of the
// tile on entry if `primed`; with `chain_next` the tile after this one is entered inside and its unit 0 is
// left in `acc`.
template <int D, int NQT, int SPT, int TK, int NB, int SLOT>
__device__ __forceinline__ void fast_tile_pass1(const Ring<D, TK, NB>& ring, int t, bool& primed, bool chain_next,
                                                UnitPipe<D, NQT, SPT, true>& pp, f32x16& acc,
                                                const bf16x8 (&qf)[NQT][D / 16], float c, float (&m)[NQT], float (&z)[NQT]) {
  constexpr int NS = D / 16, EPC = 16 / NS, U = SPT * NQT, kNextSlot = (SLOT + 1) % NB, TILE = Geo<D, TK>::TILE;
  const __bf16* cur = ring.tiles + SLOT * TILE;
  const __bf16* nxt_tile = ring.tiles + kNextSlot * TILE;
  if (!primed) pp.prime(cur, qf, acc);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int qt = u % NQT;
    const float mq = m[qt];
    f32x16 nxt = {0};
    float s0 = 0.f, s1 = 0.f;
    auto soft = [&](int i) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const float p = fast_exp2(fmaf(acc[EPC * i + e], c, -mq));
        if (e & 1) s1 += p; else s0 += p;
      }
    };
    if (u + 1 < U) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        pp.step(cur, u + 1, i, qf, nxt);
        soft(i);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (chain_next) {
      ring.template enter<kNextSlot, 0>(t + 1);
      pp.load_all(nxt_tile);
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        soft(i);
        pp.step(nxt_tile, 0, i, qf, nxt);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NS; ++i) soft(i);
    }
    // The sum is the detector: one uniform branch per unit; the exact update runs for the whole wavefront when
    // any lane needs it, and keeps the cheap result in the lanes that do not.
    const float sum = s0 + s1;
    const bool redo = !(sum < kSumLimit);                // out of range (or the very first unit)
    if (__builtin_expect(__builtin_amdgcn_ballot_w64(redo) != 0, 0)) {
      float mx = acc[0];
#pragma unroll
      for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
      const float mn = fmaxf(mq, mx * c);
      float t0 = 0.f, t1 = 0.f;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        t0 += fast_exp2(fmaf(acc[r], c, -mn));
        t1 += fast_exp2(fmaf(acc[r + 1], c, -mn));
      }
      const float zx = z[qt] * fast_exp2(mq - mn) + t0 + t1;
      z[qt] = redo ? zx : z[qt] + sum;
      m[qt] = redo ? mn : mq;
    } else {
      z[qt] += sum;
    }
    acc = nxt;
  }
  primed = chain_next;
}

// Pass 2, lane = key: s[t] = sum over the queries of exp2(x c - lse[query]); one store per sub-tile.
template <int D, int NQT, int SPT, int TK, int NB, int SLOT>
__device__ __forceinline__ void fast_tile_pass2(const Ring<D, TK, NB>& ring, int t, bool& primed, bool chain_next,
                                                UnitPipe<D, NQT, SPT, false>& pp, f32x16& acc,
                                                const bf16x8 (&qf)[NQT][D / 16], float c, const float (&lse)[NQT][16],
                                                float* out, int hi) {
  constexpr int NS = D / 16, EPC = 16 / NS, U = SPT * NQT, kNextSlot = (SLOT + 1) % NB, TILE = Geo<D, TK>::TILE;
  const __bf16* cur = ring.tiles + SLOT * TILE;
  const __bf16* nxt_tile = ring.tiles + kNextSlot * TILE;
  if (!primed) pp.prime(cur, qf, acc);
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int qt = u % NQT, sb = u / NQT;
    f32x16 nxt = {0};
    auto soft = [&](int i) {
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const int r = EPC * i + e;
        const float p = fast_exp2(fmaf(acc[r], c, -lse[qt][r]));
        if (e & 1) s1 += p; else s0 += p;
      }
    };
    if (u + 1 < U) {
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        pp.step(cur, u + 1, i, qf, nxt);
        soft(i);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else if (chain_next) {
      // the stores of this tile's earlier sub-tiles (SPT - 1 of them) were issued after the loads waited for
      ring.template enter<kNextSlot, SPT - 1>(t + 1);
      pp.load_all(nxt_tile);
#pragma unroll
      for (int i = 0; i < NS; ++i) {
        soft(i);
        pp.step(nxt_tile, 0, i, qf, nxt);
        __builtin_amdgcn_sched_barrier(0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NS; ++i) soft(i);
    }
    acc = nxt;
    if (qt == NQT - 1) {
      float colsum = s0 + s1;
      colsum += __shfl_xor(colsum, 32);
      if (hi == 0) out[32 * sb] = colsum;
      s0 = s1 = 0.f;
    }
  }
  primed = chain_next;
}

// Tiles of the chunk that every scoring query sees in full and that end inside the sequence: a prefix.
template <int TK>
__device__ __forceinline__ int fast_tiles(const ScoreArgs& a, int c_begin, int n_tiles) {
  const int x = min(a.min_pos + 1, a.L) - c_begin;
  return x <= 0 ? 0 : min(x / TK, n_tiles);
}

// HPW = query heads a workgroup serves at a time (wave_role: 4, 2 or 1 wavefronts with a head each, the others
// split the keys of a tile).  Tiles of 128 keys in a ring of two: the passes are bound by their instruction
// stream (two exponentials per MFMA), not by the stream of keys (measured: tiles of 64 keys in a ring of four,
// three in flight, are no faster and pay twice the barriers), so one tile in flight ahead is enough.
template <int HPW>
struct TileCfg {
  static constexpr int TK = 128;
  static constexpr int NB = 2;
  static constexpr int SPT = (TK / 32) / (kWaves / HPW);   // 32-key sub-tiles of a tile per wavefront
};

template <int D, int NQT, int HPW>
__global__ __launch_bounds__(kThreads, NQT <= 2 ? 2 : 1) void score_pass1(ScoreArgs a) {
  using C = TileCfg<HPW>;
  constexpr int TK = C::TK, NB = C::NB, SPT = C::SPT;
  using G = Geo<D, TK>;
  constexpr int QP = 32 * NQT;
  __shared__ __attribute__((aligned(1024))) __bf16 Ks[NB * G::TILE];
  __shared__ float2 red[kWaves][QP];
  const int chunk = blockIdx.x;
  const int bkv = blockIdx.y;                            // (batch entry, KV head): 32-bit index arithmetic, no 64-bit division
  const int kv = bkv % a.Hkv, b = bkv / a.Hkv;
  const int g = a.Hq / a.Hkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const WaveRole role = wave_role(g, wave);              // role.hpw == HPW (chosen by the host from g)
  const int c_begin = chunk * a.chunk, c_end = min(c_begin + a.chunk, a.L);
  const int n_tiles = (c_end - c_begin + TK - 1) / TK;
  const int n_fast = fast_tiles<TK>(a, c_begin, n_tiles);
  const int first_sub = role.kpart * SPT;
  int my_pos[NQT];                                       // position of this lane's query in each query sub-tile
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) my_pos[qt] = a.qpos[32 * qt + lo];
  Ring<D, TK, NB> ring;
  ring.init(a.K + a.ks.head(b, kv), a.ks.l, a.L, tid, Ks, c_begin, n_tiles);
  const int fbase = G::frag_base(lo, hi);

  for (int r0 = 0; r0 < g; r0 += role.hpw) {
    const int hh = r0 + role.hslot;
    const bool act = hh < g;
    const int head = kv * g + (act ? hh : 0);
    bf16x8 qf[NQT][D / 16];
    __syncthreads();                                   // the previous round is done with the ring and with red[]
    load_q_frags<D, NQT>(a, b, head, lo, hi, qf);           // the Q fragments (served by the L2) ahead of the first K tiles
    ring.start();
    float m[NQT], z[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { m[qt] = kNegBig; z[qt] = 0.f; }
    UnitPipe<D, NQT, SPT, true> pp;
    pp.fbase = fbase;
    pp.first_sub = first_sub;
    f32x16 acc = {0};
    bool primed = false;
    auto tile = [&](int t, auto slot_tag) {
      constexpr int SLOT = decltype(slot_tag)::value, kNextSlot = (SLOT + 1) % NB;
      if (!primed) ring.template enter<SLOT, 0>(t);
      if (t < n_fast) {
        const bool chain_next = t + 1 < n_fast;
        if (act) {
          fast_tile_pass1<D, NQT, SPT, TK, NB, SLOT>(ring, t, primed, chain_next, pp, acc, qf, a.c, m, z);
        } else {
          if (chain_next) ring.template enter<kNextSlot, 0>(t + 1);
          primed = chain_next;
        }
        return;
      }
      primed = false;
      if (!act) return;
      const __bf16* cur = Ks + SLOT * G::TILE;
      const int k0 = c_begin + t * TK;
      for (int sb = 0; sb < SPT; ++sb) {
        const int sub = first_sub + sb;
        const int t0 = k0 + 32 * sub;
        if (t0 >= a.L) break;
        const bool need_mask = t0 + 31 > a.min_pos;    // some query cannot see the whole sub-tile, or it runs past L
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
          f32x16 sc = {0};
#pragma unroll
          for (int s = 0; s < D / 16; ++s) sc = mfma32(frag<D>(cur, fbase, sub, s), qf[qt][s], sc);   // rows = keys, cols = queries
          const int qpos = my_pos[qt];
          if (need_mask) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int tk = t0 + c_row(r, hi);
              if (tk > qpos || tk >= a.L) sc[r] = -INFINITY;
            }
          }
          float mx = sc[0];
#pragma unroll
          for (int r = 1; r < 16; r += 2) mx = fmaxf(fmaxf(mx, sc[r]), sc[r == 15 ? 15 : r + 1]);
          const float mn = fmaxf(m[qt], mx * a.c);     // scale > 0: the max commutes with it
          float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
          for (int r = 0; r < 16; r += 2) {
            sum0 += fast_exp2(fmaf(sc[r], a.c, -mn));
            sum1 += fast_exp2(fmaf(sc[r + 1], a.c, -mn));
          }
          z[qt] = z[qt] * fast_exp2(m[qt] - mn) + sum0 + sum1;
          m[qt] = mn;
        }
      }
    };
    for (int t0 = 0; t0 < n_tiles; t0 += NB)
      static_for<0, NB>([&](auto s) {
        if (t0 + decltype(s)::value < n_tiles) tile(t0 + decltype(s)::value, s);
      });
    // the two halves of the wavefront hold different keys of the same query
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      const float mo = __shfl_xor(m[qt], 32), zo = __shfl_xor(z[qt], 32);
      const float mn = fmaxf(m[qt], mo);
      z[qt] = z[qt] * fast_exp2(m[qt] - mn) + zo * fast_exp2(mo - mn);
      m[qt] = mn;
      if (hi == 0) red[wave][32 * qt + lo] = make_float2(m[qt], z[qt]);
    }
    __syncthreads();
    // fold the key parts of every head of this round
    for (int i = tid; i < role.hpw * QP; i += kThreads) {
      const int slot = i / QP, q = i % QP;
      if (r0 + slot < g) {
        float mn = kNegBig;
        for (int j = 0; j < role.ksplit; ++j) mn = fmaxf(mn, red[slot + role.hpw * j][q].x);
        float zs = 0.f;
        for (int j = 0; j < role.ksplit; ++j) zs += red[slot + role.hpw * j][q].y * fast_exp2(red[slot + role.hpw * j][q].x - mn);
        const long long bh2 = (long long)b * a.Hq + kv * g + r0 + slot;
        a.part[(bh2 * a.nchunks + chunk) * QP + q] = make_float2(mn, zs);
      }
    }
  }
}

// One wavefront per (head, query): fold the chunk partials into lse2 = max + log2(sum), lanes over
// chunks.  Padded queries (index >= last_q) get +inf so that pass 2 gives them weight exp2(-inf) = 0.
__global__ __launch_bounds__(256) void score_lse(ScoreArgs a, int QP, long long n) {
  const long long i = (long long)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (i >= n) return;
  const int q = (int)(i % QP);
  const long long bh = i / QP;
  if (q >= a.Lq) {
    if (lane == 0) a.lse2[i] = INFINITY;
    return;
  }
  float mn = kNegBig;
  for (int c = lane; c < a.nchunks; c += 64) mn = fmaxf(mn, a.part[(bh * a.nchunks + c) * QP + q].x);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) mn = fmaxf(mn, __shfl_xor(mn, off));
  float zs = 0.f;
  for (int c = lane; c < a.nchunks; c += 64) {
    const float2 p = a.part[(bh * a.nchunks + c) * QP + q];
    zs += p.y * exp2f(p.x - mn);
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) zs += __shfl_xor(zs, off);     // butterfly: every lane ends with the same sum
  if (lane == 0) a.lse2[i] = mn + log2f(zs);
}

template <int D, int NQT, int HPW>
__global__ __launch_bounds__(kThreads, NQT <= 2 ? 2 : 1) void score_pass2(ScoreArgs a) {
  using C = TileCfg<HPW>;
  constexpr int TK = C::TK, NB = C::NB, SPT = C::SPT;
  using G = Geo<D, TK>;
  constexpr int QP = 32 * NQT;
  __shared__ __attribute__((aligned(1024))) __bf16 Ks[NB * G::TILE];
  __shared__ int qpos_s[kMaxQueries];                  // the position table, for the search of the masked tiles
  if (threadIdx.x < kMaxQueries) qpos_s[threadIdx.x] = a.qpos[threadIdx.x];   // visible after the first barrier below
  // Pass 2 walks the (KV head, chunk) pairs in the reverse of pass 1's order: the workgroups that start
  // first read the keys pass 1 read last, which the memory-side cache still holds when K as a whole
  // (268 MB at 128K tokens x 8 KV heads) does not fit it.
  const int chunk = (int)(gridDim.x - 1 - blockIdx.x);
  const int bkv = (int)(gridDim.y - 1 - blockIdx.y);
  const int kv = bkv % a.Hkv, b = bkv / a.Hkv;
  const int g = a.Hq / a.Hkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const WaveRole role = wave_role(g, wave);              // role.hpw == HPW (chosen by the host from g)
  const int c_begin = chunk * a.chunk, c_end = min(c_begin + a.chunk, a.L);
  const int n_tiles = (c_end - c_begin + TK - 1) / TK;
  const int n_fast = fast_tiles<TK>(a, c_begin, n_tiles);
  const int first_sub = role.kpart * SPT;
  Ring<D, TK, NB> ring;
  ring.init(a.K + a.ks.head(b, kv), a.ks.l, a.L, tid, Ks, c_begin, n_tiles);
  const int fbase = G::frag_base(lo, hi);

  for (int r0 = 0; r0 < g; r0 += role.hpw) {
    const int hh = r0 + role.hslot;
    const bool act = hh < g;
    const int head = kv * g + (act ? hh : 0);
    const long long bh = (long long)b * a.Hq + head;
    __syncthreads();                                   // the previous round is done with the ring
    bf16x8 qf[NQT][D / 16];
    load_q_frags<D, NQT>(a, b, head, lo, hi, qf);           // Q fragments and lse (served by the L2) ahead of the first K tiles
    // log2-sum-exp of the queries this lane sees as accumulator rows
    float lse[NQT][16];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) lse[qt][r] = a.lse2[bh * QP + 32 * qt + c_row(r, hi)];
    ring.start();
    UnitPipe<D, NQT, SPT, false> pp;
    pp.fbase = fbase;
    pp.first_sub = first_sub;
    f32x16 acc = {0};
    bool primed = false;
    auto tile = [&](int t, auto slot_tag) {
      constexpr int SLOT = decltype(slot_tag)::value, kNextSlot = (SLOT + 1) % NB;
      if (!primed) ring.template enter<SLOT, 0>(t);
      const int k0 = c_begin + t * TK;
      if (t < n_fast) {
        const bool chain_next = t + 1 < n_fast;
        if (act) {
          float* out = a.scores + bh * a.L + k0 + 32 * first_sub + lo;
          fast_tile_pass2<D, NQT, SPT, TK, NB, SLOT>(ring, t, primed, chain_next, pp, acc, qf, a.c, lse, out, hi);
        } else {
          if (chain_next) ring.template enter<kNextSlot, 0>(t + 1);
          primed = chain_next;
        }
        return;
      }
      primed = false;
      if (!act) return;
      const __bf16* cur = Ks + SLOT * G::TILE;
      for (int sb = 0; sb < SPT; ++sb) {
        const int sub = first_sub + sb;
        const int t0 = k0 + 32 * sub;
        if (t0 >= a.L) break;
        const int tk = t0 + lo;                        // this lane's key
        const bool need_mask = t0 + 31 > a.min_pos;
        // Queries are in ascending position order: key tk is hidden from exactly the queries with
        // index < n_hidden = #{i : qpos[i] < tk} (binary search in the position table).
        int n_hidden = 0;
        if (need_mask) {
          int lo_i = 0, hi_i = QP;
          while (lo_i < hi_i) {
            const int mid = (lo_i + hi_i) >> 1;
            if (qpos_s[mid] < tk) lo_i = mid + 1; else hi_i = mid;
          }
          n_hidden = lo_i;
        }
        float colsum = 0.f;
#pragma unroll
        for (int qt = 0; qt < NQT; ++qt) {
          f32x16 sc = {0};
#pragma unroll
          for (int s = 0; s < D / 16; ++s) sc = mfma32(qf[qt][s], frag<D>(cur, fbase, sub, s), sc);   // rows = queries, cols = keys
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            float p = fast_exp2(sc[r] * a.c - lse[qt][r]);
            if (32 * qt + c_row(r, hi) < n_hidden) p = 0.f;
            colsum += p;
          }
        }
        colsum += __shfl_xor(colsum, 32);
        if (hi == 0 && tk < a.L) a.scores[bh * a.L + tk] = colsum;
      }
    };
    for (int t0 = 0; t0 < n_tiles; t0 += NB)
      static_for<0, NB>([&](auto s) {
        if (t0 + decltype(s)::value < n_tiles) tile(t0 + decltype(s)::value, s);
      });
  }
}

// pooling(.) of Algorithm 1, read as average pooling of odd width w, stride 1, zero padding
__global__ void pool_kernel(const float* __restrict__ raw, float* __restrict__ out, int L, int w, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int t = (int)(i % L);
  const float* row = raw + (i - t);
  const int r = w / 2;
  float acc = 0.f;
  for (int u = max(0, t - r); u <= min(L - 1, t + r); ++u) acc += row[u];
  out[i] = acc / (float)w;
}

template <int D, int NQT, int HPW>
hipError_t run_split(const ScoreArgs& a, int BH, hipStream_t st) {
  constexpr int QP = 32 * NQT;
  dim3 grid(a.nchunks, BH / (a.Hq / a.Hkv));             // one workgroup per (KV head, chunk)
  score_pass1<D, NQT, HPW><<<grid, kThreads, 0, st>>>(a);
  const long long n = (long long)BH * QP;
  score_lse<<<(unsigned)((n + 3) / 4), 256, 0, st>>>(a, QP, n);
  score_pass2<D, NQT, HPW><<<grid, kThreads, 0, st>>>(a);
  if (a.pool_w > 1) {
    const long long nt = (long long)BH * a.L;
    pool_kernel<<<(unsigned)((nt + 255) / 256), 256, 0, st>>>(a.scores, a.pooled, a.L, a.pool_w, nt);
  }
  return hipGetLastError();
}

// The kernels are built per number of query heads a workgroup serves at a time (wave_role: 4, 2 or 1).
template <int D, int NQT>
hipError_t run(const ScoreArgs& a, int BH, hipStream_t st) {
  const int g = a.Hq / a.Hkv;
  if (g >= 4) return run_split<D, NQT, 4>(a, BH, st);
  if (g >= 2) return run_split<D, NQT, 2>(a, BH, st);
  return run_split<D, NQT, 1>(a, BH, st);
}

// Keys per workgroup: long enough that the start-up of a workgroup (Q fragments, first K tile)
// is amortised, short enough for two workgroups per CU (as many as the LDS tiles allow to be
// resident, so the launch runs as a single round).
inline int chunk_for(const Dims& dm) {
  const long long total = (long long)dm.L * dm.B * dm.Hkv;
  long long c = total / (256 * 2);
  c = (c + 127) / 128 * 128;
  if (c < kMinChunk) c = kMinChunk;
  if (c > 8192) c = 8192;
  return (int)c;
}

inline int nqt_for(int last_q) { return last_q <= 32 ? 1 : (last_q <= 64 ? 2 : 4); }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t score_ws_bytes(const Dims& dm) {
  const int QP = 32 * nqt_for(dm.last_q);
  const size_t nchunks = ((size_t)dm.L + kMinChunk - 1) / kMinChunk;   // upper bound for any chunk size
  const size_t BH = (size_t)dm.B * dm.Hq;
  return align256(BH * nchunks * QP * sizeof(float2)) + align256(BH * QP * sizeof(float)) +
         (dm.pool_w > 1 ? align256(BH * dm.L * sizeof(float)) : 0);
}

namespace {

hipError_t launch_common(const Dims& dm, ScoreArgs& a, const void* K, float* scores, void* ws, hipStream_t st) {
  const int nqt = nqt_for(dm.last_q);
  const int QP = 32 * nqt;
  a.K = (const __bf16*)K; a.scores = scores;
  a.ks = dm.kv;
  a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.L = dm.L; a.Lq = dm.last_q;
  a.chunk = chunk_for(dm);
  a.nchunks = (dm.L + a.chunk - 1) / a.chunk;
  a.c = dm.scale * kLog2e;
  const size_t BH = (size_t)dm.B * dm.Hq;
  a.part = (float2*)ws;
  a.lse2 = (float*)((char*)ws + align256(BH * a.nchunks * QP * sizeof(float2)));
  a.pool_w = dm.pool_w;
  a.pooled = nullptr;
  if (dm.pool_w > 1) {                                   // raw column sums go to the workspace, pooled ones out
    a.pooled = scores;
    a.scores = (float*)((char*)a.lse2 + align256(BH * QP * sizeof(float)));
  }
  const int bh = (int)BH;
  if (dm.d == 128) {
    if (nqt == 1) return run<128, 1>(a, bh, st);
    if (nqt == 2) return run<128, 2>(a, bh, st);
    return run<128, 4>(a, bh, st);
  }
  if (nqt == 1) return run<64, 1>(a, bh, st);
  if (nqt == 2) return run<64, 2>(a, bh, st);
  return run<64, 4>(a, bh, st);
}

}  // namespace

// Algorithm 1's scorer: the last last_q rows of Q at their own positions.
hipError_t launch_score(const Dims& dm, const void* Q, const void* K, float* scores, void* ws, hipStream_t st) {
  ScoreArgs a;
  a.Q = (const __bf16*)Q;
  a.qs = dm.q;
  a.q_row0 = dm.L - dm.last_q;
  a.min_pos = dm.L - dm.last_q;
  for (int i = 0; i < kMaxQueries; ++i) a.qpos[i] = i < dm.last_q ? dm.L - dm.last_q + i : dm.L - 1;
  return launch_common(dm, a, K, scores, ws, st);
}

// Scoring from caller-supplied query rows Qsel [B,Hq,last_q,d] at positions qpos (host, ascending).
hipError_t launch_score_queries(const Dims& dm, const void* Qsel, const int32_t* qpos, const void* K, float* scores,
                                void* ws, hipStream_t st) {
  ScoreArgs a;
  a.Q = (const __bf16*)Qsel;
  a.qs = Strides{(long long)dm.Hq * dm.last_q * dm.d, (long long)dm.last_q * dm.d, (long long)dm.d};
  a.q_row0 = 0;
  a.min_pos = qpos[0];
  for (int i = 0; i < kMaxQueries; ++i) a.qpos[i] = i < dm.last_q ? qpos[i] : dm.L - 1;
  return launch_common(dm, a, K, scores, ws, st);
}

// ---- the query sets of the scoring ablation

namespace {

struct GatherArgs {
  const u32x4* Q;
  u32x4* Qsel;
  Strides qs;                  // layout of Q, in 16-byte pieces
  int Hq;
  int L, n, lpr;               // lpr = 16-byte pieces per row
  int qpos[kMaxQueries];
};

// Qsel[bh, j, :] = Q[bh, qpos[j], :]
__global__ void gather_queries_kernel(GatherArgs a, long long n_pieces) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n_pieces) return;
  const int piece = (int)(i % a.lpr);
  const long long row = i / a.lpr;
  const int j = (int)(row % a.n);
  const long long bh = row / a.n;
  a.Qsel[i] = a.Q[a.qs.head(bh / a.Hq, bh % a.Hq) + a.qpos[j] * a.qs.l + piece];
}

// Segment j of the query-only pooling: rows floor(j L / n) .. ceil((j+1) L / n) - 1.
__device__ __forceinline__ void segment(int j, int L, int n, int& lo, int& hi) {
  lo = (int)(((long long)j * L) / n);
  hi = (int)((((long long)(j + 1)) * L + n - 1) / n);
}

// Stage 1: workgroup (split s, segment j, head bh) adds its slice of the segment's rows, thread = one
// d-column pair... one thread per 2 columns would leave most lanes idle at d = 128, so a thread
// owns 8 columns (16 bytes) and kPoolRows threads share a column group; they are folded in LDS.
constexpr int kPoolThreads = 256;
template <int D>
__global__ __launch_bounds__(kPoolThreads) void pool_queries_partial(const u32x4* __restrict__ Q, float* __restrict__ part,
                                                                     int L, int n_pool, int n_split, Strides qs, int Hq) {
  constexpr int LPR = D / 8, RPP = kPoolThreads / LPR;      // rows per pass
  __shared__ float red[RPP][D];
  const int s = blockIdx.x, j = blockIdx.y;
  const long long bh = blockIdx.z;
  int lo, hi;
  segment(j, L, n_pool, lo, hi);
  const int len = hi - lo, per = (len + n_split - 1) / n_split;
  const int r_begin = lo + s * per, r_end = min(hi, r_begin + per);
  const int piece = threadIdx.x % LPR, rr = threadIdx.x / LPR;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  for (int r = r_begin + rr; r < r_end; r += RPP) {
    const u32x4 v = Q[qs.head(bh / Hq, bh % Hq) + r * qs.l + piece];       // qs in 16-byte pieces
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      acc[2 * c] += __uint_as_float(v[c] << 16);
      acc[2 * c + 1] += __uint_as_float(v[c] & 0xffff0000u);
    }
  }
#pragma unroll
  for (int c = 0; c < 8; ++c) red[rr][8 * piece + c] = acc[c];
  __syncthreads();
  if (threadIdx.x < D) {
    float t = 0.f;
    for (int r = 0; r < RPP; ++r) t += red[r][threadIdx.x];                 // fixed order: deterministic
    part[((bh * n_pool + j) * n_split + s) * D + threadIdx.x] = t;
  }
}

// Stage 2: mean of the segment, rounded to bf16.
__global__ void pool_queries_final(const float* __restrict__ part, __bf16* __restrict__ Qsel, int L, int n_pool, int n_split,
                                   int D, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int c = (int)(i % D);
  const long long seg = i / D;                               // bh * n_pool + j
  int lo, hi;
  segment((int)(seg % n_pool), L, n_pool, lo, hi);
  float t = 0.f;
  for (int s = 0; s < n_split; ++s) t += part[(seg * n_split + s) * D + c];
  Qsel[i] = (__bf16)(t / (float)(hi - lo));
}

inline int pool_split(int L, int n_pool) {
  const int max_len = (L + n_pool - 1) / n_pool + 1;
  int s = (max_len + 1023) / 1024;
  return s < 1 ? 1 : (s > 64 ? 64 : s);
}

}  // namespace

hipError_t launch_gather_queries(const Dims& dm, const void* Q, const int32_t* qpos, int n, void* Qsel, hipStream_t st) {
  GatherArgs a;
  a.Q = (const u32x4*)Q; a.Qsel = (u32x4*)Qsel; a.L = dm.L; a.n = n; a.lpr = dm.d / 8;
  a.qs = Strides{dm.q.b / 8, dm.q.h / 8, dm.q.l / 8}; a.Hq = dm.Hq;
  for (int i = 0; i < kMaxQueries; ++i) a.qpos[i] = i < n ? qpos[i] : 0;
  const long long pieces = (long long)dm.B * dm.Hq * n * a.lpr;
  gather_queries_kernel<<<(unsigned)((pieces + 255) / 256), 256, 0, st>>>(a, pieces);
  return hipGetLastError();
}

size_t pool_queries_ws_bytes(const Dims& dm, int n_pool) {
  return align256((size_t)dm.B * dm.Hq * n_pool * pool_split(dm.L, n_pool) * dm.d * sizeof(float));
}

hipError_t launch_pool_queries(const Dims& dm, const void* Q, int n_pool, void* Qsel, void* ws, hipStream_t st) {
  const int n_split = pool_split(dm.L, n_pool);
  const dim3 grid((unsigned)n_split, (unsigned)n_pool, (unsigned)(dm.B * dm.Hq));
  const Strides qs8{dm.q.b / 8, dm.q.h / 8, dm.q.l / 8};
  if (dm.d == 128) pool_queries_partial<128><<<grid, kPoolThreads, 0, st>>>((const u32x4*)Q, (float*)ws, dm.L, n_pool, n_split, qs8, dm.Hq);
  else pool_queries_partial<64><<<grid, kPoolThreads, 0, st>>>((const u32x4*)Q, (float*)ws, dm.L, n_pool, n_split, qs8, dm.Hq);
  const long long n = (long long)dm.B * dm.Hq * n_pool * dm.d;
  pool_queries_final<<<(unsigned)((n + 255) / 256), 256, 0, st>>>((const float*)ws, (__bf16*)Qsel, dm.L, n_pool, n_split, dm.d, n);
  return hipGetLastError();
}

}  // namespace tsa
