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
// Tiles that every scoring query sees in full (all but the last few of a sequence) take a
// software-pipelined body: a "unit" is one 32-key x 32-query block (D/16 MFMAs, 16 scores per
// lane); the MFMAs of the next unit are issued chunk by chunk between the exponentials of the
// current one, so the matrix pipe and the vector ALU overlap inside the wavefront.  In pass 1 that
// body does not compute a row max at all: the running max only has to keep the exponentials in
// range, so the sum itself is the detector (a unit whose sum leaves the range is redone the exact
// way, with the true max; this happens once per row in practice).
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kMinChunk = 256;               // keys per workgroup: at least this, a multiple of kTK
constexpr int kTK = 128;                     // keys per staged K tile
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

template <int D, int NQT>
__device__ __forceinline__ void load_q_frags(const ScoreArgs& a, long long bh, int lo, int hi, bf16x8 (&qf)[NQT][D / 16]) {
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int qi = 32 * qt + lo;
    const bool ok = qi < a.Lq;
    const __bf16* row = a.Q + a.qs.head(bh / a.Hq, bh % a.Hq) + (long long)(a.q_row0 + (ok ? qi : 0)) * a.qs.l + 8 * hi;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      bf16x8 v = *(const bf16x8*)(row + 16 * s);
      if (!ok) v = bf16x8{};
      qf[qt][s] = v;
    }
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

// K tiles of kTK keys go through LDS: coalesced 16-byte loads (a row is 16 adjacent lanes), one
// copy per workgroup for all the heads of the group, rows padded by 16 bytes so that the
// fragment reads (16 bytes per lane, consecutive keys) are free of bank conflicts.
template <int D>
struct KStage {
  static constexpr int KS = D + 8;
  static constexpr int CH = kTK * (D / 8) / kThreads;
  static constexpr int kRowsPerPass = kThreads / (D / 8);
  const __bf16* Kh;
  long long row_stride;        // elements between consecutive keys
  int L, st_row, st_col;
  u32x4 reg[CH];
  __device__ __forceinline__ void load(int k0) {
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      const int key = k0 + st_row + kRowsPerPass * i;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (key < L) v = *(const u32x4*)(Kh + (long long)key * row_stride + 8 * st_col);
      reg[i] = v;
    }
  }
  __device__ __forceinline__ void store(__bf16* dst) const {
#pragma unroll
    for (int i = 0; i < CH; ++i) *(u32x4*)(&dst[(st_row + kRowsPerPass * i) * KS + 8 * st_col]) = reg[i];
  }
};


// ---- pipelined tile bodies (tiles without any mask).  SPT = 32-key sub-tiles of the staged tile
// that this wavefront owns, starting at `first` (LDS) = its first sub-tile.  Units run in the order
// (sub-tile, query sub-tile); while unit u is in the vector ALU the MFMAs of unit u + 1 are issued.
// The K fragments live in ONE set of registers: right after the MFMA that uses fragment i of a
// sub-tile for the last time, the register is reloaded with fragment i of the next sub-tile, which is
// consumed a whole unit later.

template <int D, int NQT, int SPT, bool KEYS_ARE_ROWS>
struct UnitPipe {
  static constexpr int NS = D / 16, KS = D + 8, U = SPT * NQT;
  const __bf16* first;
  int k_rd;
  bf16x8 kf[NS];
  __device__ __forceinline__ void load_frag(int sub, int i) { kf[i] = *(const bf16x8*)(&first[32 * sub * KS + k_rd + 16 * i]); }
  // MFMA i of unit `nu` (compile-time), then the in-place reload if unit nu + 1 starts a new sub-tile
  __device__ __forceinline__ void step(int nu, int i, const bf16x8 (&qf)[NQT][NS], f32x16& nxt) {
    if (nu >= U) return;
    const bf16x8 q = qf[nu % NQT][i];
    nxt = KEYS_ARE_ROWS ? mfma32(kf[i], q, nxt) : mfma32(q, kf[i], nxt);
    if (nu + 1 < U && (nu + 1) / NQT != nu / NQT) load_frag((nu + 1) / NQT, i);
  }
};

// Pass 1, lane = query: z[qt] += sum over the tile's keys of exp2(x c - m[qt]).
template <int D, int NQT, int SPT>
__device__ __forceinline__ void fast_tile_pass1(const __bf16* first, int k_rd, const bf16x8 (&qf)[NQT][D / 16], float c,
                                                float (&m)[NQT], float (&z)[NQT]) {
  using Pipe = UnitPipe<D, NQT, SPT, true>;
  constexpr int NS = Pipe::NS, EPC = 16 / NS, U = Pipe::U;
  Pipe pp;
  pp.first = first;
  pp.k_rd = k_rd;
#pragma unroll
  for (int i = 0; i < NS; ++i) pp.load_frag(0, i);
  f32x16 acc = {0};
#pragma unroll
  for (int i = 0; i < NS; ++i) pp.step(0, i, qf, acc);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int qt = u % NQT;
    const float mq = m[qt];
    f32x16 nxt = {0};
    float s0 = 0.f, s1 = 0.f;
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      pp.step(u + 1, i, qf, nxt);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const float p = fast_exp2(fmaf(acc[EPC * i + e], c, -mq));
        if (e & 1) s1 += p; else s0 += p;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    const float sum = s0 + s1;
    if (sum < kSumLimit) {
      z[qt] += sum;
    } else {                                             // out of range (or the very first unit): exact update
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
      z[qt] = z[qt] * fast_exp2(mq - mn) + t0 + t1;
      m[qt] = mn;
    }
    acc = nxt;
  }
}

// Pass 2, lane = key: s[t] = sum over the queries of exp2(x c - lse[query]); one store per sub-tile.
template <int D, int NQT, int SPT>
__device__ __forceinline__ void fast_tile_pass2(const __bf16* first, int k_rd, const bf16x8 (&qf)[NQT][D / 16], float c,
                                                const float (&lse)[NQT][16], float* out, int hi) {
  using Pipe = UnitPipe<D, NQT, SPT, false>;
  constexpr int NS = Pipe::NS, EPC = 16 / NS, U = Pipe::U;
  Pipe pp;
  pp.first = first;
  pp.k_rd = k_rd;
#pragma unroll
  for (int i = 0; i < NS; ++i) pp.load_frag(0, i);
  f32x16 acc = {0};
#pragma unroll
  for (int i = 0; i < NS; ++i) pp.step(0, i, qf, acc);
  float s0 = 0.f, s1 = 0.f;
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int qt = u % NQT, sb = u / NQT;
    f32x16 nxt = {0};
#pragma unroll
    for (int i = 0; i < NS; ++i) {
      pp.step(u + 1, i, qf, nxt);
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        const int r = EPC * i + e;
        const float p = fast_exp2(fmaf(acc[r], c, -lse[qt][r]));
        if (e & 1) s1 += p; else s0 += p;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    acc = nxt;
    if (qt == NQT - 1) {
      float colsum = s0 + s1;
      colsum += __shfl_xor(colsum, 32);
      if (hi == 0) out[32 * sb] = colsum;
      s0 = s1 = 0.f;
    }
  }
}

template <int D, int NQT>
__global__ __launch_bounds__(kThreads, NQT <= 2 ? 2 : 1) void score_pass1(ScoreArgs a) {
  constexpr int QP = 32 * NQT;
  constexpr int KS = D + 8;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[2][kTK * KS];
  __shared__ float2 red[kWaves][QP];
  const int chunk = blockIdx.x;
  const long long bkv = blockIdx.y;
  const int kv = (int)(bkv % a.Hkv);
  const long long b = bkv / a.Hkv;
  const int g = a.Hq / a.Hkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const WaveRole role = wave_role(g, wave);
  const int c_begin = chunk * a.chunk, c_end = min(c_begin + a.chunk, a.L);
  const int sub_per_tile = (kTK / 32) / role.ksplit;     // 32-key sub-tiles of a staged tile per wavefront
  int my_pos[NQT];                                       // position of this lane's query in each query sub-tile
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) my_pos[qt] = a.qpos[32 * qt + lo];
  KStage<D> stg;
  stg.Kh = a.K + a.ks.head(b, kv);
  stg.row_stride = a.ks.l;
  stg.L = a.L; stg.st_row = tid / (D / 8); stg.st_col = tid % (D / 8);
  const int k_rd = lo * KS + 8 * hi;

  for (int r0 = 0; r0 < g; r0 += role.hpw) {
    const int hh = r0 + role.hslot;
    const bool act = hh < g;
    const long long bh = b * a.Hq + kv * g + (act ? hh : 0);
    bf16x8 qf[NQT][D / 16];
    stg.load(c_begin);                                 // first K tile and the Q fragments are in flight together
    load_q_frags<D, NQT>(a, bh, lo, hi, qf);
    float m[NQT], z[NQT];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) { m[qt] = kNegBig; z[qt] = 0.f; }
    stg.store(Ks[0]);
    int par = 0;
    for (int k0 = c_begin; k0 < c_end; k0 += kTK) {
      __syncthreads();                                 // tile k0 is staged, the other buffer is free
      if (k0 + kTK < c_end) stg.load(k0 + kTK);        // in flight during the math below
      if (act && k0 + kTK - 1 <= a.min_pos && k0 + kTK <= a.L) {   // every query sees the whole tile
        const __bf16* first = &Ks[par][32 * role.kpart * sub_per_tile * KS];
        if (sub_per_tile == 4) fast_tile_pass1<D, NQT, 4>(first, k_rd, qf, a.c, m, z);
        else if (sub_per_tile == 2) fast_tile_pass1<D, NQT, 2>(first, k_rd, qf, a.c, m, z);
        else fast_tile_pass1<D, NQT, 1>(first, k_rd, qf, a.c, m, z);
      } else if (act) {
        for (int sb = 0; sb < sub_per_tile; ++sb) {
          const int sub = role.kpart * sub_per_tile + sb;
          const int t0 = k0 + 32 * sub;
          if (t0 >= a.L) break;
          const bool need_mask = t0 + 31 > a.min_pos;  // some query cannot see the whole sub-tile, or it runs past L
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
              const bf16x8 kf = *(const bf16x8*)(&Ks[par][32 * sub * KS + k_rd + 16 * s]);
              acc = mfma32(kf, qf[qt][s], acc);        // rows = keys, cols = queries
            }
            const int qpos = my_pos[qt];
            if (need_mask) {
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int t = t0 + c_row(r, hi);
                if (t > qpos || t >= a.L) acc[r] = -INFINITY;
              }
            }
            float mx = acc[0];
#pragma unroll
            for (int r = 1; r < 16; r += 2) mx = fmaxf(fmaxf(mx, acc[r]), acc[r == 15 ? 15 : r + 1]);
            const float mn = fmaxf(m[qt], mx * a.c);   // scale > 0: the max commutes with it
            float sum0 = 0.f, sum1 = 0.f;
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
              sum0 += fast_exp2(fmaf(acc[r], a.c, -mn));
              sum1 += fast_exp2(fmaf(acc[r + 1], a.c, -mn));
            }
            z[qt] = z[qt] * fast_exp2(m[qt] - mn) + sum0 + sum1;
            m[qt] = mn;
          }
        }
      }
      if (k0 + kTK < c_end) stg.store(Ks[par ^ 1]);
      par ^= 1;
    }
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
        const long long bh2 = b * a.Hq + kv * g + r0 + slot;
        a.part[(bh2 * a.nchunks + chunk) * QP + q] = make_float2(mn, zs);
      }
    }
    __syncthreads();
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

template <int D, int NQT>
__global__ __launch_bounds__(kThreads, NQT <= 2 ? 2 : 1) void score_pass2(ScoreArgs a) {
  constexpr int QP = 32 * NQT;
  constexpr int KS = D + 8;
  __shared__ __attribute__((aligned(16))) __bf16 Ks[2][kTK * KS];
  // Pass 2 walks the (KV head, chunk) pairs in the reverse of pass 1's order: the workgroups that start
  // first read the keys pass 1 read last, which the memory-side cache still holds when K as a whole
  // (268 MB at 128K tokens x 8 KV heads) does not fit it.
  const int chunk = (int)(gridDim.x - 1 - blockIdx.x);
  const long long bkv = gridDim.y - 1 - blockIdx.y;
  const int kv = (int)(bkv % a.Hkv);
  const long long b = bkv / a.Hkv;
  const int g = a.Hq / a.Hkv;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lo = lane & 31, hi = lane >> 5;
  const WaveRole role = wave_role(g, wave);
  const int c_begin = chunk * a.chunk, c_end = min(c_begin + a.chunk, a.L);
  const int sub_per_tile = (kTK / 32) / role.ksplit;
  KStage<D> stg;
  stg.Kh = a.K + a.ks.head(b, kv);
  stg.row_stride = a.ks.l;
  stg.L = a.L; stg.st_row = tid / (D / 8); stg.st_col = tid % (D / 8);
  const int k_rd = lo * KS + 8 * hi;

  for (int r0 = 0; r0 < g; r0 += role.hpw) {
    const int hh = r0 + role.hslot;
    const bool act = hh < g;
    const long long bh = b * a.Hq + kv * g + (act ? hh : 0);
    __syncthreads();                                   // previous round is done with both buffers
    stg.load(c_begin);                                 // first K tile, Q fragments and lse are in flight together
    bf16x8 qf[NQT][D / 16];
    load_q_frags<D, NQT>(a, bh, lo, hi, qf);
    // log2-sum-exp of the queries this lane sees as accumulator rows
    float lse[NQT][16];
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
      for (int r = 0; r < 16; ++r) lse[qt][r] = a.lse2[bh * QP + 32 * qt + c_row(r, hi)];
    stg.store(Ks[0]);
    int par = 0;
    for (int k0 = c_begin; k0 < c_end; k0 += kTK) {
      __syncthreads();
      if (k0 + kTK < c_end) stg.load(k0 + kTK);
      if (act && k0 + kTK - 1 <= a.min_pos && k0 + kTK <= a.L) {   // no query is hidden from any key of the tile
        const int sub0 = role.kpart * sub_per_tile;
        const __bf16* first = &Ks[par][32 * sub0 * KS];
        float* out = a.scores + bh * a.L + k0 + 32 * sub0 + lo;
        if (sub_per_tile == 4) fast_tile_pass2<D, NQT, 4>(first, k_rd, qf, a.c, lse, out, hi);
        else if (sub_per_tile == 2) fast_tile_pass2<D, NQT, 2>(first, k_rd, qf, a.c, lse, out, hi);
        else fast_tile_pass2<D, NQT, 1>(first, k_rd, qf, a.c, lse, out, hi);
      } else if (act) {
        for (int sb = 0; sb < sub_per_tile; ++sb) {
          const int sub = role.kpart * sub_per_tile + sb;
          const int t0 = k0 + 32 * sub;
          if (t0 >= a.L) break;
          const int t = t0 + lo;                       // this lane's key
          const bool need_mask = t0 + 31 > a.min_pos;
          // Queries are in ascending position order: key t is hidden from exactly the queries with
          // index < n_hidden = #{i : qpos[i] < t} (binary search in the position table).
          int n_hidden = 0;
          if (need_mask) {
            int lo_i = 0, hi_i = QP;
            while (lo_i < hi_i) {
              const int mid = (lo_i + hi_i) >> 1;
              if (a.qpos[mid] < t) lo_i = mid + 1; else hi_i = mid;
            }
            n_hidden = lo_i;
          }
          float colsum = 0.f;
#pragma unroll
          for (int qt = 0; qt < NQT; ++qt) {
            f32x16 acc = {0};
#pragma unroll
            for (int s = 0; s < D / 16; ++s) {
              const bf16x8 kf = *(const bf16x8*)(&Ks[par][32 * sub * KS + k_rd + 16 * s]);
              acc = mfma32(qf[qt][s], kf, acc);        // rows = queries, cols = keys
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              float p = fast_exp2(acc[r] * a.c - lse[qt][r]);
              if (32 * qt + c_row(r, hi) < n_hidden) p = 0.f;
              colsum += p;
            }
          }
          colsum += __shfl_xor(colsum, 32);
          if (hi == 0 && t < a.L) a.scores[bh * a.L + t] = colsum;
        }
      }
      if (k0 + kTK < c_end) stg.store(Ks[par ^ 1]);
      par ^= 1;
    }
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

template <int D, int NQT>
hipError_t run(const ScoreArgs& a, int BH, hipStream_t st) {
  constexpr int QP = 32 * NQT;
  dim3 grid(a.nchunks, BH / (a.Hq / a.Hkv));             // one workgroup per (KV head, chunk)
  score_pass1<D, NQT><<<grid, kThreads, 0, st>>>(a);
  const long long n = (long long)BH * QP;
  score_lse<<<(unsigned)((n + 3) / 4), 256, 0, st>>>(a, QP, n);
  score_pass2<D, NQT><<<grid, kThreads, 0, st>>>(a);
  if (a.pool_w > 1) {
    const long long nt = (long long)BH * a.L;
    pool_kernel<<<(unsigned)((nt + 255) / 256), 256, 0, st>>>(a.scores, a.pooled, a.L, a.pool_w, nt);
  }
  return hipGetLastError();
}

// Keys per workgroup: long enough that the start-up of a workgroup (Q fragments, first K tile)
// is amortised, short enough for two workgroups per CU (as many as the LDS tiles allow to be
// resident, so the launch runs as a single round).
inline int chunk_for(const Dims& dm) {
  const long long total = (long long)dm.L * dm.B * dm.Hkv;
  long long c = total / (256 * 2);
  c = (c + kTK - 1) / kTK * kTK;
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
