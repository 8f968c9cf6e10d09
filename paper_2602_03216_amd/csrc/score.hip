// Token scoring: Algorithm 1 of the paper, "attention scores using recent queries" and
// "token-level scores per head":  A = softmax(Q[-last_q:] K^T * scale) (causal inside the
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
// reduction longer than one step.  K fragments go straight from global memory to registers.
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;
constexpr int kChunk = 1024;                 // keys per workgroup
constexpr int kKeysPerWave = kChunk / kWaves;
constexpr float kNegBig = -1.0e30f;

struct ScoreArgs {
  const __bf16* Q;
  const __bf16* K;
  float* scores;
  float2* part;       // [B*Hq][nchunks][QP] (max, sum) in the log2 domain
  float* lse2;        // [B*Hq][QP]
  int Hq, Hkv, L, Lq, nchunks;
  float c;            // scale * log2(e)
};

template <int D, int NQT>
__device__ __forceinline__ void load_q_frags(const ScoreArgs& a, long long bh, int lo, int hi, bf16x8 (&qf)[NQT][D / 16]) {
  const int first = a.L - a.Lq;
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) {
    const int qi = 32 * qt + lo;
    const bool ok = qi < a.Lq;
    const __bf16* row = a.Q + ((bh * a.L) + (ok ? first + qi : 0)) * (long long)D + 8 * hi;
#pragma unroll
    for (int s = 0; s < D / 16; ++s) {
      bf16x8 v = *(const bf16x8*)(row + 16 * s);
      if (!ok) v = bf16x8{};
      qf[qt][s] = v;
    }
  }
}

template <int D>
__device__ __forceinline__ void load_k_frags(const __bf16* Kh, int L, int t, int hi, bf16x8 (&kf)[D / 16]) {
  const bool ok = t < L;
  const __bf16* row = Kh + (long long)(ok ? t : 0) * D + 8 * hi;
#pragma unroll
  for (int s = 0; s < D / 16; ++s) {
    bf16x8 v = *(const bf16x8*)(row + 16 * s);
    if (!ok) v = bf16x8{};
    kf[s] = v;
  }
}

template <int D, int NQT>
__global__ __launch_bounds__(kThreads) void score_pass1(ScoreArgs a) {
  constexpr int QP = 32 * NQT;
  __shared__ float2 red[kWaves][QP];
  const int chunk = blockIdx.x;
  const long long bh = blockIdx.y;
  const int h = (int)(bh % a.Hq);
  const long long b = bh / a.Hq;
  const int g = a.Hq / a.Hkv;
  const __bf16* Kh = a.K + ((b * a.Hkv + h / g) * (long long)a.L) * D;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lo = lane & 31, hi = lane >> 5;
  const int first = a.L - a.Lq;

  bf16x8 qf[NQT][D / 16];
  load_q_frags<D, NQT>(a, bh, lo, hi, qf);
  float m[NQT], z[NQT];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt) { m[qt] = kNegBig; z[qt] = 0.f; }

  const int t_begin = chunk * kChunk + wave * kKeysPerWave;
  const int t_end = min(t_begin + kKeysPerWave, a.L);
  bf16x8 kf[D / 16], kf_next[D / 16];
  load_k_frags<D>(Kh, a.L, t_begin + lo, hi, kf_next);
  for (int t0 = t_begin; t0 < t_end; t0 += 32) {
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kf[s] = kf_next[s];
    if (t0 + 32 < t_end) load_k_frags<D>(Kh, a.L, t0 + 32 + lo, hi, kf_next);   // in flight during the math below
    const bool need_mask = t0 + 31 > first;       // tile reaches into the window or past L
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      f32x16 acc = {0};
#pragma unroll
      for (int s = 0; s < D / 16; ++s) acc = mfma32(kf[s], qf[qt][s], acc);   // rows = keys, cols = queries
      const int qpos = first + 32 * qt + lo;       // position of this lane's query
      float x[16];
      float mx = kNegBig;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = acc[r] * a.c;
        if (need_mask) {
          const int t = t0 + c_row(r, hi);
          if (t > qpos || t >= a.L) v = -INFINITY;
        }
        x[r] = v;
        mx = fmaxf(mx, v);
      }
      const float mn = fmaxf(m[qt], mx);
      float sum = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += fast_exp2(x[r] - mn);
      z[qt] = z[qt] * fast_exp2(m[qt] - mn) + sum;
      m[qt] = mn;
    }
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
  if (threadIdx.x < QP) {
    float mn = kNegBig;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) mn = fmaxf(mn, red[w][threadIdx.x].x);
    float zs = 0.f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) zs += red[w][threadIdx.x].y * fast_exp2(red[w][threadIdx.x].x - mn);
    a.part[(bh * a.nchunks + chunk) * QP + threadIdx.x] = make_float2(mn, zs);
  }
}

// One thread per (head, query): fold the chunk partials into lse2 = max + log2(sum).
// Padded queries (index >= last_q) get +inf so that pass 2 gives them weight exp2(-inf) = 0.
__global__ void score_lse(ScoreArgs a, int QP, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int q = (int)(i % QP);
  const long long bh = i / QP;
  if (q >= a.Lq) { a.lse2[i] = INFINITY; return; }
  float mn = kNegBig;
  for (int c = 0; c < a.nchunks; ++c) mn = fmaxf(mn, a.part[(bh * a.nchunks + c) * QP + q].x);
  float zs = 0.f;
  for (int c = 0; c < a.nchunks; ++c) {
    const float2 p = a.part[(bh * a.nchunks + c) * QP + q];
    zs += p.y * exp2f(p.x - mn);
  }
  a.lse2[i] = mn + log2f(zs);
}

template <int D, int NQT>
__global__ __launch_bounds__(kThreads) void score_pass2(ScoreArgs a) {
  constexpr int QP = 32 * NQT;
  const int chunk = blockIdx.x;
  const long long bh = blockIdx.y;
  const int h = (int)(bh % a.Hq);
  const long long b = bh / a.Hq;
  const int g = a.Hq / a.Hkv;
  const __bf16* Kh = a.K + ((b * a.Hkv + h / g) * (long long)a.L) * D;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, lo = lane & 31, hi = lane >> 5;
  const int first = a.L - a.Lq;

  bf16x8 qf[NQT][D / 16];
  load_q_frags<D, NQT>(a, bh, lo, hi, qf);
  // log2-sum-exp of the queries this lane sees as accumulator rows
  float lse[NQT][16];
#pragma unroll
  for (int qt = 0; qt < NQT; ++qt)
#pragma unroll
    for (int r = 0; r < 16; ++r) lse[qt][r] = a.lse2[bh * QP + 32 * qt + c_row(r, hi)];

  const int t_begin = chunk * kChunk + wave * kKeysPerWave;
  const int t_end = min(t_begin + kKeysPerWave, a.L);
  bf16x8 kf[D / 16], kf_next[D / 16];
  load_k_frags<D>(Kh, a.L, t_begin + lo, hi, kf_next);
  for (int t0 = t_begin; t0 < t_end; t0 += 32) {
    const int t = t0 + lo;                         // this lane's key
#pragma unroll
    for (int s = 0; s < D / 16; ++s) kf[s] = kf_next[s];
    if (t0 + 32 < t_end) load_k_frags<D>(Kh, a.L, t + 32, hi, kf_next);         // in flight during the math below
    const bool need_mask = t0 + 31 > first;
    float colsum = 0.f;
#pragma unroll
    for (int qt = 0; qt < NQT; ++qt) {
      f32x16 acc = {0};
#pragma unroll
      for (int s = 0; s < D / 16; ++s) acc = mfma32(qf[qt][s], kf[s], acc);   // rows = queries, cols = keys
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = fast_exp2(acc[r] * a.c - lse[qt][r]);
        if (need_mask) {
          const int qpos = first + 32 * qt + c_row(r, hi);
          if (t > qpos) p = 0.f;
        }
        colsum += p;
      }
    }
    colsum += __shfl_xor(colsum, 32);
    if (hi == 0 && t < a.L) a.scores[bh * a.L + t] = colsum;
  }
}

template <int D, int NQT>
hipError_t run(const ScoreArgs& a, int BH, hipStream_t st) {
  constexpr int QP = 32 * NQT;
  dim3 grid(a.nchunks, BH);
  score_pass1<D, NQT><<<grid, kThreads, 0, st>>>(a);
  const long long n = (long long)BH * QP;
  score_lse<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(a, QP, n);
  score_pass2<D, NQT><<<grid, kThreads, 0, st>>>(a);
  return hipGetLastError();
}

inline int nqt_for(int last_q) { return last_q <= 32 ? 1 : (last_q <= 64 ? 2 : 4); }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t score_ws_bytes(const Dims& dm) {
  const int QP = 32 * nqt_for(dm.last_q);
  const size_t nchunks = ((size_t)dm.L + kChunk - 1) / kChunk;
  const size_t BH = (size_t)dm.B * dm.Hq;
  return align256(BH * nchunks * QP * sizeof(float2)) + align256(BH * QP * sizeof(float));
}

hipError_t launch_score(const Dims& dm, const void* Q, const void* K, float* scores, void* ws, hipStream_t st) {
  const int nqt = nqt_for(dm.last_q);
  const int QP = 32 * nqt;
  ScoreArgs a;
  a.Q = (const __bf16*)Q; a.K = (const __bf16*)K; a.scores = scores;
  a.Hq = dm.Hq; a.Hkv = dm.Hkv; a.L = dm.L; a.Lq = dm.last_q;
  a.nchunks = (dm.L + kChunk - 1) / kChunk;
  a.c = dm.scale * kLog2e;
  const size_t BH = (size_t)dm.B * dm.Hq;
  a.part = (float2*)ws;
  a.lse2 = (float*)((char*)ws + align256(BH * a.nchunks * QP * sizeof(float2)));
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

}  // namespace tsa
