// Head-wise top-k selection: Algorithm 1 of the paper, S_h = TopK(s_h, k_keep).
// Exact: the k_keep largest scores, ties to the lowest token index, emitted in ascending
// token order together with the inverse map.  Integer work on the order-preserving uint32
// image of the fp32 score:
//   1. radix select (4 passes of 8 bits, histograms in LDS) finds the k-th largest key T and
//      how many keys equal to T have to be taken;
//   2. a stable compaction (wave ballots + prefix sums) writes idx ascending and inv.
// One workgroup of 1024 threads per (batch, selection head).
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;

// fp32 -> uint32 with the same order (-0 and +0 map to the same key)
__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint32_t key_at(const float* __restrict__ s, int t, int L, int ff, int fl) {
  if (t < ff || t >= L - fl) return 0xffffffffu;   // always-kept tokens rank above every score
  return order_key(s[t]);
}

__global__ __launch_bounds__(kThreads) void select_kernel(const float* __restrict__ scores, int32_t* __restrict__ idx,
                                                          int32_t* __restrict__ inv, int L, int k, int ff, int fl) {
  __shared__ uint32_t hist[kWaves][256];
  __shared__ uint32_t total[256];
  __shared__ uint32_t sh_prefix, sh_krem;
  __shared__ uint32_t w_gt[kWaves], w_eq[kWaves], w_out[kWaves], w_eqb[kWaves];

  const long long row = blockIdx.x;
  const float* s = scores + row * L;
  int32_t* out_idx = idx + row * k;
  int32_t* out_inv = inv ? inv + row * L : nullptr;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;

  if (tid == 0) { sh_prefix = 0u; sh_krem = (uint32_t)k; }
  // ---- radix select, most significant digit first ----
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    for (int i = tid; i < kWaves * 256; i += kThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int base = 0; base < L; base += kThreads) {
      const int t = base + tid;
      bool valid = false;
      uint32_t dg = 0;
      if (t < L) {
        const uint32_t key = key_at(s, t, L, ff, fl);
        valid = (key & himask) == prefix;
        dg = (key >> shift) & 255u;
      }
      const unsigned long long act = __ballot(valid);
      if (act == 0ull) continue;
      // common case in the first pass: the whole wavefront falls into one bin
      const int leader = __ffsll((long long)act) - 1;
      const uint32_t dg0 = __shfl(dg, leader);
      const unsigned long long same = __ballot(valid && dg == dg0);
      if (same == act) {
        if (lane == leader) atomicAdd(&hist[wave][dg0], (uint32_t)__popcll(act));
      } else if (valid) {
        atomicAdd(&hist[wave][dg], 1u);
      }
    }
    __syncthreads();
    if (tid < 256) {
      uint32_t c = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) c += hist[w][tid];
      total[tid] = c;
    }
    __syncthreads();
    if (tid == 0) {
      uint32_t krem = sh_krem, above = 0;
      int bin = 255;
      for (; bin > 0; --bin) {
        if (above + total[bin] >= krem) break;
        above += total[bin];
      }
      sh_krem = krem - above;
      sh_prefix = prefix | ((uint32_t)bin << shift);
    }
    __syncthreads();
  }
  const uint32_t T = sh_prefix;          // k-th largest key
  const uint32_t need_eq = sh_krem;      // how many keys equal to T are taken (lowest tokens first)

  // ---- stable compaction: each wavefront owns a contiguous range of tokens ----
  const int seg = (((L + kWaves - 1) / kWaves) + 63) & ~63;
  const int t_lo = wave * seg;
  const int t_hi = min(L, t_lo + seg);
  uint32_t n_gt = 0, n_eq = 0;
  for (int base = t_lo; base < t_hi; base += 64) {
    const int t = base + lane;
    uint32_t key = 0;
    const bool in = t < t_hi;
    if (in) key = key_at(s, t, L, ff, fl);
    n_gt += (uint32_t)__popcll(__ballot(in && key > T));
    n_eq += (uint32_t)__popcll(__ballot(in && key == T));
  }
  if (lane == 0) { w_gt[wave] = n_gt; w_eq[wave] = n_eq; }
  __syncthreads();
  if (tid == 0) {
    uint32_t eqb = 0, outb = 0;
    for (int w = 0; w < kWaves; ++w) {
      w_eqb[w] = eqb;
      w_out[w] = outb;
      const uint32_t room = need_eq > eqb ? need_eq - eqb : 0u;
      outb += w_gt[w] + min(room, w_eq[w]);
      eqb += w_eq[w];
    }
  }
  __syncthreads();
  uint32_t eq_run = w_eqb[wave], out_run = w_out[wave];
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (int base = t_lo; base < t_hi; base += 64) {
    const int t = base + lane;
    const bool in = t < t_hi;
    uint32_t key = 0;
    if (in) key = key_at(s, t, L, ff, fl);
    const bool gt = in && key > T;
    const bool eq = in && key == T;
    const unsigned long long m_eq = __ballot(eq);
    const uint32_t eq_rank = eq_run + (uint32_t)__popcll(m_eq & lt_mask);
    const bool take = gt || (eq && eq_rank < need_eq);
    const unsigned long long m_take = __ballot(take);
    const uint32_t pos = out_run + (uint32_t)__popcll(m_take & lt_mask);
    if (take) out_idx[pos] = t;
    if (in && out_inv) out_inv[t] = take ? (int32_t)pos : -1;
    out_run += (uint32_t)__popcll(m_take);
    eq_run += (uint32_t)__popcll(m_eq);
  }
}

// scores [B,Hq,L] -> [B,Hkv,L]: sum of the g heads of each KV group, in head order
__global__ void group_sum_kernel(const float* __restrict__ s, float* __restrict__ out, int g, int L, long long n) {
  const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const long long grp = i / L;
  const int t = (int)(i % L);
  float acc = 0.f;
  for (int j = 0; j < g; ++j) acc += s[(grp * g + j) * L + t];
  out[i] = acc;
}

}  // namespace

size_t select_ws_bytes(const Dims& dm) {
  if (!dm.group_mode) return 0;
  return (((size_t)dm.B * dm.Hkv * dm.L * sizeof(float)) + 255) & ~(size_t)255;
}

hipError_t launch_select(const Dims& dm, const float* scores, int k_keep, int32_t* idx, int32_t* inv,
                         void* ws, hipStream_t st) {
  const float* src = scores;
  int rows = dm.B * dm.Hq;
  if (dm.group_mode) {
    rows = dm.B * dm.Hkv;
    const long long n = (long long)rows * dm.L;
    group_sum_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(scores, (float*)ws, dm.Hq / dm.Hkv, dm.L, n);
    src = (const float*)ws;
  }
  select_kernel<<<rows, kThreads, 0, st>>>(src, idx, inv, dm.L, k_keep, dm.force_first, dm.force_last);
  return hipGetLastError();
}

}  // namespace tsa
