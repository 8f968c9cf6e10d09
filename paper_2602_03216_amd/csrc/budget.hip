// Dynamic Token Coverage budget: Algorithm 1 of the paper, steps "aggregate and normalize token
// scores across heads", "sort tokens by ascending importance", "determine the number of sparse
// token".  s_l[t] = sum_h s_h[t] (normalised by its total); k_sparse = the smallest k whose k
// least important tokens carry a cumulative mass >= tau; k_keep = L - k_sparse.
//
// No sort is needed: the answer only depends on the value at which the ascending cumulative mass
// crosses tau * total.  A radix descent over the order-preserving uint32 image of s_l finds it
// in 4 passes of 8 bits, least important bin first: every pass builds, for the keys that match
// the prefix found so far, a 256-bin histogram of (count, mass); the next kernel walks the bins
// upwards until count/mass below plus the bin's mass reaches the target.  After the last pass
// the bin is a single fp32 value v, and the number of tied tokens to take is
// ceil((target - mass_below) / v).  Masses are accumulated in fp64 (atomics on integers and
// doubles: the result does not depend on the order beyond 1e-16 relative).
#include "tsa_internal.h"

namespace tsa {

namespace {

constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kSlice = 2048;      // tokens per workgroup: few rows (one per batch entry), so short slices fill the chip

struct BudState {
  uint32_t prefix;       // digits found so far
  uint32_t count_below;  // tokens strictly below the prefix range
  double mass_below;     // their mass
};

struct BudRow {
  double total;
  double mass[4][256];
  uint32_t count[4][256];
  BudState state[5];     // state[p]: before pass p; state[4]: final
};

struct BudArgs {
  const float* scores;   // [B,Hq,L]
  float* sl;             // [B,L]
  BudRow* rows;          // [B]
  int32_t* k_keep;       // [B]
  int Hq, L;
  double tau;
  int k_max;             // upper bound of the result (capacity of the caller's buffers)
};

__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void zero_rows_kernel(BudRow* rows, int n_words) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n_words) ((uint32_t*)rows)[i] = 0u;
}

// s_l = sum over heads, fp32, in head order; total in fp64
__global__ __launch_bounds__(kThreads) void head_sum_kernel(BudArgs a) {
  __shared__ double wsum[kWaves];
  const long long b = blockIdx.y;
  const int t = blockIdx.x * kThreads + threadIdx.x;
  float acc = 0.f;
  if (t < a.L) {
    for (int h = 0; h < a.Hq; ++h) acc += a.scores[(b * a.Hq + h) * a.L + t];
    a.sl[b * a.L + t] = acc;
  }
  double v = (double)acc;
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d);
  if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int w = 0; w < kWaves; ++w) s += wsum[w];
    atomicAdd(&a.rows[b].total, s);
  }
}

// Walks the 256 bins of one pass upwards (first wavefront): lane l owns bins 4l..4l+3.
__device__ __forceinline__ BudState next_state(const BudRow* rw, int pass, BudState st, double target, int shift, int lane) {
  double ms[4];
  uint32_t cn[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) { ms[j] = rw->mass[pass][4 * lane + j]; cn[j] = rw->count[pass][4 * lane + j]; }
  const double mine = ms[0] + ms[1] + ms[2] + ms[3];
  const uint32_t minec = cn[0] + cn[1] + cn[2] + cn[3];
  double incl = mine;
  uint32_t inclc = minec;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const double up = __shfl_up(incl, d);
    const uint32_t upc = __shfl_up(inclc, d);
    if (lane >= d) { incl += up; inclc += upc; }
  }
  // first lane whose bins reach the target; if none does (tau >= 1 up to rounding), the last lane
  // that holds any token
  const unsigned long long reach = __ballot(minec > 0 && st.mass_below + incl >= target);
  const unsigned long long any = __ballot(minec > 0);
  const int who = reach ? __ffsll((long long)reach) - 1 : (any ? 63 - __clzll((long long)any) : 0);
  double mb = st.mass_below + (incl - mine);
  uint32_t cb = st.count_below + (inclc - minec);
  int bin = 4 * lane;
  int last_nonempty = -1;
  bool found = false;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    if (!found && cn[j] > 0) {
      if (mb + ms[j] >= target) { bin = 4 * lane + j; found = true; }
      else { mb += ms[j]; cb += cn[j]; last_nonempty = j; }
    }
  }
  if (!found) {
    // target not reached inside this lane: stay on its last non-empty bin
    bin = 4 * lane + (last_nonempty < 0 ? 0 : last_nonempty);
    if (last_nonempty >= 0) { mb -= ms[last_nonempty]; cb -= cn[last_nonempty]; }
  }
  BudState out;
  out.prefix = st.prefix | ((uint32_t)__shfl(bin, who) << shift);
  out.count_below = __shfl(cb, who);
  out.mass_below = __shfl(mb, who);
  return out;
}

template <int PASS>
__global__ __launch_bounds__(kThreads) void bud_hist_kernel(BudArgs a) {
  __shared__ double hmass[256];
  __shared__ uint32_t hcount[256];
  __shared__ BudState sh_state;
  const int slice = blockIdx.x;
  const long long b = blockIdx.y;
  BudRow* rw = a.rows + b;
  const float* s = a.sl + b * a.L;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  constexpr int shift = 24 - 8 * PASS;
  if (wave == 0) {
    BudState st;
    if (PASS == 0) { st.prefix = 0u; st.count_below = 0u; st.mass_below = 0.0; }
    else st = next_state(rw, PASS - 1, rw->state[PASS - 1], a.tau * rw->total, shift + 8, lane);
    if (lane == 0) {
      sh_state = st;
      if (slice == 0) rw->state[PASS] = st;
    }
  }
  if (tid < 256) { hmass[tid] = 0.0; hcount[tid] = 0u; }
  __syncthreads();
  const uint32_t prefix = sh_state.prefix;
  constexpr uint32_t himask = PASS == 0 ? 0u : (0xffffffffu << (shift + 8));
  const int t_end = min(a.L, (slice + 1) * kSlice);
  for (int t = slice * kSlice + tid; t < t_end; t += kThreads) {
    const float v = s[t];
    const uint32_t key = order_key(v);
    if ((key & himask) == prefix) {
      const uint32_t dg = (key >> shift) & 255u;
      atomicAdd(&hcount[dg], 1u);
      atomicAdd(&hmass[dg], (double)v);
    }
  }
  __syncthreads();
  if (tid < 256 && hcount[tid]) {
    atomicAdd(&rw->count[PASS][tid], hcount[tid]);
    atomicAdd(&rw->mass[PASS][tid], hmass[tid]);
  }
}

__global__ void bud_final_kernel(BudArgs a) {
  const long long b = blockIdx.x;
  BudRow* rw = a.rows + b;
  const int lane = threadIdx.x;
  const double target = a.tau * rw->total;
  const BudState st = next_state(rw, 3, rw->state[3], target, 0, lane);
  if (lane == 0) {
    rw->state[4] = st;
    long long k_sparse = 0;
    if (a.tau > 0.0) {
      // all tokens of the final bin have the value v: take as many as are needed to reach the target
      const uint32_t bin = st.prefix & 255u;
      const uint32_t n_eq = rw->count[3][bin];
      const double v = (double)key_value(st.prefix);
      long long j = n_eq;
      if (v > 0.0) {
        const double need = (target - st.mass_below) / v;
        j = (long long)ceil(need);
        if (j < 1) j = 1;
        if (j > (long long)n_eq) j = n_eq;
      }
      k_sparse = (long long)st.count_below + j;
    }
    long long keep = (long long)a.L - k_sparse;
    if (keep < 1) keep = 1;
    if (keep > a.k_max) keep = a.k_max;
    a.k_keep[b] = (int32_t)keep;
  }
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

}  // namespace

size_t budget_ws_bytes(const Dims& dm) {
  return align256((size_t)dm.B * sizeof(BudRow)) + align256((size_t)dm.B * dm.L * sizeof(float));
}

hipError_t launch_budget(const Dims& dm, const float* scores, double tau_cov, int32_t* k_keep, void* ws, hipStream_t st,
                         int k_max) {
  BudArgs a;
  a.k_max = k_max > 0 ? k_max : dm.L;
  a.scores = scores;
  a.rows = (BudRow*)ws;
  a.sl = (float*)((char*)ws + align256((size_t)dm.B * sizeof(BudRow)));
  a.k_keep = k_keep;
  a.Hq = dm.Hq; a.L = dm.L; a.tau = tau_cov;
  const int n_words = (int)((size_t)dm.B * sizeof(BudRow) / 4);
  zero_rows_kernel<<<(n_words + 255) / 256, 256, 0, st>>>(a.rows, n_words);
  head_sum_kernel<<<dim3((dm.L + kThreads - 1) / kThreads, dm.B), kThreads, 0, st>>>(a);
  const dim3 grid((dm.L + kSlice - 1) / kSlice, dm.B);
  bud_hist_kernel<0><<<grid, kThreads, 0, st>>>(a);
  bud_hist_kernel<1><<<grid, kThreads, 0, st>>>(a);
  bud_hist_kernel<2><<<grid, kThreads, 0, st>>>(a);
  bud_hist_kernel<3><<<grid, kThreads, 0, st>>>(a);
  bud_final_kernel<<<dm.B, 64, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace tsa
