// Dynamic Token Coverage budget: the budget steps of Algorithm 1 of the paper (Section 2.3): cross-head
// sum of the token scores, normalisation, ascending order, cumulative-mass threshold.
// s_l[t] = sum_h s_h[t] (normalised by its total); k_sparse = the smallest k whose k
// least important tokens carry a cumulative mass >= tau; k_keep = L - k_sparse.
//
// No sort is needed: the answer only depends on the value at which the ascending cumulative mass
// crosses tau * total.  A radix descent over the order-preserving uint32 image of s_l finds it
// in 4 passes of 8 bits, least important bin first: every pass builds, for the keys that match
// the prefix found so far, a 256-bin histogram of (count, mass); the next kernel walks the bins
// upwards until count/mass below plus the bin's mass reaches the target.  After the last pass
// the bin is a single fp32 value v, and the number of tied tokens to take is
// ceil((target - mass_below) / v).
// Masses are EXACT and do not depend on the order of the additions: the keys of one bin differ by at
// most one step of the binary exponent (first pass) or share it (later passes), so a bin's mass is kept
// as the integer sum of the 24-bit significands (shifted by the lowest exponent bit), accumulated with
// integer atomics, and becomes a double only when the bins are walked, in a fixed order.  Two runs on
// the same scores give the same count bit for bit.
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
  double total;                        // written by the first slice of pass 1, read by the later launches
  unsigned long long isum[4][256];     // per bin: sum of significands, in units of 2^(E - 150), E = bin_exponent()
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
  int k_min;             // lower bound of the result (at least 1)
};

__device__ __forceinline__ uint32_t order_key(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u << 1) == 0u) u = 0u;
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k) {
  return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// A float as significand x 2^(exponent - 150): finite v, sig < 2^24 (subnormals: exponent field 1).
__device__ __forceinline__ void split_float(float v, uint32_t& sig, int& e) {
  const uint32_t u = __float_as_uint(v);
  e = (int)((u >> 23) & 255u);
  sig = u & 0x7fffffu;
  if (e) sig |= 0x800000u; else e = 1;
}
// Exponent unit of a bin's integer sum: the exponent field of the bin's smallest magnitude.  The first
// pass fixes sign and the upper seven exponent bits (the low bit is free: significands of the larger
// exponent are shifted left by one); later passes fix the whole exponent.  `key_prefix`: any key of the bin.
__device__ __forceinline__ int bin_exponent(uint32_t key_prefix, int pass) {
  const uint32_t u = (key_prefix & 0x80000000u) ? (key_prefix & 0x7fffffffu) : ~key_prefix;   // back to float bits
  int e = (int)((u >> 23) & 255u);
  if (pass == 0) e &= ~1;
  return e < 1 ? 1 : e;
}
__device__ __forceinline__ double bin_mass(unsigned long long isum, uint32_t key_prefix, int pass) {
  const double m = ldexp((double)isum, bin_exponent(key_prefix, pass) - 150);     // isum < 2^53: exact
  return (key_prefix & 0x80000000u) ? m : -m;                                     // keys below 2^31 are negative scores
}

// s_l = sum over heads, fp32, in head order; also clears the histograms of the four passes
__global__ __launch_bounds__(kThreads) void head_sum_kernel(BudArgs a) {
  const long long b = blockIdx.y;
  const int t = blockIdx.x * kThreads + threadIdx.x;
  if (t < a.L) {
    float acc = 0.f;
    for (int h = 0; h < a.Hq; ++h) acc += a.scores[(b * a.Hq + h) * a.L + t];
    a.sl[b * a.L + t] = acc;
  }
  constexpr int n_words = (int)(sizeof(BudRow) / 4);
  uint32_t* row = (uint32_t*)(a.rows + b);
  for (int i = t; i < n_words; i += gridDim.x * kThreads) row[i] = 0u;
}

// Walks the 256 bins of one pass upwards (first wavefront): lane l owns bins 4l..4l+3.
// `total` (may be NULL): receives the mass of all bins of the pass (every lane gets the same value).
__device__ __forceinline__ BudState next_state(const BudRow* rw, int pass, BudState st, double tau, double* total, int shift,
                                               int lane) {
  double ms[4];
  uint32_t cn[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const uint32_t key_prefix = st.prefix | ((uint32_t)(4 * lane + j) << shift);
    ms[j] = bin_mass(rw->isum[pass][4 * lane + j], key_prefix, pass);
    cn[j] = rw->count[pass][4 * lane + j];
  }
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
  double target;
  if (total) {                          // first pass: its bins hold every token, their mass is the total
    *total = __shfl(incl, 63);
    target = tau * *total;
  } else {
    target = tau * rw->total;
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
  __shared__ unsigned long long hsum[256];
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
    else {
      double total;
      st = next_state(rw, PASS - 1, rw->state[PASS - 1], a.tau, PASS == 1 ? &total : nullptr, shift + 8, lane);
      if (PASS == 1 && lane == 0 && slice == 0) rw->total = total;
    }
    if (lane == 0) {
      sh_state = st;
      if (slice == 0) rw->state[PASS] = st;
    }
  }
  if (tid < 256) { hsum[tid] = 0ull; hcount[tid] = 0u; }
  __syncthreads();
  const uint32_t prefix = sh_state.prefix;
  constexpr uint32_t himask = PASS == 0 ? 0u : (0xffffffffu << (shift + 8));
  const int t_end = min(a.L, (slice + 1) * kSlice);
  for (int t = slice * kSlice + tid; t < t_end; t += kThreads) {
    const float v = s[t];
    const uint32_t key = order_key(v);
    if ((key & himask) == prefix) {
      const uint32_t dg = (key >> shift) & 255u;
      uint32_t sig;
      int e;
      split_float(v, sig, e);
      atomicAdd(&hcount[dg], 1u);
      atomicAdd(&hsum[dg], (unsigned long long)sig << (e - bin_exponent(key, PASS)));   // shift is 0 or 1
    }
  }
  __syncthreads();
  if (tid < 256 && hcount[tid]) {
    atomicAdd(&rw->count[PASS][tid], hcount[tid]);
    atomicAdd(&rw->isum[PASS][tid], hsum[tid]);
  }
}

__global__ void bud_final_kernel(BudArgs a) {
  const long long b = blockIdx.x;
  BudRow* rw = a.rows + b;
  const int lane = threadIdx.x;
  const double target = a.tau * rw->total;
  const BudState st = next_state(rw, 3, rw->state[3], a.tau, nullptr, 0, lane);
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
    if (keep < a.k_min) keep = a.k_min;
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
                         int k_max, int k_min) {
  BudArgs a;
  a.k_max = k_max > 0 ? k_max : dm.L;
  a.k_min = k_min > 1 ? k_min : 1;
  a.scores = scores;
  a.rows = (BudRow*)ws;
  a.sl = (float*)((char*)ws + align256((size_t)dm.B * sizeof(BudRow)));
  a.k_keep = k_keep;
  a.Hq = dm.Hq; a.L = dm.L; a.tau = tau_cov;
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
