// Head-wise top-k selection: Algorithm 1 of the paper, S_h = TopK(s_h, k_keep).
// Exact: the k_keep largest scores, ties to the lowest token index, emitted in ascending
// token order together with the inverse map.  Integer work on the order-preserving uint32
// image of the fp32 score:
//   1. radix select, 4 passes of 8 bits, most significant first: every pass histograms the
//      digit of the keys that still match the prefix found so far (LDS histograms per
//      wavefront), and the next kernel derives the digit of the k-th largest key from the
//      histogram.  The first pass writes one histogram per slice (nothing has to be cleared
//      beforehand; its first slice clears the row histograms of the later passes, which are
//      built with one global atomic per bin and workgroup); the last pass also leaves, per
//      slice, the number of keys above the 24-bit prefix and the histogram of the last digit;
//   2. write: the threshold key T from the last histogram; the per-slice figures of the last
//      pass give the number of keys above T / equal to T in the slices before this one,
//      per-wavefront counts inside the slice give every wavefront its output offset; a stable
//      ballot compaction writes idx ascending and inv.
// A head is cut into at most 64 slices (a power of two of tokens, at least 2048, one workgroup of 1024
// threads each), sized so that a launch has about 512 workgroups: each of the five small kernels
// is a chain of dependent steps per thread, so it pays to spread it over the whole chip, but not
// to go below a few tokens per thread.
#include "tsa_internal.h"

#include <mutex>

namespace tsa {

namespace {

constexpr int kMaxDevices = 64;
constexpr int kThreads = 1024;
constexpr int kWaves = kThreads / 64;
constexpr int kMinSlice = 2048, kMaxSlice = 16384;   // tokens per workgroup (SelArgs::slice), unless a row needs more
constexpr int kMaxSlices = 64;                       // slices per row at most

struct SelState {
  uint32_t prefix;   // digits found so far, in place
  uint32_t krem;     // how many keys are still wanted among those that match the prefix
};

// Per selection row (batch, head or group) in the workspace:
struct RowWs {
  uint32_t hist[4][256];      // [0] is unused (the first pass keeps one histogram per slice)
  SelState state[5];          // state[p]: before pass p; state[4]: (T, number of keys equal to T to take)
  uint32_t pad[6];
};

// Per (row, slice) in the workspace:
struct SliceWs {
  uint32_t hist0[256];        // first pass: digit histogram of the slice
  uint32_t last[256];         // last pass: last digit of the slice's keys that match the 24-bit prefix
  uint32_t n_above;           // last pass: keys of the slice above the 24-bit prefix
  uint32_t pad[63];
};

struct SelArgs {
  const float* scores;
  int32_t* idx;
  int32_t* inv;
  RowWs* rows;
  SliceWs* slices;            // [row][nslices]
  int L, k, ff, fl, nslices;
  int slice;                  // tokens per workgroup; a wavefront owns slice / kWaves contiguous tokens
  // Count decided on the device (dynamic coverage budget): k_dev[b] replaces k for the rows of batch
  // entry b (NULL: every row takes k); a row of idx is k_stride entries long either way.
  const int32_t* k_dev;
  int k_stride, rows_per_b;
  __device__ __forceinline__ uint32_t k_of(long long row) const {
    return (uint32_t)(k_dev ? k_dev[row / rows_per_b] : k);
  }
};

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

// Digit of the krem-th largest key among those counted in `hist`, found by the first wavefront:
// lane l sums bins 255-4l .. 252-4l, a wave scan finds the lane where the running count from the
// top reaches krem, the lane then walks its four bins.
__device__ __forceinline__ SelState next_state(const uint32_t* __restrict__ hist, SelState st, int shift, int lane) {
  uint32_t c[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) c[j] = hist[255 - 4 * lane - j];
  const uint32_t mine = c[0] + c[1] + c[2] + c[3];
  uint32_t incl = mine;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d);
    if (lane >= d) incl += up;
  }
  const unsigned long long reach = __ballot(incl >= st.krem);
  const int who = reach ? __ffsll((long long)reach) - 1 : 63;
  uint32_t above = incl - mine, bin = 255 - 4 * lane;
#pragma unroll
  for (int j = 0; j < 3; ++j) {
    if (above + c[j] < st.krem) { above += c[j]; bin = 255 - 4 * lane - (j + 1); }
    else break;
  }
  SelState out;
  out.prefix = st.prefix | (__shfl(bin, who) << shift);
  out.krem = st.krem - __shfl(above, who);
  return out;
}

template <int PASS>
__global__ __launch_bounds__(kThreads) void hist_kernel(SelArgs a) {
  __shared__ uint32_t hist[kWaves][256];
  __shared__ uint32_t tot[256];
  __shared__ SelState sh_state;
  __shared__ uint32_t sh_above;
  const int slice = blockIdx.x;
  const long long row = blockIdx.y;
  RowWs* rw = a.rows + row;
  SliceWs* sw = a.slices + row * a.nslices + slice;
  const float* s = a.scores + row * a.L;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  constexpr int shift = 24 - 8 * PASS;

  if (PASS == 0 && slice == 0) {                          // row histograms of the later passes start at zero
    for (int i = tid; i < 3 * 256; i += kThreads) rw->hist[1 + i / 256][i % 256] = 0u;
  }
  if (PASS == 1) {                                        // the first pass left one histogram per slice: add them up
    const SliceWs* row_slices = a.slices + row * a.nslices;
    uint32_t c = 0;
    for (int sl = tid >> 8; sl < a.nslices; sl += kThreads / 256) c += row_slices[sl].hist0[tid & 255];
    hist[tid >> 8][tid & 255] = c;
    __syncthreads();
    if (tid < 256) tot[tid] = hist[0][tid] + hist[1][tid] + hist[2][tid] + hist[3][tid];
    __syncthreads();
  }
  if (wave == 0) {
    SelState st;
    if (PASS == 0) { st.prefix = 0u; st.krem = a.k_of(row); }
    else st = next_state(PASS == 1 ? tot : rw->hist[PASS - 1], rw->state[PASS - 1], shift + 8, lane);
    if (lane == 0) {
      sh_state = st;
      if (slice == 0) rw->state[PASS] = st;
    }
  }
  for (int i = tid; i < kWaves * 256; i += kThreads) (&hist[0][0])[i] = 0u;
  if (tid == 0) sh_above = 0u;
  __syncthreads();
  const uint32_t prefix = sh_state.prefix;
  constexpr uint32_t himask = PASS == 0 ? 0u : (0xffffffffu << (shift + 8));
  const int t_end = min(a.L, (slice + 1) * a.slice);
  uint32_t above = 0;
  for (int base = slice * a.slice; base < t_end; base += kThreads) {
    const int t = base + tid;
    bool valid = false;
    uint32_t dg = 0;
    if (t < t_end) {
      const uint32_t key = key_at(s, t, a.L, a.ff, a.fl);
      valid = (key & himask) == prefix;
      dg = (key >> shift) & 255u;
      if (PASS == 3 && (key & himask) > prefix) ++above;
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
  if (PASS == 3) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) above += __shfl_xor(above, d);
    if (lane == 0 && above) atomicAdd(&sh_above, above);
  }
  __syncthreads();
  if (tid < 256) {
    uint32_t c = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) c += hist[w][tid];
    if (PASS == 0) sw->hist0[tid] = c;
    else if (c) atomicAdd(&rw->hist[PASS][tid], c);
    if (PASS == 3) sw->last[tid] = c;
  }
  if (PASS == 3 && tid == 0) sw->n_above = sh_above;
}

// Keys of a wavefront's segment held in registers between the counting and the compaction: segments of up
// to kRegKeys * 64 tokens (slices of up to 16384) are read once, longer ones are read again.
constexpr int kRegKeys = 16;

__global__ __launch_bounds__(kThreads) void write_kernel(SelArgs a) {
  __shared__ SelState sh_state;
  __shared__ uint32_t before_gt, before_eq;
  __shared__ uint2 cnt[kWaves];
  const int slice = blockIdx.x;
  const long long row = blockIdx.y;
  RowWs* rw = a.rows + row;
  const SliceWs* row_slices = a.slices + row * a.nslices;
  const float* s = a.scores + row * a.L;
  int32_t* out_idx = a.idx + row * a.k_stride;
  int32_t* out_inv = a.inv ? a.inv + row * a.L : nullptr;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  // the keys of this wavefront's segment are requested first: their latency hides behind the threshold
  const int seg = a.slice / kWaves;
  const int t_lo = slice * a.slice + wave * seg;
  const int t_hi = min(a.L, t_lo + seg);
  const bool in_regs = seg <= kRegKeys * 64;
  uint32_t keys[kRegKeys];
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < kRegKeys; ++j) {
      const int t = t_lo + 64 * j + lane;
      keys[j] = t < t_hi ? key_at(s, t, a.L, a.ff, a.fl) : 0u;
    }
  }
  if (tid == 0) { before_gt = 0u; before_eq = 0u; }
  if (wave == 0) {
    const SelState st = next_state(rw->hist[3], rw->state[3], 0, lane);
    if (lane == 0) {
      sh_state = st;
      if (slice == 0) rw->state[4] = st;
    }
  }
  __syncthreads();
  const uint32_t T = sh_state.prefix;
  const uint32_t need_eq = sh_state.krem;
  // keys above T / equal to T in the slices before this one, from what the last pass left per slice
  {
    const uint32_t dT = T & 255u;
    uint32_t gt = 0, eq = 0;
    if (tid < slice) gt = row_slices[tid].n_above;
    for (int i = tid; i < slice * 256; i += kThreads) {
      const uint32_t v = row_slices[i >> 8].last[i & 255];
      const uint32_t d = (uint32_t)(i & 255);
      gt += d > dT ? v : 0u;
      eq += d == dT ? v : 0u;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
      gt += __shfl_xor(gt, d);
      eq += __shfl_xor(eq, d);
    }
    if (lane == 0) {
      if (gt) atomicAdd(&before_gt, gt);
      if (eq) atomicAdd(&before_eq, eq);
    }
  }
  // this slice: per-wavefront counts, then the stable compaction
  {
    uint32_t n_gt = 0, n_eq = 0;
    if (in_regs) {
#pragma unroll
      for (int j = 0; j < kRegKeys; ++j) {
        const bool in = t_lo + 64 * j + lane < t_hi;
        n_gt += (uint32_t)__popcll(__ballot(in && keys[j] > T));
        n_eq += (uint32_t)__popcll(__ballot(in && keys[j] == T));
      }
    } else {
      for (int base = t_lo; base < t_hi; base += 64) {
        const int t = base + lane;
        const bool in = t < t_hi;
        const uint32_t key = in ? key_at(s, t, a.L, a.ff, a.fl) : 0u;
        n_gt += (uint32_t)__popcll(__ballot(in && key > T));
        n_eq += (uint32_t)__popcll(__ballot(in && key == T));
      }
    }
    if (lane == 0) cnt[wave] = make_uint2(n_gt, n_eq);
  }
  __syncthreads();
  uint32_t gt_before = before_gt, eq_before = before_eq;
  for (int w = 0; w < wave; ++w) { gt_before += cnt[w].x; eq_before += cnt[w].y; }
  // ties are taken in token order until need_eq of them are used up
  uint32_t eq_run = eq_before, out_run = gt_before + min(need_eq, eq_before);
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  auto emit = [&](int t, uint32_t key) {
    const bool in = t < t_hi;
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
  };
  if (in_regs) {
#pragma unroll
    for (int j = 0; j < kRegKeys; ++j)
      if (t_lo + 64 * j < t_hi) emit(t_lo + 64 * j + lane, keys[j]);
  } else {
    for (int base = t_lo; base < t_hi; base += 64) {
      const int t = base + lane;
      emit(t, t < t_hi ? key_at(s, t, a.L, a.ff, a.fl) : 0u);
    }
  }
}

// Short rows (L <= kSmallL): the whole selection of a row in ONE launch by one workgroup.  The
// order-preserving keys of the row are kept in LDS (4 bytes per token), the four radix passes, the
// counting and the stable compaction all run out of LDS; same arithmetic and same result as the
// sliced kernels above, without six launches whose fixed cost dominates at this size.
constexpr int kSmallL = 16384;

__global__ __launch_bounds__(kThreads) void select_small_kernel(SelArgs a) {
  extern __shared__ uint32_t dyn[];
  uint32_t* keys = dyn;                                   // [L]
  uint32_t* hist = dyn + a.L;                             // [kWaves][256], then reused
  __shared__ uint32_t tot[256];
  __shared__ SelState sh_state;
  __shared__ uint2 cnt[kWaves];
  const long long row = blockIdx.x;
  const float* s = a.scores + row * a.L;
  int32_t* out_idx = a.idx + row * a.k_stride;
  int32_t* out_inv = a.inv ? a.inv + row * a.L : nullptr;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  for (int t = tid; t < a.L; t += kThreads) keys[t] = key_at(s, t, a.L, a.ff, a.fl);
  SelState st;
  st.prefix = 0u;
  st.krem = a.k_of(row);
#pragma unroll 1
  for (int pass = 0; pass < 4; ++pass) {
    const int shift = 24 - 8 * pass;
    const uint32_t himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
    for (int i = tid; i < kWaves * 256; i += kThreads) hist[i] = 0u;
    __syncthreads();                                      // keys (first pass) and cleared histograms are visible
    for (int base = 0; base < a.L; base += kThreads) {
      const int t = base + tid;
      bool valid = false;
      uint32_t dg = 0;
      if (t < a.L) {
        const uint32_t key = keys[t];
        valid = (key & himask) == st.prefix;
        dg = (key >> shift) & 255u;
      }
      const unsigned long long act = __ballot(valid);
      if (act == 0ull) continue;
      const int leader = __ffsll((long long)act) - 1;
      const uint32_t dg0 = __shfl(dg, leader);
      const unsigned long long same = __ballot(valid && dg == dg0);
      if (same == act) {
        if (lane == leader) atomicAdd(&hist[wave * 256 + dg0], (uint32_t)__popcll(act));
      } else if (valid) {
        atomicAdd(&hist[wave * 256 + dg], 1u);
      }
    }
    __syncthreads();
    if (tid < 256) {
      uint32_t c = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) c += hist[w * 256 + tid];
      tot[tid] = c;
    }
    __syncthreads();
    if (wave == 0) {
      const SelState nx = next_state(tot, st, shift, lane);
      if (lane == 0) sh_state = nx;
    }
    __syncthreads();
    st = sh_state;
  }
  // st.prefix = threshold key T, st.krem = number of keys equal to T to take (in token order)
  const uint32_t T = st.prefix, need_eq = st.krem;
  const int seg = ((a.L + kWaves - 1) / kWaves + 63) & ~63;
  const int t_lo = wave * seg, t_hi = min(a.L, t_lo + seg);
  uint32_t n_gt = 0, n_eq = 0;
  for (int base = t_lo; base < t_hi; base += 64) {
    const int t = base + lane;
    const bool in = t < t_hi;
    const uint32_t key = in ? keys[t] : 0u;
    n_gt += (uint32_t)__popcll(__ballot(in && key > T));
    n_eq += (uint32_t)__popcll(__ballot(in && key == T));
  }
  if (lane == 0) cnt[wave] = make_uint2(n_gt, n_eq);
  __syncthreads();
  uint32_t gt_before = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) { gt_before += cnt[w].x; eq_before += cnt[w].y; }
  uint32_t eq_run = eq_before, out_run = gt_before + min(need_eq, eq_before);
  const unsigned long long lt_mask = (1ull << lane) - 1ull;
  for (int base = t_lo; base < t_hi; base += 64) {
    const int t = base + lane;
    const bool in = t < t_hi;
    const uint32_t key = in ? keys[t] : 0u;
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

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int n_rows(const Dims& dm) { return dm.B * (dm.group_mode ? dm.Hkv : dm.Hq); }
// tokens per workgroup: the power of two that gives the launch about 512 workgroups
inline int slice_for(const Dims& dm) {
  const long long want = (long long)n_rows(dm) * dm.L / 512;
  int s = kMinSlice;
  while (s < kMaxSlice && s < want) s *= 2;
  while ((dm.L + s - 1) / s > kMaxSlices) s *= 2;
  return s;
}
inline int n_slices(const Dims& dm) { return (dm.L + slice_for(dm) - 1) / slice_for(dm); }

}  // namespace

size_t select_ws_bytes(const Dims& dm) {
  size_t n = align256((size_t)n_rows(dm) * sizeof(RowWs));
  n += align256((size_t)n_rows(dm) * n_slices(dm) * sizeof(SliceWs));
  if (dm.group_mode) n += align256((size_t)dm.B * dm.Hkv * dm.L * sizeof(float));
  return n;
}

hipError_t launch_select(const Dims& dm, const float* scores, int k_keep, int32_t* idx, int32_t* inv,
                         void* ws, hipStream_t st, const int32_t* k_dev) {
  const int rows = n_rows(dm);
  SelArgs a;
  a.rows = (RowWs*)ws;
  a.slices = (SliceWs*)((char*)ws + align256((size_t)rows * sizeof(RowWs)));
  a.scores = scores;
  if (dm.group_mode) {
    float* gs = (float*)((char*)a.slices + align256((size_t)rows * n_slices(dm) * sizeof(SliceWs)));
    const long long n = (long long)rows * dm.L;
    group_sum_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(scores, gs, dm.Hq / dm.Hkv, dm.L, n);
    a.scores = gs;
  }
  a.idx = idx; a.inv = inv;
  a.L = dm.L; a.k = k_keep; a.ff = dm.force_first; a.fl = dm.force_last; a.nslices = n_slices(dm);
  a.k_dev = k_dev; a.k_stride = k_keep; a.rows_per_b = rows / dm.B;
  a.slice = slice_for(dm);
  if (dm.L <= kSmallL) {
    const size_t lds = ((size_t)dm.L + kWaves * 256) * sizeof(uint32_t);
    // the attribute belongs to the kernel as loaded on ONE device: set it once per device, under a lock
    {
      static std::mutex mu;
      static bool attr_set[kMaxDevices] = {};
      int dev = 0;
      hipError_t e = hipGetDevice(&dev);
      if (e != hipSuccess) return e;
      if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
      std::lock_guard<std::mutex> lock(mu);
      if (!attr_set[dev]) {
        e = hipFuncSetAttribute((const void*)select_small_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 4096);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
      }
    }
    select_small_kernel<<<rows, kThreads, lds, st>>>(a);
    return hipGetLastError();
  }
  const dim3 grid(a.nslices, rows);
  hist_kernel<0><<<grid, kThreads, 0, st>>>(a);
  hist_kernel<1><<<grid, kThreads, 0, st>>>(a);
  hist_kernel<2><<<grid, kThreads, 0, st>>>(a);
  hist_kernel<3><<<grid, kThreads, 0, st>>>(a);
  write_kernel<<<grid, kThreads, 0, st>>>(a);
  return hipGetLastError();
}

}  // namespace tsa
