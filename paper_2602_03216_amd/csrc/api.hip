// C-ABI layer of libtsa: argument validation on the host, workspace carving, kernel launches.
// Nothing here allocates device memory or synchronises with the host.
#include "../../include/tsa.h"
#include "../../include/tsa_bench.h"
#include "tsa_internal.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>

#ifndef TSA_STATIC_SCRATCH_BYTES
#define TSA_STATIC_SCRATCH_BYTES (8u << 20)
#endif

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

inline bool misaligned(const void* p) { return ((uintptr_t)p & 15u) != 0; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Checks the descriptor; on success fills the launcher's view of it.
int check_desc(const tsa_desc* d, tsa::Dims* out) {
  if (!d) return fail(TSA_ERR_ARG, "desc is NULL");
  if (d->B < 1 || d->Hq < 1 || d->Hkv < 1 || d->L < 1) return fail(TSA_ERR_ARG, "B, Hq, Hkv, L must be >= 1");
  if (d->Hq % d->Hkv != 0) return fail(TSA_ERR_ARG, "Hq (%d) is not a multiple of Hkv (%d)", d->Hq, d->Hkv);
  if (d->d != 64 && d->d != 128) return fail(TSA_ERR_UNSUPPORTED, "head dimension %d: only 64 and 128 are built", d->d);
  if (d->last_q < 1 || d->last_q > d->L || d->last_q > 128)
    return fail(TSA_ERR_ARG, "last_q (%d) must lie in [1, min(L, 128)]", d->last_q);
  if (d->pool_w < 1 || d->pool_w % 2 == 0 || d->pool_w > 1023)
    return fail(TSA_ERR_ARG, "pool_w (%d) must be odd and lie in [1, 1023]", d->pool_w);
  if (d->group_mode != 0 && d->group_mode != 1) return fail(TSA_ERR_ARG, "group_mode must be 0 or 1");
  if (d->block_list_per_head != 0 && d->block_list_per_head != 1) return fail(TSA_ERR_ARG, "block_list_per_head must be 0 or 1");
  if (d->force_first < 0 || d->force_last < 0 || (long long)d->force_first + d->force_last > d->L)
    return fail(TSA_ERR_ARG, "force_first / force_last out of range");
  if (!(d->scale >= 0.0f) || !std::isfinite(d->scale)) return fail(TSA_ERR_ARG, "scale must be finite and >= 0");
  if ((long long)d->B * d->Hq > 65535) return fail(TSA_ERR_UNSUPPORTED, "B*Hq > 65535");
  // one head of Q / K / V / inv is addressed with 32-bit byte offsets inside the kernels
  if ((long long)d->L * d->d * 2 >= (1LL << 31)) return fail(TSA_ERR_UNSUPPORTED, "L (%d) too long: one head must stay below 2 GiB", d->L);
  out->B = d->B; out->Hq = d->Hq; out->Hkv = d->Hkv; out->L = d->L; out->d = d->d;
  out->last_q = d->last_q; out->pool_w = d->pool_w; out->group_mode = d->group_mode;
  out->force_first = d->force_first; out->force_last = d->force_last;
  out->block_list_per_head = d->block_list_per_head;
  out->scale = d->scale > 0.0f ? d->scale : 1.0f / std::sqrt((float)d->d);
  struct { const char* name; int64_t b, h, l; int heads; tsa::Strides* dst; } lay[3] = {
      {"q", d->q_stride_b, d->q_stride_h, d->q_stride_l, d->Hq, &out->q},
      {"kv", d->kv_stride_b, d->kv_stride_h, d->kv_stride_l, d->Hkv, &out->kv},
      {"o", d->o_stride_b, d->o_stride_h, d->o_stride_l, d->Hq, &out->o}};
  for (auto& t : lay) {
    if (t.b == 0 && t.h == 0 && t.l == 0) {
      *t.dst = tsa::Strides{(long long)t.heads * d->L * d->d, (long long)d->L * d->d, (long long)d->d};
      continue;
    }
    if (t.b < 0 || t.h < 0 || t.l < d->d || (t.b | t.h | t.l) % 8 != 0)
      return fail(TSA_ERR_ARG, "%s strides: multiples of 8 elements, stride_l >= d, none negative (or all three 0)", t.name);
    if ((d->Hq > 1 || d->Hkv > 1) && t.heads > 1 && t.h == 0) return fail(TSA_ERR_ARG, "%s_stride_h is 0", t.name);
    if (d->B > 1 && t.b == 0) return fail(TSA_ERR_ARG, "%s_stride_b is 0", t.name);
    // rows of one head are addressed with 32-bit byte offsets inside the kernels
    if ((long long)d->L * t.l >= (1LL << 30)) return fail(TSA_ERR_UNSUPPORTED, "%s: L * stride_l must stay below 2^30 elements", t.name);
    if (t.l >= (1LL << 23) || d->L >= (1 << 24)) return fail(TSA_ERR_UNSUPPORTED, "%s: stride_l must stay below 2^23 elements and L below 2^24", t.name);
    *t.dst = tsa::Strides{(long long)t.b, (long long)t.h, (long long)t.l};
  }
  return TSA_OK;
}

int check_k(const tsa::Dims& dm, int32_t k_keep) {
  if (k_keep < 1 || k_keep > dm.L) return fail(TSA_ERR_ARG, "k_keep (%d) must lie in [1, L=%d]", k_keep, dm.L);
  return TSA_OK;
}

// The always-kept tokens must fit into the set (selection only: the other steps ignore them).
int check_forced(const tsa::Dims& dm, int32_t k_keep) {
  if (dm.force_first + dm.force_last > k_keep)
    return fail(TSA_ERR_ARG, "force_first + force_last (%d) exceeds k_keep (%d): the forced tokens would not all be kept",
                dm.force_first + dm.force_last, k_keep);
  return TSA_OK;
}

int check_ptr(const void* p, const char* name, bool optional = false) {
  if (!p) return optional ? TSA_OK : fail(TSA_ERR_ARG, "%s is NULL", name);
  if (misaligned(p)) return fail(TSA_ERR_ARG, "%s is not 16-byte aligned", name);
  return TSA_OK;
}

int check_ws(const void* ws, size_t have, size_t need) {
  if (need == 0) return TSA_OK;
  if (!ws) return fail(TSA_ERR_WORKSPACE, "ws is NULL but %zu bytes are needed", need);
  if (((uintptr_t)ws & 255u) != 0) return fail(TSA_ERR_WORKSPACE, "ws is not 256-byte aligned");
  if (have < need) return fail(TSA_ERR_WORKSPACE, "workspace too small: %zu bytes given, %zu needed", have, need);
  return TSA_OK;
}

int hip_status(hipError_t e, const char* what) {
  if (e == hipSuccess) return TSA_OK;
  return fail(TSA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int check_block_list(const int32_t* bl, int32_t block_size, int32_t max_blocks) {
  if (!bl) return TSA_OK;
  if (block_size != 64 && block_size != 128 && block_size != 256)
    return fail(TSA_ERR_UNSUPPORTED, "block_size %d: 64, 128 and 256 are built", block_size);
  if (max_blocks < 1) return fail(TSA_ERR_ARG, "max_blocks_per_row must be >= 1 with a block list");
  if (((uintptr_t)bl & 3u) != 0) return fail(TSA_ERR_ARG, "block_list is not 4-byte aligned");
  return TSA_OK;
}

// Carving of the workspace used by tsa_forward (every piece 256-byte aligned).
struct ForwardWs {
  size_t scores, score_ws, select_ws, idx, inv, Vt, total;
  size_t budget_ws, k_dev, total_dynamic;    // tsa_forward_dynamic: the budget's scratch and the counts it writes
};

ForwardWs forward_layout(const tsa::Dims& dm, int32_t k) {
  ForwardWs w;
  const size_t BHq = (size_t)dm.B * dm.Hq, BHkv = (size_t)dm.B * dm.Hkv;
  const size_t Hs = dm.group_mode ? BHkv : BHq;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t at = off; off += align256(bytes); return at; };
  w.scores = take(BHq * dm.L * sizeof(float));
  w.score_ws = take(tsa::score_ws_bytes(dm));
  w.select_ws = take(tsa::select_ws_bytes(dm));
  w.idx = take(Hs * k * sizeof(int32_t));
  w.inv = take(Hs * dm.L * sizeof(int32_t));
  w.Vt = take(tsa::v_tiles_bytes(dm.B, dm.group_mode ? dm.Hkv : dm.Hq, k, dm.d));
  w.total = off > tsa::budget_ws_bytes(dm) ? off : tsa::budget_ws_bytes(dm);
  w.budget_ws = take(tsa::budget_ws_bytes(dm));
  w.k_dev = take((size_t)dm.B * sizeof(int32_t));
  w.total_dynamic = off;
  return w;
}

}  // namespace

extern "C" {

int tsa_version(void) { return 10; }

const char* tsa_last_error(void) { return g_err; }

int32_t tsa_keep_count(int32_t L, double tau) {
  if (L < 1 || !(tau >= 0.0) || !(tau <= 1.0)) return 0;
  const long long drop = (long long)std::floor(tau * (double)L);
  long long keep = (long long)L - drop;
  if (keep < 1) keep = 1;
  if (keep > L) keep = L;
  return (int32_t)keep;
}

size_t tsa_workspace_bytes(const tsa_desc* desc, int32_t k_keep) {
  tsa::Dims dm;
  if (check_desc(desc, &dm) != TSA_OK) return 0;
  if (check_k(dm, k_keep) != TSA_OK) return 0;
  return forward_layout(dm, k_keep).total;
}

int tsa_score(const tsa_desc* desc, const void* Q, const void* K, float* scores,
              void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(scores, "scores"))) return rc;
  if ((rc = check_ws(ws, ws_bytes, tsa::score_ws_bytes(dm)))) return rc;
  return hip_status(tsa::launch_score(dm, Q, K, scores, ws, (hipStream_t)stream), "tsa_score");
}

namespace {
int check_positions(const int32_t* qpos, int32_t n, int32_t L) {
  if (!qpos) return fail(TSA_ERR_ARG, "qpos is NULL");
  for (int32_t i = 0; i < n; ++i) {
    if (qpos[i] < 0 || qpos[i] >= L) return fail(TSA_ERR_ARG, "qpos[%d] = %d is outside [0, L)", i, qpos[i]);
    if (i > 0 && qpos[i] < qpos[i - 1]) return fail(TSA_ERR_ARG, "qpos must be ascending");
  }
  return TSA_OK;
}
}  // namespace

int tsa_score_queries(const tsa_desc* desc, const void* Qsel, const int32_t* qpos, int32_t n, const void* K,
                      float* scores, void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if (n < 1 || n > 128) return fail(TSA_ERR_ARG, "n (%d) must lie in [1, 128]", n);
  dm.last_q = n;                                         // the query set of this call replaces the recent-query window
  if ((rc = check_positions(qpos, n, dm.L))) return rc;
  if ((rc = check_ptr(Qsel, "Qsel")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(scores, "scores"))) return rc;
  if ((rc = check_ws(ws, ws_bytes, tsa::score_ws_bytes(dm)))) return rc;
  return hip_status(tsa::launch_score_queries(dm, Qsel, qpos, K, scores, ws, (hipStream_t)stream), "tsa_score_queries");
}

size_t tsa_score_queries_workspace_bytes(const tsa_desc* desc, int32_t n) {
  tsa::Dims dm;
  if (check_desc(desc, &dm) != TSA_OK) return 0;
  if (n < 1 || n > 128) return 0;
  dm.last_q = n;
  return tsa::score_ws_bytes(dm);
}

int tsa_gather_queries(const tsa_desc* desc, const void* Q, const int32_t* qpos, int32_t n, void* Qsel, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if (n < 1 || n > 128) return fail(TSA_ERR_ARG, "n (%d) must lie in [1, 128]", n);
  if ((rc = check_positions(qpos, n, dm.L))) return rc;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(Qsel, "Qsel"))) return rc;
  return hip_status(tsa::launch_gather_queries(dm, Q, qpos, n, Qsel, (hipStream_t)stream), "tsa_gather_queries");
}

size_t tsa_pool_queries_workspace_bytes(const tsa_desc* desc, int32_t n_pool) {
  tsa::Dims dm;
  if (check_desc(desc, &dm) != TSA_OK) return 0;
  if (n_pool < 1 || n_pool > 128 || n_pool > dm.L) return 0;
  return tsa::pool_queries_ws_bytes(dm, n_pool);
}

int tsa_pool_queries(const tsa_desc* desc, const void* Q, int32_t n_pool, void* Qsel, int32_t* qpos,
                     void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if (n_pool < 1 || n_pool > 128 || n_pool > dm.L) return fail(TSA_ERR_ARG, "n_pool (%d) must lie in [1, min(L, 128)]", n_pool);
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(Qsel, "Qsel"))) return rc;
  if ((rc = check_ws(ws, ws_bytes, tsa::pool_queries_ws_bytes(dm, n_pool)))) return rc;
  if (qpos)
    for (int32_t j = 0; j < n_pool; ++j) qpos[j] = (int32_t)((((long long)(j + 1)) * dm.L + n_pool - 1) / n_pool) - 1;
  return hip_status(tsa::launch_pool_queries(dm, Q, n_pool, Qsel, ws, (hipStream_t)stream), "tsa_pool_queries");
}

int tsa_coverage_budget(const tsa_desc* desc, const float* scores, double tau_cov, int32_t* k_keep,
                        void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if (!(tau_cov >= 0.0) || !(tau_cov <= 1.0)) return fail(TSA_ERR_ARG, "tau_cov must lie in [0, 1]");
  if ((rc = check_ptr(scores, "scores"))) return rc;
  if (!k_keep || ((uintptr_t)k_keep & 3u)) return fail(TSA_ERR_ARG, "k_keep is NULL or not 4-byte aligned");
  if ((rc = check_ws(ws, ws_bytes, tsa::budget_ws_bytes(dm)))) return rc;
  return hip_status(tsa::launch_budget(dm, scores, tau_cov, k_keep, ws, (hipStream_t)stream), "tsa_coverage_budget");
}

int tsa_select(const tsa_desc* desc, const float* scores, int32_t k_keep,
               int32_t* idx, int32_t* inv, void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep)) || (rc = check_forced(dm, k_keep))) return rc;
  if ((rc = check_ptr(scores, "scores")) || (rc = check_ptr(idx, "idx")) || (rc = check_ptr(inv, "inv", true))) return rc;
  if ((rc = check_ws(ws, ws_bytes, tsa::select_ws_bytes(dm)))) return rc;
  return hip_status(tsa::launch_select(dm, scores, k_keep, idx, inv, ws, (hipStream_t)stream), "tsa_select");
}

}  // extern "C"

// ---- tsa_select_static: selection whose scratch is a static device array of the library ----
namespace {

constexpr size_t kStaticScratchBytes = TSA_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

// Histograms, thresholds and per-slice counts of the selection kernels (what tsa_select takes through
// `ws`).  One copy per GPU the library runs on, resident until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress: kernels and copies get the address looked up below.
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device, looked up once per device.
int static_scratch(void** out) {
  int dev = 0, rc;
  if ((rc = hip_status(hipGetDevice(&dev), "hipGetDevice"))) return rc;
  if (dev < 0 || dev >= kMaxDevices) return fail(TSA_ERR_UNSUPPORTED, "device ordinal %d: at most %d devices", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if ((rc = hip_status(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)"))) return rc;
    if (!p) return fail(TSA_ERR_HIP, "hipGetSymbolAddress(scratch) returned NULL");
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TSA_OK;
}

}  // namespace

extern "C" {

size_t tsa_select_static_capacity(void) { return kStaticScratchBytes; }

int tsa_select_static(const tsa_desc* desc, const float* scores, int32_t k_keep,
                      int32_t* idx, int32_t* inv, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep)) || (rc = check_forced(dm, k_keep))) return rc;
  if ((rc = check_ptr(scores, "scores")) || (rc = check_ptr(idx, "idx")) || (rc = check_ptr(inv, "inv", true))) return rc;
  const size_t need = tsa::select_ws_bytes(dm);
  if (need > kStaticScratchBytes)
    return fail(TSA_ERR_UNSUPPORTED, "tsa_select_static: this problem needs %zu bytes of scratch, the static buffer holds %zu "
                "(use tsa_select with a workspace)", need, kStaticScratchBytes);
  void* ws = nullptr;
  if ((rc = static_scratch(&ws))) return rc;
  // the kernels clear the part of the scratch that has to start at zero themselves
  return hip_status(tsa::launch_select(dm, scores, k_keep, idx, inv, ws, (hipStream_t)stream), "tsa_select_static");
}

int tsa_compress(const tsa_desc* desc, const void* Q, const void* K, const void* V,
                 const int32_t* idx, int32_t k_keep, void* Qc, void* Kc, void* Vc, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep))) return rc;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(V, "V")) || (rc = check_ptr(idx, "idx")) ||
      (rc = check_ptr(Qc, "Qc")) || (rc = check_ptr(Kc, "Kc")) || (rc = check_ptr(Vc, "Vc")))
    return rc;
  return hip_status(tsa::launch_compress(dm, Q, K, V, idx, k_keep, Qc, Kc, Vc, (hipStream_t)stream), "tsa_compress");
}

size_t tsa_attend_workspace_bytes(const tsa_desc* desc, int32_t Lc, int32_t kv_heads) {
  tsa::Dims dm;
  if (check_desc(desc, &dm) != TSA_OK) return 0;
  if (Lc < 1 || kv_heads < 1 || dm.Hq % kv_heads != 0) return 0;
  return align256(tsa::v_tiles_bytes(dm.B, kv_heads, Lc, dm.d));
}

int tsa_attend(const tsa_desc* desc, const void* Qc, const void* Kc, const void* Vc,
               int32_t Lc, int32_t kv_heads,
               const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
               void* Oc, float* lse, void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm))) return rc;
  if (Lc < 1) return fail(TSA_ERR_ARG, "Lc (%d) must be >= 1", Lc);
  if ((long long)Lc * dm.d * 2 >= (1LL << 31)) return fail(TSA_ERR_UNSUPPORTED, "Lc (%d) too long: one head must stay below 2 GiB", Lc);
  if (kv_heads < 1 || dm.Hq % kv_heads != 0) return fail(TSA_ERR_ARG, "kv_heads (%d) must divide Hq (%d)", kv_heads, dm.Hq);
  if ((rc = check_ptr(Qc, "Qc")) || (rc = check_ptr(Kc, "Kc")) || (rc = check_ptr(Vc, "Vc")) || (rc = check_ptr(Oc, "Oc")))
    return rc;
  if (lse && ((uintptr_t)lse & 3u)) return fail(TSA_ERR_ARG, "lse is not 4-byte aligned");
  if ((rc = check_block_list(block_list, block_size, max_blocks_per_row))) return rc;
  if ((long long)dm.B * dm.Hq * ((Lc + 127) / 128 + 7) > 0x7fffffffLL)      // upper bound of the launch's workgroups
    return fail(TSA_ERR_UNSUPPORTED, "grid too large");
  if ((rc = check_ws(ws, ws_bytes, tsa::v_tiles_bytes(dm.B, kv_heads, Lc, dm.d)))) return rc;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = hip_status(tsa::launch_v_tiles(dm.B, kv_heads, Lc, dm.d, Vc, ws, st), "tsa_attend(V tiles)"))) return rc;
  return hip_status(tsa::launch_attend(dm.B, dm.Hq, kv_heads, Lc, dm.d, dm.scale, Qc, Kc, ws, block_list,
                                       block_size, max_blocks_per_row, dm.block_list_per_head, Oc, lse, st), "tsa_attend");
}

int tsa_decompress(const tsa_desc* desc, const void* Oc, const int32_t* idx, const int32_t* inv,
                   int32_t k_keep, void* O, void* residual, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep))) return rc;
  if ((rc = check_ptr(Oc, "Oc"))) return rc;
  if (!O && !residual) return fail(TSA_ERR_ARG, "both O and residual are NULL");
  if ((rc = check_ptr(O, "O", true)) || (rc = check_ptr(residual, "residual", true))) return rc;
  if (O && (rc = check_ptr(inv, "inv"))) return rc;
  if (residual && (rc = check_ptr(idx, "idx"))) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (O && (rc = hip_status(tsa::launch_decompress(dm, Oc, idx, inv, k_keep, O, st), "tsa_decompress"))) return rc;
  if (residual && (rc = hip_status(tsa::launch_residual(dm, Oc, idx, k_keep, residual, st), "tsa_decompress(residual)"))) return rc;
  return TSA_OK;
}

int tsa_compress_v_tiles(const tsa_desc* desc, const void* V, const int32_t* idx, int32_t k_keep,
                         void* Vt, size_t vt_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep))) return rc;
  if ((rc = check_ptr(V, "V")) || (rc = check_ptr(idx, "idx"))) return rc;
  if ((rc = check_ws(Vt, vt_bytes, tsa::v_tiles_bytes(dm.B, dm.group_mode ? dm.Hkv : dm.Hq, k_keep, dm.d)))) return rc;
  return hip_status(tsa::launch_compress_tiled(dm, nullptr, nullptr, V, idx, k_keep, nullptr, nullptr, Vt, (hipStream_t)stream),
                    "tsa_compress_v_tiles");
}

int tsa_attend_fused(const tsa_desc* desc, const void* Q, const void* K, const void* Vt,
                     const int32_t* idx, const int32_t* inv, int32_t k_keep,
                     const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                     void* O, void* Oc, void* residual, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep))) return rc;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(Vt, "Vt")) || (rc = check_ptr(idx, "idx"))) return rc;
  if (!O && !Oc && !residual) return fail(TSA_ERR_ARG, "O, Oc and residual are all NULL");
  if ((rc = check_ptr(O, "O", true)) || (rc = check_ptr(Oc, "Oc", true)) || (rc = check_ptr(residual, "residual", true))) return rc;
  if (O && (rc = check_ptr(inv, "inv"))) return rc;
  if ((rc = check_block_list(block_list, block_size, max_blocks_per_row))) return rc;
  return hip_status(tsa::launch_attend_fused(dm, Q, K, Vt, idx, inv, k_keep, block_list, block_size, max_blocks_per_row,
                                             Oc, O, residual, (hipStream_t)stream), "tsa_attend_fused");
}

int tsa_forward(const tsa_desc* desc, const void* Q, const void* K, const void* V, int32_t k_keep,
                const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                void* O, void* residual, int32_t* idx_out,
                void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_keep)) || (rc = check_forced(dm, k_keep))) return rc;
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(V, "V"))) return rc;
  if (!O && !residual) return fail(TSA_ERR_ARG, "both O and residual are NULL");
  if ((rc = check_ptr(O, "O", true)) || (rc = check_ptr(residual, "residual", true)) || (rc = check_ptr(idx_out, "idx_out", true)))
    return rc;
  if ((rc = check_block_list(block_list, block_size, max_blocks_per_row))) return rc;
  const ForwardWs w = forward_layout(dm, k_keep);
  if ((rc = check_ws(ws, ws_bytes, w.total))) return rc;
  char* base = (char*)ws;
  float* scores = (float*)(base + w.scores);
  int32_t* idx = (int32_t*)(base + w.idx);
  int32_t* inv = (int32_t*)(base + w.inv);
  void* Vt = base + w.Vt;
  hipStream_t st = (hipStream_t)stream;
  if ((rc = hip_status(tsa::launch_score(dm, Q, K, scores, base + w.score_ws, st), "tsa_forward(score)"))) return rc;
  if ((rc = hip_status(tsa::launch_select(dm, scores, k_keep, idx, inv, base + w.select_ws, st), "tsa_forward(select)"))) return rc;
  // Compression and decompression are folded into the attention kernel: it gathers Q and K rows
  // through idx in its loads, writes the rows of O in its epilogue and clears the other rows; only
  // V is gathered beforehand (into the transposed tiles the kernel's operands want).  The compacted
  // output is materialised only for the residual update.
  if ((rc = hip_status(tsa::launch_compress_tiled(dm, Q, K, V, idx, k_keep, nullptr, nullptr, Vt, st), "tsa_forward(V tiles)"))) return rc;
  if ((rc = hip_status(tsa::launch_attend_fused(dm, Q, K, Vt, idx, inv, k_keep, block_list, block_size,
                                                max_blocks_per_row, nullptr, O, residual, st), "tsa_forward(attend)"))) return rc;
  if (idx_out) {
    const size_t Hs = (size_t)dm.B * (dm.group_mode ? dm.Hkv : dm.Hq);
    if ((rc = hip_status(hipMemcpyAsync(idx_out, idx, Hs * k_keep * sizeof(int32_t), hipMemcpyDeviceToDevice, st),
                         "tsa_forward(idx copy)"))) return rc;
  }
  return TSA_OK;
}

size_t tsa_forward_dynamic_workspace_bytes(const tsa_desc* desc, int32_t k_max) {
  tsa::Dims dm;
  if (check_desc(desc, &dm) || check_k(dm, k_max)) return 0;
  return forward_layout(dm, k_max).total_dynamic;
}

int tsa_forward_dynamic(const tsa_desc* desc, const void* Q, const void* K, const void* V, double tau_cov, int32_t k_max,
                        const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                        void* O, void* residual, int32_t* k_keep_out, int32_t* idx_out,
                        void* ws, size_t ws_bytes, void* stream) {
  tsa::Dims dm;
  int rc;
  if ((rc = check_desc(desc, &dm)) || (rc = check_k(dm, k_max)) || (rc = check_forced(dm, k_max))) return rc;
  if (!(tau_cov >= 0.0) || !(tau_cov <= 1.0)) return fail(TSA_ERR_ARG, "tau_cov must lie in [0, 1]");
  if ((rc = check_ptr(Q, "Q")) || (rc = check_ptr(K, "K")) || (rc = check_ptr(V, "V"))) return rc;
  if (!O && !residual) return fail(TSA_ERR_ARG, "both O and residual are NULL");
  if ((rc = check_ptr(O, "O", true)) || (rc = check_ptr(residual, "residual", true)) || (rc = check_ptr(idx_out, "idx_out", true)))
    return rc;
  if (k_keep_out && ((uintptr_t)k_keep_out & 3)) return fail(TSA_ERR_ARG, "k_keep_out is not 4-byte aligned");
  if ((rc = check_block_list(block_list, block_size, max_blocks_per_row))) return rc;
  const ForwardWs w = forward_layout(dm, k_max);
  if ((rc = check_ws(ws, ws_bytes, w.total_dynamic))) return rc;
  char* base = (char*)ws;
  float* scores = (float*)(base + w.scores);
  int32_t* idx = (int32_t*)(base + w.idx);
  int32_t* inv = (int32_t*)(base + w.inv);
  int32_t* k_dev = (int32_t*)(base + w.k_dev);
  void* Vt = base + w.Vt;
  hipStream_t st = (hipStream_t)stream;
  // Algorithm 1 in its own order: scores, budget from the cross-head mass, selection with that budget;
  // every later launch is sized for k_max and reads the count of its batch entry from k_dev.
  if ((rc = hip_status(tsa::launch_score(dm, Q, K, scores, base + w.score_ws, st), "tsa_forward_dynamic(score)"))) return rc;
  if ((rc = hip_status(tsa::launch_budget(dm, scores, tau_cov, k_dev, base + w.budget_ws, st, k_max, dm.force_first + dm.force_last),
                       "tsa_forward_dynamic(budget)"))) return rc;
  if ((rc = hip_status(tsa::launch_select(dm, scores, k_max, idx, inv, base + w.select_ws, st, k_dev), "tsa_forward_dynamic(select)"))) return rc;
  if ((rc = hip_status(tsa::launch_compress_tiled(dm, Q, K, V, idx, k_max, nullptr, nullptr, Vt, st, k_dev), "tsa_forward_dynamic(V tiles)"))) return rc;
  if ((rc = hip_status(tsa::launch_attend_fused(dm, Q, K, Vt, idx, inv, k_max, block_list, block_size, max_blocks_per_row,
                                                nullptr, O, residual, st, k_dev),
                       "tsa_forward_dynamic(attend)"))) return rc;
  if (k_keep_out && (rc = hip_status(hipMemcpyAsync(k_keep_out, k_dev, (size_t)dm.B * sizeof(int32_t), hipMemcpyDeviceToDevice, st),
                                     "tsa_forward_dynamic(count copy)"))) return rc;
  if (idx_out) {
    const size_t Hs = (size_t)dm.B * (dm.group_mode ? dm.Hkv : dm.Hq);
    if ((rc = hip_status(hipMemcpyAsync(idx_out, idx, Hs * k_max * sizeof(int32_t), hipMemcpyDeviceToDevice, st),
                         "tsa_forward_dynamic(idx copy)"))) return rc;
  }
  return TSA_OK;
}

size_t tsa_layer_drift_workspace_bytes(int64_t n_tokens) {
  if (n_tokens < 1) return 0;
  return tsa::drift_ws_bytes(n_tokens);
}

int tsa_layer_drift(const void* h_in, const void* h_out, int64_t n_tokens, int32_t width, float eps,
                    float* drift_out, void* ws, size_t ws_bytes, void* stream) {
  int rc;
  if (n_tokens < 1 || n_tokens > ((int64_t)1 << 31) * 64) return fail(TSA_ERR_ARG, "n_tokens out of range");
  if (width < 8 || width % 8 != 0) return fail(TSA_ERR_ARG, "width (%d) must be a positive multiple of 8", width);
  if (!(eps >= 0.0f) || !std::isfinite(eps)) return fail(TSA_ERR_ARG, "eps must be finite and >= 0");
  if ((rc = check_ptr(h_in, "h_in")) || (rc = check_ptr(h_out, "h_out"))) return rc;
  if (!drift_out || ((uintptr_t)drift_out & 3u)) return fail(TSA_ERR_ARG, "drift_out is NULL or not 4-byte aligned");
  if ((rc = check_ws(ws, ws_bytes, tsa::drift_ws_bytes(n_tokens)))) return rc;
  return hip_status(tsa::launch_drift(h_in, h_out, n_tokens, width, eps, drift_out, ws, (hipStream_t)stream), "tsa_layer_drift");
}

int tsa_sparse_layers(const float* drift, int32_t n_layers, double delta, int32_t* is_sparse) {
  if (!drift || !is_sparse) return fail(TSA_ERR_ARG, "drift or is_sparse is NULL");
  if (n_layers < 1) return fail(TSA_ERR_ARG, "n_layers must be >= 1");
  for (int32_t l = 0; l < n_layers; ++l) {
    int32_t not_above = 0;
    for (int32_t k = 0; k < n_layers; ++k) not_above += drift[k] <= drift[l] ? 1 : 0;
    is_sparse[l] = (double)not_above / (double)n_layers <= delta ? 1 : 0;
  }
  return TSA_OK;
}

int tsa_mfma_probe(const void* operands, int32_t iters, int32_t blocks, float* sink, int64_t* clocks,
                   double* flops, int32_t* wall_clock_khz, void* stream) {
  int rc;
  if ((rc = check_ptr(operands, "operands")) || (rc = check_ptr(sink, "sink")) || (rc = check_ptr(clocks, "clocks"))) return rc;
  if (iters < 1 || iters > (1 << 24) || blocks < 1 || blocks > 65536) return fail(TSA_ERR_ARG, "iters or blocks out of range");
  if (flops) *flops = (double)blocks * 4.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  if (wall_clock_khz) {
    int dev = 0, khz = 0;
    if ((rc = hip_status(hipGetDevice(&dev), "hipGetDevice"))) return rc;
    if ((rc = hip_status(hipDeviceGetAttribute(&khz, hipDeviceAttributeWallClockRate, dev), "wall clock rate"))) return rc;
    *wall_clock_khz = khz;
  }
  return hip_status(tsa::launch_mfma_probe(operands, iters, blocks, sink, (long long*)clocks, (hipStream_t)stream), "tsa_mfma_probe");
}

int tsa_mix_probe(int32_t mix, const void* operands, int32_t iters, int32_t blocks, float* sink, double* flops, void* stream) {
  int rc;
  if ((rc = check_ptr(operands, "operands")) || (rc = check_ptr(sink, "sink"))) return rc;
  if (mix < 0 || mix > 3) return fail(TSA_ERR_ARG, "mix must be 0..3");
  if (iters < 1 || iters > (1 << 24) || blocks < 1 || blocks > 65536) return fail(TSA_ERR_ARG, "iters or blocks out of range");
  if (flops) *flops = (double)blocks * 4.0 * (double)iters * (mix <= 1 ? 16.0 : 8.0) * (2.0 * 32 * 32 * 16);
  return hip_status(tsa::launch_mix_probe(mix, operands, iters, blocks, sink, (hipStream_t)stream), "tsa_mix_probe");
}

int tsa_read_probe(const void* src, size_t bytes, void* sink, void* stream) {
  int rc;
  if ((rc = check_ptr(src, "src"))) return rc;
  if (!sink) return fail(TSA_ERR_ARG, "sink is NULL");
  if (bytes % 16 != 0) return fail(TSA_ERR_ARG, "bytes must be a multiple of 16");
  return hip_status(tsa::launch_read_probe(src, bytes, sink, (hipStream_t)stream), "tsa_read_probe");
}

int tsa_bench_set_attend_form(int32_t form) {
  if (form < 0 || form > 2) return fail(TSA_ERR_ARG, "form must be 0, 1 or 2");
  tsa::set_attend_form(form);
  return TSA_OK;
}

int tsa_copy_probe(const void* src, void* dst, size_t bytes, void* stream) {
  int rc;
  if ((rc = check_ptr(src, "src")) || (rc = check_ptr(dst, "dst"))) return rc;
  if (bytes % 16 != 0) return fail(TSA_ERR_ARG, "bytes must be a multiple of 16");
  return hip_status(tsa::launch_copy_probe(src, dst, bytes, (hipStream_t)stream), "tsa_copy_probe");
}

}  // extern "C"
