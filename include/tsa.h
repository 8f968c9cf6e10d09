/*
 * libtsa -- Token Sparse Attention prefill hot path for AMD MI355X (gfx950).
 *
 * C ABI.  Every tensor argument is a DEVICE pointer owned by the caller, 16-byte
 * aligned, contiguous row-major in the stated shape (the full-length tensors Q, K,
 * V and O may instead follow the strides of the descriptor, wherever an entry point
 * takes them in full length); bf16 tensors are passed as
 * `const void*` / `void*` (2 bytes per element).  The library never allocates or
 * frees device memory: scratch space comes in through the `ws` argument (256-byte
 * aligned), sized with tsa_workspace_bytes() or the entry point's own size query.
 * All work is queued asynchronously on `stream` (a hipStream_t passed as void*,
 * NULL = the default stream); no call synchronises with the host, and buffers
 * must stay valid until the stream has finished the work.
 *
 * Every entry point returns a status code.  Arguments are validated on the
 * host before anything is launched; on error nothing has been queued and
 * tsa_last_error() (thread-local) describes the problem.  Inputs must be
 * finite; behaviour for NaN / Inf inputs is undefined.
 *
 * Notation follows the paper: B batch, Hq query heads, Hkv key/value heads
 * (g = Hq / Hkv query heads share a KV head: query head h reads KV head h / g),
 * L tokens, d head dimension, S_h the per-head index set, k_keep = |S_h| = L'.
 */
#ifndef TSA_H
#define TSA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  TSA_OK = 0,
  TSA_ERR_ARG = 1,          /* null / misaligned pointer, size out of range */
  TSA_ERR_UNSUPPORTED = 2,  /* valid request this build has no kernel for */
  TSA_ERR_WORKSPACE = 3,    /* ws == NULL or ws_bytes too small */
  TSA_ERR_HIP = 4           /* a HIP launch or query failed */
};

/* Problem statement of one attention layer (Section 2.2 of the paper: per-head
 * Q, K, V of L tokens) plus the parameters of Algorithm 1 the paper leaves open. */
typedef struct tsa_desc {
  int32_t B;            /* batch, >= 1 */
  int32_t Hq;           /* query heads */
  int32_t Hkv;          /* key/value heads, Hq % Hkv == 0 */
  int32_t L;            /* tokens, >= 1 */
  int32_t d;            /* head dimension: 64 or 128 */
  int32_t last_q;       /* number of most recent queries used for scoring (Algorithm 1), 1..min(L,128) */
  int32_t pool_w;       /* width of Algorithm 1's pooling(.) on s_h: odd, 1 = none; average pooling, stride 1,
                           zero padding (the paper does not give the kernel) */
  int32_t group_mode;   /* 0: every query head selects its own S_h; 1: the g heads of a KV group share
                           one set chosen from the sum of their scores */
  int32_t force_first;  /* tokens t < force_first are always kept (score treated as +inf); default 0 */
  int32_t force_last;   /* tokens t >= L - force_last are always kept; default 0.  Selection needs
                           force_first + force_last <= k_keep (TSA_ERR_ARG otherwise); with a count decided
                           on the device the count is raised to force_first + force_last where the budget
                           asks for fewer */
  float   scale;        /* softmax scale; 0 means 1/sqrt(d) */
  int32_t block_list_per_head; /* 0: one block list shared by all heads; 1: one list per (b, h),
                                  block_list is [B,Hq,ceil(Lc/block_size),max_blocks_per_row] (block-sparse
                                  methods pick a different pattern for every head) */
  /* Layout of the full-length tensors Q [B,Hq,L,d], K and V [B,Hkv,L,d] (one layout for both) and
   * O [B,Hq,L,d], in elements: element (b, h, t, c) sits at b * stride_b + h * stride_h + t * stride_l + c.
   * All three strides of a tensor zero (the default) means contiguous [B,H,L,d]; a [B,L,H,d] tensor (the
   * layout a fused QKV projection leaves behind) is stride_b = L*H*d, stride_h = d, stride_l = H*d.
   * Every stride must be a multiple of 8 (rows stay 16-byte aligned), stride_l >= d, and L * stride_l
   * below 2^30 elements.  Compacted tensors, scores, index sets, workspaces and the residual stream are
   * always contiguous in the shapes stated at their entry points. */
  int64_t q_stride_b, q_stride_h, q_stride_l;
  int64_t kv_stride_b, kv_stride_h, kv_stride_l;
  int64_t o_stride_b, o_stride_h, o_stride_l;
} tsa_desc;

/* Version of this ABI (increases when a signature changes). */
int tsa_version(void);

/* Text of the last error on the calling thread ("" if none).  Host pointer, owned by the library. */
const char* tsa_last_error(void);

/* Fixed token-sparsity ratio (the "fixed sparsity" policy the paper compares against in
 * its dynamic-vs-fixed table): drop floor(tau * L) tokens.  Returns k_keep = L - floor(tau*L)
 * clamped to [1, L]; returns 0 if L < 1 or tau is outside [0, 1]. */
int32_t tsa_keep_count(int32_t L, double tau);

/* Bytes of workspace that tsa_score, tsa_coverage_budget, tsa_select and tsa_forward need for this
 * problem and k_keep (tsa_forward needs the most: scores, index sets and the gathered V; it also
 * covers the workspace of tsa_attend on the compacted tensors).
 * Returns 0 if the descriptor or k_keep is invalid. */
size_t tsa_workspace_bytes(const tsa_desc* desc, int32_t k_keep);

/* Token scoring -- Algorithm 1, first two steps: A = softmax(Q[-last_q:] K^T * scale) with
 * query i seeing keys t <= i, then the column sums s[b,h,t] = sum_i A[i,t].
 *   Q      [B,Hq,L,d]  bf16, device (only the last last_q rows of each head are read)
 *   K      [B,Hkv,L,d] bf16, device
 *   scores [B,Hq,L]    fp32, device, fully overwritten
 * With pool_w > 1 the column sums are then average-pooled along t (width pool_w, zero padding).
 * Arithmetic: bf16 products accumulated in fp32 (MFMA), exact two-pass softmax in fp32. */
int tsa_score(const tsa_desc* desc, const void* Q, const void* K, float* scores,
              void* ws, size_t ws_bytes, void* stream);

/* Scoring from other query sets -- the paper's scoring ablation (appendix, "Token Scoring Methods":
 * randomly selected queries, or a pooled query tensor, in place of the most recent queries).
 *
 * tsa_score_queries: as tsa_score, but the scoring queries are the rows of Qsel [B,Hq,n,d] bf16 (device),
 *   query j sitting at position qpos[j]: s[b,h,t] = sum_j softmax_t(scale Qsel[b,h,j].k_t) over keys
 *   t <= qpos[j].  qpos: HOST array of n ints in [0, L), ascending (it travels in the kernel
 *   arguments); 1 <= n <= 128 (desc->last_q is not used);  ws: tsa_score_queries_workspace_bytes(desc, n)
 *   bytes.  tsa_score is the case Qsel = Q[:, :, L-n:], qpos = L-n .. L-1.
 * tsa_gather_queries: Qsel[b,h,j,:] = Q[b,h,qpos[j],:] -- the rows of randomly selected queries; the
 *   caller draws the positions (seeded, sorted) and passes them in, 1 <= n <= 128.
 * tsa_pool_queries: query-only pooling: the L rows of every head are cut into n_pool contiguous
 *   segments (rows floor(j L / n_pool) .. ceil((j+1) L / n_pool) - 1) and averaged (fp32 sums in a
 *   fixed order, one rounding to bf16): Qsel [B,Hq,n_pool,d] out; qpos (HOST, out, may be NULL)
 *   receives the last row of each segment, the position a pooled query scores from.  The paper
 *   does not give the pooling window or the causal treatment: n_pool = 1 is a single mean query
 *   that sees every key. */
size_t tsa_score_queries_workspace_bytes(const tsa_desc* desc, int32_t n);
int tsa_score_queries(const tsa_desc* desc, const void* Qsel, const int32_t* qpos, int32_t n, const void* K,
                      float* scores, void* ws, size_t ws_bytes, void* stream);
int tsa_gather_queries(const tsa_desc* desc, const void* Q, const int32_t* qpos, int32_t n, void* Qsel, void* stream);
size_t tsa_pool_queries_workspace_bytes(const tsa_desc* desc, int32_t n_pool);
int tsa_pool_queries(const tsa_desc* desc, const void* Q, int32_t n_pool, void* Qsel, int32_t* qpos,
                     void* ws, size_t ws_bytes, void* stream);

/* Dynamic Token Coverage budget -- Algorithm 1, its budget steps (Section 2.3): cross-head sum of the
 * token scores, normalisation, ascending order, cumulative-mass threshold:
 * s_l[t] = sum_h scores[b,h,t] (fp32, head order), normalised by its total over t; k_sparse is the
 * smallest k in {0..L} such that the k least important tokens carry a cumulative mass >= tau_cov;
 * k_keep[b] = L - k_sparse, at least 1.  The result stays on the device; a caller that sizes buffers
 * with it reads it back after synchronising the stream, then calls tsa_select with it.
 * The masses are accumulated exactly (integer sums of significands), so the count does not depend on
 * the order in which the hardware adds them: repeated calls give the same count.
 *   scores [B,Hq,L] fp32, device;  k_keep [B] int32, device, out;  tau_cov in [0, 1]
 *   ws: at least tsa_workspace_bytes() bytes (uses a part of it) */
int tsa_coverage_budget(const tsa_desc* desc, const float* scores, double tau_cov, int32_t* k_keep,
                        void* ws, size_t ws_bytes, void* stream);

/* Top-k selection -- Algorithm 1, last step, S_h = TopK(s_h, k_keep): for every (b, hs)
 * the k_keep tokens of largest score, ties to the lowest token index, written in ascending
 * token order.  hs runs over Hs = Hq heads (group_mode 0) or Hs = Hkv groups (group_mode 1,
 * where the g heads' scores are summed first, in head order, in fp32).
 *   scores [B,Hq,L]  fp32, device
 *   idx    [B,Hs,k_keep] int32, device, out: S_h ascending
 *   inv    [B,Hs,L]  int32, device, out (may be NULL): inv[t] = r if idx[r] == t, else -1 */
int tsa_select(const tsa_desc* desc, const float* scores, int32_t k_keep,
               int32_t* idx, int32_t* inv, void* ws, size_t ws_bytes, void* stream);

/* tsa_select for callers that cannot allocate device memory or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments and same results as
 * tsa_select, but the histograms, thresholds and per-slice counts live in a static device array of the
 * library, tsa_select_static_capacity() bytes (8 MiB) per GPU the library runs on, held until the process
 * ends.  Allocates nothing.  A problem whose scratch does not fit (group_mode 1 keeps B*Hkv*L fp32 sums
 * there) is rejected with TSA_ERR_UNSUPPORTED.  All calls on one GPU share the array: calls that
 * overlap on one GPU (different streams, or different threads) race; the array keeps the last call's
 * contents and every call clears what it needs at zero itself. */
size_t tsa_select_static_capacity(void);
int tsa_select_static(const tsa_desc* desc, const float* scores, int32_t k_keep,
                      int32_t* idx, int32_t* inv, void* stream);

/* Stage 1, compression: gather the rows S_h of Q, K, V into dense contiguous tensors.
 *   idx [B,Hs,k_keep] int32 (from tsa_select)
 *   Qc  [B,Hq,k_keep,d] out.  group_mode 0: Kc, Vc [B,Hq,k_keep,d] (row idx[b,h,r] of KV head h/g);
 *                             group_mode 1: Kc, Vc [B,Hkv,k_keep,d].
 * Bit-exact row copies.  Index values must lie in [0, L). */
int tsa_compress(const tsa_desc* desc, const void* Q, const void* K, const void* V,
                 const int32_t* idx, int32_t k_keep, void* Qc, void* Kc, void* Vc, void* stream);

/* Attention in the compressed space (Stage 1, last step; cost O(L'^2 d)): causal softmax
 * attention over Lc rows, row r attending to columns c <= r.  Because S_h is ascending this
 * is causal in the original positions, i.e. the hard mask of Stage 2.
 *   Qc [B,Hq,Lc,d] bf16;  Kc, Vc [B,kv_heads,Lc,d] bf16 with Hq % kv_heads == 0
 *   Oc [B,Hq,Lc,d] bf16 out;  lse [B,Hq,Lc] fp32 out or NULL (natural-log sum-exp of the scaled logits)
 *   block_list: NULL for plain causal attention.  Otherwise [ceil(Lc/block_size), max_blocks_per_row]
 *   int32 on the device, shared by all heads (or one such table per (b, h), see
 *   tsa_desc.block_list_per_head): row qb lists, in ascending order and padded with -1,
 *   the key blocks that query block qb may see (composition with a block-sparse pattern in
 *   compacted index space, Section 1 / Appendix "other sparse attention methods").  Entries > qb
 *   are ignored; the diagonal block is causal inside.  block_size: 64, 128 or 256.
 * The dense baseline is this same call with Qc=Q, Kc=K, Vc=V, Lc=L, kv_heads=Hkv.
 *   ws: tsa_attend_workspace_bytes(desc, Lc, kv_heads) bytes (only B, Hq, d of desc are used): the
 *   call first rewrites Vc into 64-key transposed tiles there, the layout the kernel's matrix
 *   operands want; Vc itself is not modified.
 * Arithmetic: bf16 MFMA with fp32 accumulation, online softmax in fp32, probabilities rounded
 * to bf16 before the PV product, output rounded to bf16 (nearest even); the products are scaled in
 * fp32. */
size_t tsa_attend_workspace_bytes(const tsa_desc* desc, int32_t Lc, int32_t kv_heads);
int tsa_attend(const tsa_desc* desc, const void* Qc, const void* Kc, const void* Vc,
               int32_t Lc, int32_t kv_heads,
               const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
               void* Oc, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Stage 2, decompression: scatter the compressed output back to the full sequence.
 *   Oc  [B,Hq,k_keep,d] bf16;  idx [B,Hs,k_keep];  inv [B,Hs,L] (both from tsa_select)
 *   O   [B,Hq,L,d] bf16 out or NULL: O[b,h,t,:] = Oc[b,h,inv[t],:] if inv[t] >= 0 else 0; every
 *       element is written, the caller need not clear it.
 *   residual [B,L,Hq*d] bf16 in/out or NULL: residual[b,t,h*d:(h+1)*d] += Oc[b,h,r,:] for
 *       t = idx[r] (fp32 add, one rounding to bf16); rows of unselected tokens are untouched.  This is
 *       the residual connection of Stage 2 with the identity in place of the output projection.
 * At least one of O, residual must be non-NULL.  inv is required for O, idx for residual; idx may be
 * NULL when only O is wanted (with both given, the copies can be driven by idx and the zero rows by
 * inv as two independent streams, which is the faster form at moderate sparsity); idx and inv must be
 * each other's inverse, as tsa_select writes them. */
int tsa_decompress(const tsa_desc* desc, const void* Oc, const int32_t* idx, const int32_t* inv,
                   int32_t k_keep, void* O, void* residual, void* stream);

/* Stage 1 + attention + Stage 2 in two launches, the form tsa_forward uses.  Same results as
 * tsa_compress -> tsa_attend -> tsa_decompress, but the compacted Q, K and O never exist in memory.
 *
 * tsa_compress_v_tiles: gathers the rows S_h of V into 64-key transposed tiles,
 *   Vt [B,Hs',ceil(k_keep/64),d,64] bf16 (Hs' = Hq, or Hkv with group_mode 1; keys past k_keep zero),
 *   vt_bytes >= tsa_attend_workspace_bytes(desc, k_keep, Hs'), Vt 256-byte aligned.
 * tsa_attend_fused: causal attention over the compacted set, reading row r of head h as
 *   Q[b,h,idx[r],:], K[b,h/g,idx[r],:] (original tensors) and the V tiles; writes
 *   O [B,Hq,L,d] (may be NULL): O[b,h,idx[r],:] = output row r, every other row zero (needs inv), and/or
 *   Oc [B,Hq,k_keep,d] (may be NULL): the compacted output, as tsa_attend would;
 *   residual [B,L,Hq*d] (may be NULL): as in tsa_decompress, residual[b,idx[r],h*d:(h+1)*d] += output row r
 *   (rounded to bf16 first, then added in fp32 and rounded once: bit-identical to tsa_decompress).
 *   At least one of the three must be given.  block_list as in tsa_attend.
 *   idx and inv must be what tsa_select wrote (ascending sets with values in [0, L), inv their
 *   inverse): the kernel addresses Q, K and O through them without further checks. */
int tsa_compress_v_tiles(const tsa_desc* desc, const void* V, const int32_t* idx, int32_t k_keep,
                         void* Vt, size_t vt_bytes, void* stream);
int tsa_attend_fused(const tsa_desc* desc, const void* Q, const void* K, const void* Vt,
                     const int32_t* idx, const int32_t* inv, int32_t k_keep,
                     const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                     void* O, void* Oc, void* residual, void* stream);

/* The whole layer on one stream, no host synchronisation:
 * score -> select -> compress -> attend -> decompress (Figure 3 of the paper).  Same results as the
 * five calls in a row; inside, the gather of Q and K rows happens in the attention kernel's loads
 * and the scatter (with the zero rows) in its epilogue, so the compacted Q, K, O never touch HBM.
 *   Q [B,Hq,L,d], K, V [B,Hkv,L,d] bf16;  O [B,Hq,L,d] bf16 out (or NULL when only residual is wanted)
 *   idx_out [B,Hs,k_keep] int32 out or NULL;  residual as in tsa_decompress or NULL
 *   block_list / block_size / max_blocks_per_row as in tsa_attend (NULL, 0, 0 for plain causal) */
int tsa_forward(const tsa_desc* desc, const void* Q, const void* K, const void* V, int32_t k_keep,
                const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                void* O, void* residual, int32_t* idx_out,
                void* ws, size_t ws_bytes, void* stream);

/* The layer with Dynamic Token Coverage (Section 2.3, Algorithm 1 in full) on one stream, no host
 * synchronisation: score -> coverage budget -> select -> compress -> attend -> decompress.  The number
 * of kept tokens is decided on the device, per batch entry, from the cross-head mass threshold
 * tau_cov (as tsa_coverage_budget), clamped to k_max; every launch is sized for k_max and reads the
 * count it works on from device memory, so the call can be recorded into a HIP graph.  The result
 * equals tsa_forward with k_keep = the count the budget found (batch entry by batch entry).
 *   k_max: capacity, 1..L (k_max = L never clamps; a smaller k_max keeps the k_max best tokens when the
 *          budget asks for more)
 *   O [B,Hq,L,d] bf16 out or NULL;  residual as in tsa_decompress or NULL
 *   k_keep_out [B] int32, device, out or NULL: the counts used
 *   idx_out [B,Hs,k_max] int32, device, out or NULL: row (b, h) holds k_keep_out[b] indices, the rest
 *          of the row is unspecified
 *   block_list / block_size / max_blocks_per_row as in tsa_attend, laid out for k_max compacted rows
 *          ([ceil(k_max/block_size), max_blocks_per_row], per (b, h) if the descriptor says so): a batch
 *          entry that keeps fewer rows uses the first ceil(k_keep/block_size) rows of its table, so
 *          the pattern must not depend on the total (sink + window and vertical + slash lists do not)
 *   ws: tsa_forward_dynamic_workspace_bytes(desc, k_max) bytes */
size_t tsa_forward_dynamic_workspace_bytes(const tsa_desc* desc, int32_t k_max);
int tsa_forward_dynamic(const tsa_desc* desc, const void* Q, const void* K, const void* V, double tau_cov, int32_t k_max,
                        const int32_t* block_list, int32_t block_size, int32_t max_blocks_per_row,
                        void* O, void* residual, int32_t* k_keep_out, int32_t* idx_out,
                        void* ws, size_t ws_bytes, void* stream);

/* Sparse layer selection (Section 2.4).  Offline preprocessing in the paper; here as kernels on
 * caller-supplied hidden states.
 *
 * tsa_layer_drift -- Eq. 1, Inter-Layer Representation Drift of one layer:
 *   R = mean_t ||h_out[t] - h_in[t]||_2 / (||h_in[t]||_2 + eps)
 *   h_in, h_out [n_tokens, width] bf16, device (the layer's input and output hidden states);
 *   width a multiple of 8;  drift_out: one fp32 on the device;  ws: tsa_layer_drift_workspace_bytes().
 *   fp32 sums of squares per token, fp64 mean; deterministic. */
size_t tsa_layer_drift_workspace_bytes(int64_t n_tokens);
int tsa_layer_drift(const void* h_in, const void* h_out, int64_t n_tokens, int32_t width, float eps,
                    float* drift_out, void* ws, size_t ws_bytes, void* stream);

/* tsa_sparse_layers -- Eq. 2, normalised drift rank and layer set, on the HOST:
 *   rank[l] = (1/n) * #{k : R_k <= R_l};  is_sparse[l] = rank[l] <= delta  (the paper uses delta = 0.5).
 *   drift [n_layers] fp32, host;  is_sparse [n_layers] int32, host, out (1 = apply Token Sparse Attention). */
int tsa_sparse_layers(const float* drift, int32_t n_layers, double delta, int32_t* is_sparse);

#ifdef __cplusplus
}
#endif
#endif /* TSA_H */
