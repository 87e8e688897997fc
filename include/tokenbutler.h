/*
 * tokenbutler.h -- C ABI of the MI355X (gfx950) implementation of TokenButler's decode-time
 * hot path: score every cached token with a low-dimensional importance query against the
 * projected key cache, keep a fixed top-k budget per query head (sink prefix and local window
 * always kept), optionally widen a reused selection with neighbours, and run decode attention
 * over the selected K/V rows only.
 *
 * Conventions shared by every entry point
 *  - All tensor pointers are DEVICE pointers owned by the caller.  The library never
 *    allocates, frees or keeps them.  Scratch memory comes in through `ws` (see
 *    tb_workspace_bytes / tb_workspace_init).
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Every call only
 *    enqueues work on that stream and returns; nothing synchronises.
 *  - Errors are return codes.  All argument checks happen on the host before anything is
 *    launched; a failing call launches nothing.
 *  - K, V, K_imp, W, q, q_imp share one element type (tb_dtype).  Scores, attention output
 *    and log-sum-exp are always fp32; index lists and counts are int32.
 *  - Query head h reads KV head h / (Hq / Hkv)  (consecutive query heads share a KV head).
 *  - Supported shapes: D in {64, 128}; Dimp in {16, 32, 64}; Hq / Hkv in {1, 2, 4, 8};
 *    N <= 2^20 for selection.  Row starts must be 16-byte aligned: base pointers 16-byte
 *    aligned and all strides multiples of 8 elements.  Anything else -> TB_ERR_UNSUPPORTED.
 */
#ifndef TOKENBUTLER_H_
#define TOKENBUTLER_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum tb_status {
  TB_OK = 0,
  TB_ERR_INVALID_ARG = 1, /* null pointer, negative size, inconsistent shape, capacity too small */
  TB_ERR_UNSUPPORTED = 2, /* well-formed but outside the supported shapes / alignments          */
  TB_ERR_WORKSPACE = 3,   /* ws is NULL or ws_bytes below tb_workspace_bytes()                  */
  TB_ERR_HIP = 4          /* a HIP launch reported an error                                     */
} tb_status;

typedef enum tb_dtype { TB_F32 = 0, TB_BF16 = 1 } tb_dtype;

/* One layer's cache view.  Plain data, read during the call only.
 * K, V   : [B][Hkv][>=N][D]     element (b,h,n,d) at  b*stride_b + h*stride_h + n*stride_n + d
 * K_imp  : [B][Hkv][>=N][Dimp]  same addressing with the ki_ strides
 * Strides are in elements; the innermost dimension is contiguous. */
typedef struct tb_cache_desc {
  int32_t B, Hq, Hkv, D, Dimp;
  int32_t dtype; /* tb_dtype */
  int64_t N;     /* tokens currently valid in the cache */
  int64_t k_stride_b, k_stride_h, k_stride_n;
  int64_t v_stride_b, v_stride_h, v_stride_n;
  int64_t ki_stride_b, ki_stride_h, ki_stride_n;
} tb_cache_desc;

/* Operation selector for tb_workspace_bytes. */
enum { TB_OP_SELECT = 1, TB_OP_ATTN = 2, TB_OP_DECODE_STEP = 3 };

/* Key-cache projection (Sec. 3.1, "Key-cache projection": K_imp = K W_K, W_K in R^{D x Dimp}).
 * Fills K_imp[b,h,n,:] = round(K[b,h,n,:] . W[hw]) for n_begin <= n < n_end, fp32 accumulation,
 * one round-to-nearest-even to the storage type.  Covers both the one-row append and the
 * batched deferred projection of a whole window of rows (Sec. 3.3).
 * W: [Hw][D][Dimp] contiguous; Hw == 1 (one matrix per layer, as the paper writes it) or
 * Hw == Hkv.  Requires 0 <= n_begin <= n_end <= desc->N.  Empty range: no-op, TB_OK. */
tb_status tb_project_keys(const tb_cache_desc* desc, const void* K, const void* W, int32_t Hw, void* Kimp,
                          int64_t n_begin, int64_t n_end, void* stream);

/* Importance scoring (abstract; Sec. 3.4, prediction steps).
 * scores[b,h,n] = scale * sum_j q_imp[b,h,j] * K_imp[b,h/g,n,j]   for 0 <= n < desc->N.
 * q_imp: [B][Hq][Dimp] contiguous.  scores: fp32 [B][Hq][score_stride], score_stride >= N and
 * a multiple of 4.  The paper gives no normalisation of the score; `scale` is explicit. */
tb_status tb_score(const tb_cache_desc* desc, const void* q_imp, const void* Kimp, float scale, float* scores,
                   int64_t score_stride, void* stream);

/* Token selection policy (Sec. 4 "Token Selection Policy").  Per (b,h): candidates are the
 * positions [lo, hi) with lo = min(sink, N), hi = max(lo, N - window); the kk = min(k, hi-lo)
 * candidates with the largest score are kept.  Ordering: larger score first, NaN counts as
 * -inf, -0 equals +0, equal scores -> lower index first.  Output per (b,h), ascending:
 *   idx = [0,lo) ++ ascending(kept) ++ [hi,N),   count = lo + kk + (N - hi).
 * idx: int32 [B][Hq][idx_cap], idx_cap >= lo + kk + (N - hi); entries beyond count are left
 * untouched.  count: int32 [B][Hq].  ws / ws_bytes are optional (NULL / 0 is fine): the selection
 * keeps its scratch on chip, except that long rows (N > 65536 with a budget of at most an
 * eighth of the candidates) are cut into pieces that are filtered by several compute units and
 * then combined, which needs tb_workspace_bytes(TB_OP_SELECT, desc, sink + k + window) bytes
 * (8 bytes per slot for a kept score: at most min(2k + 4096, piece length) slots per piece of
 * 16384 scores, so up to 8 N bytes per (b,h) -- 201 MB for B*Hq = 256, N = 131072, k = 4096);
 * with less, one workgroup selects the whole row (same result, slower).  The batch axis may
 * just as well run over the consumer layers of a producer (Sec. 3.3: their scoring and
 * selection are batched): stack the layers' projected-key caches and queries along B. */
tb_status tb_select_topk(const tb_cache_desc* desc, const float* scores, int64_t score_stride, int32_t k,
                         int32_t sink, int32_t window, int32_t* idx, int32_t* count, int64_t idx_cap, void* ws,
                         size_t ws_bytes, void* stream);

/* Neighbour fetching (Sec. 3.4 "Neighbor fetching").  idx_in lists must be strictly ascending
 * and within [0, N).
 * mode 0: idx_out = ascending, duplicate-free union over the input of [i-radius, i+radius]
 *         clipped to [0, N).  cap_out >= min(N, (2*radius+1) * cap_in) is required.
 * mode 1: cluster-aware fetch: consecutive selected positions form clusters and every
 *         selected token adds the next free position past its cluster (left-to-right; free
 *         positions taken by an earlier cluster are skipped), 2*count positions unless the
 *         sweep reaches N.  radius is ignored.  cap_out >= min(N, 2 * cap_in).
 * Units are the B*Hq lists; count_out[u] receives the output length. */
tb_status tb_expand_neighbors(int32_t B, int32_t Hq, int64_t N, int32_t radius, int32_t mode,
                              const int32_t* idx_in, const int32_t* count_in, int64_t cap_in, int32_t* idx_out,
                              int32_t* count_out, int64_t cap_out, void* stream);

/* Decode attention over the selected rows (Sec. 3.3: attention touches sink, window and
 * important tokens only; with every token selected it is dense decode attention).
 *   out[b,h,:] = sum_i softmax_i(sm_scale * q[b,h] . K[b,h/g,n_i]) * V[b,h/g,n_i]
 * where n_i runs over idx[b,h,0:count[b,h]] followed by the dense range [tail_begin, tail_end)
 * (tokens appended since the list was made, which are always attended while a selection is
 * reused across a prediction interval; pass tail_begin == tail_end for none).
 * q: [B][Hq][D] contiguous.  idx entries must lie in [0, desc->N); tail_end <= desc->N.
 * max_count: host-side upper bound on count[b,h] (<= idx_cap) used to size the launch; a list
 * longer than max_count is truncated to it.  out: fp32 [B][Hq][D]; lse: fp32 [B][Hq] or NULL.
 * An empty list gives out = 0 and lse = -inf.  ws: tb_workspace_bytes(TB_OP_ATTN, ...). */
tb_status tb_sparse_decode_attn(const tb_cache_desc* desc, const void* q, const void* K, const void* V,
                                const int32_t* idx, const int32_t* count, int64_t idx_cap, int64_t max_count,
                                int64_t tail_begin, int64_t tail_end, float sm_scale, float* out, float* lse,
                                void* ws, size_t ws_bytes, void* stream);

/* Head-less form of tb_sparse_decode_attn (Appendix "Additional Efficiency Evaluation": the
 * predictor gives one importance per token per layer, with no head dimension, so one token list
 * serves every head of the layer).  idx: [B][idx_cap], count: [B]; every query head h of batch
 * element b attends over idx[b,0:count[b]] followed by [tail_begin, tail_end).  Such a list is
 * what tb_score and tb_select_topk produce under a descriptor with Hq = Hkv = 1 (one importance
 * head).  All other arguments, results and errors as tb_sparse_decode_attn. */
tb_status tb_sparse_decode_attn_shared(const tb_cache_desc* desc, const void* q, const void* K, const void* V,
                                       const int32_t* idx, const int32_t* count, int64_t idx_cap,
                                       int64_t max_count, int64_t tail_begin, int64_t tail_end, float sm_scale,
                                       float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/* tb_sparse_decode_attn for callers that cannot allocate device memory or hand over a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same
 * arguments minus ws / ws_bytes, same kernels and bit-identical results.  The scratch (arrival
 * counters and split partials) lives in a device array inside the library, 4 MiB per GPU, held
 * from the first call on that GPU until the process ends.  A shape whose scratch would exceed
 * that (tb_workspace_bytes(TB_OP_ATTN, ...) > 4 MiB) is rejected with TB_ERR_WORKSPACE before
 * anything is launched.  The call allocates nothing and enqueues a small fill kernel (the
 * counters are cleared on every call) followed by the attention kernel.  All calls on one GPU
 * share the array: calls that overlap in time on one GPU (different streams) race. */
tb_status tb_sparse_decode_attn_static(const tb_cache_desc* desc, const void* q, const void* K, const void* V,
                                       const int32_t* idx, const int32_t* count, int64_t idx_cap,
                                       int64_t max_count, int64_t tail_begin, int64_t tail_end, float sm_scale,
                                       float* out, float* lse, void* stream);

/* Migration of selected rows into the "Important Buffer" (Sec. 3.3 "Inference Setup": the
 * paper keeps the attended tokens in contiguous buffers and copies the selection there on
 * prediction steps).  Kbuf/Vbuf[b,h,i,:] = K/V[b,h/g,idx[b,h,i],:] for i < min(count[b,h], max_count).
 * Kbuf, Vbuf: [B][Hq][buf_cap][D] contiguous, element type of the cache, buf_cap >= max_count;
 * rows at and beyond the count are left untouched.  The buffers are per *query* head, because
 * every query head selects its own tokens. */
tb_status tb_gather_kv(const tb_cache_desc* desc, const void* K, const void* V, const int32_t* idx,
                       const int32_t* count, int64_t idx_cap, int64_t max_count, void* Kbuf, void* Vbuf,
                       int64_t buf_cap, void* stream);

/* tb_gather_kv for the layout with a Sink Buffer and a Local Window Buffer of their own (Sec. 3.3
 * "Inference Setup"): a list made by tb_select_topk (and widened by tb_expand_neighbors) begins
 * with the sink positions and ends with the local-window positions; those rows live in their own
 * buffers, so only the entries in between are migrated:
 *   Kbuf/Vbuf[b,h,i,:] = K/V[b,h/g,idx[b,h,skip_front + i],:]   for 0 <= i < count_out[b,h],
 *   count_out[b,h] = max(0, min(count[b,h], max_count) - skip_front - skip_back).
 * buf_cap >= max(0, max_count - skip_front - skip_back); count_out: int32 [B][Hq], always written. */
tb_status tb_gather_important(const tb_cache_desc* desc, const void* K, const void* V, const int32_t* idx,
                              const int32_t* count, int64_t idx_cap, int64_t max_count, int32_t skip_front,
                              int32_t skip_back, void* Kbuf, void* Vbuf, int64_t buf_cap, int32_t* count_out,
                              void* stream);

/* tb_sparse_decode_attn over rows that tb_gather_kv has migrated: the rows 0 .. count[b,h]-1 of
 * the per-query-head buffers (no index list is read) followed by the dense range
 * [tail_begin, tail_end) of the cache K, V (the local window of tokens appended since the
 * migration).  Same result, bit for bit, as tb_sparse_decode_attn with the list the buffers
 * were filled from.  ws: tb_workspace_bytes(TB_OP_ATTN, ...). */
tb_status tb_buffered_decode_attn(const tb_cache_desc* desc, const void* q, const void* Kbuf, const void* Vbuf,
                                  int64_t buf_cap, const int32_t* count, int64_t max_count, const void* K,
                                  const void* V, int64_t tail_begin, int64_t tail_end, float sm_scale,
                                  float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/* One prediction step in a single enqueue: tb_score -> tb_select_topk -> tb_sparse_decode_attn
 * with one validation pass and one launch plan.  Results (scores, idx, count, out, lse) are
 * identical to calling the three entry points one after the other.
 * ws: tb_workspace_bytes(TB_OP_DECODE_STEP, ...). */
tb_status tb_decode_step(const tb_cache_desc* desc, const void* q_imp, const void* Kimp, float score_scale,
                         const void* q, const void* K, const void* V, int32_t k, int32_t sink, int32_t window,
                         float sm_scale, float* scores, int64_t score_stride, int32_t* idx, int32_t* count,
                         int64_t idx_cap, float* out, float* lse, void* ws, size_t ws_bytes, void* stream);

/* Query prediction of a producer layer (Sec. 3.1 "Query prediction"): from the hidden state of
 * the token being decoded, a LayerNorm and a two-layer MLP give one importance query per query
 * head for each of the G consumer layers ("slots") that follow the producer:
 *   x = LN(h) = (h - mean) / sqrt(var + ln_eps) * gamma + beta      (over E, biased variance)
 *   z = gelu(W1 x + b1)          (exact erf form; the paper does not name the nonlinearity)
 *   y = W2 z + b2,   q_imp[s][b][hq][j] = y[(s*Hq + hq)*Dimp + j]
 * h: [B][E]; gamma, beta: [E]; W1: [hidden][E]; b1: [hidden]; W2: [G*Hq*Dimp][hidden];
 * b2: [G*Hq*Dimp] -- all contiguous, all of element type `dtype`; fp32 accumulation, one rounding
 * when q_imp is stored.  q_imp: [G][B][Hq][Dimp] of `dtype`: slot s is the [B][Hq][Dimp] array that
 * tb_score takes for consumer layer s.  hidden_act: fp32 [B][hidden], receives z; ln_act: fp32
 * [B][E], receives LN(h) when B > 2 (both are scratch that the caller owns; 16-byte aligned, as
 * are h, gamma, beta, W1, W2).  E and hidden must be multiples of 8, E <= 8192, hidden <= 2048. */
typedef struct {
  int32_t E, hidden, G, Hq, Dimp;
  tb_dtype dtype;
  float ln_eps;
} tb_predictor_desc;
tb_status tb_predict_queries(const tb_predictor_desc* p, int32_t B, const void* h, const void* gamma,
                             const void* beta, const void* W1, const void* b1, const void* W2, const void* b2,
                             float* hidden_act, float* ln_act, void* q_imp, void* stream);

/* Scratch size in bytes for `op` on this cache shape.  max_count is the longest list the
 * attention will see, tail included; for TB_OP_SELECT and TB_OP_DECODE_STEP it is the list
 * length the selection policy produces, lo + kk + N - hi (TB_OP_SELECT returns 0 for every
 * shape whose rows are selected by one workgroup each).  Returns 0 on invalid
 * input.  A workspace of the TB_OP_DECODE_STEP size serves all three operations on that
 * shape.  The workspace pointer must be 16-byte aligned. */
size_t tb_workspace_bytes(int32_t op, const tb_cache_desc* desc, int64_t max_count);

/* A workspace must be zero-filled once before its first use (this call enqueues that fill;
 * any other device memset does as well).  Every entry point leaves the workspace ready for the
 * next call, provided the calls that share it run one after the other on one stream and use
 * the same B and Hq.  Calls that overlap in time need separate workspaces. */
tb_status tb_workspace_init(void* ws, size_t ws_bytes, void* stream);

/* Measurement aid, not a step of the method: reads `bytes` (rounded down to 16) of device
 * memory at `src` (16-byte aligned) once with plain 128-bit streaming loads and writes nothing
 * (sink: one device word that is written only if the data fold to one particular value).  The
 * rate it reaches is the practical read ceiling of the box for the bandwidth-bound kernels of
 * the path, to be quoted next to the data-sheet HBM bandwidth. */
tb_status tb_read_stream_probe(const void* src, size_t bytes, uint32_t* sink, void* stream);

const char* tb_status_string(tb_status s);

/* Library version: major*10000 + minor*100 + patch. */
int32_t tb_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TOKENBUTLER_H_ */
