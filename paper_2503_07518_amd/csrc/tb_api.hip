// C ABI of libtokenbutler: argument validation on the host, workspace layout, launch plans.
// Every entry point only enqueues kernels on the caller's stream.
#include <cmath>
#include <mutex>

#include "tb_internal.h"

namespace tb {

constexpr int64_t kAttnTargetWgs = 512;   // workgroups a launch of the split attention aims at
constexpr int64_t kAttnMinTiles = 2;      // a workgroup is worth its hand-over from two tiles per wave on

AttnPlan attn_plan(int64_t units, int64_t max_rows, int tile_rows_per_wg, bool grouped) {
  // Aim for two workgroups per compute unit (256 CUs): the gathers of the whole chip are in
  // flight together, and fewer, longer workgroups mean fewer partials to hand over (measured
  // best across the five configurations; 1024 was 1 µs slower on the smallest and 2 µs on the
  // largest).  A workgroup takes whole wave tiles.
  AttnPlan p;
  if (max_rows <= 0 || units <= 0) {
    p.rows_per_wg = tile_rows_per_wg;
    p.nsplit = 1;
    p.max_split = 1;
    return p;
  }
  const int64_t target_wgs = kAttnTargetWgs;  // (the same for one workgroup per KV group)
  int64_t want = (target_wgs + units - 1) / units;
  (void)grouped;
  const int64_t max_split = max_rows / (kAttnMinTiles * tile_rows_per_wg);
  if (want > max_split) want = max_split;
  if (want < 1) want = 1;
  // equal shares, rounded up to whole wave instructions (4 rows x 4 waves for 256-byte rows) rather
  // than whole tiles: a ragged last tile per wave costs less than a last workgroup round that
  // only some compute units take part in
  const int64_t granule = tile_rows_per_wg / kAttnLoadsPerTile;
  int64_t rows = (max_rows + want - 1) / want;
  rows = (rows + granule - 1) / granule * granule;
  p.rows_per_wg = static_cast<int>(rows);
  p.nsplit = static_cast<int>((max_rows + rows - 1) / rows);
  p.max_split = static_cast<int>(want);
  return p;
}

// A shared list with grouped queries: one workgroup per (KV group, split) loads every row once
// for all heads of the group.  That pays when there are enough KV groups to fill the chip with
// few splits each (the last workgroup of a group combines heads x splits partials with
// device-scope loads, about 0.1 us per split); with fewer groups the per-head kernel, whose
// heads share rows through the L2 of their XCD, is faster (8 groups, 3277 rows: 10.9 against 18.7 us).
bool attn_shared_list_grouped(const tb_cache_desc* d) {
  return d->Hq > d->Hkv && static_cast<int64_t>(d->B) * d->Hkv >= 32;
}

SelectPlan select_plan(int64_t units, int64_t candidates, int64_t N, int64_t kk) {
  SelectPlan p{1, 0, 0, 2, 16, 16};
  // worth it when the budget is a small share of the candidates (the kept keys are then a small
  // share of the row as well) and the row is longer than the 65536 scores one workgroup holds in
  // registers (beyond that it would stream the row again in every phase: 44 against 27 us just
  // past 65536); up to 65536 scores two launches cost more than the one-workgroup selection
  if (units <= 0 || kk <= 0 || N <= 65536 || kk * 8 > candidates) return p;
  int waves = 8, tiles = 8;
  auto len_of = [&]() { return static_cast<int64_t>(waves) * 256 * tiles; };
  // few rows (a head-less selection has one per batch element): shorter pieces, so that more
  // compute units take part
  while (units * ((N + len_of() - 1) / len_of()) < 256 && (tiles > 2 || waves > 4)) {
    if (tiles > 2) tiles /= 2; else waves /= 2;
  }
  while ((N + len_of() - 1) / len_of() > 256 && tiles < 16) tiles *= 2;  // the table of stage B has 256 entries
  const int64_t len = len_of();
  const int64_t pieces = (N + len - 1) / len;
  if (pieces < 2 || pieces > 256) return p;
  p.pieces = static_cast<int>(pieces);
  p.piece_len = len;
  p.piece_waves = waves;
  p.piece_tiles = tiles;
  const int64_t cap = 2 * kk + 4096;                      // the budget, the bracket's slack, a coarse top bin
  p.cap = ((cap < len ? cap : len) + 3) / 4 * 4;
  // what the pieces keep together, give or take: the share of the row above the lower end of the
  // bracket (the rank of the threshold in a sample of 4 keys per thread plus twice the bracket's
  // slack: the lower end lies one slack below the expected rank, and its 12-bit bin reaches further
  // down), every piece padded to a multiple of 4
  const double n_s = 4.0 * 64 * waves, frac = static_cast<double>(kk) / static_cast<double>(candidates);
  const double ks = frac * n_s, slack = 6.0 * sqrt(ks * (1.0 - frac)) + 4.0;
  double kept = (ks + 2.0 * slack) / n_s * static_cast<double>(candidates) + 3.0 * static_cast<double>(pieces);
  if (kept > static_cast<double>(pieces * p.cap)) kept = static_cast<double>(pieces * p.cap);
  const int64_t t4k = (static_cast<int64_t>(kept) + 4095) / 4096;
  p.stage_b_tiles = t4k <= 2 ? 2 : (t4k <= 4 ? 4 : (t4k <= 8 ? 8 : 16));
  return p;
}

WsLayout ws_layout(int64_t units, int D, int nsplit) {
  WsLayout w;
  w.part_off = align_up(static_cast<size_t>(units) * kCounterStrideWords * sizeof(uint32_t), 256);
  w.total = w.part_off + align_up(static_cast<size_t>(units) * nsplit * (D + 2) * sizeof(float), 256);
  return w;
}

namespace {

// Scratch of tb_sparse_decode_attn_static: device memory that the library owns, one copy per
// GPU, held from the first use on that GPU until the process ends.  Host code never passes the
// array's name to a kernel (on the host it is only a stand-in for the symbol): the device
// address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = size_t{4} << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device (looked up on the first call per device).
tb_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return TB_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return TB_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return TB_OK;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

tb_status check_desc(const tb_cache_desc* d) {
  if (!d) return TB_ERR_INVALID_ARG;
  if (d->B < 0 || d->Hq < 0 || d->Hkv < 0 || d->N < 0) return TB_ERR_INVALID_ARG;
  if (d->dtype != TB_F32 && d->dtype != TB_BF16) return TB_ERR_INVALID_ARG;
  if (d->Hkv == 0 ? d->Hq != 0 : (d->Hq % d->Hkv) != 0) return TB_ERR_INVALID_ARG;
  if (d->D != 64 && d->D != 128) return TB_ERR_UNSUPPORTED;
  if (d->Dimp != 16 && d->Dimp != 32 && d->Dimp != 64) return TB_ERR_UNSUPPORTED;
  if (d->Hkv > 0) {
    const int g = d->Hq / d->Hkv;
    if (g != 1 && g != 2 && g != 4 && g != 8) return TB_ERR_UNSUPPORTED;
  }
  if (d->B > 65535 || d->Hq > 65535) return TB_ERR_UNSUPPORTED;
  return TB_OK;
}

tb_status check_strides(const tb_cache_desc* d, int64_t sb, int64_t sh, int64_t sn, int inner) {
  if (sb < 0 || sh < 0 || sn < inner) return TB_ERR_INVALID_ARG;
  if ((sb | sh | sn) % 8) return TB_ERR_UNSUPPORTED;
  (void)d;
  return TB_OK;
}

#define TB_TRY(expr)                 \
  do {                               \
    const tb_status _s = (expr);     \
    if (_s != TB_OK) return _s;      \
  } while (0)

struct Policy {
  int64_t lo, hi, kk, count;
};
Policy policy(int64_t N, int32_t k, int32_t sink, int32_t window) {
  Policy p;
  p.lo = sink < N ? sink : N;
  p.hi = (N - window > p.lo) ? (N - window) : p.lo;
  const int64_t nc = p.hi - p.lo;
  p.kk = k < nc ? k : nc;
  p.count = p.lo + p.kk + (N - p.hi);
  return p;
}

tb_status check_score_args(const tb_cache_desc* d, const void* q_imp, const void* Kimp, const float* scores,
                           int64_t score_stride) {
  TB_TRY(check_desc(d));
  if (!q_imp || !Kimp || !scores) return TB_ERR_INVALID_ARG;
  if (score_stride < d->N) return TB_ERR_INVALID_ARG;
  if (score_stride % 4) return TB_ERR_UNSUPPORTED;
  TB_TRY(check_strides(d, d->ki_stride_b, d->ki_stride_h, d->ki_stride_n, d->Dimp));
  if (!aligned16(q_imp) || !aligned16(Kimp) || !aligned16(scores)) return TB_ERR_UNSUPPORTED;
  return TB_OK;
}

tb_status check_select_args(const tb_cache_desc* d, const float* scores, int64_t score_stride, int32_t k,
                            int32_t sink, int32_t window, const int32_t* idx, const int32_t* count,
                            int64_t idx_cap) {
  TB_TRY(check_desc(d));
  if (!scores || !idx || !count) return TB_ERR_INVALID_ARG;
  if (k < 0 || sink < 0 || window < 0) return TB_ERR_INVALID_ARG;
  if (score_stride < d->N) return TB_ERR_INVALID_ARG;
  if (score_stride % 4 || !aligned16(scores)) return TB_ERR_UNSUPPORTED;
  if (d->N > kSelectMaxN) return TB_ERR_UNSUPPORTED;
  const Policy p = policy(d->N, k, sink, window);
  if (idx_cap < p.count) return TB_ERR_INVALID_ARG;
  return TB_OK;
}

tb_status check_attn_args(const tb_cache_desc* d, const void* q, const void* K, const void* V, const int32_t* idx,
                          const int32_t* count, int64_t idx_cap, int64_t max_count, int64_t tail_begin,
                          int64_t tail_end, const float* out) {
  TB_TRY(check_desc(d));
  if (!q || !K || !V || !idx || !count || !out) return TB_ERR_INVALID_ARG;
  if (idx_cap < 0 || max_count < 0 || max_count > idx_cap) return TB_ERR_INVALID_ARG;
  if (tail_begin < 0 || tail_begin > tail_end || tail_end > d->N) return TB_ERR_INVALID_ARG;
  if (d->N == 0 && max_count > 0) return TB_ERR_INVALID_ARG;
  TB_TRY(check_strides(d, d->k_stride_b, d->k_stride_h, d->k_stride_n, d->D));
  TB_TRY(check_strides(d, d->v_stride_b, d->v_stride_h, d->v_stride_n, d->D));
  if (!aligned16(q) || !aligned16(K) || !aligned16(V)) return TB_ERR_UNSUPPORTED;
  if (max_count + (tail_end - tail_begin) > (int64_t{1} << 30)) return TB_ERR_UNSUPPORTED;
  // the gather addresses rows with 32-bit byte offsets inside one (b, kv-head) slab
  const int64_t elt = d->dtype == TB_F32 ? 4 : 2;
  if (d->N * d->k_stride_n * elt >= (int64_t{1} << 32) || d->N * d->v_stride_n * elt >= (int64_t{1} << 32))
    return TB_ERR_UNSUPPORTED;
  return TB_OK;
}

}  // namespace
}  // namespace tb

using namespace tb;

extern "C" {

tb_status tb_project_keys(const tb_cache_desc* d, const void* K, const void* W, int32_t Hw, void* Kimp,
                          int64_t n_begin, int64_t n_end, void* stream) {
  TB_TRY(check_desc(d));
  if (!K || !W || !Kimp) return TB_ERR_INVALID_ARG;
  if (Hw != 1 && Hw != d->Hkv) return TB_ERR_INVALID_ARG;
  if (n_begin < 0 || n_begin > n_end || n_end > d->N) return TB_ERR_INVALID_ARG;
  TB_TRY(check_strides(d, d->k_stride_b, d->k_stride_h, d->k_stride_n, d->D));
  TB_TRY(check_strides(d, d->ki_stride_b, d->ki_stride_h, d->ki_stride_n, d->Dimp));
  if (!aligned16(K) || !aligned16(W) || !aligned16(Kimp)) return TB_ERR_UNSUPPORTED;
  return launch_project(d, K, W, Hw, Kimp, n_begin, n_end, static_cast<hipStream_t>(stream));
}

tb_status tb_score(const tb_cache_desc* d, const void* q_imp, const void* Kimp, float scale, float* scores,
                   int64_t score_stride, void* stream) {
  TB_TRY(check_score_args(d, q_imp, Kimp, scores, score_stride));
  if (d->B == 0 || d->Hq == 0) return TB_OK;
  ScoreLaunch L{d, q_imp, Kimp, scale, scores, score_stride};
  return launch_score(L, static_cast<hipStream_t>(stream));
}

tb_status tb_select_topk(const tb_cache_desc* d, const float* scores, int64_t score_stride, int32_t k, int32_t sink,
                         int32_t window, int32_t* idx, int32_t* count, int64_t idx_cap, void* ws, size_t ws_bytes,
                         void* stream) {
  TB_TRY(check_select_args(d, scores, score_stride, k, sink, window, idx, count, idx_cap));
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  if (units == 0) return TB_OK;
  const Policy p = policy(d->N, k, sink, window);
  SelectLaunch L;
  L.units = units;
  L.N = d->N;
  L.scores = scores;
  L.score_stride = score_stride;
  L.kk = static_cast<int32_t>(p.kk);
  L.lo = static_cast<int32_t>(p.lo);
  L.hi = static_cast<int32_t>(p.hi);
  L.idx = idx;
  L.count = count;
  L.idx_cap = idx_cap;
  // scratch of the two-stage selection: behind the arrival counters, which stay untouched
  const size_t off = ws_layout(units, d->D, 1).part_off;
  const bool usable = ws && aligned16(ws) && ws_bytes > off;
  L.scratch = usable ? static_cast<char*>(ws) + off : nullptr;
  L.scratch_bytes = usable ? ws_bytes - off : 0;
  return launch_select(L, static_cast<hipStream_t>(stream));
}

tb_status tb_expand_neighbors(int32_t B, int32_t Hq, int64_t N, int32_t radius, int32_t mode, const int32_t* idx_in,
                              const int32_t* count_in, int64_t cap_in, int32_t* idx_out, int32_t* count_out,
                              int64_t cap_out, void* stream) {
  if (B < 0 || Hq < 0 || N < 0 || radius < 0 || cap_in < 0 || cap_out < 0) return TB_ERR_INVALID_ARG;
  if (mode != 0 && mode != 1) return TB_ERR_INVALID_ARG;
  if (!idx_in || !count_in || !idx_out || !count_out) return TB_ERR_INVALID_ARG;
  if (idx_in == idx_out) return TB_ERR_INVALID_ARG;
  if (B > 65535 || Hq > 65535 || N > (int64_t{1} << 30) || radius > (1 << 20)) return TB_ERR_UNSUPPORTED;
  const int64_t mult = (mode == 0) ? (2 * static_cast<int64_t>(radius) + 1) : 2;
  int64_t need = mult * cap_in;
  if (need > N) need = N;
  if (cap_out < need) return TB_ERR_INVALID_ARG;
  return launch_expand(static_cast<int64_t>(B) * Hq, N, radius, mode, idx_in, count_in, cap_in, idx_out, count_out,
                       cap_out, static_cast<hipStream_t>(stream));
}

namespace {
tb_status sparse_attn(const tb_cache_desc* d, const void* q, const void* K, const void* V, const int32_t* idx,
                      const int32_t* count, int64_t idx_cap, int64_t max_count, int64_t tail_begin,
                      int64_t tail_end, float sm_scale, float* out, float* lse, void* ws, size_t ws_bytes,
                      void* stream, bool shared_list) {
  TB_TRY(check_attn_args(d, q, K, V, idx, count, idx_cap, max_count, tail_begin, tail_end, out));
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  if (units == 0) return TB_OK;
  const int64_t rows = max_count + (tail_end - tail_begin);
  const bool grouped = shared_list && attn_shared_list_grouped(d);
  const int64_t wg_units = grouped ? static_cast<int64_t>(d->B) * d->Hkv : units;
  const AttnPlan plan = attn_plan(wg_units, rows, attn_tile_rows_per_wg(d->dtype, d->D), wg_units != units);
  const WsLayout w = ws_layout(units, d->D, plan.nsplit);
  if (!ws || !aligned16(ws) || ws_bytes < w.total) return TB_ERR_WORKSPACE;
  AttnLaunch L{d,   q,   K,   V,
               idx, count, idx_cap, max_count, tail_begin, tail_end,
               sm_scale, out, lse,
               reinterpret_cast<float*>(static_cast<char*>(ws) + w.part_off),
               reinterpret_cast<uint32_t*>(ws), plan};
  L.shared_list = shared_list;
  L.grouped = grouped;
  return launch_attn(L, static_cast<hipStream_t>(stream));
}
}  // namespace

tb_status tb_sparse_decode_attn(const tb_cache_desc* d, const void* q, const void* K, const void* V,
                                const int32_t* idx, const int32_t* count, int64_t idx_cap, int64_t max_count,
                                int64_t tail_begin, int64_t tail_end, float sm_scale, float* out, float* lse,
                                void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn(d, q, K, V, idx, count, idx_cap, max_count, tail_begin, tail_end, sm_scale, out, lse, ws,
                     ws_bytes, stream, false);
}

tb_status tb_sparse_decode_attn_shared(const tb_cache_desc* d, const void* q, const void* K, const void* V,
                                       const int32_t* idx, const int32_t* count, int64_t idx_cap,
                                       int64_t max_count, int64_t tail_begin, int64_t tail_end, float sm_scale,
                                       float* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  return sparse_attn(d, q, K, V, idx, count, idx_cap, max_count, tail_begin, tail_end, sm_scale, out, lse, ws,
                     ws_bytes, stream, true);
}

tb_status tb_sparse_decode_attn_static(const tb_cache_desc* d, const void* q, const void* K, const void* V,
                                       const int32_t* idx, const int32_t* count, int64_t idx_cap,
                                       int64_t max_count, int64_t tail_begin, int64_t tail_end, float sm_scale,
                                       float* out, float* lse, void* stream) {
  TB_TRY(check_attn_args(d, q, K, V, idx, count, idx_cap, max_count, tail_begin, tail_end, out));
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  if (units == 0) return TB_OK;
  const AttnPlan plan = attn_plan(units, max_count + (tail_end - tail_begin), attn_tile_rows_per_wg(d->dtype, d->D));
  const WsLayout w = ws_layout(units, d->D, plan.nsplit);
  if (w.total > kStaticScratchBytes) return TB_ERR_WORKSPACE;  // beyond the library's own scratch
  void* ws = nullptr;
  TB_TRY(static_scratch(&ws));
  hipStream_t st = static_cast<hipStream_t>(stream);
  // the arrival counters must be zero when the kernel starts; the array keeps whatever the
  // last call on this GPU left, so they are cleared here (a fill kernel, not a memset node:
  // callers may be capturing a graph)
  TB_TRY(launch_fill_zero(ws, w.part_off, st));
  AttnLaunch L{d,   q,   K,   V,
               idx, count, idx_cap, max_count, tail_begin, tail_end,
               sm_scale, out, lse,
               reinterpret_cast<float*>(static_cast<char*>(ws) + w.part_off),
               reinterpret_cast<uint32_t*>(ws), plan};
  return launch_attn(L, st);
}

tb_status tb_gather_kv(const tb_cache_desc* d, const void* K, const void* V, const int32_t* idx, const int32_t* count,
                       int64_t idx_cap, int64_t max_count, void* Kbuf, void* Vbuf, int64_t buf_cap, void* stream) {
  TB_TRY(check_desc(d));
  if (!K || !V || !idx || !count || !Kbuf || !Vbuf) return TB_ERR_INVALID_ARG;
  if (idx_cap < 0 || max_count < 0 || max_count > idx_cap || max_count > buf_cap) return TB_ERR_INVALID_ARG;
  if (d->N == 0 && max_count > 0) return TB_ERR_INVALID_ARG;
  TB_TRY(check_strides(d, d->k_stride_b, d->k_stride_h, d->k_stride_n, d->D));
  TB_TRY(check_strides(d, d->v_stride_b, d->v_stride_h, d->v_stride_n, d->D));
  if (!aligned16(K) || !aligned16(V) || !aligned16(Kbuf) || !aligned16(Vbuf)) return TB_ERR_UNSUPPORTED;
  if (max_count > (int64_t{1} << 30)) return TB_ERR_UNSUPPORTED;
  GatherLaunch L{d, K, V, idx, count, idx_cap, max_count, Kbuf, Vbuf, buf_cap};
  return launch_gather(L, static_cast<hipStream_t>(stream));
}

tb_status tb_gather_important(const tb_cache_desc* d, const void* K, const void* V, const int32_t* idx,
                              const int32_t* count, int64_t idx_cap, int64_t max_count, int32_t skip_front,
                              int32_t skip_back, void* Kbuf, void* Vbuf, int64_t buf_cap, int32_t* count_out,
                              void* stream) {
  TB_TRY(check_desc(d));
  if (!K || !V || !idx || !count || !Kbuf || !Vbuf || !count_out) return TB_ERR_INVALID_ARG;
  if (idx_cap < 0 || max_count < 0 || max_count > idx_cap || skip_front < 0 || skip_back < 0) return TB_ERR_INVALID_ARG;
  const int64_t rows = max_count > static_cast<int64_t>(skip_front) + skip_back ? max_count - skip_front - skip_back : 0;
  if (rows > buf_cap) return TB_ERR_INVALID_ARG;
  if (d->N == 0 && max_count > 0) return TB_ERR_INVALID_ARG;
  TB_TRY(check_strides(d, d->k_stride_b, d->k_stride_h, d->k_stride_n, d->D));
  TB_TRY(check_strides(d, d->v_stride_b, d->v_stride_h, d->v_stride_n, d->D));
  if (!aligned16(K) || !aligned16(V) || !aligned16(Kbuf) || !aligned16(Vbuf)) return TB_ERR_UNSUPPORTED;
  if (max_count > (int64_t{1} << 30)) return TB_ERR_UNSUPPORTED;
  GatherLaunch L{d, K, V, idx, count, idx_cap, max_count, Kbuf, Vbuf, buf_cap};
  L.skip_front = skip_front;
  L.skip_back = skip_back;
  L.count_out = count_out;
  return launch_gather(L, static_cast<hipStream_t>(stream));
}

tb_status tb_buffered_decode_attn(const tb_cache_desc* d, const void* q, const void* Kbuf, const void* Vbuf,
                                  int64_t buf_cap, const int32_t* count, int64_t max_count, const void* K,
                                  const void* V, int64_t tail_begin, int64_t tail_end, float sm_scale, float* out,
                                  float* lse, void* ws, size_t ws_bytes, void* stream) {
  if (!Kbuf || !Vbuf || buf_cap < 0 || max_count > buf_cap) return TB_ERR_INVALID_ARG;
  // the list itself is not read: its place in the argument check is taken by the count array
  TB_TRY(check_attn_args(d, q, K, V, count, count, buf_cap, max_count, tail_begin, tail_end, out));
  if (!aligned16(Kbuf) || !aligned16(Vbuf)) return TB_ERR_UNSUPPORTED;
  const int64_t elt = d->dtype == TB_F32 ? 4 : 2;
  if (buf_cap * d->D * elt >= (int64_t{1} << 32)) return TB_ERR_UNSUPPORTED;  // 32-bit offsets inside a head's buffer
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  if (units == 0) return TB_OK;
  const int64_t rows = max_count + (tail_end - tail_begin);
  const AttnPlan plan = attn_plan(units, rows, attn_tile_rows_per_wg(d->dtype, d->D));
  const WsLayout w = ws_layout(units, d->D, plan.nsplit);
  if (!ws || !aligned16(ws) || ws_bytes < w.total) return TB_ERR_WORKSPACE;
  AttnLaunch L{d,   q,   K,   V,
               nullptr, count, buf_cap, max_count, tail_begin, tail_end,
               sm_scale, out, lse,
               reinterpret_cast<float*>(static_cast<char*>(ws) + w.part_off),
               reinterpret_cast<uint32_t*>(ws), plan};
  L.Kbuf = Kbuf;
  L.Vbuf = Vbuf;
  L.buf_cap = buf_cap;
  return launch_attn(L, static_cast<hipStream_t>(stream));
}

tb_status tb_predict_queries(const tb_predictor_desc* p, int32_t B, const void* h, const void* gamma,
                             const void* beta, const void* W1, const void* b1, const void* W2, const void* b2,
                             float* hidden_act, float* ln_act, void* q_imp, void* stream) {
  if (!p || B < 0) return TB_ERR_INVALID_ARG;
  if (p->E <= 0 || p->hidden <= 0 || p->G <= 0 || p->Hq <= 0 || p->Dimp <= 0) return TB_ERR_INVALID_ARG;
  if (p->dtype != TB_F32 && p->dtype != TB_BF16) return TB_ERR_INVALID_ARG;
  if (!(p->ln_eps >= 0.f)) return TB_ERR_INVALID_ARG;
  if (!h || !gamma || !beta || !W1 || !b1 || !W2 || !b2 || !hidden_act || !ln_act || !q_imp)
    return TB_ERR_INVALID_ARG;
  if (p->E % 8 || p->hidden % 8 || p->E > 8192 || p->hidden > 2048 || B > 65535) return TB_ERR_UNSUPPORTED;
  if (static_cast<int64_t>(p->G) * p->Hq * p->Dimp > (int64_t{1} << 24)) return TB_ERR_UNSUPPORTED;
  if (!aligned16(W1) || !aligned16(W2) || !aligned16(h) || !aligned16(gamma) || !aligned16(beta) ||
      !aligned16(ln_act))
    return TB_ERR_UNSUPPORTED;
  PredictLaunch L{p->dtype, B, p->E, p->hidden, p->G, p->Hq, p->Dimp, p->ln_eps, h, gamma, beta, W1, b1, W2, b2,
                  hidden_act, ln_act, q_imp};
  return launch_predict(L, static_cast<hipStream_t>(stream));
}

tb_status tb_decode_step(const tb_cache_desc* d, const void* q_imp, const void* Kimp, float score_scale,
                         const void* q, const void* K, const void* V, int32_t k, int32_t sink, int32_t window,
                         float sm_scale, float* scores, int64_t score_stride, int32_t* idx, int32_t* count,
                         int64_t idx_cap, float* out, float* lse, void* ws, size_t ws_bytes, void* stream) {
  TB_TRY(check_score_args(d, q_imp, Kimp, scores, score_stride));
  TB_TRY(check_select_args(d, scores, score_stride, k, sink, window, idx, count, idx_cap));
  const Policy p = policy(d->N, k, sink, window);
  TB_TRY(check_attn_args(d, q, K, V, idx, count, idx_cap, p.count, 0, 0, out));
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  if (units == 0) return TB_OK;
  const AttnPlan plan = attn_plan(units, p.count, attn_tile_rows_per_wg(d->dtype, d->D));
  const WsLayout w = ws_layout(units, d->D, plan.nsplit);
  if (!ws || !aligned16(ws) || ws_bytes < w.total) return TB_ERR_WORKSPACE;
  hipStream_t st = static_cast<hipStream_t>(stream);
  ScoreLaunch S{d, q_imp, Kimp, score_scale, scores, score_stride};

  SelectLaunch L;
  L.units = units;
  L.N = d->N;
  L.scores = scores;
  L.score_stride = score_stride;
  L.kk = static_cast<int32_t>(p.kk);
  L.lo = static_cast<int32_t>(p.lo);
  L.hi = static_cast<int32_t>(p.hi);
  L.idx = idx;
  L.count = count;
  L.idx_cap = idx_cap;
  L.scratch = static_cast<char*>(ws) + w.part_off;
  L.scratch_bytes = ws_bytes - w.part_off;
  TB_TRY(launch_score(S, st));
  TB_TRY(launch_select(L, st));

  AttnLaunch A{d,   q,   K,   V,
               idx, count, idx_cap, p.count, 0, 0,
               sm_scale, out, lse,
               reinterpret_cast<float*>(static_cast<char*>(ws) + w.part_off),
               reinterpret_cast<uint32_t*>(ws), plan};
  return launch_attn(A, st);
}

size_t tb_workspace_bytes(int32_t op, const tb_cache_desc* d, int64_t max_count) {
  if (check_desc(d) != TB_OK || max_count < 0) return 0;
  const int64_t units = static_cast<int64_t>(d->B) * d->Hq;
  // two-stage selection of long rows (none for most shapes): max_count bounds the budget
  // (sized for the largest budget that still takes the two-stage path on this row length)
  int64_t kk_bound = max_count < d->N / 8 ? max_count : d->N / 8;
  const size_t sel = select_scratch_bytes(units, select_plan(units, d->N, d->N, kk_bound));
  const size_t sel_total = sel ? ws_layout(units, d->D, 1).part_off + align_up(sel, 256) : 0;
  if (op == TB_OP_SELECT) return sel_total;
  if (op == TB_OP_ATTN || op == TB_OP_DECODE_STEP) {
    const AttnPlan plan = attn_plan(units, max_count, attn_tile_rows_per_wg(d->dtype, d->D));
    // sized for the largest split count a shorter list could get, so that one workspace serves
    // every call whose list is no longer than max_count
    size_t att = ws_layout(units, d->D, plan.max_split).total;
    if (attn_shared_list_grouped(d)) {  // the head-less form splits per KV group, possibly finer
      const AttnPlan gp = attn_plan(static_cast<int64_t>(d->B) * d->Hkv, max_count, attn_tile_rows_per_wg(d->dtype, d->D), true);
      const size_t g_att = ws_layout(units, d->D, gp.max_split).total;
      if (g_att > att) att = g_att;
    }
    return (op == TB_OP_DECODE_STEP && sel_total > att) ? sel_total : att;
  }
  return 0;
}

tb_status tb_workspace_init(void* ws, size_t ws_bytes, void* stream) {
  if (!ws && ws_bytes) return TB_ERR_INVALID_ARG;
  if (ws_bytes % 4 || (reinterpret_cast<uintptr_t>(ws) & 3u)) return TB_ERR_INVALID_ARG;
  return launch_fill_zero(ws, ws_bytes, static_cast<hipStream_t>(stream));
}

tb_status tb_read_stream_probe(const void* src, size_t bytes, uint32_t* sink, void* stream) {
  if (!src || !sink) return TB_ERR_INVALID_ARG;
  if (!aligned16(src)) return TB_ERR_UNSUPPORTED;
  return launch_read_stream(src, bytes, sink, static_cast<hipStream_t>(stream));
}

const char* tb_status_string(tb_status s) {
  switch (s) {
    case TB_OK: return "ok";
    case TB_ERR_INVALID_ARG: return "invalid argument";
    case TB_ERR_UNSUPPORTED: return "unsupported shape, dtype or alignment";
    case TB_ERR_WORKSPACE: return "workspace missing or too small";
    case TB_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int32_t tb_version(void) { return 100; }

}  // extern "C"
