// Host-side declarations shared by the translation units of libtokenbutler: one launcher per
// kernel family, the workspace layout and the launch plan of the split attention.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "tokenbutler.h"

namespace tb {

constexpr int64_t kSelectMaxN = 1 << 20;
// Arrival counters sit 256 bytes apart so that the device-scope atomics of different heads do
// not queue up on one cache line / memory channel.
constexpr int kCounterStrideWords = 64;

// Workspace layout (byte offsets), fixed by B*Hq so that all operations agree on it:
//   [0, part_off)              uint32 arrival counters, one per (b,h), 256 B apart -- zero between calls
//   [part_off, ...)            fp32 split-attention partials [B*Hq][nsplit][D+2]; the two-stage
//                              selection of long rows keeps its candidates in the same region
//                              (it has finished before the attention of the same stream starts)
struct WsLayout {
  size_t part_off, total;
};

struct AttnPlan {
  int rows_per_wg;  // list entries handled by one workgroup
  int nsplit;       // workgroups per (b,h)
  int max_split;    // upper bound of nsplit for any list no longer than the one planned for
};

AttnPlan attn_plan(int64_t units, int64_t max_rows, int tile_rows_per_wg, bool grouped = false);
bool attn_shared_list_grouped(const tb_cache_desc* d);
WsLayout ws_layout(int64_t units, int D, int nsplit);

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct ScoreLaunch {
  const tb_cache_desc* desc;
  const void* q_imp;
  const void* Kimp;
  float scale;
  float* scores;
  int64_t score_stride;
};
tb_status launch_score(const ScoreLaunch& a, hipStream_t st);

// Long rows are selected in two stages so that several compute units work on a head: the row
// is cut into `pieces` pieces, every piece keeps the candidates that a sample of the row puts
// at or above the k-th largest (stage A, one workgroup per piece), and the final kk are
// selected among the kept ones (stage B, a second kernel).  pieces == 1: one workgroup per row,
// no scratch.
struct SelectPlan {
  int pieces;
  int64_t piece_len;  // scores per piece
  int64_t cap;        // kept keys a piece has room for (a multiple of 4)
  int stage_b_tiles;  // 4096-key tiles of kept keys that stage B holds in registers: 2, 4, 8 or 16
  int piece_waves;    // waves of a stage-A workgroup: 4, 8 or 16
  int piece_tiles;    // 256-key tiles that each of them keeps in registers: 2, 4, 8 or 16
};
SelectPlan select_plan(int64_t units, int64_t candidates, int64_t N, int64_t kk);
// kept positions int32 and keys uint32, [units][pieces][cap] each, then 4 words of header per piece
inline size_t select_scratch_bytes(int64_t units, const SelectPlan& p) {
  return p.pieces > 1 ? static_cast<size_t>(units) * p.pieces * (p.cap * 8 + 16) : 0;
}

struct SelectLaunch {
  int64_t units;
  int64_t N;
  const float* scores;
  int64_t score_stride;
  int32_t kk, lo, hi;
  int32_t* idx;
  int32_t* count;
  int64_t idx_cap;
  void* scratch;         // 16-byte aligned, or NULL
  size_t scratch_bytes;  // below select_scratch_bytes(): one workgroup per row is used instead
  const SelectPlan* plan = nullptr;  // NULL: select_plan() decides
};
tb_status launch_select(const SelectLaunch& a, hipStream_t st);

struct AttnLaunch {
  const tb_cache_desc* desc;
  const void* q;
  const void* K;
  const void* V;
  const int32_t* idx;
  const int32_t* count;
  int64_t idx_cap, max_count, tail_begin, tail_end;
  float sm_scale;
  float* out;
  float* lse;
  float* partials;
  uint32_t* counters;
  AttnPlan plan;
  // buffered form (Kbuf != NULL): list slot i is row i of the per-query-head buffers
  const void* Kbuf = nullptr;
  const void* Vbuf = nullptr;
  int64_t buf_cap = 0;
  // head-less form: idx is [B][idx_cap] and count [B], one list for all heads of a batch element
  bool shared_list = false;
  bool grouped = false;  // shared list served by one workgroup per KV group (plan made for that)
};

// Copies the listed rows of K and V into per-query-head buffers [B][Hq][buf_cap][D].
struct GatherLaunch {
  const tb_cache_desc* desc;
  const void* K;
  const void* V;
  const int32_t* idx;
  const int32_t* count;
  int64_t idx_cap, max_count;
  void* Kbuf;
  void* Vbuf;
  int64_t buf_cap;
  int32_t skip_front = 0, skip_back = 0;  // list entries left out at the two ends
  int32_t* count_out = nullptr;           // receives count - skip_front - skip_back (>= 0) per list
};
tb_status launch_gather(const GatherLaunch& a, hipStream_t st);
int attn_tile_rows_per_wg(int dtype, int D);
constexpr int kAttnLoadsPerTile = 4;  // K (and V) gathers of a lane per tile
tb_status launch_attn(const AttnLaunch& a, hipStream_t st);

// Query predictor of a producer layer (LN + two-layer MLP), see tb_predict.hip.
struct PredictLaunch {
  int dtype;
  int32_t B, E, hidden, G, Hq, Dimp;
  float eps;
  const void *h, *gamma, *beta, *W1, *b1, *W2, *b2;
  float* z;
  float* xln;
  void* q_imp;
};
tb_status launch_predict(const PredictLaunch& a, hipStream_t st);

tb_status launch_project(const tb_cache_desc* d, const void* K, const void* W, int32_t Hw, void* Kimp,
                         int64_t n_begin, int64_t n_end, hipStream_t st);

tb_status launch_expand(int64_t units, int64_t N, int32_t radius, int32_t mode, const int32_t* idx_in,
                        const int32_t* count_in, int64_t cap_in, int32_t* idx_out, int32_t* count_out,
                        int64_t cap_out, hipStream_t st);

tb_status launch_fill_zero(void* p, size_t bytes, hipStream_t st);
tb_status launch_read_stream(const void* src, size_t bytes, uint32_t* sink, hipStream_t st);

inline tb_status hip_status(hipError_t e) { return e == hipSuccess ? TB_OK : TB_ERR_HIP; }

}  // namespace tb
