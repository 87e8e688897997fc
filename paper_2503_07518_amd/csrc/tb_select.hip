// Top-k selection under the policy "candidates = [lo, hi); keep the kk largest scores, lowest
// index wins ties; emit ascending".
//
// The selection of one row (b,h) by one workgroup of W waves: wave w owns the contiguous span
// [w*span, (w+1)*span) of the row's scores and keeps their order-preserving 32-bit keys in
// registers (up to 64 per thread; longer rows are streamed again in every phase).  The exact
// threshold key T (the kk-th largest) and the number r of keys equal to T that are still
// needed are found by an MSB-first radix descent over LDS histograms:
//
//   bracket   a 12-bit histogram of a strided SAMPLE of the keys (one per thread) gives a range
//             of top-12-bit bins [b_lo, b_hi] that contains T unless the sample is wildly
//             unrepresentative (the rank of T in the sample, +- 6 standard deviations);
//   level 1   exact: every key above the bracket is counted, every key inside it goes into a
//             histogram of up to 4096 sub-bins; if the exact counts show that T is NOT inside
//             the bracket, the level is repeated with the bracket widened to all bins (slow
//             path, same result);
//   level 2+  the remaining low bits, 12 at a time, over the few keys of the chosen sub-bin.
//
// Output: {key > T} U {first r keys == T by index} in ascending order.  Positions come from
// prefix sums (DPP scans inside a 256-key wave tile, running totals along the wave's span, the
// wave totals across the workgroup) -- no atomic slot grabbing, so the result is ordered and
// reproducible.
//
// Launch forms:
//   select_kernel                      one 1024-thread workgroup per row, no global scratch;
//   prefilter_kernel + stage_b_kernel  long rows: the row is cut into pieces, one workgroup per
//                                      piece keeps the keys at or above the lower end of a bracket
//                                      that every piece derives from the same sample of the row,
//                                      and a second kernel selects among the kept keys.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kWaveTile = kWave * 4;  // scores per wave tile: one float4 per lane
constexpr int kHistBins = 4096;       // LDS histogram size (12 bits per level)
constexpr int kTopShift = 20;         // key >> 20 = top 12 bits
constexpr int kMaxPieces = 256;       // pieces of a row (the table of the second stage)

struct SelectArgs {
  const float* scores;
  int64_t score_stride;
  int64_t N;
  int32_t kk, lo, hi;  // selection: the kk largest of the candidates [lo, hi)
  int32_t* idx;
  int32_t* count;
  int64_t idx_cap;
  int32_t tiles_per_wave;  // of a workgroup that takes the whole row
  // Selection by pieces.  Stage A cuts the row into `pieces` pieces and keeps, per piece, the
  // candidates whose key is not below a threshold that a sample of the whole row puts safely
  // under the kk-th largest key: positions (of the whole row) and keys go to cand_idx /
  // cand_key [unit][piece][cap] in position order, and the piece's header {number found,
  // b_lo, b_hi, 0} to piece_hdr[unit][piece].  Stage B selects the kk largest among the kept
  // ones, read as one row through the table of the pieces' counts; if the pieces hold fewer
  // than kk keys together or more than stage B has registers for -- the sample misled -- it
  // selects on the original row instead.
  int32_t pieces;
  int64_t piece_len;
  int64_t cap;
  int64_t units;  // rows of the launch (stage A maps its workgroups to rows and pieces itself)
  int32_t* cand_idx;
  uint32_t* cand_key;
  uint32_t* piece_hdr;
};

// The four scores at positions n0 .. n0+3 (n0 a multiple of 4) as one 128-bit load without any
// branch, so that a thread's loads can all be in flight together.  A row's allocation covers
// score_stride >= N entries and score_stride is a multiple of 4, so the vector that holds the
// last score lies inside it; a position past that vector (`last4`) is clamped to it, and
// keys_of4 -- which gets the unclamped position -- masks what was read.
__device__ inline float4 load_scores4(const float* s, int64_t last4, int64_t n0) {
  return *reinterpret_cast<const float4*>(s + (n0 < last4 ? n0 : last4));
}

// Keys of the positions n0 .. n0+3.  Positions outside the candidate range [lo, hi) get key 0
// (no real score has a key below 0x007FFFFF).
__device__ inline void keys_of4(const float4& f, int lo, int hi, int64_t n0, uint32_t (&key)[4]) {
  const float v[4] = {f.x, f.y, f.z, f.w};
  if (n0 >= lo && n0 + 3 < hi) {  // the usual case: all four are candidates
#pragma unroll
    for (int c = 0; c < 4; ++c) key[c] = score_key(v[c]);
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int64_t n = n0 + c;
      key[c] = (n >= lo && n < hi) ? score_key(v[c]) : 0u;
    }
  }
}

// The W per-wave values in s_w (complete after a barrier): returns the sum of the entries of
// the waves before this one and, in `total`, the sum of all.  Every wave scans the values in
// one DPP row (lane i < W of each row holds entry i) instead of adding up W LDS reads per thread.
template <int W>
__device__ inline uint32_t wave_entries_scan(const uint32_t* s_w, uint32_t& total) {
  static_assert(W <= 16, "one DPP row holds the per-wave entries");
  constexpr int kRowShr = 0x110;
  const int l16 = threadIdx.x & 15;
  const uint32_t v = l16 < W ? s_w[l16] : 0u;
  uint32_t incl = v;
  incl += __builtin_amdgcn_update_dpp(0u, incl, kRowShr + 1, 0xF, 0xF, false);
  incl += __builtin_amdgcn_update_dpp(0u, incl, kRowShr + 2, 0xF, 0xF, false);
  if (W > 4) incl += __builtin_amdgcn_update_dpp(0u, incl, kRowShr + 4, 0xF, 0xF, false);
  if (W > 8) incl += __builtin_amdgcn_update_dpp(0u, incl, kRowShr + 8, 0xF, 0xF, false);
  total = __builtin_amdgcn_readlane(incl, W - 1);
  return __builtin_amdgcn_readlane(incl - v, wave_id());
}

// Number of set bits of a lane mask below this lane, added to acc; number of set bits.
__device__ inline uint32_t mbcnt64(unsigned long long m, uint32_t acc) {
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(m >> 32), __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(m), acc));
}
__device__ inline uint32_t popc64(unsigned long long m) { return static_cast<uint32_t>(__popcll(m)); }

// Result of a histogram walk, published in LDS for the whole workgroup.
struct Found {
  uint32_t bin_a, above_a;  // bin in which the running count (from the top bin down) reaches target a, count above it
  uint32_t bin_b, above_b;  // same for target b
  uint32_t extra_total;     // block-wide sum of `extra`
  uint32_t total;           // sum of all bins
  uint32_t need_a, need_b;  // the targets that were searched
  uint32_t count_a;         // entries in bin_a (the histogram itself may be cleared for reuse once the walk is done)
  uint32_t count_b;         // entries in bin_b
  uint32_t pad[2];
};
static_assert(sizeof(Found) == 48, "three 128-bit LDS reads");
constexpr int kFoundWords = sizeof(Found) / 4;

// Walk the 4096-entry LDS histogram (entries the caller does not use are 0) from the highest
// bin down and find, for each of two targets, the bin in which the running count reaches it
// and the count in strictly higher bins.  A target of 0 or beyond the total finds nothing and
// leaves the preset {0, 0}.  The targets may depend on a second block-wide sum: every wave
// reduces `extra`, and `targets(extra_total, need_a, need_b)` turns the total into the targets.
//
// All W waves take part: wave w owns the 4096/W bins below 4096 - (4096/W) w, lane l a run of
// BL = 64/W adjacent bins (128-bit reads), so that (wave, lane, slot) ascending is bin
// descending.  A DPP scan gives the running count inside the wave, the wave totals go through
// LDS and are scanned by every wave; the one lane whose bins contain a target resolves it and
// publishes the result.  Three barriers: the first completes the histogram that the callers
// fill with LDS atomics.  s_extra (W words) is per call site, s_wsum (W words) may be shared by
// all call sites, s_found is per call site and preset to 0.
template <int W, typename Targets>
__device__ inline Found find_bins(const uint32_t* s_hist, uint32_t extra, uint32_t* s_extra, uint32_t* s_wsum,
                                  Found* s_found, Targets&& targets) {
  constexpr int BW = kHistBins / W;  // bins per wave
  constexpr int BL = BW / kWave;     // bins per lane
  static_assert(BL >= 4 && BL % 4 == 0, "whole 128-bit reads per lane");
  const int lane = lane_id();
  const int wave = wave_id();
  const uint32_t extra_incl = wave_incl_scan_u32(extra);
  if (lane == kWave - 1) s_extra[wave] = extra_incl;
  __syncthreads();  // the histogram and s_extra are complete
  const uint32_t bin0 = static_cast<uint32_t>(kHistBins - BW * (wave + 1) + BL * (kWave - 1 - lane));
  uint32_t c[BL];  // ascending bins bin0 .. bin0 + BL - 1
  uint32_t lsum = 0;
#pragma unroll
  for (int i = 0; i < BL / 4; ++i) {
    const uint4 q = *reinterpret_cast<const uint4*>(s_hist + bin0 + 4 * i);
    c[4 * i] = q.x;
    c[4 * i + 1] = q.y;
    c[4 * i + 2] = q.z;
    c[4 * i + 3] = q.w;
    lsum += (q.x + q.y) + (q.z + q.w);
  }
  const uint32_t incl = wave_incl_scan_u32(lsum);
  if (lane == kWave - 1) s_wsum[wave] = incl;
  __syncthreads();
  uint32_t total, extra_total;
  const uint32_t before = wave_entries_scan<W>(s_wsum, total) + incl - lsum;  // count in bins above this lane's
  wave_entries_scan<W>(s_extra, extra_total);
  uint32_t need[2];
  targets(extra_total, need[0], need[1]);
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    if (before < need[t] && need[t] <= before + lsum) {  // at most one thread of the workgroup
      uint32_t run = before, bin = bin0 + BL - 1, cnt = c[BL - 1];
#pragma unroll
      for (int i = BL - 2; i >= 0; --i) {
        if (need[t] > run + cnt) {  // not in this bin: go one down
          run += cnt;
          cnt = c[i];
          --bin;
        }
      }
      if (t == 0) {
        s_found->bin_a = bin;
        s_found->above_a = run;
        s_found->count_a = cnt;
      } else {
        s_found->bin_b = bin;
        s_found->above_b = run;
        s_found->count_b = cnt;
      }
    }
  }
  if (threadIdx.x == 0) {
    s_found->extra_total = extra_total;
    s_found->total = total;
    s_found->need_a = need[0];
    s_found->need_b = need[1];
  }
  __syncthreads();
  return *s_found;
}

// The bracket of top-12-bit bins that a sample of n_s keys (histogram s_hist) gives for the
// kk-th largest of n_cand candidates: the rank of the threshold inside the sample and its
// spread (binomial), in fp32 -- a heuristic only: exact counts decide afterwards whether the
// bracket holds.
template <int W>
__device__ inline void sample_bracket(const uint32_t* s_hist, uint32_t n_valid, uint32_t* s_extra, uint32_t* s_wsum,
                                      Found* s_found, int kk, int64_t n_cand, uint32_t& b_lo, uint32_t& b_hi,
                                      uint32_t* key_lo = nullptr) {
  const Found fb = find_bins<W>(s_hist, n_valid, s_extra, s_wsum, s_found, [&](uint32_t n_s, uint32_t& na, uint32_t& nb) {
    // (hardware reciprocal and square root: approximate, which is all a heuristic needs)
    const float frac = static_cast<float>(kk) * __builtin_amdgcn_rcpf(static_cast<float>(n_cand));
    const float ks_f = frac * static_cast<float>(n_s);
    const float margin = 6.0f * __builtin_amdgcn_sqrtf(ks_f * (1.0f - frac)) + 4.0f;
    const float hi_f = ks_f - margin, lo_f = ks_f + margin;
    na = hi_f < 1.0f ? 0u : static_cast<uint32_t>(hi_f);  // 0: no bin is safely above T
    nb = lo_f >= static_cast<float>(n_s) ? n_s + 1u : static_cast<uint32_t>(lo_f) + 1u;
  });
  b_hi = fb.need_a ? fb.bin_a : (kHistBins - 1);         // top bin of the bracket
  const bool have_lo = fb.need_b <= fb.extra_total && fb.bin_b >= 1u;
  b_lo = have_lo ? fb.bin_b : 1u;                        // bottom bin of the bracket (bin 0 holds only "not a candidate")
  if (b_hi < b_lo) b_hi = b_lo;
  if (key_lo) {
    // A key inside the bottom bin from which up a filter may keep: the bin is a sixteenth of an
    // octave wide, and a distribution that is dense around the threshold puts several times the
    // budget into it.  The sample's target rank is its j-th largest entry of count_b; with the
    // bin's entries taken as evenly spread, everything from one spacing below that entry up is
    // kept (a heuristic like the bracket itself: what decides is the exact count afterwards).
    uint32_t lo_key = b_lo << kTopShift;
    if (have_lo && fb.count_b > 0u) {
      const uint32_t j = fb.need_b - fb.above_b;  // 1 .. count_b
      const uint32_t width = 1u << kTopShift;
      const uint32_t below = fb.count_b > j + 1u ? fb.count_b - (j + 1u) : 0u;  // spacings between the bin's lower edge and the cut
      lo_key += static_cast<uint32_t>((static_cast<unsigned long long>(width) * below) / fb.count_b);
    }
    *key_lo = lo_key;
  }
}

// Streamed rows (NT == 0) may keep the keys that fall inside the bracket in LDS, so that only
// two passes read the scores: the bracketed level and the final write-out.
constexpr int kListCap = 16384;
constexpr int kStreamBatch = 8;  // tiles in flight per wave while streaming
constexpr int kMaxLevels = 4;    // bracketed level (possibly repeated once over all bins) + up to 2 levels of low bits

// LDS of one selection (shared by the bodies that run one after the other in a kernel).
template <int W>
struct SelLds {
  uint32_t hist[2][kHistBins];  // alternating: one in use, the other being cleared
  __attribute__((aligned(16))) Found found[kMaxLevels + 1];
  uint32_t part[2][W];
  uint32_t wsum[W];
  uint32_t wgt[W], weq[W];
  uint32_t wabove[W];  // streamed rows: every wave's count of keys above the bracket
  uint32_t nlist;      // streamed rows: keys appended to the list (unusable when beyond its capacity)
  uint32_t ntiny;      // keys gathered from a sparsely populated sub-bin
  uint32_t tiny[kWave];
};
// Streamed rows that keep a list: keys inside the bracket (with the wave whose span they come
// from) and per-(counting wave, owning wave) tallies of kept / tied keys.
template <int W>
struct ListLds {
  uint32_t ckey[kListCap];
  uint8_t cwave[kListCap];
  uint32_t lcnt[W][W][2];
};
// Stage B: where the pieces' kept keys lie in the row that stage B selects on.
struct PieceTab {
  uint32_t start[kMaxPieces];  // position of piece c's first kept key in that row (pieces padded to multiples of 4)
  uint32_t n[kMaxPieces];      // kept keys of piece c
  uint32_t len;                // length of the row
  uint32_t b_lo, b_hi;         // the bracket the pieces agreed on
  uint32_t ok;                 // the row of kept keys can be selected on
};

// STAGE 0: the selection of a row of scores; 2: stage B of a selection by pieces (the row is
// what the pieces kept, read through the piece table).
// W: waves of the workgroup.  NT > 0: the wave's tiles are cached in registers (NT >= tiles per
// wave); NT == 0: the row is streamed again in every phase; with LIST the keys inside the
// bracket are kept in LDS and only two passes read the scores.
// u: the row (b*Hq + h) this workgroup selects for.
template <int W, int NT, int STAGE, bool LIST>
__device__ __forceinline__ void select_body(const SelectArgs& a, const int u, const PieceTab* tab, SelLds<W>& sl,
                                            ListLds<W>* ll) {
  static_assert(!LIST || NT == 0, "only streamed rows keep a list");
  constexpr int kThreads = W * kWave;
  constexpr int kTileElts = W * kWaveTile;  // scores per workgroup-wide tile
  constexpr bool kStream = LIST;
  constexpr bool kStageB = STAGE == 2;
  uint32_t (&s_hist)[2][kHistBins] = sl.hist;
  Found (&s_found)[kMaxLevels + 1] = sl.found;
  uint32_t (&s_part)[2][W] = sl.part;
  uint32_t (&s_wgt)[W] = sl.wgt;
  uint32_t (&s_weq)[W] = sl.weq;
  uint32_t (&s_wabove)[W] = sl.wabove;
  uint32_t& s_nlist = sl.nlist;
  uint32_t* s_ckey = kStream ? ll->ckey : nullptr;
  uint8_t* s_cwave = kStream ? ll->cwave : nullptr;
  uint32_t (*s_lcnt)[W][2] = kStream ? ll->lcnt : nullptr;

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int kk = a.kk;
  // stage B: the row is the concatenation of the pieces' kept keys, every piece padded to a
  // multiple of 4; every key of it is a candidate
  const int64_t N = kStageB ? static_cast<int64_t>(tab->len) : a.N;
  const int lo = kStageB ? 0 : a.lo, hi = kStageB ? static_cast<int>(N) : a.hi;
  const float* s = a.scores + static_cast<int64_t>(u) * a.score_stride;
  int32_t* out = a.idx + static_cast<int64_t>(u) * a.idx_cap;
  // stage B: as many tiles per wave as the row needs (its length is not known at launch)
  const int tpw_b = static_cast<int>((N + kTileElts - 1) / kTileElts);
  const int tpw = (NT > 0) ? (kStageB ? (tpw_b < 1 ? 1 : (tpw_b < NT ? tpw_b : NT)) : NT) : a.tiles_per_wave;
  const int64_t wbase = static_cast<int64_t>(wave) * tpw * kWaveTile + lane * 4;
  const bool refine = kk > 0 && kk < hi - lo;
  const int64_t last4 = N > 0 ? ((N - 1) & ~int64_t{3}) : 0;  // the vector that holds the last score
  uint32_t keys[NT > 0 ? NT : 1][4];
  int32_t cidx[(kStageB && NT > 0) ? NT : 1][4];  // stage B: positions in the original row
  if (NT > 0 && kk > 0) {
    if constexpr (kStageB) {
      // where position n (a multiple of 4) of the row lies in the [piece][cap] arrays, and how
      // many of the four keys from there on are real (the rest is padding)
      const uint32_t* ckeys = a.cand_key + static_cast<int64_t>(u) * a.pieces * a.cap;
      const int32_t* cpos = a.cand_idx + static_cast<int64_t>(u) * a.pieces * a.cap;
      uint4 rk[NT], ri[NT];
      int valid[NT];
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int64_t n0 = wbase + j * kWaveTile;
        valid[j] = 0;
        int64_t phys = 0;
        if (j < tpw && n0 < N) {
          int c = 0;  // the last piece that starts at or before n0 (binary search over the starts)
#pragma unroll
          for (int step = kMaxPieces / 2; step >= 1; step >>= 1)
            if (c + step < a.pieces && static_cast<int64_t>(tab->start[c + step]) <= n0) c += step;
          const int64_t off = n0 - tab->start[c];
          valid[j] = static_cast<int>(tab->n[c]) - static_cast<int>(off);
          phys = c * a.cap + off;
        }
        rk[j] = *reinterpret_cast<const uint4*>(ckeys + phys);
        ri[j] = *reinterpret_cast<const uint4*>(cpos + phys);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const uint32_t kv[4] = {rk[j].x, rk[j].y, rk[j].z, rk[j].w};
        const uint32_t iv[4] = {ri[j].x, ri[j].y, ri[j].z, ri[j].w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          keys[j][c] = c < valid[j] ? kv[c] : 0u;
          cidx[(kStageB && NT > 0) ? j : 0][c] = static_cast<int32_t>(iv[c]);
        }
      }
    } else {
      float4 raw[NT > 0 ? NT : 1];  // every load of the thread is issued before the first is used
#pragma unroll
      for (int j = 0; j < NT; ++j) raw[j] = load_scores4(s, last4, wbase + j * kWaveTile);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int j = 0; j < NT; ++j) keys_of4(raw[j], lo, hi, wbase + j * kWaveTile, keys[j]);
    }
  }
  for (int i = tid; i < 2 * kHistBins; i += kThreads) (&s_hist[0][0])[i] = 0;
  for (int i = tid; i < (kMaxLevels + 1) * kFoundWords; i += kThreads) reinterpret_cast<uint32_t*>(&s_found[0])[i] = 0;
  if (tid == 0) {
    s_nlist = 0;
    sl.ntiny = 0;
  }

  // always-kept ranges: sink prefix [0, lo) and local window [hi, N) of the original row (in
  // stage B these are the ranges of the original row: a.lo, a.hi, a.N).  Written last: a global
  // store that is still on its way would hold up the first barrier of the selection.
  auto write_fixed_ranges = [&]() {
    for (int64_t n = tid; n < a.lo; n += kThreads) out[n] = static_cast<int32_t>(n);
    for (int64_t n = a.hi + tid; n < a.N; n += kThreads) out[a.lo + kk + (n - a.hi)] = static_cast<int32_t>(n);
    if (tid == 0) a.count[u] = static_cast<int32_t>(a.lo + kk + (a.N - a.hi));
  };
  int32_t* sel_out = out + a.lo;
  if (kk == 0) {
    write_fixed_ranges();
    return;
  }

  // visit every tile of this wave's span: body(j, keys of the tile)
  auto for_each_tile = [&](auto&& body) {
    if constexpr (NT > 0) {
#pragma unroll
      for (int j = 0; j < NT; ++j)
        if (!kStageB || j < tpw) body(j, keys[j]);
    } else {
      // streamed: the loads of kStreamBatch tiles are issued before the first tile is used (one
      // load per iteration would leave a wave with 1 KiB in flight and the pass latency-bound)
      for (int j0 = 0; j0 < tpw; j0 += kStreamBatch) {
        float4 raw[kStreamBatch];
#pragma unroll
        for (int t = 0; t < kStreamBatch; ++t)  // tiles past the wave's span read a clamped address and are dropped
          raw[t] = load_scores4(s, last4, wbase + static_cast<int64_t>(j0 + t) * kWaveTile);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < kStreamBatch; ++t) {
          if (j0 + t < tpw) {
            uint32_t k4[4];
            keys_of4(raw[t], lo, hi, wbase + static_cast<int64_t>(j0 + t) * kWaveTile, k4);
            body(j0 + t, k4);
          }
        }
      }
    }
  };

  uint32_t T = 0;        // threshold key: everything above is kept
  uint32_t r_eq = 0;     // how many keys equal to T are kept (lowest indices first)
  bool list_ok = false;  // streamed rows: the LDS list holds every key inside the bracket
  if (refine) {
    __syncthreads();  // LDS initialised
    uint32_t b_lo, b_hi;
    if constexpr (kStageB) {
      // the pieces have already derived the bracket from their sample of the row
      b_lo = tab->b_lo;
      b_hi = tab->b_hi;
    } else {
      // ---- bracket from a sample: one key per thread, the first key of a tile that varies with
      // the lane so that the sample is spread over the wave's span.  (More keys would narrow the
      // bracket a little, but they land in a handful of exponent bins and their LDS atomics
      // serialise.)
      uint32_t n_valid = 0;
      const int st = lane % tpw;  // tile sampled by this lane
      uint32_t ks;
      if constexpr (NT > 0) {
        ks = keys[0][0];
#pragma unroll
        for (int j = 1; j < NT; ++j) ks = (j == st) ? keys[j][0] : ks;
      } else {
        const int64_t n0 = wbase + static_cast<int64_t>(st) * kWaveTile;
        uint32_t k4[4];
        keys_of4(load_scores4(s, last4, n0), lo, hi, n0, k4);
        ks = k4[0];
      }
      if (ks) {
        atomicAdd(&s_hist[0][ks >> kTopShift], 1u);
        n_valid = 1;
      }
      sample_bracket<W>(s_hist[0], n_valid, s_part[0], sl.wsum, &s_found[0], kk, hi - lo, b_lo, b_hi);
    }

    // ---- radix descent.  Level state: candidates are the keys with lo_key <= key < lo_key +
    // span, histogrammed by (key - lo_key) >> shift; keys above `above_key` (only on the
    // first, bracketed level) are counted instead.  If the exact counts of the first level
    // show that T is not inside the bracket, the level is repeated over every real bin.
    uint32_t lo_key, span, above_key, need = static_cast<uint32_t>(kk);
    int shift;
    {
      const uint32_t nb = b_hi - b_lo + 1;                         // 12-bit bins in the bracket
      const int e = 31 - __clz(static_cast<int>(kHistBins / nb));  // extra bits of resolution
      shift = kTopShift - e;
      lo_key = b_lo << kTopShift;
      span = nb << kTopShift;
      above_key = (b_hi == kHistBins - 1) ? 0xFFFFFFFFu : ((b_hi + 1) << kTopShift) - 1u;
    }
    int cur = 1;  // s_hist[cur] is clear and becomes this level's histogram
    bool dense_level = true;
    bool take_whole_bin = false;
#pragma nounroll
    for (int call = 1; call <= kMaxLevels; ++call) {
      uint32_t* h = s_hist[cur];
      uint32_t n_above = 0;
      if (kStream && call == 1) {
        // the bracketed level of a streamed row: as the dense level below, and the keys inside
        // the bracket are appended to the LDS list (one slot reservation per wave tile)
        for_each_tile([&](int, const uint32_t(&k4)[4]) {
          uint32_t d[4], nin = 0;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            d[c] = k4[c] - lo_key;
            n_above += (k4[c] > above_key) ? 1u : 0u;
            if (d[c] < span) {
              atomicAdd(&h[d[c] >> shift], 1u);
              ++nin;
            }
          }
          const uint32_t incl = wave_incl_scan_u32(nin);
          const uint32_t tot = __builtin_amdgcn_readlane(incl, kWave - 1);
          if (tot) {
            uint32_t base = 0;
            if (lane == kWave - 1) base = atomicAdd(&s_nlist, tot);
            uint32_t pos = __builtin_amdgcn_readlane(base, kWave - 1) + incl - nin;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              if (d[c] < span) {
                if (pos < static_cast<uint32_t>(kListCap)) {
                  s_ckey[kStream ? pos : 0] = k4[c];
                  s_cwave[kStream ? pos : 0] = static_cast<uint8_t>(wave);
                }
                ++pos;
              }
            }
          }
        });
      } else if (dense_level) {
        // a sizeable share of the keys falls into the range: test every key on its own.
        // (key > above_key implies key - lo_key >= span, so the two cases are disjoint.)
        for_each_tile([&](int, const uint32_t(&k4)[4]) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t d = k4[c] - lo_key;  // wraps to a large value for keys below lo_key
            n_above += (k4[c] > above_key) ? 1u : 0u;
            if (d < span) atomicAdd(&h[d >> shift], 1u);
          }
        });
      } else if (kStream && list_ok) {
        // streamed row: the keys of the chosen sub-bin are all in the LDS list
        const uint32_t nl = s_nlist;
        for (uint32_t i = tid; i < nl; i += kThreads) {
          const uint32_t d = s_ckey[kStream ? i : 0] - lo_key;
          if (d < span) atomicAdd(&h[d >> shift], 1u);
        }
      } else {
        // only the handful of keys of one sub-bin take part: skip wave-uniformly
        for_each_tile([&](int, const uint32_t(&k4)[4]) {
          const uint32_t d0 = k4[0] - lo_key, d1 = k4[1] - lo_key, d2 = k4[2] - lo_key, d3 = k4[3] - lo_key;
          const uint32_t dmin = min(min(d0, d1), min(d2, d3));
          if (__any(dmin < span)) {
            if (d0 < span) atomicAdd(&h[d0 >> shift], 1u);
            if (d1 < span) atomicAdd(&h[d1 >> shift], 1u);
            if (d2 < span) atomicAdd(&h[d2 >> shift], 1u);
            if (d3 < span) atomicAdd(&h[d3 >> shift], 1u);
          }
        });
      }
      // clear the other histogram for the next level while this one is being filled
      for (int i = tid; i < kHistBins; i += kThreads) s_hist[cur ^ 1][i] = 0;
      const Found f = find_bins<W>(h, n_above, s_part[call & 1], sl.wsum, &s_found[call],
                                   [&](uint32_t c_above, uint32_t& na, uint32_t& nb) {
                                     na = (c_above < need) ? need - c_above : 0u;
                                     nb = 0u;
                                   });
      const uint32_t want = f.need_a, total_in = f.total;
      if (kStream && call == 1) {
        list_ok = s_nlist <= static_cast<uint32_t>(kListCap);
        if (tid < W) s_wabove[tid] = s_part[1][tid];  // per-wave counts of keys above the bracket
      }
      cur ^= 1;
      if (want >= 1u && want <= total_in) {  // T lies inside this level's range: descend
        lo_key += f.bin_a << shift;
        need = want - f.above_a;
        if (need == f.count_a) {
          // every key of this sub-bin is needed: no reason to look at its low bits
          take_whole_bin = true;
          break;
        }
        if (shift == 0) break;
        if (NT > 0 && f.count_a <= static_cast<uint32_t>(kWave)) {
          // A handful of keys share the sub-bin (the usual case after the bracketed level: its
          // sub-bins are a few thousand key values wide): instead of another histogram level,
          // gather them -- one lane each -- and rank them against each other in every wave.
          const uint32_t sub = 1u << shift;
          for_each_tile([&](int, const uint32_t(&k4)[4]) {
            const uint32_t d0 = k4[0] - lo_key, d1 = k4[1] - lo_key, d2 = k4[2] - lo_key, d3 = k4[3] - lo_key;
            const uint32_t dmin = min(min(d0, d1), min(d2, d3));
            if (__any(dmin < sub)) {
#pragma unroll
              for (int c = 0; c < 4; ++c)
                if (k4[c] - lo_key < sub) sl.tiny[atomicAdd(&sl.ntiny, 1u)] = k4[c];
            }
          });
          __syncthreads();
          const int n_tiny = static_cast<int>(f.count_a);
          const uint32_t mine = lane < n_tiny ? sl.tiny[lane] : 0u;
          uint32_t greater = 0, equal = 0;
          for (int j = 0; j < n_tiny; ++j) {
            const uint32_t other = __builtin_amdgcn_readlane(mine, j);
            greater += other > mine ? 1u : 0u;
            equal += other == mine ? 1u : 0u;
          }
          // the key whose ranks (greater, greater + equal] contain `need` is the threshold
          const unsigned long long hit = __ballot(lane < n_tiny && greater < need && need <= greater + equal);
          const int L = __ffsll(hit) - 1;  // (several lanes when the threshold value repeats: they agree)
          lo_key = static_cast<uint32_t>(__builtin_amdgcn_readlane(mine, L));
          need -= static_cast<uint32_t>(__builtin_amdgcn_readlane(greater, L));
          if (need == static_cast<uint32_t>(__builtin_amdgcn_readlane(equal, L))) take_whole_bin = true;  // every key equal to it is kept
          break;
        }
        const int nshift = shift > 12 ? shift - 12 : 0;
        span = 1u << shift;
        shift = nshift;
        above_key = 0xFFFFFFFFu;
        dense_level = false;
      } else {
        // the sample misled us (possible on the bracketed level only): widen to every real
        // bin and count again.  Bin 0 holds only "not a candidate".
        lo_key = 1u << kTopShift;
        span = static_cast<uint32_t>(kHistBins - 1) << kTopShift;
        shift = kTopShift;
        above_key = 0xFFFFFFFFu;
        list_ok = false;
      }
    }
    T = lo_key;
    r_eq = need;
    if (take_whole_bin) {  // keep everything from the start of the sub-bin upwards
      T = lo_key - 1u;
      r_eq = 0u;
    }
  }
  // kk == hi - lo: T = 0 keeps every candidate (all real keys are > 0)

  // ---- ordered compaction.  Pass A: prefix of {key > T} (low half) and {key == T} (high
  // half) inside each wave tile, and the wave's totals.  TIES == false: no key equal to T has
  // to be cut (r_eq == 0: every kept key is > T), so the equal-to-T bookkeeping is left out.
  auto compact = [&](auto ties_tag) {
    constexpr bool TIES = decltype(ties_tag)::value;
    auto tile_count = [&](const uint32_t(&k4)[4]) {
      uint32_t cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        cnt += k4[c] > T ? 1u : 0u;
        if (TIES) cnt += (k4[c] == T) ? 0x10000u : 0u;
      }
      return cnt;
    };
    if constexpr (!TIES && NT > 0) {
      // Keys in registers and no tie to cut: the lane masks of the compares (scalar registers)
      // give the counts (bit counts, scalar) and the positions (mask counts below the lane).
      uint32_t run = 0;
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if (kStageB && j >= tpw) break;
        run += popc64(__ballot(keys[j][0] > T)) + popc64(__ballot(keys[j][1] > T)) + popc64(__ballot(keys[j][2] > T)) +
               popc64(__ballot(keys[j][3] > T));
      }
      if (lane == 0) s_wgt[wave] = run;
      __syncthreads();
      uint32_t unused;
      uint32_t at = wave_entries_scan<W>(s_wgt, unused);  // kept keys of the waves and tiles before
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if (kStageB && j >= tpw) break;
        const bool t0 = keys[j][0] > T, t1 = keys[j][1] > T, t2 = keys[j][2] > T, t3 = keys[j][3] > T;
        const unsigned long long m0 = __ballot(t0), m1 = __ballot(t1), m2 = __ballot(t2), m3 = __ballot(t3);
        const uint32_t tot = popc64(m0) + popc64(m1) + popc64(m2) + popc64(m3);
        if (at + tot <= static_cast<uint32_t>(kk)) {  // (always, when the counts above add up)
          int32_t* o = sel_out + at + mbcnt64(m3, mbcnt64(m2, mbcnt64(m1, mbcnt64(m0, 0u))));
          const int32_t nn = static_cast<int32_t>(wbase) + j * kWaveTile;
          if (t0) *o++ = kStageB ? cidx[(kStageB && NT > 0) ? j : 0][0] : nn;
          if (t1) *o++ = kStageB ? cidx[(kStageB && NT > 0) ? j : 0][1] : nn + 1;
          if (t2) *o++ = kStageB ? cidx[(kStageB && NT > 0) ? j : 0][2] : nn + 2;
          if (t3) *o = kStageB ? cidx[(kStageB && NT > 0) ? j : 0][3] : nn + 3;
        }
        at += tot;
      }
      return;
    }
    constexpr bool kKeepPre = NT > 0 && NT <= 8;  // keep the in-tile prefixes when registers allow
    uint32_t pre[kKeepPre ? NT : 1];
    if (kStream && list_ok) {
      // streamed row: the per-wave totals come from the list instead of another pass over the
      // scores (a key above the bracket is kept for sure; a key below it never is)
      for (int i = tid; i < (kStream ? W : 1) * W * 2; i += kThreads) (&s_lcnt[0][0][0])[i] = 0;
      __syncthreads();
      const uint32_t nl = s_nlist;
      for (uint32_t i = tid; i < nl; i += kThreads) {
        const uint32_t key = s_ckey[kStream ? i : 0];
        const uint32_t w = s_cwave[kStream ? i : 0];
        if (key > T) {
          atomicAdd(&s_lcnt[kStream ? wave : 0][w][0], 1u);
        } else if (key == T) {
          atomicAdd(&s_lcnt[kStream ? wave : 0][w][1], 1u);
        }
      }
      __syncthreads();
      if (tid < W) {
        uint32_t gt = s_wabove[tid], eq = 0;
        for (int cw = 0; cw < (kStream ? W : 1); ++cw) {
          gt += s_lcnt[cw][tid][0];
          eq += s_lcnt[cw][tid][1];
        }
        s_wgt[tid] = gt;
        s_weq[tid] = eq;
      }
    } else {
      uint32_t run_gt = 0, run_eq = 0;
      for_each_tile([&](int j, const uint32_t(&k4)[4]) {
        const uint32_t cnt = tile_count(k4);
        const uint32_t incl = wave_incl_scan_u32(cnt);
        if (kKeepPre) pre[kKeepPre ? j : 0] = incl - cnt;
        const uint32_t tot = __builtin_amdgcn_readlane(incl, kWave - 1);
        run_gt += tot & 0xFFFFu;
        run_eq += tot >> 16;
      });
      if (lane == 0) {
        s_wgt[wave] = run_gt;
        s_weq[wave] = run_eq;
      }
    }
    __syncthreads();
    // kept / tied keys in the spans of the waves before this one
    uint32_t unused_total;
    uint32_t base_gt = wave_entries_scan<W>(s_wgt, unused_total);
    uint32_t base_eq = TIES ? wave_entries_scan<W>(s_weq, unused_total) : 0u;

    // Pass B: position of a kept key = (#greater before it) + min(#equal before it, r_eq)
    for_each_tile([&](int j, const uint32_t(&k4)[4]) {
      const uint32_t cnt = tile_count(k4);
      uint32_t excl;
      if (kKeepPre) {
        excl = pre[kKeepPre ? j : 0];
      } else {
        excl = wave_incl_scan_u32(cnt) - cnt;
      }
      const uint32_t tot = __builtin_amdgcn_readlane(excl + cnt, kWave - 1);
      uint32_t gt_before = base_gt + (excl & 0xFFFFu);
      uint32_t eq_before = base_eq + (excl >> 16);
      const int32_t nn = static_cast<int32_t>(wbase + static_cast<int64_t>(j) * kWaveTile);
      auto emit = [&](uint32_t pos, int c) {
        if (pos < static_cast<uint32_t>(kk)) sel_out[pos] = kStageB ? cidx[(kStageB && NT > 0) ? j : 0][c] : nn + c;
      };
      if (!TIES || (tot >> 16) == 0) {
        // no key of this wave tile equals T: the tie count is the same for every slot
        uint32_t pos = gt_before + (TIES ? (eq_before < r_eq ? eq_before : r_eq) : 0u);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (k4[c] > T) {
            emit(pos, c);
            ++pos;
          }
        }
      } else {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          const bool gt = k4[c] > T;
          const bool eq = k4[c] == T;
          if (gt || (eq && eq_before < r_eq)) emit(gt_before + (eq_before < r_eq ? eq_before : r_eq), c);
          gt_before += gt ? 1u : 0u;
          eq_before += eq ? 1u : 0u;
        }
      }
      base_gt += tot & 0xFFFFu;
      base_eq += tot >> 16;
    });
  };
  if (r_eq != 0)
    compact(std::true_type{});
  else
    compact(std::false_type{});
  write_fixed_ranges();
}

// ---- moving the scores at or above a bound into a list, with few instructions per score ----------
// A SIMD issues about one instruction in four cycles whatever its kind, so a pass over a row
// costs what it spends per score.  This pass spends one floating-point compare per score (the
// lane masks of a wave tile's four compares stay in scalar registers), eight mask-count
// instructions per tile for the number of entries in lower lanes, and per score one store of
// (score bits, position) -- to the next free slot of the wave's region in LDS, or to a spare
// slot of the lane when the score is below the bound, instead of a branch.  The regions hold
// their entries in position order.
template <int W, int NT, int CAP_PER_TILE>
struct RegionLds {
  static constexpr int kCap = NT * CAP_PER_TILE;  // entries per wave (a tile has 256 scores)
  // The waves' regions one after the other, then one spare slot per lane.  pos mirrors key at a
  // fixed distance, so that one instruction writes both.  A wave with more entries than its
  // region holds runs on into what follows -- the caller then discards the list, but the stores
  // must stay inside the arrays: the last wave's can reach NT * 256 - kCap entries past its
  // region, which `spill` covers.
  uint32_t key[W * kCap + kWave];  // raw score bits
  int32_t pos[W * kCap + kWave];   // position in the row
  uint32_t spill[NT * kWaveTile - kCap];
  uint32_t cnt[W];
};

// Smallest score whose key is `key` (a key that a real score produces).
__device__ inline float score_of_key(uint32_t key) {
  return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}
constexpr uint32_t kKeyOfMinusInf = 0x007FFFFFu;

// Appends the candidates (positions in [lo, hi)) among the wave's NT tiles `raw` -- tile j holds
// the positions pos0 + 256 j + 4 lane .. + 3 -- whose score is at least f_lo (`all`: every
// candidate, NaN included) to the wave's region, and returns their number, the same in every
// lane; beyond RegionLds::kCap the region has overflowed.
template <int W, int NT, int CPT>
__device__ __forceinline__ uint32_t append_at_least(const float4 (&raw)[NT], const int pos0, const int lo, const int hi,
                                                    const float f_lo, const bool all, RegionLds<W, NT, CPT>& rl, const int wave,
                                                    const int lane) {
  using R = RegionLds<W, NT, CPT>;
  constexpr int kCap = R::kCap;
  constexpr int kPosOff = static_cast<int>(sizeof(rl.key) / 4);  // pos[i] is key[i + kPosOff]
  static_assert(offsetof(R, pos) == sizeof(rl.key), "pos follows key");
  static_assert(offsetof(R, spill) == offsetof(R, pos) + sizeof(rl.pos), "the spill area follows pos");
  uint32_t* const lkey = rl.key + wave * kCap;
  uint32_t* const spare = rl.key + W * kCap + lane;
  uint32_t run = 0;
  auto append = [&](int j, bool t0, bool t1, bool t2, bool t3) {
    const float v0 = raw[j].x, v1 = raw[j].y, v2 = raw[j].z, v3 = raw[j].w;
    const int p0 = pos0 + j * kWaveTile + lane * 4;
    const unsigned long long m0 = __ballot(t0), m1 = __ballot(t1), m2 = __ballot(t2), m3 = __ballot(t3);
    uint32_t* w = lkey + run + mbcnt64(m3, mbcnt64(m2, mbcnt64(m1, mbcnt64(m0, 0u))));  // after the entries of lower lanes and earlier tiles
    uint32_t* d;
    d = t0 ? w : spare;
    d[0] = __float_as_uint(v0);
    d[kPosOff] = static_cast<uint32_t>(p0);
    w += t0 ? 1 : 0;
    d = t1 ? w : spare;
    d[0] = __float_as_uint(v1);
    d[kPosOff] = static_cast<uint32_t>(p0 + 1);
    w += t1 ? 1 : 0;
    d = t2 ? w : spare;
    d[0] = __float_as_uint(v2);
    d[kPosOff] = static_cast<uint32_t>(p0 + 2);
    w += t2 ? 1 : 0;
    d = t3 ? w : spare;
    d[0] = __float_as_uint(v3);
    d[kPosOff] = static_cast<uint32_t>(p0 + 3);
    run += popc64(m0) + popc64(m1) + popc64(m2) + popc64(m3);  // (scalar instructions)
  };
  if (pos0 >= lo && pos0 + NT * kWaveTile <= hi) {  // the usual case: every score of the wave's span is a candidate
#pragma unroll
    for (int j = 0; j < NT; ++j) append(j, all || raw[j].x >= f_lo, all || raw[j].y >= f_lo, all || raw[j].z >= f_lo, all || raw[j].w >= f_lo);
  } else {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n_t = pos0 + j * kWaveTile;
      if (n_t >= hi || n_t + kWaveTile <= lo) continue;
      const int p0 = n_t + lane * 4;
      append(j, (all || raw[j].x >= f_lo) && p0 >= lo && p0 < hi, (all || raw[j].y >= f_lo) && p0 + 1 >= lo && p0 + 1 < hi,
             (all || raw[j].z >= f_lo) && p0 + 2 >= lo && p0 + 2 < hi, (all || raw[j].w >= f_lo) && p0 + 3 >= lo && p0 + 3 < hi);
    }
  }
  return run;
}

constexpr int kSelWaves = 16;  // one workgroup per row
constexpr int kSelThreads = kSelWaves * kWave;

template <int NT>
__global__ __launch_bounds__(kSelThreads, (NT >= 1 && NT <= 4) ? 8 : 4) void select_kernel(SelectArgs a) {
  __shared__ SelLds<kSelWaves> sl;
  if constexpr (NT == 0) {
    __shared__ ListLds<kSelWaves> ll;
    select_body<kSelWaves, 0, 0, true>(a, blockIdx.x, nullptr, sl, &ll);
  } else {
    select_body<kSelWaves, NT, 0, false>(a, blockIdx.x, nullptr, sl, nullptr);
  }
}

// ---- selection of a row by pieces, stage A.  The piece's scores are in registers (NT tiles per
// wave).  Every piece of a row takes the same sample of the row's candidates (one 128-bit load
// per thread at positions spread evenly over [lo, hi)) and so arrives at the same bracket as its
// siblings.  The scores whose keys are at or above the bracket's lower end are kept, in position
// order: collected per wave in LDS, then copied out behind the entries of the waves before.
constexpr int kPieceCapPerTile = 56;  // a wave's region holds 22% of its span: several times what a piece keeps
template <int W, int NT>
struct PieceLds {
  uint32_t hist[kHistBins];
  __attribute__((aligned(16))) Found found;
  uint32_t part[W], wsum[W];
  RegionLds<W, NT, kPieceCapPerTile> reg;
};

template <int W, int NT>
__device__ __forceinline__ void piece_body(const SelectArgs& a, const int u, const int c, PieceLds<W, NT>& pl) {
  constexpr int kThreads = W * kWave;
  constexpr int kCap = RegionLds<W, NT, kPieceCapPerTile>::kCap;
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int64_t base = c * a.piece_len;
  int64_t n_c = a.N - base;
  n_c = n_c < 0 ? 0 : (n_c > a.piece_len ? a.piece_len : n_c);
  const float* row = a.scores + static_cast<int64_t>(u) * a.score_stride;
  const float* s = row + base;
  const int last4 = n_c > 0 ? static_cast<int>((n_c - 1) & ~int64_t{3}) : 0;
  const int wspan0 = wave * NT * kWaveTile;  // the wave's span, as positions inside the piece
  // the sample of the whole row: four adjacent scores at each of `kThreads` positions spread
  // evenly over the candidates
  const int64_t span = a.hi - a.lo;
  const int64_t sp = (a.lo + (tid * span) / kThreads) & ~int64_t{3};
  const int64_t row_last4 = (a.N - 1) & ~int64_t{3};
  float4 raw[NT];
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n0 = wspan0 + j * kWaveTile + lane * 4;
    raw[j] = *reinterpret_cast<const float4*>(s + (n0 < last4 ? n0 : last4));  // (past the piece's end: excluded by position below)
  }
  const float4 sraw = load_scores4(row, row_last4, sp);
  __builtin_amdgcn_sched_barrier(0);

  {
    uint4* z = reinterpret_cast<uint4*>(pl.hist);
    for (int i = tid; i < kHistBins / 4; i += kThreads) z[i] = make_uint4(0u, 0u, 0u, 0u);
  }
  if (tid < kFoundWords) reinterpret_cast<uint32_t*>(&pl.found)[tid] = 0;
  __syncthreads();
  uint32_t n_valid = 0;
  {
    uint32_t sk[4];
    keys_of4(sraw, a.lo, a.hi, sp, sk);  // (the four may straddle an end of the candidate range)
    // all four enter the histogram: a narrower bracket means fewer kept keys to store and to
    // select among
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (sk[i]) {
        atomicAdd(&pl.hist[sk[i] >> kTopShift], 1u);
        ++n_valid;
      }
    }
  }
  uint32_t b_lo, b_hi, t_lo;  // t_lo: keys from here up are kept (inside the bracket's bottom bin)
  sample_bracket<W>(pl.hist, n_valid, pl.part, pl.wsum, &pl.found, a.kk, span, b_lo, b_hi, &t_lo);
  // a score is kept when it is at least f_lo; a lower end at or below the key of -inf keeps
  // every candidate (NaN, whose key is that of -inf, included)
  const bool all = t_lo <= kKeyOfMinusInf;
  const float f_lo = all ? 0.f : score_of_key(t_lo);

  // positions are those of the whole row; candidates past the piece's end do not exist (the
  // last piece ends with the row, and hi <= N)
  const int pos0 = static_cast<int>(base) + wspan0;
  const uint32_t run = append_at_least<W, NT>(raw, pos0, a.lo, a.hi, f_lo, all, pl.reg, wave, lane);
  if (lane == 0) pl.reg.cnt[wave] = run;
  __syncthreads();
  uint32_t total;
  const uint32_t wave_base = wave_entries_scan<W>(pl.reg.cnt, total);
  const int l16 = lane & 15;
  const bool overflowed = __ballot(l16 < W && pl.reg.cnt[l16 < W ? l16 : 0] > static_cast<uint32_t>(kCap)) != 0ull;
  int32_t* out_idx = a.cand_idx + (static_cast<int64_t>(u) * a.pieces + c) * a.cap;
  uint32_t* out_key = a.cand_key + (static_cast<int64_t>(u) * a.pieces + c) * a.cap;
  uint32_t* hdr = a.piece_hdr + (static_cast<int64_t>(u) * a.pieces + c) * 4;
  if (!overflowed) {
    if (tid < 3) hdr[tid] = tid == 0 ? total : (tid == 1 ? b_lo : b_hi);
    const uint32_t* lkey = pl.reg.key + wave * kCap;
    const int32_t* lpos = pl.reg.pos + wave * kCap;
    for (uint32_t e = lane; e < run; e += kWave) {
      const uint32_t at = wave_base + e;
      if (at < static_cast<uint32_t>(a.cap)) {
        out_idx[at] = lpos[e];
        out_key[at] = score_key(__uint_as_float(lkey[e]));
      }
    }
    return;
  }

  // A wave of this piece holds more kept scores than its region (a dense cluster of large
  // scores).  The counts of the pass above are right all the same, so every wave knows where
  // its kept scores go: they are stored from the registers, positions from the compare masks.
  uint32_t at = wave_base;  // kept scores of the waves and tiles before (the same in every lane)
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n_t = pos0 + j * kWaveTile;
    if (n_t >= a.hi || n_t + kWaveTile <= a.lo) continue;
    const int p0 = n_t + lane * 4;
    const float v[4] = {raw[j].x, raw[j].y, raw[j].z, raw[j].w};
    bool t[4];
    unsigned long long m[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      t[e] = (all || v[e] >= f_lo) && p0 + e >= a.lo && p0 + e < a.hi;  // (the test of the pass above)
      m[e] = __ballot(t[e]);
    }
    uint32_t o = mbcnt64(m[3], mbcnt64(m[2], mbcnt64(m[1], mbcnt64(m[0], at))));
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (t[e]) {
        if (o < static_cast<uint32_t>(a.cap)) {
          out_idx[o] = p0 + e;
          out_key[o] = score_key(v[e]);
        }
        ++o;
      }
    }
    at += popc64(m[0]) + popc64(m[1]) + popc64(m[2]) + popc64(m[3]);
  }
  if (tid < 3) hdr[tid] = tid == 0 ? total : (tid == 1 ? b_lo : b_hi);
}

// ---- stage B.  One workgroup per row: builds the table of the pieces' kept keys and selects
// among them, or -- when the pieces kept fewer than kk keys, one of them ran out of room, or they
// kept more than this instance holds in registers -- selects on the original row (one streaming
// workgroup: slow, but it only happens when the sample of stage A was wildly unrepresentative).
template <int NT>
__global__ __launch_bounds__(kSelThreads, 4) void stage_b_kernel(SelectArgs a) {
  constexpr int W = kSelWaves;
  __shared__ SelLds<W> sl;
  __shared__ ListLds<W> ll;
  __shared__ PieceTab tab;
  __shared__ uint32_t s_scan[2][W + 1];
  const int tid = threadIdx.x;
  const int u = blockIdx.x;
  const uint32_t* hdr = a.piece_hdr + static_cast<int64_t>(u) * a.pieces * 4;
  uint32_t n = 0;
  if (tid < a.pieces) n = hdr[tid * 4];
  const uint32_t padded = (n + 3u) & ~3u;
  uint32_t len, kept;
  const uint32_t start = block_excl_scan<W>(padded, s_scan[0], len);
  block_excl_scan<W>(n, s_scan[1], kept);
  const int over = __syncthreads_or(n > static_cast<uint32_t>(a.cap));
  if (tid < kMaxPieces) {
    tab.start[tid] = start;
    tab.n[tid] = n;
  }
  if (tid == 0) {
    tab.len = len;
    tab.b_lo = hdr[1];
    tab.b_hi = hdr[2];
    tab.ok = (!over && len <= static_cast<uint32_t>(NT * W * kWaveTile) && kept >= static_cast<uint32_t>(a.kk)) ? 1u : 0u;
  }
  __syncthreads();
  if (tab.ok) {
    select_body<W, NT, 2, false>(a, u, &tab, sl, nullptr);
  } else {
    select_body<W, 0, 0, true>(a, u, nullptr, sl, &ll);
  }
}

// Stage A.  All pieces of a row run on one XCD (workgroups go to the eight XCDs round-robin by
// their linear index), close together in time: the sample of the row that every piece takes is
// then served by that XCD's L2, out of the lines that the row's pieces fetch anyway.
template <int W, int NT>
__global__ __launch_bounds__(W * kWave) void prefilter_kernel(SelectArgs a) {
  __shared__ PieceLds<W, NT> sl;
  const int64_t xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int64_t u = (slot / a.pieces) * 8 + xcd;
  if (u >= a.units) return;  // (the launch is padded to a multiple of eight rows)
  // the pieces of a row from its end backwards: with scores that favour recent positions the
  // last pieces keep the most and take the longest, so they should not be the last to start
  piece_body<W, NT>(a, static_cast<int>(u), a.pieces - 1 - static_cast<int>(slot % a.pieces), sl);
}

template <int W>
tb_status launch_prefilter_w(const SelectArgs& a, int tiles, dim3 grid, hipStream_t st) {
  const dim3 block(W * kWave);
  if (tiles <= 2)
    hipLaunchKernelGGL((prefilter_kernel<W, 2>), grid, block, 0, st, a);
  else if (tiles <= 4)
    hipLaunchKernelGGL((prefilter_kernel<W, 4>), grid, block, 0, st, a);
  else if (tiles <= 8)
    hipLaunchKernelGGL((prefilter_kernel<W, 8>), grid, block, 0, st, a);
  else
    hipLaunchKernelGGL((prefilter_kernel<W, 16>), grid, block, 0, st, a);
  return hip_status(hipGetLastError());
}

tb_status launch_whole(const SelectArgs& a, int64_t units, hipStream_t st) {
  SelectArgs b = a;
  const int32_t tiles = static_cast<int32_t>((a.N + kSelWaves * kWaveTile - 1) / (kSelWaves * kWaveTile));  // per wave
  b.tiles_per_wave = tiles;
  dim3 grid(static_cast<unsigned>(units));
  dim3 block(kSelThreads);
  if (tiles <= 1)
    hipLaunchKernelGGL(select_kernel<1>, grid, block, 0, st, b);
  else if (tiles <= 2)
    hipLaunchKernelGGL(select_kernel<2>, grid, block, 0, st, b);
  else if (tiles <= 4)
    hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, st, b);
  else if (tiles <= 8)
    hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, st, b);
  else if (tiles <= 16)
    hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, st, b);
  else
    hipLaunchKernelGGL(select_kernel<0>, grid, block, 0, st, b);
  return hip_status(hipGetLastError());
}

// Second stage over kept keys that are in place (layout of SelectArgs::cand_*).
tb_status launch_stage_b(const SelectLaunch& L, const SelectPlan& plan, hipStream_t st) {
  SelectArgs a;
  a.scores = L.scores;
  a.score_stride = L.score_stride;
  a.N = L.N;
  a.kk = L.kk;
  a.lo = L.lo;
  a.hi = L.hi;
  a.idx = L.idx;
  a.count = L.count;
  a.idx_cap = L.idx_cap;
  const int64_t per_unit = static_cast<int64_t>(plan.pieces) * plan.cap;
  a.pieces = plan.pieces;
  a.piece_len = plan.piece_len;
  a.cap = plan.cap;
  a.units = L.units;
  a.cand_idx = static_cast<int32_t*>(L.scratch);
  a.cand_key = reinterpret_cast<uint32_t*>(a.cand_idx + L.units * per_unit);
  a.piece_hdr = a.cand_key + L.units * per_unit;
  a.tiles_per_wave = static_cast<int32_t>((L.N + kSelWaves * kWaveTile - 1) / (kSelWaves * kWaveTile));  // fall-back on the whole row
  const dim3 grid(static_cast<unsigned>(L.units)), block(kSelThreads);
  if (plan.stage_b_tiles <= 2)
    hipLaunchKernelGGL(stage_b_kernel<2>, grid, block, 0, st, a);
  else if (plan.stage_b_tiles <= 4)
    hipLaunchKernelGGL(stage_b_kernel<4>, grid, block, 0, st, a);
  else if (plan.stage_b_tiles <= 8)
    hipLaunchKernelGGL(stage_b_kernel<8>, grid, block, 0, st, a);
  else  // (more than 65536 kept keys falls back to the whole row inside the kernel)
    hipLaunchKernelGGL(stage_b_kernel<16>, grid, block, 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace

tb_status launch_select(const SelectLaunch& L, hipStream_t st) {
  if (L.units == 0) return TB_OK;
  SelectArgs a;
  a.scores = L.scores;
  a.score_stride = L.score_stride;
  a.N = L.N;
  a.kk = L.kk;
  a.lo = L.lo;
  a.hi = L.hi;
  a.idx = L.idx;
  a.count = L.count;
  a.idx_cap = L.idx_cap;
  a.tiles_per_wave = 0;
  a.pieces = 1;
  a.piece_len = 0;
  a.cap = 0;
  a.units = L.units;
  a.cand_idx = nullptr;
  a.cand_key = nullptr;
  a.piece_hdr = nullptr;
  const SelectPlan plan = L.plan ? *L.plan : select_plan(L.units, L.hi - L.lo, L.N, L.kk);
  if (plan.pieces <= 1 || !L.scratch || L.scratch_bytes < select_scratch_bytes(L.units, plan))
    return launch_whole(a, L.units, st);

  // scratch: kept positions, kept keys ([units][pieces][cap] each), then the pieces' headers
  const int64_t per_unit = static_cast<int64_t>(plan.pieces) * plan.cap;
  a.pieces = plan.pieces;
  a.piece_len = plan.piece_len;
  a.cap = plan.cap;
  a.cand_idx = static_cast<int32_t*>(L.scratch);
  a.cand_key = reinterpret_cast<uint32_t*>(a.cand_idx + L.units * per_unit);
  a.piece_hdr = a.cand_key + L.units * per_unit;
  a.units = L.units;
  const dim3 grid(static_cast<unsigned>((L.units + 7) / 8 * 8 * plan.pieces));
  tb_status rc;
  if (plan.piece_waves == 4)
    rc = launch_prefilter_w<4>(a, plan.piece_tiles, grid, st);
  else if (plan.piece_waves == 8)
    rc = launch_prefilter_w<8>(a, plan.piece_tiles, grid, st);
  else
    rc = launch_prefilter_w<16>(a, plan.piece_tiles, grid, st);
  if (rc != TB_OK) return rc;
  return launch_stage_b(L, plan, st);
}

}  // namespace tb
