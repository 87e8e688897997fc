// Top-k selection under the policy "candidates = [lo, hi); keep the kk largest scores, lowest
// index wins ties; emit ascending".
//
// One 1024-thread workgroup per (b,h).  Wave w owns the contiguous span [w*span, (w+1)*span)
// of the head's scores and keeps their order-preserving 32-bit keys in registers (up to 64
// per thread = 65536 scores; longer rows are streamed again in every phase).  The exact
// threshold key T (the kk-th largest) and the number r of keys equal to T that are still
// needed are found by an MSB-first radix descent over LDS histograms:
//
//   bracket   a 12-bit histogram of a strided SAMPLE of the keys (4 per thread) gives a range of
//             top-12-bit bins [b_lo, b_hi] that contains T unless the sample is wildly
//             unrepresentative (the rank of T in the sample, +- 6 standard deviations);
//   level 1   exact: every key above the bracket is counted, every key inside it goes into a
//             histogram of up to 4096 sub-bins; if the exact counts show that T is NOT inside
//             the bracket, the level is repeated with the bracket widened to all bins (slow
//             path, same result);
//   level 2+  the remaining low bits, 12 at a time, over the few keys of the chosen sub-bin.
//
// Output: {key > T} U {first r keys == T by index} in ascending order.  Positions come from
// prefix sums (DPP scans inside a 256-key wave tile, running totals along the wave's span, 16
// wave totals across the workgroup) -- no atomic slot grabbing, so the result is ordered and
// reproducible.  No global scratch is used.
#include "tb_device.h"
#include "tb_internal.h"

#ifdef TB_PROBE
__device__ unsigned long long tb_probe_buf[64];
#define TB_MARK(i)                                                             \
  do {                                                                         \
    if (blockIdx.x == 0 && threadIdx.x == 0) tb_probe_buf[i] = wall_clock64(); \
  } while (0)
#else
#define TB_MARK(i)
#endif

namespace tb {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kWaveTile = kWave * 4;              // scores per wave tile: one float4 per lane
constexpr int kTileElts = kSelWaves * kWaveTile;  // scores per workgroup-wide tile (4096)
constexpr int kHistBins = 4096;                   // LDS histogram size (12 bits per level)
constexpr int kTopShift = 20;                     // key >> 20 = top 12 bits
constexpr int kPerThread = kHistBins / kSelThreads;

struct SelectArgs {
  const float* scores;
  int64_t score_stride;
  int64_t N;
  int32_t kk, lo, hi;
  int32_t* idx;
  int32_t* count;
  int64_t idx_cap;
  int32_t tiles_per_wave;
};

// Keys of the four consecutive positions n0 .. n0+3 (n0 a multiple of 4).  Positions outside
// the candidate range get key 0 (no real score has a key below 0x007FFFFF).
__device__ inline void load_keys4(const float* s, int64_t N, int lo, int hi, int64_t n0, uint32_t (&key)[4]) {
  float v[4] = {0.f, 0.f, 0.f, 0.f};
  if (n0 + 3 < N) {
    const float4 f = *reinterpret_cast<const float4*>(s + n0);
    v[0] = f.x;
    v[1] = f.y;
    v[2] = f.z;
    v[3] = f.w;
  } else {
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (n0 + c < N) v[c] = s[n0 + c];
  }
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

// Walk an LDS histogram of `nbins` (<= 4096) bins from the highest bin down and report, for
// each of two targets need_a <= need_b, the bin in which the running count reaches it and the
// count in strictly higher bins.  A target beyond the total (or 0) reports nothing and leaves
// the preset {0, 0}.  Results in s_found[0..1] (a) and s_found[2..3] (b); returns the total.
// Two barriers; s_scan (16 words) and s_found (4 words, preset to 0) are per call site.
__device__ inline uint32_t find_bins(const uint32_t* s_hist, int nbins, uint32_t need_a, uint32_t need_b,
                                     uint32_t* s_scan, uint32_t* s_found) {
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  uint32_t v[kPerThread];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const int bin = nbins - 1 - (kPerThread * tid + i);  // thread t owns 4 consecutive bins, descending
    v[i] = bin >= 0 ? s_hist[bin] : 0u;
    sum += v[i];
  }
  const uint32_t incl = wave_incl_scan_u32(sum);
  if (lane == kWave - 1) s_scan[wave] = incl;
  __syncthreads();
  uint32_t run = incl - sum, total = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    const uint32_t t = s_scan[w];
    run += (w < wave) ? t : 0u;
    total += t;
  }
#pragma unroll
  for (int i = 0; i < kPerThread; ++i) {
    const uint32_t bin = static_cast<uint32_t>(nbins - 1 - (kPerThread * tid + i));
    if (run < need_a && need_a <= run + v[i]) {
      s_found[0] = bin;
      s_found[1] = run;
    }
    if (run < need_b && need_b <= run + v[i]) {
      s_found[2] = bin;
      s_found[3] = run;
    }
    run += v[i];
  }
  __syncthreads();
  return total;
}

__device__ inline uint32_t block_sum_u32(uint32_t v, uint32_t* s_part) {
  const uint32_t incl = wave_incl_scan_u32(v);
  if (lane_id() == kWave - 1) s_part[threadIdx.x / kWave] = incl;
  __syncthreads();
  uint32_t total = 0;
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) total += s_part[w];
  return total;
}

constexpr int kMaxLevels = 4;  // bracketed level (possibly repeated once over all bins) + up to 2 levels of low bits

template <int NT>  // NT > 0: the wave's tiles are cached in registers (NT >= tiles per wave);
                   // NT == 0: streamed again in every phase
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a) {
  __shared__ uint32_t s_hist[2][kHistBins];  // alternating: one in use, the other being cleared
  __shared__ uint32_t s_scan[kMaxLevels + 2][kSelWaves];
  __shared__ uint32_t s_found[kMaxLevels + 1][4];
  __shared__ uint32_t s_part[2][kSelWaves];
  __shared__ uint32_t s_wgt[kSelWaves], s_weq[kSelWaves];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int u = blockIdx.x;
  const float* s = a.scores + static_cast<int64_t>(u) * a.score_stride;
  int32_t* out = a.idx + static_cast<int64_t>(u) * a.idx_cap;
  const int lo = a.lo, hi = a.hi, kk = a.kk;
  const int tpw = (NT > 0) ? NT : a.tiles_per_wave;
  const int64_t wbase = static_cast<int64_t>(wave) * tpw * kWaveTile + lane * 4;
  const bool refine = kk > 0 && kk < hi - lo;

  TB_MARK(0);
  uint32_t keys[NT > 0 ? NT : 1][4];
  if (NT > 0 && kk > 0) {
#pragma unroll
    for (int j = 0; j < NT; ++j) load_keys4(s, a.N, lo, hi, wbase + j * kWaveTile, keys[j]);
  }
  for (int i = tid; i < 2 * kHistBins; i += kSelThreads) (&s_hist[0][0])[i] = 0;
  if (tid < (kMaxLevels + 1) * 4) (&s_found[0][0])[tid] = 0;

  // always-kept ranges: sink prefix [0, lo) and local window [hi, N)
  for (int64_t n = tid; n < lo; n += kSelThreads) out[n] = static_cast<int32_t>(n);
  for (int64_t n = hi + tid; n < a.N; n += kSelThreads) out[lo + kk + (n - hi)] = static_cast<int32_t>(n);
  if (tid == 0) a.count[u] = static_cast<int32_t>(lo + kk + (a.N - hi));
  if (kk == 0) return;

  // visit every tile of this wave's span: body(j, keys of the tile)
  auto for_each_tile = [&](auto&& body) {
    if constexpr (NT > 0) {
#pragma unroll
      for (int j = 0; j < NT; ++j) body(j, keys[j]);
    } else {
      for (int j = 0; j < tpw; ++j) {
        uint32_t k4[4];
        load_keys4(s, a.N, lo, hi, wbase + static_cast<int64_t>(j) * kWaveTile, k4);
        body(j, k4);
      }
    }
  };

  uint32_t T = 0;     // threshold key: everything above is kept
  uint32_t r_eq = 0;  // how many keys equal to T are kept (lowest indices first)
  if (refine) {
    __syncthreads();  // LDS initialised
    TB_MARK(1);
    // ---- bracket from a sample: the first key of (up to) four tiles per thread
    constexpr int kSamples = (NT > 0 && NT < 4) ? NT : 4;
    uint32_t n_valid = 0;
#pragma unroll
    for (int i = 0; i < kSamples; ++i) {
      uint32_t ks;
      if constexpr (NT > 0) {
        ks = keys[(i * NT) / kSamples][0];
      } else {
        uint32_t k4[4];
        load_keys4(s, a.N, lo, hi, wbase + static_cast<int64_t>((i * tpw) / kSamples) * kWaveTile, k4);
        ks = k4[0];
      }
      if (ks) {
        atomicAdd(&s_hist[0][ks >> kTopShift], 1u);
        ++n_valid;
      }
    }
    const uint32_t n_s = block_sum_u32(n_valid, s_part[0]);  // barrier inside: the sample histogram is complete
    // rank of the threshold inside the sample and its spread (binomial), in fp32: a heuristic
    // only -- the exact counts of level 1 decide whether the bracket holds
    const float frac = static_cast<float>(kk) / static_cast<float>(hi - lo);
    const float ks_f = frac * static_cast<float>(n_s);
    const float margin = 6.0f * sqrtf(ks_f * (1.0f - frac)) + 4.0f;
    const float hi_f = ks_f - margin, lo_f = ks_f + margin;
    const uint32_t need_hi = hi_f < 1.0f ? 0u : static_cast<uint32_t>(hi_f);  // 0: no bin is safely above T
    const uint32_t need_lo = lo_f >= static_cast<float>(n_s) ? n_s + 1u : static_cast<uint32_t>(lo_f) + 1u;
    find_bins(s_hist[0], kHistBins, need_hi, need_lo, s_scan[0], s_found[0]);
    uint32_t b_hi = need_hi ? s_found[0][0] : (kHistBins - 1);  // top bin of the bracket
    uint32_t b_lo = (need_lo <= n_s) ? s_found[0][2] : 1u;      // bottom bin of the bracket
    if (b_lo < 1u) b_lo = 1u;                                   // bin 0 holds only "not a candidate"
    if (b_hi < b_lo) b_hi = b_lo;
    TB_MARK(2);

    // ---- radix descent.  Level state: candidates are the keys with lo_key <= key < lo_key +
    // span, histogrammed by (key - lo_key) >> shift; keys above `above_key` (only on the
    // first, bracketed level) are counted instead.  If the exact counts of the first level
    // show that T is not inside the bracket, the level is repeated over every real bin.
    uint32_t lo_key, span, above_key, nbins, need = static_cast<uint32_t>(kk);
    int shift;
    {
      const uint32_t nb = b_hi - b_lo + 1;                         // 12-bit bins in the bracket
      const int e = 31 - __clz(static_cast<int>(kHistBins / nb));  // extra bits of resolution
      shift = kTopShift - e;
      nbins = nb << e;
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
      if (dense_level) {
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
      } else {
        // only the handful of keys of one sub-bin take part: skip wave-uniformly
        for_each_tile([&](int, const uint32_t(&k4)[4]) {
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t d = k4[c] - lo_key;
            if (__any(d < span)) {
              if (d < span) atomicAdd(&h[d >> shift], 1u);
            }
          }
        });
      }
      // clear the other histogram for the next level while this one is being filled
      for (int i = tid; i < kHistBins; i += kSelThreads) s_hist[cur ^ 1][i] = 0;
      const uint32_t c_above = block_sum_u32(n_above, s_part[call & 1]);  // barrier inside
      const uint32_t want = (c_above < need) ? need - c_above : 0u;
      const uint32_t total_in = find_bins(h, static_cast<int>(nbins), want, want, s_scan[call], s_found[call]);
      cur ^= 1;
      if (want >= 1u && want <= total_in) {  // T lies inside this level's range: descend
        lo_key += s_found[call][0] << shift;
        need = want - s_found[call][1];
        if (shift == 0) break;
        if (need == h[s_found[call][0]]) {
          // every key of this sub-bin is needed: no reason to look at its low bits
          take_whole_bin = true;
          break;
        }
        const int nshift = shift > 12 ? shift - 12 : 0;
        nbins = 1u << (shift - nshift);
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
        nbins = kHistBins - 1;
        above_key = 0xFFFFFFFFu;
      }
    }
    TB_MARK(3);
    T = lo_key;
    r_eq = need;
    if (take_whole_bin) {  // keep everything from the start of the sub-bin upwards
      T = lo_key - 1u;
      r_eq = 0u;
    }
    TB_MARK(4);
  }
  // kk == hi - lo: T = 0 keeps every candidate (all real keys are > 0)

  // ---- ordered compaction.  Pass A: prefix of {key > T} (low half) and {key == T} (high
  // half) inside each wave tile, and the wave's totals.
  auto tile_count = [&](const uint32_t(&k4)[4]) {
    uint32_t cnt = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) cnt += (k4[c] > T ? 1u : 0u) + ((k4[c] == T && T) ? 0x10000u : 0u);
    return cnt;
  };
  constexpr bool kKeepPre = NT > 0 && NT <= 8;  // keep the in-tile prefixes when registers allow
  uint32_t pre[kKeepPre ? NT : 1];
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
  __syncthreads();
  TB_MARK(5);
  uint32_t base_gt = 0, base_eq = 0;  // kept / tied keys in the spans of the waves before this one
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    base_gt += (w < wave) ? s_wgt[w] : 0u;
    base_eq += (w < wave) ? s_weq[w] : 0u;
  }

  // Pass B: position of a kept key = (#greater before it) + min(#equal before it, r_eq)
  int32_t* sel_out = out + lo;
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
    if ((tot >> 16) == 0) {
      // no key of this wave tile equals T: the tie count is the same for every slot
      uint32_t pos = gt_before + (eq_before < r_eq ? eq_before : r_eq);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (k4[c] > T) {
          if (pos < static_cast<uint32_t>(kk)) sel_out[pos] = nn + c;
          ++pos;
        }
      }
    } else {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool gt = k4[c] > T;
        const bool eq = (k4[c] == T) && T;
        if (gt || (eq && eq_before < r_eq)) {
          const uint32_t pos = gt_before + (eq_before < r_eq ? eq_before : r_eq);
          if (pos < static_cast<uint32_t>(kk)) sel_out[pos] = nn + c;
        }
        gt_before += gt ? 1u : 0u;
        eq_before += eq ? 1u : 0u;
      }
    }
    base_gt += tot & 0xFFFFu;
    base_eq += tot >> 16;
  });
  TB_MARK(6);
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
  const int32_t tiles = static_cast<int32_t>((L.N + kTileElts - 1) / kTileElts);  // per wave
  a.tiles_per_wave = tiles;
  dim3 grid(static_cast<unsigned>(L.units));
  dim3 block(kSelThreads);
  if (tiles <= 1)
    hipLaunchKernelGGL(select_kernel<1>, grid, block, 0, st, a);
  else if (tiles <= 2)
    hipLaunchKernelGGL(select_kernel<2>, grid, block, 0, st, a);
  else if (tiles <= 4)
    hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, st, a);
  else if (tiles <= 8)
    hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, st, a);
  else if (tiles <= 16)
    hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, st, a);
  else
    hipLaunchKernelGGL(select_kernel<0>, grid, block, 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace tb
