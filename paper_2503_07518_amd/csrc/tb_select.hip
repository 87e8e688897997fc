// Top-k selection under the policy "candidates = [lo, hi); keep the kk largest scores, lowest
// index wins ties; emit ascending".
//
// Exact MSB-first radix select on the order-preserving 32-bit key (11 + 11 + 10 bits):
//   level 1  histogram of the top 11 bits over all candidates.  Either accumulated by the
//            scoring kernel while the scores are still in registers, or by hist_kernel below
//            (many workgroups per head, LDS-private histograms, one global atomic per
//            non-empty bin).
//   select_kernel, one 1024-thread workgroup per (b,h):
//            wave w owns the contiguous span [w*span, (w+1)*span) of the head's scores and
//            keeps its keys in registers (up to 64 per thread = 65536 scores; longer rows are
//            streamed again per phase).  It finds the level-1 bin that contains the kk-th
//            largest key, refines inside that bin with two LDS histograms (only the few keys
//            of the bin take part), which gives the exact threshold key T and the number r of
//            keys equal to T that are still needed, then writes
//            {key > T} U {first r keys == T by index} in ascending order.  Positions come from
//            prefix sums (DPP scans inside a wave tile, running totals along the wave's span,
//            16 wave totals across the workgroup) -- no atomic slot grabbing, so the output
//            is ordered and reproducible.
#include "tb_device.h"
#include "tb_internal.h"

#ifdef TB_PROBE
__device__ unsigned long long tb_probe_buf[64];
#define TB_MARK(i)                                                                  \
  do {                                                                              \
    if (blockIdx.x == 0 && threadIdx.x == 0) tb_probe_buf[i] = wall_clock64();      \
  } while (0)
#else
#define TB_MARK(i)
#endif

namespace tb {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kWaveTile = kWave * 4;                       // scores per wave tile: one float4 per lane
constexpr int kTileElts = kSelWaves * kWaveTile;           // scores per workgroup-wide tile (4096)

struct SelectArgs {
  const float* scores;
  int64_t score_stride;
  int64_t N;
  int32_t kk, lo, hi;
  int32_t* idx;
  int32_t* count;
  int64_t idx_cap;
  uint32_t* hist;
  int32_t tiles_per_wave;
};

// Keys of the four consecutive positions n0 .. n0+3 (n0 a multiple of 4).  Positions outside
// the candidate range get key 0.
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

// Standalone level-1 histogram: grid (chunks, units), a chunk is 4 workgroup-wide tiles.
constexpr int kHistTilesPerWg = 4;
__global__ __launch_bounds__(kSelThreads) void hist_kernel(SelectArgs a) {
  __shared__ uint32_t s_hist[kBins1];
  const int u = blockIdx.y;
  for (int i = threadIdx.x; i < kBins1; i += kSelThreads) s_hist[i] = 0;
  __syncthreads();
  const float* s = a.scores + static_cast<int64_t>(u) * a.score_stride;
#pragma unroll
  for (int t = 0; t < kHistTilesPerWg; ++t) {
    const int64_t n0 = (static_cast<int64_t>(blockIdx.x) * kHistTilesPerWg + t) * kTileElts + threadIdx.x * 4;
    if (n0 < a.N) {
      uint32_t key[4];
      load_keys4(s, a.N, a.lo, a.hi, n0, key);
#pragma unroll
      for (int c = 0; c < 4; ++c)
        if (key[c]) atomicAdd(&s_hist[key[c] >> kShift1], 1u);
    }
  }
  __syncthreads();
  uint32_t* gh = a.hist + static_cast<int64_t>(u) * kBins1;
  for (int i = threadIdx.x; i < kBins1; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// Walk a histogram from its highest bin down and find the bin in which the running count
// reaches `need` (1 <= need <= total).  Thread t brings the counts of bins nbins-1-2t (v0) and
// nbins-2-2t (v1).  Returns the bin; c_gt = count in strictly higher bins.  Two barriers;
// s_scan (16 words) and s_found (2 words, preset to 0) must not be shared between calls.
__device__ inline uint32_t find_bin(uint32_t v0, uint32_t v1, int nbins, uint32_t need, uint32_t* s_scan,
                                    uint32_t* s_found, uint32_t& c_gt) {
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const uint32_t incl = wave_incl_scan_u32(v0 + v1);
  if (lane == kWave - 1) s_scan[wave] = incl;
  __syncthreads();
  uint32_t excl = incl - (v0 + v1);
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) excl += (w < wave) ? s_scan[w] : 0u;
  if (excl < need && need <= excl + v0) {
    s_found[0] = static_cast<uint32_t>(nbins - 1 - 2 * tid);
    s_found[1] = excl;
  } else if (excl + v0 < need && need <= excl + v0 + v1) {
    s_found[0] = static_cast<uint32_t>(nbins - 2 - 2 * tid);
    s_found[1] = excl + v0;
  }
  __syncthreads();
  c_gt = s_found[1];
  return s_found[0];
}

template <int NT>  // NT > 0: the wave's tiles are cached in registers (NT >= tiles per wave);
                   // NT == 0: streamed again in every phase
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a) {
  __shared__ uint32_t s_h2[kBins2];
  __shared__ uint32_t s_h3[kBins3];
  __shared__ uint32_t s_scan[3][kSelWaves];
  __shared__ uint32_t s_found[3][2];
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
  // loads first: the wave's keys, and this thread's two bins of the level-1 histogram
  // (bins 2047-2t and 2046-2t, adjacent in memory)
  uint32_t keys[NT > 0 ? NT : 1][4];
  if (NT > 0 && kk > 0) {
#pragma unroll
    for (int j = 0; j < NT; ++j) load_keys4(s, a.N, lo, hi, wbase + j * kWaveTile, keys[j]);
  }
  uint32_t hv0 = 0, hv1 = 0;
  if (refine) {
    uint2* gh = reinterpret_cast<uint2*>(a.hist + static_cast<int64_t>(u) * kBins1 + (kBins1 - 2 - 2 * tid));
    const uint2 h = *gh;
    hv0 = h.y;
    hv1 = h.x;
    *gh = make_uint2(0u, 0u);  // leave the histogram zeroed for the next call
  }
  for (int i = tid; i < kBins2; i += kSelThreads) s_h2[i] = 0;
  for (int i = tid; i < kBins3; i += kSelThreads) s_h3[i] = 0;
  if (tid < 6) s_found[tid / 2][tid % 2] = 0;

  // always-kept ranges: sink prefix [0, lo) and local window [hi, N)
  for (int64_t n = tid; n < lo; n += kSelThreads) out[n] = static_cast<int32_t>(n);
  for (int64_t n = hi + tid; n < a.N; n += kSelThreads) out[lo + kk + (n - hi)] = static_cast<int32_t>(n);
  if (tid == 0) a.count[u] = static_cast<int32_t>(lo + kk + (a.N - hi));
  if (kk == 0) return;

  auto tile_keys = [&](int j, uint32_t(&k4)[4]) {
    if (NT > 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) k4[c] = keys[NT > 0 ? j : 0][c];
    } else {
      load_keys4(s, a.N, lo, hi, wbase + static_cast<int64_t>(j) * kWaveTile, k4);
    }
  };

  uint32_t T = 0;     // threshold key: everything above is kept
  uint32_t r_eq = 0;  // how many keys equal to T are kept (lowest indices first)
  if (refine) {
    __syncthreads();  // s_found / s_h2 / s_h3 initialised
    TB_MARK(1);
    uint32_t c_gt;
    const uint32_t b1 = find_bin(hv0, hv1, kBins1, static_cast<uint32_t>(kk), s_scan[0], s_found[0], c_gt);
    uint32_t need = static_cast<uint32_t>(kk) - c_gt;
    TB_MARK(2);

    // level 2: next 11 bits, only keys inside bin b1 take part (key 0 is never in a real bin)
#pragma unroll
    for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
      if (NT > 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((keys[j][c] >> kShift1) == b1) atomicAdd(&s_h2[(keys[j][c] >> kShift2) & (kBins2 - 1)], 1u);
      }
    }
    if (NT == 0) {
      for (int j = 0; j < tpw; ++j) {
        uint32_t k4[4];
        tile_keys(j, k4);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((k4[c] >> kShift1) == b1) atomicAdd(&s_h2[(k4[c] >> kShift2) & (kBins2 - 1)], 1u);
      }
    }
    __syncthreads();
    TB_MARK(3);
    const uint32_t b2 = find_bin(s_h2[kBins2 - 1 - 2 * tid], s_h2[kBins2 - 2 - 2 * tid], kBins2, need, s_scan[1],
                                 s_found[1], c_gt);
    need -= c_gt;
    const uint32_t prefix22 = (b1 << (kShift1 - kShift2)) | b2;
    TB_MARK(4);

    // level 3: last 10 bits
#pragma unroll
    for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
      if (NT > 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((keys[j][c] >> kShift2) == prefix22) atomicAdd(&s_h3[keys[j][c] & (kBins3 - 1)], 1u);
      }
    }
    if (NT == 0) {
      for (int j = 0; j < tpw; ++j) {
        uint32_t k4[4];
        tile_keys(j, k4);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((k4[c] >> kShift2) == prefix22) atomicAdd(&s_h3[k4[c] & (kBins3 - 1)], 1u);
      }
    }
    __syncthreads();
    TB_MARK(5);
    const bool has3 = 2 * tid + 1 < kBins3;
    const uint32_t b3 = find_bin(has3 ? s_h3[kBins3 - 1 - 2 * tid] : 0u, has3 ? s_h3[kBins3 - 2 - 2 * tid] : 0u, kBins3,
                                 need, s_scan[2], s_found[2], c_gt);
    r_eq = need - c_gt;
    T = (prefix22 << kShift2) | b3;
    TB_MARK(6);
  }
  // kk == hi - lo: T = 0 keeps every candidate (all real keys are > 0)

  // ---- ordered compaction.  Pass A: prefix of {key > T} (low half) and {key == T} (high
  // half) inside each wave tile, and the wave's totals.
  uint32_t pre[NT > 0 ? NT : 1];
  uint32_t run_gt = 0, run_eq = 0;
#pragma unroll
  for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
    if (NT > 0) {
      uint32_t cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) cnt += (keys[j][c] > T ? 1u : 0u) + ((keys[j][c] == T && T) ? 0x10000u : 0u);
      const uint32_t incl = wave_incl_scan_u32(cnt);
      pre[j] = incl - cnt;
      const uint32_t tot = __builtin_amdgcn_readlane(incl, kWave - 1);
      run_gt += tot & 0xFFFFu;
      run_eq += tot >> 16;
    }
  }
  if (NT == 0) {
    for (int j = 0; j < tpw; ++j) {
      uint32_t k4[4];
      tile_keys(j, k4);
      uint32_t cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) cnt += (k4[c] > T ? 1u : 0u) + ((k4[c] == T && T) ? 0x10000u : 0u);
      const uint32_t tot = __builtin_amdgcn_readlane(wave_incl_scan_u32(cnt), kWave - 1);
      run_gt += tot & 0xFFFFu;
      run_eq += tot >> 16;
    }
  }
  if (lane == 0) {
    s_wgt[wave] = run_gt;
    s_weq[wave] = run_eq;
  }
  __syncthreads();
  TB_MARK(7);
  uint32_t base_gt = 0, base_eq = 0;  // kept / tied keys in the spans of the waves before this one
#pragma unroll
  for (int w = 0; w < kSelWaves; ++w) {
    base_gt += (w < wave) ? s_wgt[w] : 0u;
    base_eq += (w < wave) ? s_weq[w] : 0u;
  }

  // Pass B: position of a kept key = (#greater before it) + min(#equal before it, r_eq)
  int32_t* sel_out = out + lo;
  auto emit = [&](const uint32_t(&k4)[4], uint32_t gt_before, uint32_t eq_before, int64_t n0, bool tile_has_eq) {
    const int32_t nn = static_cast<int32_t>(n0);
    if (!tile_has_eq) {
      // no key of this wave tile equals T: the tie count is the same for every slot
      uint32_t pos = gt_before + (eq_before < r_eq ? eq_before : r_eq);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (k4[c] > T) {
          if (pos < static_cast<uint32_t>(kk)) sel_out[pos] = nn + c;
          ++pos;
        }
      }
      return;
    }
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
  };
#pragma unroll
  for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
    if (NT > 0) {
      uint32_t cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) cnt += (keys[j][c] > T ? 1u : 0u) + ((keys[j][c] == T && T) ? 0x10000u : 0u);
      const uint32_t tot = __builtin_amdgcn_readlane(pre[j] + cnt, kWave - 1);
      emit(keys[j], base_gt + (pre[j] & 0xFFFFu), base_eq + (pre[j] >> 16), wbase + j * kWaveTile, (tot >> 16) != 0);
      base_gt += tot & 0xFFFFu;
      base_eq += tot >> 16;
    }
  }
  if (NT == 0) {
    for (int j = 0; j < tpw; ++j) {
      uint32_t k4[4];
      tile_keys(j, k4);
      uint32_t cnt = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) cnt += (k4[c] > T ? 1u : 0u) + ((k4[c] == T && T) ? 0x10000u : 0u);
      const uint32_t incl = wave_incl_scan_u32(cnt);
      const uint32_t tot = __builtin_amdgcn_readlane(incl, kWave - 1);
      emit(k4, base_gt + ((incl - cnt) & 0xFFFFu), base_eq + ((incl - cnt) >> 16),
           wbase + static_cast<int64_t>(j) * kWaveTile, (tot >> 16) != 0);
      base_gt += tot & 0xFFFFu;
      base_eq += tot >> 16;
    }
  }
  TB_MARK(8);
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
  a.hist = L.hist;
  const int32_t tiles = static_cast<int32_t>((L.N + kTileElts - 1) / kTileElts);  // per wave
  a.tiles_per_wave = tiles;
  const bool need_hist = L.kk > 0 && L.kk < L.hi - L.lo;
  if (need_hist && !L.hist_ready) {
    dim3 grid((tiles + kHistTilesPerWg - 1) / kHistTilesPerWg, static_cast<unsigned>(L.units));
    hipLaunchKernelGGL(hist_kernel, grid, dim3(kSelThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
  }
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
