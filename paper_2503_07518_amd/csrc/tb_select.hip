// Top-k selection under the policy "candidates = [lo, hi); keep the kk largest scores, lowest
// index wins ties; emit ascending".
//
// Exact MSB-first radix select on the order-preserving 32-bit key (11 + 11 + 10 bits):
//   level 1  histogram of the top 11 bits over all candidates.  Either accumulated by the
//            scoring kernel while the scores are still in registers, or by hist_kernel below
//            (many workgroups per head, LDS-private histograms, one global atomic per
//            non-empty bin).
//   select_kernel, one 1024-thread workgroup per (b,h):
//            keeps the head's keys in registers (up to 64 per thread = 65536 scores; longer
//            rows are streamed again per phase), finds the level-1 bin that contains the
//            kk-th largest key, refines inside that bin with two LDS histograms (only the few
//            keys of the bin take part), which gives the exact threshold key T and the number
//            r of keys equal to T that are still needed, then writes
//            {key > T} U {first r keys == T by index} in ascending order using prefix sums
//            (no atomic slot grabbing, so the output is ordered and reproducible).
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / kWave;
constexpr int kTileElts = kSelThreads * 4;       // scores per tile: one float4 per thread
constexpr int kMaxTiles = kSelectMaxN / kTileElts;  // 256

struct SelectArgs {
  const float* scores;
  int64_t score_stride;
  int64_t N;
  int32_t kk, lo, hi;
  int32_t* idx;
  int32_t* count;
  int64_t idx_cap;
  uint32_t* hist;
  int32_t ntiles;
};

// Keys of tile j for this thread: positions ((j*1024 + tid)*4 + c), c = 0..3.  Positions
// outside the candidate range get key 0.
__device__ inline void load_tile_keys(const float* s, int64_t N, int lo, int hi, int j, uint32_t (&key)[4]) {
  const int64_t n0 = (static_cast<int64_t>(j) * kSelThreads + threadIdx.x) * 4;
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
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int64_t n = n0 + c;
    key[c] = (n >= lo && n < hi) ? score_key(v[c]) : 0u;
  }
}

// Standalone level-1 histogram: grid (chunks, units), chunk = 4 tiles.
constexpr int kHistTilesPerWg = 4;
__global__ __launch_bounds__(kSelThreads) void hist_kernel(SelectArgs a) {
  __shared__ uint32_t s_hist[kBins1];
  const int u = blockIdx.y;
  for (int i = threadIdx.x; i < kBins1; i += kSelThreads) s_hist[i] = 0;
  __syncthreads();
  const float* s = a.scores + static_cast<int64_t>(u) * a.score_stride;
  for (int t = 0; t < kHistTilesPerWg; ++t) {
    const int j = blockIdx.x * kHistTilesPerWg + t;
    if (j >= a.ntiles) break;
    uint32_t key[4];
    load_tile_keys(s, a.N, a.lo, a.hi, j, key);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      if (key[c]) atomicAdd(&s_hist[key[c] >> kShift1], 1u);
  }
  __syncthreads();
  uint32_t* gh = a.hist + static_cast<int64_t>(u) * kBins1;
  for (int i = threadIdx.x; i < kBins1; i += kSelThreads) {
    const uint32_t c = s_hist[i];
    if (c) atomicAdd(&gh[i], c);
  }
}

// Walk the histogram from the highest bin down and find the bin in which the running count
// reaches `need` (1 <= need <= total).  Returns the bin; c_gt = count in strictly higher bins.
// All threads get the same answer.  nbins is 2048 or 1024.
__device__ inline uint32_t find_bin(const uint32_t* s_hist, int nbins, uint32_t need, uint32_t* s_scan,
                                    uint32_t* s_found, uint32_t& c_gt) {
  const int tid = threadIdx.x;
  const int r0 = 2 * tid, r1 = 2 * tid + 1;  // reversed bin numbers handled by this thread
  const uint32_t v0 = (r0 < nbins) ? s_hist[nbins - 1 - r0] : 0u;
  const uint32_t v1 = (r1 < nbins) ? s_hist[nbins - 1 - r1] : 0u;
  uint32_t total;
  const uint32_t excl = block_excl_scan<kSelWaves>(v0 + v1, s_scan, total);
  if (excl < need && need <= excl + v0) {
    s_found[0] = static_cast<uint32_t>(nbins - 1 - r0);
    s_found[1] = excl;
  } else if (excl + v0 < need && need <= excl + v0 + v1) {
    s_found[0] = static_cast<uint32_t>(nbins - 1 - r1);
    s_found[1] = excl + v0;
  }
  __syncthreads();
  const uint32_t bin = s_found[0];
  c_gt = s_found[1];
  __syncthreads();
  return bin;
}

template <int NT>  // NT > 0: tiles cached in registers (NT >= ntiles); NT == 0: streamed per phase
__global__ __launch_bounds__(kSelThreads) void select_kernel(SelectArgs a) {
  __shared__ uint32_t s_hist[kBins1];
  __shared__ uint32_t s_scan[kSelWaves + 1];
  __shared__ unsigned long long s_scan64[kSelWaves + 1];
  __shared__ uint32_t s_found[2];
  __shared__ uint32_t s_tot_gt[(NT > 0 ? NT : kMaxTiles) * kSelWaves];
  __shared__ uint32_t s_tot_eq[(NT > 0 ? NT : kMaxTiles) * kSelWaves];

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = tid / kWave;
  const int u = blockIdx.x;
  const float* s = a.scores + static_cast<int64_t>(u) * a.score_stride;
  int32_t* out = a.idx + static_cast<int64_t>(u) * a.idx_cap;
  const int lo = a.lo, hi = a.hi, kk = a.kk;
  const int ntiles = (NT > 0) ? NT : a.ntiles;

  // always-kept ranges: sink prefix [0, lo) and local window [hi, N)
  for (int64_t n = tid; n < lo; n += kSelThreads) out[n] = static_cast<int32_t>(n);
  for (int64_t n = hi + tid; n < a.N; n += kSelThreads) out[lo + kk + (n - hi)] = static_cast<int32_t>(n);
  if (tid == 0) a.count[u] = static_cast<int32_t>(lo + kk + (a.N - hi));
  if (kk == 0) return;

  uint32_t keys[NT > 0 ? NT : 1][4];
  if (NT > 0) {
#pragma unroll
    for (int j = 0; j < NT; ++j) load_tile_keys(s, a.N, lo, hi, j, keys[j]);
  }
  auto tile_keys = [&](int j, uint32_t(&k4)[4]) {
    if (NT > 0) {
#pragma unroll
      for (int c = 0; c < 4; ++c) k4[c] = keys[NT > 0 ? j : 0][c];
    } else {
      load_tile_keys(s, a.N, lo, hi, j, k4);
    }
  };

  uint32_t T = 0;      // threshold key: everything above is kept
  uint32_t r_eq = 0;   // how many keys equal to T are kept (lowest indices first)
  if (tid == 0) {
    s_found[0] = 0;
    s_found[1] = 0;
  }

  if (kk < hi - lo) {
    // ---- level 1: histogram from global memory; leave it zeroed for the next call
    uint32_t* gh = a.hist + static_cast<int64_t>(u) * kBins1;
    for (int i = tid; i < kBins1; i += kSelThreads) {
      s_hist[i] = gh[i];
      gh[i] = 0;
    }
    __syncthreads();
    uint32_t c_gt;
    const uint32_t b1 = find_bin(s_hist, kBins1, static_cast<uint32_t>(kk), s_scan, s_found, c_gt);
    uint32_t need = static_cast<uint32_t>(kk) - c_gt;

    // ---- level 2: next 11 bits, only keys inside bin b1 take part
    for (int i = tid; i < kBins2; i += kSelThreads) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
      if (NT > 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((keys[j][c] >> kShift1) == b1 && keys[j][c]) atomicAdd(&s_hist[(keys[j][c] >> kShift2) & (kBins2 - 1)], 1u);
      }
    }
    if (NT == 0) {
      for (int j = 0; j < ntiles; ++j) {
        uint32_t k4[4];
        load_tile_keys(s, a.N, lo, hi, j, k4);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((k4[c] >> kShift1) == b1 && k4[c]) atomicAdd(&s_hist[(k4[c] >> kShift2) & (kBins2 - 1)], 1u);
      }
    }
    __syncthreads();
    const uint32_t b2 = find_bin(s_hist, kBins2, need, s_scan, s_found, c_gt);
    need -= c_gt;
    const uint32_t prefix22 = (b1 << (kShift1 - kShift2)) | b2;

    // ---- level 3: last 10 bits
    for (int i = tid; i < kBins3; i += kSelThreads) s_hist[i] = 0;
    __syncthreads();
#pragma unroll
    for (int j = 0; j < (NT > 0 ? NT : 1); ++j) {
      if (NT > 0) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((keys[j][c] >> kShift2) == prefix22) atomicAdd(&s_hist[keys[j][c] & (kBins3 - 1)], 1u);
      }
    }
    if (NT == 0) {
      for (int j = 0; j < ntiles; ++j) {
        uint32_t k4[4];
        load_tile_keys(s, a.N, lo, hi, j, k4);
#pragma unroll
        for (int c = 0; c < 4; ++c)
          if ((k4[c] >> kShift2) == prefix22) atomicAdd(&s_hist[k4[c] & (kBins3 - 1)], 1u);
      }
    }
    __syncthreads();
    const uint32_t b3 = find_bin(s_hist, kBins3, need, s_scan, s_found, c_gt);
    r_eq = need - c_gt;
    T = (prefix22 << kShift2) | b3;
  }
  // kk == hi - lo: T = 0 keeps every candidate (all real keys are > 0)

  // ---- ordered compaction.  Pass A: per (tile, wave) totals of {key > T} and {key == T}.
  for (int j = 0; j < ntiles; ++j) {
    uint32_t k4[4];
    tile_keys(j, k4);
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) packed += (k4[c] > T ? 1u : 0u) + (k4[c] == T && T ? 0x10000u : 0u);
    packed = wave_sum(packed);
    if (lane == 0) {
      s_tot_gt[j * kSelWaves + wave] = packed & 0xFFFFu;
      s_tot_eq[j * kSelWaves + wave] = packed >> 16;
    }
  }
  __syncthreads();
  // exclusive scan of the totals in (tile, wave) order, both counters at once in 64 bits
  {
    const int entries = ntiles * kSelWaves;
    const int per = (entries + kSelThreads - 1) / kSelThreads;
    const int e0 = tid * per;
    unsigned long long local = 0;
    for (int e = e0; e < e0 + per && e < entries; ++e)
      local += static_cast<unsigned long long>(s_tot_gt[e]) | (static_cast<unsigned long long>(s_tot_eq[e]) << 32);
    unsigned long long total;
    unsigned long long run = block_excl_scan<kSelWaves>(local, s_scan64, total);
    for (int e = e0; e < e0 + per && e < entries; ++e) {
      const unsigned long long v =
          static_cast<unsigned long long>(s_tot_gt[e]) | (static_cast<unsigned long long>(s_tot_eq[e]) << 32);
      s_tot_gt[e] = static_cast<uint32_t>(run);
      s_tot_eq[e] = static_cast<uint32_t>(run >> 32);
      run += v;
    }
  }
  __syncthreads();
  // Pass B: position of a kept key = (#greater before it) + min(#equal before it, r_eq)
  int32_t* sel_out = out + lo;
  for (int j = 0; j < ntiles; ++j) {
    uint32_t k4[4];
    tile_keys(j, k4);
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) packed += (k4[c] > T ? 1u : 0u) + (k4[c] == T && T ? 0x10000u : 0u);
    const uint32_t incl = wave_incl_scan(packed);
    const uint32_t excl = incl - packed;
    uint32_t gt_before = s_tot_gt[j * kSelWaves + wave] + (excl & 0xFFFFu);
    uint32_t eq_before = s_tot_eq[j * kSelWaves + wave] + (excl >> 16);
    const int64_t n0 = (static_cast<int64_t>(j) * kSelThreads + tid) * 4;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool gt = k4[c] > T;
      const bool eq = (k4[c] == T) && T;
      if (gt || (eq && eq_before < r_eq)) {
        const uint32_t pos = gt_before + (eq_before < r_eq ? eq_before : r_eq);
        if (pos < static_cast<uint32_t>(kk)) sel_out[pos] = static_cast<int32_t>(n0 + c);
      }
      gt_before += gt ? 1u : 0u;
      eq_before += eq ? 1u : 0u;
    }
  }
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
  a.ntiles = static_cast<int32_t>((L.N + kTileElts - 1) / kTileElts);
  const bool need_hist = L.kk > 0 && L.kk < L.hi - L.lo;
  if (need_hist && !L.hist_ready) {
    dim3 grid((a.ntiles + kHistTilesPerWg - 1) / kHistTilesPerWg, static_cast<unsigned>(L.units));
    hipLaunchKernelGGL(hist_kernel, grid, dim3(kSelThreads), 0, st, a);
    if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
  }
  dim3 grid(static_cast<unsigned>(L.units));
  dim3 block(kSelThreads);
  if (a.ntiles <= 1)
    hipLaunchKernelGGL(select_kernel<1>, grid, block, 0, st, a);
  else if (a.ntiles <= 2)
    hipLaunchKernelGGL(select_kernel<2>, grid, block, 0, st, a);
  else if (a.ntiles <= 4)
    hipLaunchKernelGGL(select_kernel<4>, grid, block, 0, st, a);
  else if (a.ntiles <= 8)
    hipLaunchKernelGGL(select_kernel<8>, grid, block, 0, st, a);
  else if (a.ntiles <= 16)
    hipLaunchKernelGGL(select_kernel<16>, grid, block, 0, st, a);
  else
    hipLaunchKernelGGL(select_kernel<0>, grid, block, 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace tb
