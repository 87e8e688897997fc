// Neighbour fetching on an ascending, duplicate-free index list; one workgroup per (b,h) list.
//
// mode 0 (radius): the output is the union of [i-r, i+r] clipped to [0,N).  Because the input
// ascends, entry j adds exactly the positions of its interval that lie beyond the interval of
// entry j-1, so the output length is a prefix sum and every entry writes its own run.
//
// mode 1 (cluster-aware): every selected token adds the next free position past its cluster.
// With D_j = number of still-owed positions right after entry j (itself counted) and
// gap_j = free positions between entries j and j+1, D_j = max(D_{j-1} - gap_{j-1}, 0) + 1 and
// entry j is followed by min(D_j, gap_j) fetched positions.  The recurrence is a composition
// of maps x -> max(x + a, c), which is associative, so it runs as a block-wide prefix scan.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kExpThreads = 1024;
constexpr int kExpWaves = kExpThreads / kWave;

struct ExpandArgs {
  int64_t N;
  int32_t radius;
  const int32_t* idx_in;
  const int32_t* count_in;
  int64_t cap_in;
  int32_t* idx_out;
  int32_t* count_out;
  int64_t cap_out;
};

__global__ __launch_bounds__(kExpThreads) void expand_radius_kernel(ExpandArgs a) {
  __shared__ unsigned long long s_scan[kExpWaves + 1];
  const int tid = threadIdx.x;
  const int64_t u = blockIdx.x;
  const int32_t* in = a.idx_in + u * a.cap_in;
  int32_t* out = a.idx_out + u * a.cap_out;
  int64_t c = a.count_in[u];
  c = c < 0 ? 0 : (c > a.cap_in ? a.cap_in : c);
  const int64_t per = (c + kExpThreads - 1) / kExpThreads;
  const int64_t j0 = tid * per;
  const int64_t j1 = (j0 + per < c) ? j0 + per : c;
  const int64_t r = a.radius;
  const int64_t last = a.N - 1;

  auto hi_of = [&](int64_t i) { return (i + r < last) ? i + r : last; };

  int64_t covered = -1;  // last position already emitted by earlier entries
  if (j0 > 0 && j0 < c) covered = hi_of(in[j0 - 1]);
  unsigned long long mine = 0;
  {
    int64_t cov = covered;
    for (int64_t j = j0; j < j1; ++j) {
      const int64_t i = in[j];
      int64_t s = i - r;
      if (s < 0) s = 0;
      if (s <= cov) s = cov + 1;
      const int64_t e = hi_of(i);
      if (e >= s) {
        mine += static_cast<unsigned long long>(e - s + 1);
        cov = e;
      }
    }
  }
  unsigned long long total;
  unsigned long long pos = block_excl_scan<kExpWaves>(mine, s_scan, total);
  {
    int64_t cov = covered;
    for (int64_t j = j0; j < j1; ++j) {
      const int64_t i = in[j];
      int64_t s = i - r;
      if (s < 0) s = 0;
      if (s <= cov) s = cov + 1;
      const int64_t e = hi_of(i);
      for (int64_t p = s; p <= e; ++p) {
        if (pos < static_cast<unsigned long long>(a.cap_out)) out[pos] = static_cast<int32_t>(p);
        ++pos;
      }
      if (e >= s) cov = e;
    }
  }
  if (tid == 0)
    a.count_out[u] = static_cast<int32_t>(total < static_cast<unsigned long long>(a.cap_out) ? total : a.cap_out);
}

// x -> max(x + add, floor): the debt carried across a run of entries.
struct DebtMap {
  long long add, floor;
};
__device__ inline DebtMap compose(const DebtMap& first, const DebtMap& then) {
  // then(first(x)) = max(max(x + a1, c1) + a2, c2) = max(x + a1 + a2, max(c1 + a2, c2))
  DebtMap o;
  o.add = first.add + then.add;
  const long long t = first.floor + then.add;
  o.floor = t > then.floor ? t : then.floor;
  return o;
}
constexpr long long kNegBig = -(1LL << 60);

__global__ __launch_bounds__(kExpThreads) void expand_cluster_kernel(ExpandArgs a) {
  __shared__ unsigned long long s_scan[kExpWaves + 1];
  __shared__ DebtMap s_map[kExpWaves];
  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int64_t u = blockIdx.x;
  const int32_t* in = a.idx_in + u * a.cap_in;
  int32_t* out = a.idx_out + u * a.cap_out;
  int64_t c = a.count_in[u];
  c = c < 0 ? 0 : (c > a.cap_in ? a.cap_in : c);
  const int64_t per = (c + kExpThreads - 1) / kExpThreads;
  const int64_t j0 = tid * per;
  const int64_t j1 = (j0 + per < c) ? j0 + per : c;

  // map of entry j applied to the debt after entry j-1: D_j = max(D_{j-1} - gap_{j-1}, 0) + 1
  auto entry_map = [&](int64_t j) {
    DebtMap mp;
    const long long gap = (j > 0) ? static_cast<long long>(in[j]) - in[j - 1] - 1 : (1LL << 40);
    mp.add = 1 - gap;
    mp.floor = 1;
    return mp;
  };
  DebtMap mine{0, kNegBig};  // identity
  for (int64_t j = j0; j < j1; ++j) mine = compose(mine, entry_map(j));

  // inclusive scan of the maps across the wave, then across waves (thread order = list order)
  DebtMap incl = mine;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    DebtMap o;
    o.add = __shfl_up(incl.add, off, kWave);
    o.floor = __shfl_up(incl.floor, off, kWave);
    if (lane >= off) incl = compose(o, incl);
  }
  if (lane == kWave - 1) s_map[wave] = incl;
  __syncthreads();
  DebtMap before{0, kNegBig};
  for (int w = 0; w < wave; ++w) before = compose(before, s_map[w]);
  {
    DebtMap prev;
    prev.add = __shfl_up(incl.add, 1, kWave);
    prev.floor = __shfl_up(incl.floor, 1, kWave);
    if (lane > 0) before = compose(before, prev);
  }
  // debt after the last entry handled by earlier threads (0 before the first entry)
  long long debt0 = before.add > before.floor ? before.add : before.floor;  // map applied to x = 0
  if (j0 == 0) debt0 = 0;

  unsigned long long mine_out = 0;
  {
    long long debt = debt0;
    for (int64_t j = j0; j < j1; ++j) {
      const long long gap_prev = (j > 0) ? static_cast<long long>(in[j]) - in[j - 1] - 1 : 0;
      debt = (debt - gap_prev > 0 ? debt - gap_prev : 0) + 1;
      const long long gap = (j + 1 < c) ? static_cast<long long>(in[j + 1]) - in[j] - 1 : (a.N - 1 - in[j]);
      const long long fill = debt < gap ? debt : gap;
      mine_out += static_cast<unsigned long long>(1 + (fill > 0 ? fill : 0));
    }
  }
  unsigned long long total;
  unsigned long long pos = block_excl_scan<kExpWaves>(mine_out, s_scan, total);
  {
    long long debt = debt0;
    for (int64_t j = j0; j < j1; ++j) {
      const long long gap_prev = (j > 0) ? static_cast<long long>(in[j]) - in[j - 1] - 1 : 0;
      debt = (debt - gap_prev > 0 ? debt - gap_prev : 0) + 1;
      const long long gap = (j + 1 < c) ? static_cast<long long>(in[j + 1]) - in[j] - 1 : (a.N - 1 - in[j]);
      const long long fill = debt < gap ? debt : gap;
      for (long long f = 0; f <= (fill > 0 ? fill : 0); ++f) {
        if (pos < static_cast<unsigned long long>(a.cap_out)) out[pos] = static_cast<int32_t>(in[j] + f);
        ++pos;
      }
    }
  }
  if (tid == 0)
    a.count_out[u] = static_cast<int32_t>(total < static_cast<unsigned long long>(a.cap_out) ? total : a.cap_out);
}

}  // namespace

tb_status launch_expand(int64_t units, int64_t N, int32_t radius, int32_t mode, const int32_t* idx_in,
                        const int32_t* count_in, int64_t cap_in, int32_t* idx_out, int32_t* count_out,
                        int64_t cap_out, hipStream_t st) {
  if (units == 0) return TB_OK;
  ExpandArgs a{N, radius, idx_in, count_in, cap_in, idx_out, count_out, cap_out};
  if (mode == 0)
    hipLaunchKernelGGL(expand_radius_kernel, dim3(static_cast<unsigned>(units)), dim3(kExpThreads), 0, st, a);
  else
    hipLaunchKernelGGL(expand_cluster_kernel, dim3(static_cast<unsigned>(units)), dim3(kExpThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace tb
