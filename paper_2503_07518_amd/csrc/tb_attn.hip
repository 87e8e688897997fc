// Decode attention over a per-head list of selected rows (gather fused into the kernel: no
// intermediate "important buffer" copy is made).
//
// Work split: nsplit workgroups per (b, h) (placed per XCD when heads share KV rows, see the
// kernel).  A workgroup of 4 waves takes a contiguous slice of the
// head's list; each wave walks its part in tiles of 4*GPW rows, where GPW = 64/LPR row groups
// and LPR = D*sizeof(T)/16 lanes cover one row with a 128-bit load each (bf16, D=128: 16
// lanes per 256 B row, 4 rows per wave instruction, 16-row tiles).  All K and V loads of a
// tile are issued before the first one is consumed, so a wave keeps 8 KiB of gathers in
// flight (measured best: 32-row tiles were 3-5% slower on the batched configurations).  Every lane group runs its own online softmax (running max, running sum, fp32
// accumulator slice of D/LPR elements) in the base-2 domain; groups are merged by wave
// shuffles, waves through LDS, and workgroups through fp32 partials in the workspace: the
// last workgroup of a head to arrive (device-scope counter) combines the partials in split
// order, so the result does not depend on arrival order.  The counter is reset by that
// workgroup, which leaves the workspace ready for the next call.
//
// Head-less lists (one list per batch element for all heads) go through the same kernel with
// the list shared, or, when there are enough KV groups to fill the chip, through
// attn_group_kernel: one workgroup per (b, kv head, split) that serves all query heads of the
// KV head, so that every listed row is loaded once.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kAttnThreads = 256;
constexpr int kXcds = 8;  // accelerator complex dies of the chip, each with its own L2
constexpr int kAttnWaves = kAttnThreads / kWave;
constexpr int kLoadsPerTile = kAttnLoadsPerTile;
// occupancy the register allocation is held to: 4 waves per SIMD = 4 workgroups per CU, so that a
// launch of up to 1024 workgroups is resident at once (no second round of workgroups)
constexpr int kAttnWavesPerSimd = 4;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct AttnArgs {
  const void* q;
  const void* K;
  const void* V;
  const int32_t* idx;
  const int32_t* count;
  int64_t idx_cap, max_count, tail_begin, tail_end, N;
  int64_t k_stride_b, k_stride_h, k_stride_n;
  int64_t v_stride_b, v_stride_h, v_stride_n;
  float sm_scale_log2;
  float* out;
  float* lse;
  float* partials;
  uint32_t* counters;
  int32_t Hq, g, rows_per_wg, nsplit, n_kv_groups, xcd_map;
  int32_t shared_list;  // one list and count per batch element, read by all of its heads
  // buffered form: the listed rows have been copied to per-query-head buffers
  // [B][Hq][buf_cap][D] in list order (slot i of the list is buffer row i); idx is unused
  const void* Kbuf;
  const void* Vbuf;
  int64_t buf_cap;
};

constexpr int32_t kTailFlag = 0x40000000;  // buffered form: the row number refers to the cache, not the buffer

__device__ inline float exp2_safe(float d) { return __builtin_amdgcn_exp2f(d); }

// Waits until every vector-memory operation this wave has issued, stores included, has been
// acknowledged (s_waitcnt with all counters at zero).
__device__ inline void publish_fence() { __builtin_amdgcn_s_waitcnt(0); }

template <typename T, int D, bool BUF>
__global__ __launch_bounds__(kAttnThreads, kAttnWavesPerSimd) void attn_kernel(AttnArgs a) {
  constexpr int EPL = Pack16<T>::kElts;    // elements per lane
  constexpr int LPR = D / EPL;             // lanes per row
  constexpr int GPW = kWave / LPR;         // row groups per wave
  constexpr int TILE = kLoadsPerTile * GPW;  // rows per wave tile
  static_assert(LPR >= 4 && LPR <= 32, "row must span 4..32 lanes");

  __shared__ float s_m[kAttnWaves], s_l[kAttnWaves];
  __shared__ float s_acc[kAttnWaves][D];
  __shared__ uint32_t s_last;

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int grp = lane / LPR;
  const int sub = lane % LPR;
  // Workgroups go to the 8 XCDs round-robin by their linear index, and every XCD has an L2 of
  // its own: with grouped queries, the query heads that share a KV head are given to one XCD, so
  // that rows picked by several of them are fetched into one L2 once.  KV group (b, hkv) number
  // k lives on XCD k % 8; slot s of an XCD is (its k-th group, head of the group, split).  (If
  // the hardware places workgroups differently, the mapping is just another order of the work.)
  int split, h, b, hkv;
  if (a.xcd_map) {
    const int per_group = a.g * a.nsplit;
    const int xcd = blockIdx.x % kXcds, slot = blockIdx.x / kXcds;
    const int kvg = xcd + kXcds * (slot / per_group);
    if (kvg >= a.n_kv_groups) return;  // the last round of groups does not fill all XCDs
    const int within = slot % per_group;
    split = within % a.nsplit;
    hkv = kvg % (a.Hq / a.g);
    b = kvg / (a.Hq / a.g);
    h = hkv * a.g + within / a.nsplit;
  } else {
    split = blockIdx.x;
    h = blockIdx.y;
    b = blockIdx.z;
    hkv = h / a.g;
  }
  const int64_t u = static_cast<int64_t>(b) * a.Hq + h;

  const int64_t wg_beg = static_cast<int64_t>(split) * a.rows_per_wg;
  const int rows_per_wave = a.rows_per_wg / kAttnWaves;
  const int64_t w_beg0 = wg_beg + static_cast<int64_t>(wave) * rows_per_wave;
  const int64_t w_beg = w_beg0;
  int64_t cnt, total, w_end;  // set once the count has arrived (first-tile block below)

  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.K) + b * a.k_stride_b +
                                                   hkv * a.k_stride_h) + sub * 16;
  const char* vbase = reinterpret_cast<const char*>(static_cast<const T*>(a.V) + b * a.v_stride_b +
                                                   hkv * a.v_stride_h) + sub * 16;
  const uint32_t k_row_bytes = static_cast<uint32_t>(a.k_stride_n * sizeof(T));
  const uint32_t v_row_bytes = static_cast<uint32_t>(a.v_stride_n * sizeof(T));
  const int64_t lu = (!BUF && a.shared_list) ? b : u;  // which list this head reads
  const int32_t* list = BUF ? nullptr : a.idx + lu * a.idx_cap;
  const char* kbuf = nullptr;
  const char* vbuf = nullptr;
  if (BUF) {
    kbuf = reinterpret_cast<const char*>(static_cast<const T*>(a.Kbuf) + u * a.buf_cap * D) + sub * 16;
    vbuf = reinterpret_cast<const char*>(static_cast<const T*>(a.Vbuf) + u * a.buf_cap * D) + sub * 16;
  }

  float qv[EPL];
  Pack16<T>::load(static_cast<const T*>(a.q) + u * D + sub * EPL, qv);
#pragma unroll
  for (int e = 0; e < EPL; ++e) qv[e] *= a.sm_scale_log2;

  float m = -INFINITY, l = 0.f;
  float acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.f;

  // row numbers of a tile: lanes 0..TILE-1 fetch one entry each (selected list, then the
  // dense tail); -1 marks a slot past the end.  The next tile's entries are fetched while the
  // current tile is being processed.
  auto fetch_rows = [&](int64_t t0) -> int32_t {
    const int64_t i = t0 + lane;
    if (lane < TILE && i < w_end) {
      if (BUF) {  // slot i of the list is row i of the buffer; the tail is read from the cache
        if (i < cnt) return static_cast<int32_t>(i);
        const int64_t n = a.tail_begin + (i - cnt);
        return static_cast<int32_t>(n < 0 ? 0 : (n >= a.N ? a.N - 1 : n)) | kTailFlag;
      }
      int64_t n = (i < cnt) ? static_cast<int64_t>(list[i]) : a.tail_begin + (i - cnt);
      n = n < 0 ? 0 : (n >= a.N ? a.N - 1 : n);  // keep the gather inside the cache whatever the list holds
      return static_cast<int32_t>(n);
    }
    return -1;
  };
  int32_t n_next;
  if (BUF) {
    int64_t cnt_now = a.count[u];
    cnt_now = cnt_now < 0 ? 0 : (cnt_now > a.max_count ? a.max_count : cnt_now);
    cnt = cnt_now;
    total = cnt + (a.tail_end - a.tail_begin);
    w_end = (w_beg0 + rows_per_wave < total) ? w_beg0 + rows_per_wave : total;
    n_next = fetch_rows(w_beg0);
  } else {
    // first tile: the list entry is read without waiting for the count (the slot is inside
    // the list's capacity whatever the count is) and sorted out afterwards
    const int64_t i = w_beg0 + lane;
    const int64_t i_safe = (i < a.idx_cap) ? i : (a.idx_cap > 0 ? a.idx_cap - 1 : 0);
    const int32_t raw = (lane < TILE && a.idx_cap > 0) ? list[i_safe] : 0;
    int64_t cnt_now = a.count[lu];
    cnt_now = cnt_now < 0 ? 0 : (cnt_now > a.max_count ? a.max_count : cnt_now);
    cnt = cnt_now;
    total = cnt + (a.tail_end - a.tail_begin);
    w_end = (w_beg0 + rows_per_wave < total) ? w_beg0 + rows_per_wave : total;
    int64_t n = (i < cnt) ? static_cast<int64_t>(raw) : a.tail_begin + (i - cnt);
    n = n < 0 ? 0 : (n >= a.N ? a.N - 1 : n);
    n_next = (lane < TILE && i < w_end) ? static_cast<int32_t>(n) : -1;
  }
  for (int64_t t0 = w_beg; t0 < w_end; t0 += TILE) {
    const int32_t n_mine = n_next;
    typename Pack16<T>::Raw kraw[kLoadsPerTile], vraw[kLoadsPerTile];  // kept packed until used
    bool valid[kLoadsPerTile];
#pragma unroll
    for (int t = 0; t < kLoadsPerTile; ++t) {
      const int32_t n = __shfl(n_mine, t * GPW + grp, kWave);
      valid[t] = n >= 0;
      // 32-bit byte offsets from a per-workgroup base (the host checks that a head's slab is
      // below 4 GiB): one address register per gather instead of two
      if (BUF) {
        const bool tail = valid[t] && (n & kTailFlag);
        const uint32_t row = valid[t] ? static_cast<uint32_t>(n & (kTailFlag - 1)) : 0u;
        const char* kp = tail ? kbase + row * k_row_bytes : kbuf + row * static_cast<uint32_t>(D * sizeof(T));
        const char* vp = tail ? vbase + row * v_row_bytes : vbuf + row * static_cast<uint32_t>(D * sizeof(T));
        kraw[t] = Pack16<T>::load_raw(kp);
        vraw[t] = Pack16<T>::load_raw(vp);
      } else {
        const uint32_t row = valid[t] ? static_cast<uint32_t>(n) : 0u;
        kraw[t] = Pack16<T>::load_raw(kbase + row * k_row_bytes);
        vraw[t] = Pack16<T>::load_raw(vbase + row * v_row_bytes);
      }
    }
    n_next = fetch_rows(t0 + TILE);
    // every gather of the tile is in flight before the first one is consumed
    __builtin_amdgcn_sched_barrier(0);
    float sc[kLoadsPerTile];
    float tmax = -INFINITY;
#pragma unroll
    for (int t = 0; t < kLoadsPerTile; ++t) {
      float kf[EPL];
      Pack16<T>::unpack(kraw[t], kf);
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) s = fmaf(qv[e], kf[e], s);
      s = group_allreduce_sum<LPR>(s);
      sc[t] = valid[t] ? s : -INFINITY;
      tmax = fmaxf(tmax, sc[t]);
    }
    const float m_new = fmaxf(m, tmax);
    if (m_new > -INFINITY) {
      const float alpha = exp2_safe(m - m_new);  // m = -inf -> 0
      l *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] *= alpha;
#pragma unroll
      for (int t = 0; t < kLoadsPerTile; ++t) {
        const float p = exp2_safe(sc[t] - m_new);  // invalid -> 0
        l += p;
        float vf[EPL];
        Pack16<T>::unpack(vraw[t], vf);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[e] = fmaf(p, vf[e], acc[e]);
      }
      m = m_new;
    }
  }
  // merge the row groups of the wave
#pragma unroll
  for (int off = LPR; off < kWave; off <<= 1) {
    const float m_o = __shfl_xor(m, off, kWave);
    const float l_o = __shfl_xor(l, off, kWave);
    const float m_n = fmaxf(m, m_o);
    const float wa = (m_n > -INFINITY) ? exp2_safe(m - m_n) : 0.f;
    const float wb = (m_n > -INFINITY) ? exp2_safe(m_o - m_n) : 0.f;
    l = l * wa + l_o * wb;
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
      const float a_o = __shfl_xor(acc[e], off, kWave);
      acc[e] = acc[e] * wa + a_o * wb;
    }
    m = m_n;
  }
  if (grp == 0) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) s_acc[wave][sub * EPL + e] = acc[e];
    if (sub == 0) {
      s_m[wave] = m;
      s_l[wave] = l;
    }
  }
  __syncthreads();

  // merge the waves of the workgroup: thread d < D owns output element d
  float M = -INFINITY, L = 0.f, o = 0.f;
  if (tid < D) {
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) M = fmaxf(M, s_m[w]);
    if (M > -INFINITY) {
#pragma unroll
      for (int w = 0; w < kAttnWaves; ++w) {
        const float wgt = exp2_safe(s_m[w] - M);
        L += s_l[w] * wgt;
        o += s_acc[w][tid] * wgt;
      }
    }
  }

  if (a.nsplit == 1) {
    if (tid < D) a.out[u * D + tid] = (L > 0.f) ? o / L : 0.f;
    if (tid == 0 && a.lse) a.lse[u] = (L > 0.f) ? M * kLn2 + logf(L) : -INFINITY;
    return;
  }

  // Several workgroups per head: publish the partial, the last one to arrive combines.
  // Partials are written and read with agent-scope accesses, which go through the L2 of the
  // XCD to the memory side where the L2s of all XCDs meet, so the hand-over needs no cache
  // write-back or invalidate.  Ordering: a store counts against the wave's vector-memory
  // counter until the memory side has acknowledged it, so after publish_fence() (s_waitcnt
  // vmcnt(0)) in every storing wave and the workgroup barrier, the partial of this workgroup is
  // in place; only then does thread 0 issue the ticket, a read-modify-write performed at the
  // memory side.  The drawer of the last ticket issues its agent-scope loads after the ticket
  // has returned (branch on its value behind a barrier), so they find every partial whose
  // ticket preceded its own.
  float* part = a.partials + (u * a.nsplit + split) * (D + 2);
  if (tid < D) __hip_atomic_store(&part[tid], o, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (tid == 0) {
    __hip_atomic_store(&part[D], M, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&part[D + 1], L, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  publish_fence();
  __syncthreads();
  if (tid == 0) {
    const uint32_t ticket = __hip_atomic_fetch_add(&a.counters[u * kCounterStrideWords], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (ticket == static_cast<uint32_t>(a.nsplit - 1)) ? 1u : 0u;
  }
  __syncthreads();
  if (!s_last) return;
  // Combine the partials: thread (d, lane-group j) walks splits j, j+G, ... in chunks whose
  // loads are all issued before the first is used (a dependent chain of device-scope loads
  // would cost one memory round trip per split); the G groups are then merged through LDS in
  // group order.  The order of combination is fixed, so the result is reproducible.
  {
    constexpr int G = kAttnThreads / D;  // split groups: 2 for D=128, 4 for D=64
    const int d = tid % D, j = tid / D;
    const float* p0 = a.partials + u * a.nsplit * (D + 2);
    float Mg = -INFINITY, Lg = 0.f, og = 0.f;
    // CH loads in flight per thread and field.  A device-scope load is paid per instruction
    // even when its result is not needed, so the chunk is sized to the split count.
    auto walk = [&](auto ch_tag) {
      constexpr int CH = decltype(ch_tag)::value;
      for (int s0 = j; s0 < a.nsplit; s0 += G * CH) {
        float mv[CH], lv[CH], ov[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int sp = s0 + c * G;
          const int sl = sp < a.nsplit ? sp : a.nsplit - 1;
          mv[c] = __hip_atomic_load(&p0[sl * (D + 2) + D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          lv[c] = __hip_atomic_load(&p0[sl * (D + 2) + D + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          ov[c] = __hip_atomic_load(&p0[sl * (D + 2) + d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          if (sp >= a.nsplit) {
            mv[c] = -INFINITY;
            lv[c] = 0.f;
            ov[c] = 0.f;
          }
        }
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const float Mn = fmaxf(Mg, mv[c]);
          if (Mn > -INFINITY) {
            const float wa = exp2_safe(Mg - Mn), wb = exp2_safe(mv[c] - Mn);
            Lg = Lg * wa + lv[c] * wb;
            og = og * wa + ov[c] * wb;
            Mg = Mn;
          }
        }
      }
    };
    if (a.nsplit <= G)
      walk(std::integral_constant<int, 1>{});
    else if (a.nsplit <= 2 * G)
      walk(std::integral_constant<int, 2>{});
    else if (a.nsplit <= 4 * G)
      walk(std::integral_constant<int, 4>{});
    else
      walk(std::integral_constant<int, 8>{});
    __syncthreads();  // s_acc / s_m / s_l were last read before the partial was published
    s_acc[j][d] = og;
    if (d == 0) {
      s_m[j] = Mg;
      s_l[j] = Lg;
    }
    __syncthreads();
    if (tid < D) {
      float Mt = -INFINITY;
#pragma unroll
      for (int jj = 0; jj < G; ++jj) Mt = fmaxf(Mt, s_m[jj]);
      float Lt = 0.f, ot = 0.f;
      if (Mt > -INFINITY) {
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
          const float wgt = exp2_safe(s_m[jj] - Mt);
          Lt += s_l[jj] * wgt;
          ot += s_acc[jj][tid] * wgt;
        }
      }
      a.out[u * D + tid] = (Lt > 0.f) ? ot / Lt : 0.f;
      if (tid == 0 && a.lse) a.lse[u] = (Lt > 0.f) ? Mt * kLn2 + logf(Lt) : -INFINITY;
    }
  }
  if (tid == 0) __hip_atomic_store(&a.counters[u * kCounterStrideWords], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Head-less lists with grouped queries: the GH query heads of a KV head read the same rows, so
// one workgroup serves all of them: every listed row is loaded once and used GH times (the
// loads, not the arithmetic, bound this kernel).  Work split and tiling as in attn_kernel, with
// one workgroup per (b, kv head, split); every lane group keeps GH softmax states and GH
// accumulator slices.  The partial hand-over uses the counter of the group's first head.
template <typename T, int D, int GH>
__global__ __launch_bounds__(kAttnThreads) void attn_group_kernel(AttnArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int LPR = D / EPL;
  constexpr int GPW = kWave / LPR;
  constexpr int TILE = kLoadsPerTile * GPW;
  constexpr int OUTS = GH * D;                                     // outputs of the workgroup
  constexpr int R = (OUTS + kAttnThreads - 1) / kAttnThreads;      // outputs per thread in the merges
  static_assert(LPR >= 4 && LPR <= 32, "row must span 4..32 lanes");

  __shared__ float s_m[kAttnWaves][GH], s_l[kAttnWaves][GH];
  __shared__ float s_acc[kAttnWaves][GH][D];
  __shared__ uint32_t s_last;

  const int tid = threadIdx.x;
  const int lane = tid & (kWave - 1);
  const int wave = wave_id();
  const int grp = lane / LPR;
  const int sub = lane % LPR;
  const int split = blockIdx.x, hkv = blockIdx.y, b = blockIdx.z;
  const int64_t u0 = static_cast<int64_t>(b) * a.Hq + static_cast<int64_t>(hkv) * GH;  // first head of the group

  const int rows_per_wave = a.rows_per_wg / kAttnWaves;
  const int64_t w_beg = static_cast<int64_t>(split) * a.rows_per_wg + static_cast<int64_t>(wave) * rows_per_wave;

  const char* kbase = reinterpret_cast<const char*>(static_cast<const T*>(a.K) + b * a.k_stride_b +
                                                   hkv * a.k_stride_h) + sub * 16;
  const char* vbase = reinterpret_cast<const char*>(static_cast<const T*>(a.V) + b * a.v_stride_b +
                                                   hkv * a.v_stride_h) + sub * 16;
  const uint32_t k_row_bytes = static_cast<uint32_t>(a.k_stride_n * sizeof(T));
  const uint32_t v_row_bytes = static_cast<uint32_t>(a.v_stride_n * sizeof(T));
  const int32_t* list = a.idx + b * a.idx_cap;

  float qv[GH][EPL];
#pragma unroll
  for (int j = 0; j < GH; ++j) {
    Pack16<T>::load(static_cast<const T*>(a.q) + (u0 + j) * D + sub * EPL, qv[j]);
#pragma unroll
    for (int e = 0; e < EPL; ++e) qv[j][e] *= a.sm_scale_log2;
  }
  float m[GH], l[GH], acc[GH][EPL];
#pragma unroll
  for (int j = 0; j < GH; ++j) {
    m[j] = -INFINITY;
    l[j] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[j][e] = 0.f;
  }

  int64_t cnt = a.count[b];
  cnt = cnt < 0 ? 0 : (cnt > a.max_count ? a.max_count : cnt);
  const int64_t total = cnt + (a.tail_end - a.tail_begin);
  const int64_t w_end = (w_beg + rows_per_wave < total) ? w_beg + rows_per_wave : total;
  // row numbers of a tile: lanes 0..TILE-1 fetch one entry each (list, then the dense tail)
  auto fetch_rows = [&](int64_t t0) -> int32_t {
    const int64_t i = t0 + lane;
    if (lane < TILE && i < w_end) {
      int64_t n = (i < cnt) ? static_cast<int64_t>(list[i]) : a.tail_begin + (i - cnt);
      n = n < 0 ? 0 : (n >= a.N ? a.N - 1 : n);  // keep the gather inside the cache whatever the list holds
      return static_cast<int32_t>(n);
    }
    return -1;
  };
  int32_t n_next = fetch_rows(w_beg);
  for (int64_t t0 = w_beg; t0 < w_end; t0 += TILE) {
    const int32_t n_mine = n_next;
    typename Pack16<T>::Raw kraw[kLoadsPerTile], vraw[kLoadsPerTile];
    bool valid[kLoadsPerTile];
#pragma unroll
    for (int t = 0; t < kLoadsPerTile; ++t) {
      const int32_t n = __shfl(n_mine, t * GPW + grp, kWave);
      valid[t] = n >= 0;
      const uint32_t row = valid[t] ? static_cast<uint32_t>(n) : 0u;
      kraw[t] = Pack16<T>::load_raw(kbase + row * k_row_bytes);
      vraw[t] = Pack16<T>::load_raw(vbase + row * v_row_bytes);
    }
    n_next = fetch_rows(t0 + TILE);
    __builtin_amdgcn_sched_barrier(0);  // every gather of the tile is in flight before the first is consumed
    float sc[GH][kLoadsPerTile];
#pragma unroll
    for (int t = 0; t < kLoadsPerTile; ++t) {
      float kf[EPL];
      Pack16<T>::unpack(kraw[t], kf);
#pragma unroll
      for (int j = 0; j < GH; ++j) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(qv[j][e], kf[e], s);
        s = group_allreduce_sum<LPR>(s);
        sc[j][t] = valid[t] ? s : -INFINITY;
      }
    }
#pragma unroll
    for (int j = 0; j < GH; ++j) {
      float tmax = sc[j][0];
#pragma unroll
      for (int t = 1; t < kLoadsPerTile; ++t) tmax = fmaxf(tmax, sc[j][t]);
      const float m_new = fmaxf(m[j], tmax);
      const float m_ref = (m_new > -INFINITY) ? m_new : 0.f;  // nothing seen yet: all weights 0
      const float alpha = exp2_safe(m[j] - m_ref);
      l[j] *= alpha;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[j][e] *= alpha;
#pragma unroll
      for (int t = 0; t < kLoadsPerTile; ++t) {
        sc[j][t] = exp2_safe(sc[j][t] - m_ref);  // invalid -> 0
        l[j] += sc[j][t];
      }
      m[j] = m_new;
    }
#pragma unroll
    for (int t = 0; t < kLoadsPerTile; ++t) {
      float vf[EPL];
      Pack16<T>::unpack(vraw[t], vf);
#pragma unroll
      for (int j = 0; j < GH; ++j)
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[j][e] = fmaf(sc[j][t], vf[e], acc[j][e]);
    }
  }

  // merge the row groups of the wave, head by head
#pragma unroll
  for (int j = 0; j < GH; ++j) {
#pragma unroll
    for (int off = LPR; off < kWave; off <<= 1) {
      const float m_o = __shfl_xor(m[j], off, kWave);
      const float l_o = __shfl_xor(l[j], off, kWave);
      const float m_n = fmaxf(m[j], m_o);
      const float wa = (m_n > -INFINITY) ? exp2_safe(m[j] - m_n) : 0.f;
      const float wb = (m_n > -INFINITY) ? exp2_safe(m_o - m_n) : 0.f;
      l[j] = l[j] * wa + l_o * wb;
#pragma unroll
      for (int e = 0; e < EPL; ++e) {
        const float a_o = __shfl_xor(acc[j][e], off, kWave);
        acc[j][e] = acc[j][e] * wa + a_o * wb;
      }
      m[j] = m_n;
    }
    if (grp == 0) {
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_acc[wave][j][sub * EPL + e] = acc[j][e];
      if (sub == 0) {
        s_m[wave][j] = m[j];
        s_l[wave][j] = l[j];
      }
    }
  }
  __syncthreads();

  // merge the waves: thread owns outputs (head, element) number tid, tid + 256, ...
  float M[R], L[R], o[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = tid + r * kAttnThreads;
    const int hh = (e < OUTS) ? e / D : 0, d = e % D;
    M[r] = -INFINITY;
    L[r] = 0.f;
    o[r] = 0.f;
#pragma unroll
    for (int w = 0; w < kAttnWaves; ++w) M[r] = fmaxf(M[r], s_m[w][hh]);
    if (M[r] > -INFINITY) {
#pragma unroll
      for (int w = 0; w < kAttnWaves; ++w) {
        const float wgt = exp2_safe(s_m[w][hh] - M[r]);
        L[r] += s_l[w][hh] * wgt;
        o[r] += s_acc[w][hh][d] * wgt;
      }
    }
  }

  if (a.nsplit == 1) {
#pragma unroll
    for (int r = 0; r < R; ++r) {
      const int e = tid + r * kAttnThreads;
      if (e < OUTS) {
        const int hh = e / D, d = e % D;
        a.out[(u0 + hh) * D + d] = (L[r] > 0.f) ? o[r] / L[r] : 0.f;
        if (d == 0 && a.lse) a.lse[u0 + hh] = (L[r] > 0.f) ? M[r] * kLn2 + logf(L[r]) : -INFINITY;
      }
    }
    return;
  }

  // several workgroups per KV group: publish the partials (agent-scope accesses and the same
  // ordering as in attn_kernel), take a ticket, the last to arrive combines in split order
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = tid + r * kAttnThreads;
    if (e < OUTS) {
      const int hh = e / D, d = e % D;
      float* part = a.partials + ((u0 + hh) * a.nsplit + split) * (D + 2);
      __hip_atomic_store(&part[d], o[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (d == 0) {
        __hip_atomic_store(&part[D], M[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&part[D + 1], L[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
    }
  }
  publish_fence();
  __syncthreads();
  if (tid == 0) {
    const uint32_t ticket = __hip_atomic_fetch_add(&a.counters[u0 * kCounterStrideWords], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_last = (ticket == static_cast<uint32_t>(a.nsplit - 1)) ? 1u : 0u;
  }
  __syncthreads();
  if (!s_last) return;
  // Combine: the device-scope loads of a chunk are issued together: per thread its R outputs
  // of CH splits; the (max, sum) pairs of those splits, the same for all elements of a head,
  // are fetched once by GH * CH threads and passed through LDS.  Splits are merged in order.
  // A device-scope load is paid per instruction even when its result is not needed, so the
  // chunk is sized to the split count.
  constexpr int kMaxCH = (R <= 2) ? 32 : 16;
  static_assert(GH * kMaxCH <= kAttnThreads, "one thread per (head, split) pair of a chunk");
  __shared__ float s_pm[GH][kMaxCH], s_pl[GH][kMaxCH];
  float Mg[R], Lg[R], og[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    Mg[r] = -INFINITY;
    Lg[r] = 0.f;
    og[r] = 0.f;
  }
  auto walk = [&](auto ch_tag) {
    constexpr int CH = decltype(ch_tag)::value < kMaxCH ? decltype(ch_tag)::value : kMaxCH;
    for (int s0 = 0; s0 < a.nsplit; s0 += CH) {
      float ov[R][CH];
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int e = tid + r * kAttnThreads;
        const int hh = (e < OUTS) ? e / D : 0, d = e % D;
        const float* p0 = a.partials + (u0 + hh) * a.nsplit * (D + 2);
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const int sl = (s0 + c < a.nsplit) ? s0 + c : a.nsplit - 1;
          ov[r][c] = __hip_atomic_load(&p0[sl * (D + 2) + d], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
      }
      if (tid < GH * CH) {
        const int hh = tid / CH, c = tid % CH;
        const float* p0 = a.partials + (u0 + hh) * a.nsplit * (D + 2);
        const int sl = (s0 + c < a.nsplit) ? s0 + c : a.nsplit - 1;
        const float pm = __hip_atomic_load(&p0[sl * (D + 2) + D], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const float pl = __hip_atomic_load(&p0[sl * (D + 2) + D + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_pm[hh][c] = (s0 + c < a.nsplit) ? pm : -INFINITY;  // a slot past the last split weighs nothing
        s_pl[hh][c] = (s0 + c < a.nsplit) ? pl : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const int e = tid + r * kAttnThreads;
        const int hh = (e < OUTS) ? e / D : 0;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
          const float mv = s_pm[hh][c];
          const float Mn = fmaxf(Mg[r], mv);
          if (Mn > -INFINITY) {
            const float wa = exp2_safe(Mg[r] - Mn), wb = exp2_safe(mv - Mn);
            Lg[r] = Lg[r] * wa + s_pl[hh][c] * wb;
            og[r] = og[r] * wa + ov[r][c] * wb;
            Mg[r] = Mn;
          }
        }
      }
      __syncthreads();  // the pairs are overwritten by the next chunk
    }
  };
  if (a.nsplit <= 2)
    walk(std::integral_constant<int, 2>{});
  else if (a.nsplit <= 4)
    walk(std::integral_constant<int, 4>{});
  else if (a.nsplit <= 8)
    walk(std::integral_constant<int, 8>{});
  else if (a.nsplit <= 16)
    walk(std::integral_constant<int, 16>{});
  else
    walk(std::integral_constant<int, 32>{});
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int e = tid + r * kAttnThreads;
    if (e < OUTS) {
      const int hh = e / D, d = e % D;
      a.out[(u0 + hh) * D + d] = (Lg[r] > 0.f) ? og[r] / Lg[r] : 0.f;
      if (d == 0 && a.lse) a.lse[u0 + hh] = (Lg[r] > 0.f) ? Mg[r] * kLn2 + logf(Lg[r]) : -INFINITY;
    }
  }
  if (tid == 0) __hip_atomic_store(&a.counters[u0 * kCounterStrideWords], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <typename T, int D, int GH>
tb_status launch_group(const AttnArgs& a, const AttnLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  hipLaunchKernelGGL((attn_group_kernel<T, D, GH>), dim3(L.plan.nsplit, d.Hkv, d.B), dim3(kAttnThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

template <typename T, int D>
tb_status launch_td(const AttnLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  AttnArgs a;
  a.q = L.q;
  a.K = L.K;
  a.V = L.V;
  a.idx = L.idx;
  a.count = L.count;
  a.idx_cap = L.idx_cap;
  a.max_count = L.max_count;
  a.tail_begin = L.tail_begin;
  a.tail_end = L.tail_end;
  a.N = d.N;
  a.k_stride_b = d.k_stride_b;
  a.k_stride_h = d.k_stride_h;
  a.k_stride_n = d.k_stride_n;
  a.v_stride_b = d.v_stride_b;
  a.v_stride_h = d.v_stride_h;
  a.v_stride_n = d.v_stride_n;
  a.sm_scale_log2 = L.sm_scale * kLog2e;
  a.out = L.out;
  a.lse = L.lse;
  a.partials = L.partials;
  a.counters = L.counters;
  a.Hq = d.Hq;
  a.g = d.Hq / d.Hkv;
  a.rows_per_wg = L.plan.rows_per_wg;
  a.nsplit = L.plan.nsplit;
  a.Kbuf = L.Kbuf;
  a.Vbuf = L.Vbuf;
  a.buf_cap = L.buf_cap;
  a.shared_list = L.shared_list ? 1 : 0;
  a.n_kv_groups = d.B * d.Hkv;
  // per-XCD placement pays when heads share KV rows and the KV groups spread evenly over the XCDs
  a.xcd_map = (a.g > 1 && (a.n_kv_groups % kXcds == 0 || a.n_kv_groups >= 8 * kXcds)) ? 1 : 0;
  if (L.grouped) {  // the plan was made for one workgroup per KV group
    if (a.g == 2) return launch_group<T, D, 2>(a, L, st);
    if (a.g == 4) return launch_group<T, D, 4>(a, L, st);
    if (a.g == 8) return launch_group<T, D, 8>(a, L, st);
    return TB_ERR_UNSUPPORTED;
  }
  dim3 grid(L.plan.nsplit, d.Hq, d.B);
  if (a.xcd_map) grid = dim3(static_cast<unsigned>(kXcds * ((a.n_kv_groups + kXcds - 1) / kXcds) * a.g * a.nsplit));
  if (L.Kbuf)
    hipLaunchKernelGGL((attn_kernel<T, D, true>), grid, dim3(kAttnThreads), 0, st, a);
  else
    hipLaunchKernelGGL((attn_kernel<T, D, false>), grid, dim3(kAttnThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace

int attn_tile_rows_per_wg(int dtype, int D) {
  const int elt = dtype == TB_F32 ? 4 : 2;
  const int lpr = D * elt / 16;
  return kAttnWaves * kLoadsPerTile * (kWave / lpr);
}

tb_status launch_attn(const AttnLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  if (d.B == 0 || d.Hq == 0) return TB_OK;
  if (d.dtype == TB_F32) {
    if (d.D == 64) return launch_td<float, 64>(L, st);
    if (d.D == 128) return launch_td<float, 128>(L, st);
  } else {
    if (d.D == 64) return launch_td<bf16_t, 64>(L, st);
    if (d.D == 128) return launch_td<bf16_t, 128>(L, st);
  }
  return TB_ERR_UNSUPPORTED;
}

}  // namespace tb
