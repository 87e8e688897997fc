// Migration of the selected K/V rows into per-query-head "important" buffers (the paper's
// physical layout, Sec. 3.3): Kbuf/Vbuf[b,h,i,:] = K/V[b,h/g,idx[b,h,skip_front + i],:] for
// i < count[b,h] - skip_front - skip_back (the entries at the two ends of a list are the sink
// prefix and the local window, which live in buffers of their own).
// A pure copy: LPR = D*sizeof(T)/16 adjacent lanes move one row with a 128-bit load and store
// each; a thread issues the loads of all its rows (K and V) before the first store.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kGatherThreads = 256;
constexpr int kGatherRowsPerThread = 4;

struct GatherArgs {
  const void* K;
  const void* V;
  const int32_t* idx;
  const int32_t* count;
  int64_t idx_cap, max_count, N;
  int64_t k_stride_b, k_stride_h, k_stride_n;
  int64_t v_stride_b, v_stride_h, v_stride_n;
  void* Kbuf;
  void* Vbuf;
  int64_t buf_cap;
  int32_t Hq, g;
  int32_t skip_front, skip_back;  // list entries left out at the two ends
  int32_t* count_out;             // nullable: receives the number of rows migrated per (b,h)
};

template <typename T, int D>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(GatherArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int LPR = D / EPL;                  // lanes per row
  constexpr int RPP = kGatherThreads / LPR;     // rows per pass of the workgroup
  typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
  const int tid = threadIdx.x;
  const int sub = tid % LPR, rsub = tid / LPR;
  const int h = blockIdx.y, b = blockIdx.z;
  const int64_t u = static_cast<int64_t>(b) * a.Hq + h;
  const int hkv = h / a.g;
  int64_t cnt = a.count[u];
  cnt = cnt < 0 ? 0 : (cnt > a.max_count ? a.max_count : cnt);
  cnt -= a.skip_front + a.skip_back;
  cnt = cnt < 0 ? 0 : cnt;
  if (a.count_out && blockIdx.x == 0 && tid == 0) a.count_out[u] = static_cast<int32_t>(cnt);
  const int64_t i0 = static_cast<int64_t>(blockIdx.x) * RPP * kGatherRowsPerThread + rsub;
  if (i0 - rsub >= cnt) return;
  const int32_t* list = a.idx + u * a.idx_cap + a.skip_front;
  const T* kb = static_cast<const T*>(a.K) + b * a.k_stride_b + hkv * a.k_stride_h + sub * EPL;
  const T* vb = static_cast<const T*>(a.V) + b * a.v_stride_b + hkv * a.v_stride_h + sub * EPL;
  T* ko = static_cast<T*>(a.Kbuf) + u * a.buf_cap * D + sub * EPL;
  T* vo = static_cast<T*>(a.Vbuf) + u * a.buf_cap * D + sub * EPL;
  u32x4 kr[kGatherRowsPerThread], vr[kGatherRowsPerThread];
#pragma unroll
  for (int r = 0; r < kGatherRowsPerThread; ++r) {
    const int64_t i = i0 + r * RPP;
    int64_t n = (i < cnt) ? static_cast<int64_t>(list[i]) : 0;
    n = n < 0 ? 0 : (n >= a.N ? a.N - 1 : n);  // stay inside the cache whatever the list holds
    kr[r] = *reinterpret_cast<const u32x4*>(kb + n * a.k_stride_n);
    vr[r] = *reinterpret_cast<const u32x4*>(vb + n * a.v_stride_n);
  }
#pragma unroll
  for (int r = 0; r < kGatherRowsPerThread; ++r) {
    const int64_t i = i0 + r * RPP;
    if (i < cnt) {
      *reinterpret_cast<u32x4*>(ko + i * D) = kr[r];
      *reinterpret_cast<u32x4*>(vo + i * D) = vr[r];
    }
  }
}

template <typename T, int D>
tb_status launch_td(const GatherLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  GatherArgs a;
  a.K = L.K;
  a.V = L.V;
  a.idx = L.idx;
  a.count = L.count;
  a.idx_cap = L.idx_cap;
  a.max_count = L.max_count;
  a.N = d.N;
  a.k_stride_b = d.k_stride_b;
  a.k_stride_h = d.k_stride_h;
  a.k_stride_n = d.k_stride_n;
  a.v_stride_b = d.v_stride_b;
  a.v_stride_h = d.v_stride_h;
  a.v_stride_n = d.v_stride_n;
  a.Kbuf = L.Kbuf;
  a.Vbuf = L.Vbuf;
  a.buf_cap = L.buf_cap;
  a.Hq = d.Hq;
  a.g = d.Hq / d.Hkv;
  a.skip_front = L.skip_front;
  a.skip_back = L.skip_back;
  a.count_out = L.count_out;
  constexpr int rows_per_wg = kGatherThreads / (D / Pack16<T>::kElts) * kGatherRowsPerThread;
  // (at least one workgroup per list, so that count_out is written for an empty one too)
  const int64_t rows = L.max_count > L.skip_front + L.skip_back ? L.max_count - L.skip_front - L.skip_back : 1;
  dim3 grid(static_cast<unsigned>((rows + rows_per_wg - 1) / rows_per_wg), d.Hq, d.B);
  hipLaunchKernelGGL((gather_kernel<T, D>), grid, dim3(kGatherThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

}  // namespace

tb_status launch_gather(const GatherLaunch& L, hipStream_t st) {
  const tb_cache_desc& d = *L.desc;
  if (d.B == 0 || d.Hq == 0 || (L.max_count == 0 && !L.count_out)) return TB_OK;
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
