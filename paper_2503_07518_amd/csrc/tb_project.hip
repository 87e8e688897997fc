// Key-cache projection K_imp = K W: rows [n_begin, n_end) of every (b, kv-head).
//
// One workgroup projects a tile of 64 cache rows.  W (D x Dimp) and the K tile are staged in
// LDS as fp32, 64 columns of the head dimension per round; thread (row, quarter) accumulates
// Dimp/4 adjacent outputs in fp32 and rounds once (round to nearest even) to the storage type.
// The same kernel serves the one-row append of a decode step and the batched projection of a
// window of rows.
#include "tb_device.h"
#include "tb_internal.h"

namespace tb {
namespace {

constexpr int kProjThreads = 256;
constexpr int kProjRows = 64;

struct ProjectArgs {
  const void* K;
  const void* W;
  void* Kimp;
  int64_t n_begin, n_end;
  int64_t k_stride_b, k_stride_h, k_stride_n;
  int64_t ki_stride_b, ki_stride_h, ki_stride_n;
  int32_t per_head_w;
};

template <typename T, int D, int DIMP>
__global__ __launch_bounds__(kProjThreads) void project_kernel(ProjectArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int OPT = DIMP / 4;  // outputs per thread
  constexpr int DC = 64;         // slice of the head dimension staged per round
  constexpr int KS = DC + 1;     // padded row stride of the K tile in LDS
  static_assert(D % DC == 0, "head_dim must be a multiple of 64");
  __shared__ float s_w[DC * DIMP];
  __shared__ float s_k[kProjRows * KS];

  const int tid = threadIdx.x;
  const int b = blockIdx.z, h = blockIdx.y;
  const int64_t row0 = a.n_begin + static_cast<int64_t>(blockIdx.x) * kProjRows;
  const T* w = static_cast<const T*>(a.W) + (a.per_head_w ? static_cast<int64_t>(h) * D * DIMP : 0);
  const T* kb = static_cast<const T*>(a.K) + b * a.k_stride_b + h * a.k_stride_h;
  constexpr int CPR = DC / EPL;  // 16-byte chunks per staged row slice

  const int r = tid / 4;
  const int j0 = (tid % 4) * OPT;
  float acc[OPT];
#pragma unroll
  for (int j = 0; j < OPT; ++j) acc[j] = 0.f;

  for (int d0 = 0; d0 < D; d0 += DC) {
    if (d0) __syncthreads();
    for (int i = tid * EPL; i < DC * DIMP; i += kProjThreads * EPL) {
      float f[EPL];
      Pack16<T>::load(w + d0 * DIMP + i, f);
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_w[i + e] = f[e];
    }
    for (int ch = tid; ch < kProjRows * CPR; ch += kProjThreads) {
      const int rr = ch / CPR, cc = ch % CPR;
      const int64_t row = row0 + rr;
      float f[EPL];
      if (row < a.n_end) {
        Pack16<T>::load(kb + row * a.k_stride_n + d0 + cc * EPL, f);
      } else {
#pragma unroll
        for (int e = 0; e < EPL; ++e) f[e] = 0.f;
      }
#pragma unroll
      for (int e = 0; e < EPL; ++e) s_k[rr * KS + cc * EPL + e] = f[e];
    }
    __syncthreads();
#pragma unroll 4
    for (int d = 0; d < DC; ++d) {
      const float kd = s_k[r * KS + d];
#pragma unroll
      for (int j = 0; j < OPT; ++j) acc[j] = fmaf(kd, s_w[d * DIMP + j0 + j], acc[j]);
    }
  }
  const int64_t row = row0 + r;
  if (row < a.n_end) {
    T* o = static_cast<T*>(a.Kimp) + b * a.ki_stride_b + h * a.ki_stride_h + row * a.ki_stride_n + j0;
#pragma unroll
    for (int j = 0; j < OPT; ++j) store_elt(o + j, acc[j]);
  }
}

template <typename T, int D, int DIMP>
tb_status launch_tdd(const tb_cache_desc& d, const ProjectArgs& a, hipStream_t st) {
  const int64_t rows = a.n_end - a.n_begin;
  dim3 grid(static_cast<unsigned>((rows + kProjRows - 1) / kProjRows), d.Hkv, d.B);
  hipLaunchKernelGGL((project_kernel<T, D, DIMP>), grid, dim3(kProjThreads), 0, st, a);
  return hip_status(hipGetLastError());
}

template <typename T, int D>
tb_status launch_td(const tb_cache_desc& d, const ProjectArgs& a, hipStream_t st) {
  switch (d.Dimp) {
    case 16: return launch_tdd<T, D, 16>(d, a, st);
    case 32: return launch_tdd<T, D, 32>(d, a, st);
    case 64: return launch_tdd<T, D, 64>(d, a, st);
    default: return TB_ERR_UNSUPPORTED;
  }
}

template <typename T>
tb_status launch_t(const tb_cache_desc& d, const ProjectArgs& a, hipStream_t st) {
  switch (d.D) {
    case 64: return launch_td<T, 64>(d, a, st);
    case 128: return launch_td<T, 128>(d, a, st);
    default: return TB_ERR_UNSUPPORTED;
  }
}

}  // namespace

tb_status launch_project(const tb_cache_desc* d, const void* K, const void* W, int32_t Hw, void* Kimp,
                         int64_t n_begin, int64_t n_end, hipStream_t st) {
  if (n_end <= n_begin || d->B == 0 || d->Hkv == 0) return TB_OK;
  ProjectArgs a;
  a.K = K;
  a.W = W;
  a.Kimp = Kimp;
  a.n_begin = n_begin;
  a.n_end = n_end;
  a.k_stride_b = d->k_stride_b;
  a.k_stride_h = d->k_stride_h;
  a.k_stride_n = d->k_stride_n;
  a.ki_stride_b = d->ki_stride_b;
  a.ki_stride_h = d->ki_stride_h;
  a.ki_stride_n = d->ki_stride_n;
  a.per_head_w = (Hw != 1) ? 1 : 0;
  return d->dtype == TB_F32 ? launch_t<float>(*d, a, st) : launch_t<bf16_t>(*d, a, st);
}

}  // namespace tb
