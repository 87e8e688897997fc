// Importance-query prediction of a producer layer: q_imp = f(LN(h)) with f a two-layer MLP
// (Sec. 3.1 "Query prediction"; hidden size 512 in the paper's experiments).  At decode time h is
// one hidden state per sequence, so both layers are matrix-vector products bound by reading
// the weights once: a wave owns an output row (torch Linear layout, [out][in], contiguous),
// its lanes stride over the row with 128-bit loads, and up to 8 batch rows of the workgroup sit
// in LDS as fp32 (the weights are read once per 8 sequences).
//
// hidden_kernel:  LN over E (two-pass mean / variance, fp32), z = gelu(W1 x + b1)
// output_kernel:  y = W2 z + b2, rounded once to the storage type and scattered to
//                 q_imp[slot][b][head][j]   (row o of W2 is (slot, head, j), slot outermost)
#include "tb_device.h"
#include "tb_internal.h"

#ifdef TB_PROBE
__device__ unsigned long long tb_pred_probe[16];
#define TB_PMARK(i)                                                                              \
  do {                                                                                           \
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) tb_pred_probe[i] = wall_clock64(); \
  } while (0)
#else
#define TB_PMARK(i)
#endif

namespace tb {
namespace {

constexpr int kPredThreads = 256;
constexpr int kPredWaves = kPredThreads / kWave;
constexpr int kMaxE = 8192;
constexpr size_t kLdsBudget = 144 * 1024;  // of the 160 KiB of a compute unit, for the staged hidden states
constexpr int kMaxHidden = 2048;
constexpr int kOutRowsPerWave = 8;

struct PredictArgs {
  const void* h;
  const void* gamma;
  const void* beta;
  const void* W1;
  const void* b1;
  const void* W2;
  const void* b2;
  float* z;    // [B][hidden] fp32
  float* xln;  // [B][E] fp32: LN(h), written by ln_kernel for the batched form
  void* q_imp;
  int32_t B, E, hidden, G, Hq, Dimp;
  float eps;
};

// Sum over the 64 lanes with DPP moves (row shifts, then the row broadcasts); every lane gets it.
__device__ inline float wave_total(float v) {
  constexpr int kRowShr = 0x110, kRowBcast15 = 0x142, kRowBcast31 = 0x143;
  auto dpp = [](float x, auto ctrl, auto row_mask) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value,
                                                      decltype(row_mask)::value, 0xF, false));
  };
  using std::integral_constant;
  v += dpp(v, integral_constant<int, kRowShr + 1>{}, integral_constant<int, 0xF>{});
  v += dpp(v, integral_constant<int, kRowShr + 2>{}, integral_constant<int, 0xF>{});
  v += dpp(v, integral_constant<int, kRowShr + 4>{}, integral_constant<int, 0xF>{});
  v += dpp(v, integral_constant<int, kRowShr + 8>{}, integral_constant<int, 0xF>{});
  v += dpp(v, integral_constant<int, kRowBcast15>{}, integral_constant<int, 0xA>{});
  v += dpp(v, integral_constant<int, kRowBcast31>{}, integral_constant<int, 0xC>{});
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), kWave - 1));
}

// LDS position of element e of a staged fp32 row.  A lane of the dot products owns EPL adjacent
// elements (one 128-bit piece of the weight row) and the 64 lanes own adjacent pieces, so in
// natural order the lanes would read 16-byte groups that lie 4*EPL bytes apart (bank conflicts);
// inside every block of 64*EPL elements the row is therefore stored with the 4-element groups
// transposed: group g of piece p at (g*64 + p)*4, which lets the 64 lanes read one group each
// from 64 adjacent 16-byte slots with a single 128-bit LDS read.
template <int EPL>
__device__ inline int staged_pos(int e) {
  constexpr int kBlock = kWave * EPL;
  const int in_block = e % kBlock;
  const int piece = in_block / EPL, within = in_block % EPL;
  return e - in_block + ((within / 4) * kWave + piece) * 4 + within % 4;
}
template <int EPL>
__host__ __device__ inline int staged_len(int n) {  // row length in LDS: whole blocks
  constexpr int kBlock = kWave * EPL;
  return (n + kBlock - 1) / kBlock * kBlock;
}

// Workgroup-wide sums of BC values per thread in one go (two barriers for all of them).
template <int BC>
__device__ inline void block_sums(const float (&v)[BC], float (*s_red)[BC], float (&total)[BC]) {
  float w[BC];
#pragma unroll
  for (int i = 0; i < BC; ++i) w[i] = wave_total(v[i]);
  __syncthreads();  // s_red may still be read from the previous reduction
  if (lane_id() == 0) {
#pragma unroll
    for (int i = 0; i < BC; ++i) s_red[threadIdx.x / kWave][i] = w[i];
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < BC; ++i) {
    total[i] = 0.f;
#pragma unroll
    for (int k = 0; k < kPredWaves; ++k) total[i] += s_red[k][i];
  }
}

__device__ inline float gelu_erf(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }

constexpr int kRowLoads = 8;  // 128-bit loads of a weight row that a lane issues ahead of their use

// LayerNorm of one hidden state per workgroup, written as fp32 (batched form: the matrix-vector
// kernel then only stages the normalised rows instead of normalising them again in each of
// its workgroups).  The row stays in registers for the two passes.
template <typename T>
__global__ __launch_bounds__(kPredThreads) void ln_kernel(PredictArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int kMaxChunks = kMaxE / EPL / kPredThreads;
  __shared__ float s_red[kPredWaves][1];
  const int tid = threadIdx.x;
  const int n_chunks = a.E / EPL;
  const T* row = static_cast<const T*>(a.h) + static_cast<int64_t>(blockIdx.x) * a.E;
  typename Pack16<T>::Raw raw[kMaxChunks], graw[kMaxChunks], braw[kMaxChunks];
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {  // every load first; pieces past the row read piece 0 and are dropped
    const int ch = tid + c * kPredThreads;
    const int off = (ch < n_chunks ? ch : 0) * EPL;
    raw[c] = Pack16<T>::load_raw(row + off);
    graw[c] = Pack16<T>::load_raw(static_cast<const T*>(a.gamma) + off);
    braw[c] = Pack16<T>::load_raw(static_cast<const T*>(a.beta) + off);
  }
  float hv[kMaxChunks][EPL];
  float part[1] = {0.f}, mean[1], var[1];
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    Pack16<T>::unpack(raw[c], hv[c]);
    if (tid + c * kPredThreads < n_chunks) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) part[0] += hv[c][i];
    }
  }
  block_sums<1>(part, s_red, mean);
  mean[0] /= static_cast<float>(a.E);
  part[0] = 0.f;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    if (tid + c * kPredThreads < n_chunks) {
#pragma unroll
      for (int i = 0; i < EPL; ++i) {
        hv[c][i] -= mean[0];
        part[0] += hv[c][i] * hv[c][i];
      }
    }
  }
  block_sums<1>(part, s_red, var);
  const float rstd = 1.0f / sqrtf(var[0] / static_cast<float>(a.E) + a.eps);
  float* out = a.xln + static_cast<int64_t>(blockIdx.x) * a.E;
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int ch = tid + c * kPredThreads;
    if (ch < n_chunks) {
      float gm[EPL], bt[EPL];
      Pack16<T>::unpack(graw[c], gm);
      Pack16<T>::unpack(braw[c], bt);
#pragma unroll
      for (int i = 0; i < EPL; i += 4)
        *reinterpret_cast<float4*>(out + ch * EPL + i) =
            make_float4(hv[c][i] * rstd * gm[i] + bt[i], hv[c][i + 1] * rstd * gm[i + 1] + bt[i + 1],
                        hv[c][i + 2] * rstd * gm[i + 2] + bt[i + 2], hv[c][i + 3] * rstd * gm[i + 3] + bt[i + 3]);
    }
  }
}

// BC batch rows per workgroup (1, 2, 4 or 8): the weights are read once per BC sequences.
// FUSED_LN: the workgroup normalises its rows itself (small batches: one launch less);
// otherwise it stages the rows that ln_kernel has normalised.
template <typename T, int BC, bool FUSED_LN>
__global__ __launch_bounds__(kPredThreads) void hidden_kernel(PredictArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int kStep = kWave * EPL;  // elements of a row that the wave covers per load
  constexpr int kMaxChunks = kMaxE / EPL / kPredThreads;  // 16-byte pieces of a hidden state per thread
  extern __shared__ float s_x[];  // [BC][staged_len(E)]
  const int e_pad = staged_len<EPL>(a.E);
  __shared__ float s_red[kPredWaves][BC];
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b0 = blockIdx.y * BC;
  const int nb = min(BC, a.B - b0);
  const T* h = static_cast<const T*>(a.h);

  TB_PMARK(0);
  // the first loads of this wave's weight row go out before the LayerNorm (they do not depend on it)
  const int r = blockIdx.x * kPredWaves + wave;       // hidden unit of this wave
  const int r_safe = r < a.hidden ? r : a.hidden - 1;
  const T* w = static_cast<const T*>(a.W1) + static_cast<int64_t>(r_safe) * a.E;
  typename Pack16<T>::Raw wraw[kRowLoads];
#pragma unroll
  for (int i = 0; i < kRowLoads; ++i) {
    const int e0 = lane * EPL + i * kStep;
    wraw[i] = Pack16<T>::load_raw(w + (e0 < a.E ? e0 : 0));
  }

  if constexpr (!FUSED_LN) {
    // stage the normalised rows (fp32, contiguous [nb][E]) with 128-bit loads, eight in flight
    // four rows at a time, four 128-bit loads per row and thread: sixteen loads in flight
    const int per_row = a.E / 4;
    constexpr int kRowsAtOnce = BC < 4 ? BC : 4;
    for (int bc0 = 0; bc0 < nb; bc0 += kRowsAtOnce) {
      for (int p0 = tid; p0 < per_row; p0 += kPredThreads * 4) {
        float4 v[kRowsAtOnce][4];
#pragma unroll
        for (int rr = 0; rr < kRowsAtOnce; ++rr) {
          const int bc = bc0 + rr < nb ? bc0 + rr : nb - 1;
          const float4* src = reinterpret_cast<const float4*>(a.xln + static_cast<int64_t>(b0 + bc) * a.E);
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const int p = p0 + k * kPredThreads;
            v[rr][k] = src[p < per_row ? p : per_row - 1];
          }
        }
#pragma unroll
        for (int rr = 0; rr < kRowsAtOnce; ++rr) {
          if (bc0 + rr < nb) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
              const int p = p0 + k * kPredThreads;
              if (p < per_row)
                *reinterpret_cast<float4*>(s_x + (bc0 + rr) * e_pad + staged_pos<EPL>(p * 4)) = v[rr][k];  // a whole group
            }
          }
        }
      }
    }
    for (int i = nb * e_pad + tid; i < BC * e_pad; i += kPredThreads) s_x[i] = 0.f;  // rows past the batch
  } else {
  // LayerNorm of the workgroup's batch rows, all rows together: a thread stages its 16-byte
  // pieces of every row in LDS as fp32 (re-reading only what it wrote itself), the per-row sums
  // of all rows go through one workgroup reduction per pass (mean, then squared deviations)
  const int n_chunks = a.E / EPL;
  float psum[BC];
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) {
    psum[bc] = 0.f;
    if (bc < nb) {
      const T* row = h + static_cast<int64_t>(b0 + bc) * a.E;
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) {
        const int ch = tid + c * kPredThreads;
        if (ch < n_chunks) {
          float hv[EPL];
          Pack16<T>::load(row + ch * EPL, hv);
#pragma unroll
          for (int i = 0; i < EPL; ++i) {
            s_x[bc * e_pad + staged_pos<EPL>(ch * EPL + i)] = hv[i];
            psum[bc] += hv[i];
          }
        }
      }
    }
  }
  for (int i = nb * e_pad + tid; i < BC * e_pad; i += kPredThreads) s_x[i] = 0.f;  // rows past the batch
  float mean[BC], rstd[BC];
  TB_PMARK(1);
  block_sums<BC>(psum, s_red, mean);
  TB_PMARK(2);
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) {
    mean[bc] /= static_cast<float>(a.E);
    psum[bc] = 0.f;
    if (bc < nb) {
#pragma unroll
      for (int c = 0; c < kMaxChunks; ++c) {
        const int ch = tid + c * kPredThreads;
        if (ch < n_chunks) {
#pragma unroll
          for (int i = 0; i < EPL; ++i) {
            const float d = s_x[bc * e_pad + staged_pos<EPL>(ch * EPL + i)] - mean[bc];
            psum[bc] += d * d;
          }
        }
      }
    }
  }
  block_sums<BC>(psum, s_red, rstd);
  TB_PMARK(3);
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) rstd[bc] = 1.0f / sqrtf(rstd[bc] / static_cast<float>(a.E) + a.eps);
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const int ch = tid + c * kPredThreads;
    if (ch < n_chunks) {
      float gm[EPL], bt[EPL];
      Pack16<T>::load(static_cast<const T*>(a.gamma) + ch * EPL, gm);
      Pack16<T>::load(static_cast<const T*>(a.beta) + ch * EPL, bt);
#pragma unroll
      for (int bc = 0; bc < BC; ++bc) {
        if (bc < nb) {
#pragma unroll
          for (int i = 0; i < EPL; ++i) {
            float& x = s_x[bc * e_pad + staged_pos<EPL>(ch * EPL + i)];
            x = (x - mean[bc]) * rstd[bc] * gm[i] + bt[i];
          }
        }
      }
    }
  }
  }  // FUSED_LN
  __syncthreads();
  TB_PMARK(4);
  if (r >= a.hidden) return;

  float acc[BC];
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) acc[bc] = 0.f;
  // piece `lane` of block e0 / kStep: its 4-element group g sits at block start + (g*64 + lane)*4 (see staged_pos)
  auto consume = [&](const typename Pack16<T>::Raw& raw, int e0) {
    float wf[EPL];
    Pack16<T>::unpack(raw, wf);
    const float* x = s_x + (e0 - lane * EPL) + lane * 4;
    // every staged row takes part (rows past the batch hold zeros): no branch between the LDS
    // reads, so that all of a piece's reads are in flight together
#pragma unroll
    for (int g = 0; g < EPL / 4; ++g) {
#pragma unroll
      for (int bc = 0; bc < BC; ++bc) {
        const float4 xv = *reinterpret_cast<const float4*>(x + bc * e_pad + g * kWave * 4);
        acc[bc] = fmaf(wf[4 * g], xv.x, acc[bc]);
        acc[bc] = fmaf(wf[4 * g + 1], xv.y, acc[bc]);
        acc[bc] = fmaf(wf[4 * g + 2], xv.z, acc[bc]);
        acc[bc] = fmaf(wf[4 * g + 3], xv.w, acc[bc]);
      }
    }
  };
#pragma unroll
  for (int i = 0; i < kRowLoads; ++i) {
    const int e0 = lane * EPL + i * kStep;
    if (e0 < a.E) consume(wraw[i], e0);
  }
  for (int e0 = lane * EPL + kRowLoads * kStep; e0 < a.E; e0 += kStep) consume(Pack16<T>::load_raw(w + e0), e0);
  TB_PMARK(5);
#pragma unroll
  for (int bc = 0; bc < BC; ++bc) {
    const float s = wave_total(acc[bc]);
    if (lane == 0 && bc < nb)
      a.z[static_cast<int64_t>(b0 + bc) * a.hidden + r] = gelu_erf(s + to_float(static_cast<const T*>(a.b1)[r]));
  }
  TB_PMARK(6);
}

template <typename T, int BC>
__global__ __launch_bounds__(kPredThreads) void output_kernel(PredictArgs a) {
  constexpr int EPL = Pack16<T>::kElts;
  constexpr int kStep = kWave * EPL;
  extern __shared__ float s_z[];  // [BC][staged_len(hidden)]
  const int h_pad = staged_len<EPL>(a.hidden);
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int b0 = blockIdx.y * BC;
  const int nb = min(BC, a.B - b0);
  const int n_out = a.G * a.Hq * a.Dimp;
  const int o0 = (blockIdx.x * kPredWaves + wave) * kOutRowsPerWave;
  // first piece of every row of this wave, issued before the activations are staged
  typename Pack16<T>::Raw wraw[kOutRowsPerWave];
  const int e_first = lane * EPL;
#pragma unroll
  for (int rr = 0; rr < kOutRowsPerWave; ++rr) {
    const int o = (o0 + rr < n_out) ? o0 + rr : n_out - 1;
    wraw[rr] = Pack16<T>::load_raw(static_cast<const T*>(a.W2) + static_cast<int64_t>(o) * a.hidden +
                                   (e_first < a.hidden ? e_first : 0));
  }
  for (int i = tid; i < nb * a.hidden; i += kPredThreads)
    s_z[(i / a.hidden) * h_pad + staged_pos<EPL>(i % a.hidden)] = a.z[static_cast<int64_t>(b0) * a.hidden + i];
  for (int i = nb * h_pad + tid; i < BC * h_pad; i += kPredThreads) s_z[i] = 0.f;  // rows past the batch
  __syncthreads();
#pragma unroll
  for (int rr = 0; rr < kOutRowsPerWave; ++rr) {
    const int o = o0 + rr;
    if (o >= n_out) break;  // the same for the whole wave
    const T* w = static_cast<const T*>(a.W2) + static_cast<int64_t>(o) * a.hidden;
    float acc[BC];
#pragma unroll
    for (int bc = 0; bc < BC; ++bc) acc[bc] = 0.f;
    auto consume = [&](const typename Pack16<T>::Raw& raw, int e0) {
      float wf[EPL];
      Pack16<T>::unpack(raw, wf);
      const float* zz = s_z + (e0 - lane * EPL) + lane * 4;
#pragma unroll
      for (int g = 0; g < EPL / 4; ++g) {
#pragma unroll
        for (int bc = 0; bc < BC; ++bc) {
          const float4 zv = *reinterpret_cast<const float4*>(zz + bc * h_pad + g * kWave * 4);
          acc[bc] = fmaf(wf[4 * g], zv.x, acc[bc]);
          acc[bc] = fmaf(wf[4 * g + 1], zv.y, acc[bc]);
          acc[bc] = fmaf(wf[4 * g + 2], zv.z, acc[bc]);
          acc[bc] = fmaf(wf[4 * g + 3], zv.w, acc[bc]);
        }
      }
    };
    if (e_first < a.hidden) consume(wraw[rr], e_first);
    for (int e0 = e_first + kStep; e0 < a.hidden; e0 += kStep) consume(Pack16<T>::load_raw(w + e0), e0);
    const int slot = o / (a.Hq * a.Dimp), rest = o % (a.Hq * a.Dimp);
    const float bias = to_float(static_cast<const T*>(a.b2)[o]);
#pragma unroll
    for (int bc = 0; bc < BC; ++bc) {
      const float s = wave_total(acc[bc]);
      if (lane == 0 && bc < nb) {
        T* dst = static_cast<T*>(a.q_imp) +
                 (static_cast<int64_t>(slot) * a.B + (b0 + bc)) * (a.Hq * a.Dimp) + rest;
        store_elt(dst, s + bias);
      }
    }
  }
}

template <typename T, int BC>
tb_status launch_tb(const PredictArgs& a, hipStream_t st) {
  const unsigned chunks = static_cast<unsigned>((a.B + BC - 1) / BC);
  {
    dim3 grid(static_cast<unsigned>((a.hidden + kPredWaves - 1) / kPredWaves), chunks);
    const size_t lds = static_cast<size_t>(BC) * staged_len<Pack16<T>::kElts>(a.E) * sizeof(float);
    if (lds + 64 > 64 * 1024) {
      // more than the default 64 KiB of LDS per workgroup has to be asked for (once per process)
      static const hipError_t raised =
          hipFuncSetAttribute(reinterpret_cast<const void*>(&hidden_kernel<T, BC, (BC <= 2)>),
                              hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBudget);
      if (raised != hipSuccess) return TB_ERR_HIP;
    }
    if constexpr (BC > 2) {
      if (!a.xln) return TB_ERR_INVALID_ARG;
      hipLaunchKernelGGL((ln_kernel<T>), dim3(a.B), dim3(kPredThreads), 0, st, a);
      if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
    }
    hipLaunchKernelGGL((hidden_kernel<T, BC, (BC <= 2)>), grid, dim3(kPredThreads), lds, st, a);
    if (hipGetLastError() != hipSuccess) return TB_ERR_HIP;
  }
  {
    const int n_out = a.G * a.Hq * a.Dimp;
    const int rows_per_wg = kPredWaves * kOutRowsPerWave;
    dim3 grid(static_cast<unsigned>((n_out + rows_per_wg - 1) / rows_per_wg), chunks);
    const size_t lds = static_cast<size_t>(BC) * staged_len<Pack16<T>::kElts>(a.hidden) * sizeof(float);
    hipLaunchKernelGGL((output_kernel<T, BC>), grid, dim3(kPredThreads), lds, st, a);
  }
  return hip_status(hipGetLastError());
}

template <typename T>
tb_status launch_t(const PredictArgs& a, hipStream_t st) {
  // as many batch rows per workgroup as the batch has and the LDS holds (fp32 rows of E)
  int bc = 8;
  while (bc > 1 && (bc / 2 >= a.B || static_cast<size_t>(bc) * staged_len<Pack16<T>::kElts>(a.E) * sizeof(float) > kLdsBudget)) bc >>= 1;
  switch (bc) {
    case 1: return launch_tb<T, 1>(a, st);
    case 2: return launch_tb<T, 2>(a, st);
    case 4: return launch_tb<T, 4>(a, st);
    default: return launch_tb<T, 8>(a, st);
  }
}

}  // namespace

tb_status launch_predict(const PredictLaunch& L, hipStream_t st) {
  if (L.B == 0) return TB_OK;
  if (L.E > kMaxE || L.hidden > kMaxHidden) return TB_ERR_UNSUPPORTED;
  PredictArgs a;
  a.h = L.h;
  a.gamma = L.gamma;
  a.beta = L.beta;
  a.W1 = L.W1;
  a.b1 = L.b1;
  a.W2 = L.W2;
  a.b2 = L.b2;
  a.z = L.z;
  a.xln = L.xln;
  a.q_imp = L.q_imp;
  a.B = L.B;
  a.E = L.E;
  a.hidden = L.hidden;
  a.G = L.G;
  a.Hq = L.Hq;
  a.Dimp = L.Dimp;
  a.eps = L.eps;
  return L.dtype == TB_F32 ? launch_t<float>(a, st) : launch_t<bf16_t>(a, st);
}

}  // namespace tb
